"""Seeded synthetic inputs for the pruned prefill layer.

This module only draws random tensors with the shapes and value distributions of the five
workloads; it contains none of the method's arithmetic, so both the HIP path's tests and the CPU
checker can be fed from it.  Everything is generated on the host with NumPy's PCG64 and, for the
bf16 workloads, rounded to bfloat16 once, so every consumer reads the same bits.

Draw order per workload (fixed): hidden states x, planted-token indices or block ranks, then for a
layer Wq, Wk, Wv, Wo, Wgate, Wup, Wdown, each from its own generator seeded with (seed, 1000 + layer,
index), so a process never has to hold all layers on the host and matrices can be drawn in parallel.
Weights are N(0, 0.02^2); RMSNorm gains are exactly 1.  The LLaMA-shaped workloads have no biases; the
Qwen2.5-shaped ones add bq, bk, bv ~ N(0, 0.5^2) from generators (seed, 1000 + layer, 7..9).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace

import numpy as np
import torch


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str            # "fp32" | "bf16"
    seq: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    block: int
    unit: int
    window: int
    keep_ratio: float
    seed: int
    x_kind: str           # "planted" | "zipf" | "normal"
    planted: int = 0      # number of x4 tokens
    n_layers: int = 1
    schedule: dict = field(default_factory=dict)   # layer -> keep ratio of incoming blocks
    rope_theta: float = 500000.0
    rms_eps: float = 1e-5
    qkv_bias: bool = False
    family: str = "LLaMA-3.1-8B"

    @property
    def n_blocks(self) -> int:
        return (self.seq + self.block - 1) // self.block

    @property
    def n_keep(self) -> int:
        return keep_count(self.keep_ratio, self.n_blocks)

    @property
    def n_kept_tokens(self) -> int:
        return kept_tokens(self.seq, self.block, self.n_keep)


def keep_count(ratio: float, nb: int, n_forced: int = 2) -> int:
    """Blocks retained for a keep ratio: ceil(ratio*nb) clamped to [#forced, nb]."""
    return int(min(nb, max(min(n_forced, nb), math.ceil(ratio * nb - 1e-12))))


def kept_tokens(n_tokens: int, block: int, n_keep: int) -> int:
    """Tokens in n_keep blocks when the (possibly short) last block is among them."""
    nb = (n_tokens + block - 1) // block
    if n_keep >= nb:
        return n_tokens
    return (n_keep - 1) * block + (n_tokens - (nb - 1) * block)


_LLAMA = dict(hidden=4096, n_q_heads=32, n_kv_heads=8, head_dim=128, ffn=14336, unit=8)
_QWEN = dict(hidden=3584, n_q_heads=28, n_kv_heads=4, head_dim=128, ffn=18944, unit=8, rope_theta=1000000.0,
             rms_eps=1e-6, qkv_bias=True, family="Qwen2.5-7B")

WORKLOADS = {
    "cfg1": Workload("cfg1", "fp32", 512, 256, 4, 2, 64, 688, 16, 8, 32, 0.5, 0, "planted", planted=8),
    "cfg2": Workload("cfg2", "bf16", 8192, block=64, window=64, keep_ratio=0.5, seed=1,
                     x_kind="planted", planted=82, **_LLAMA),
    "cfg3": Workload("cfg3", "bf16", 32768, block=64, window=64, keep_ratio=0.3, seed=2,
                     x_kind="zipf", **_LLAMA),
    "cfg4": Workload("cfg4", "bf16", 131072, block=128, window=128, keep_ratio=0.2, seed=3,
                     x_kind="planted", planted=655, **_LLAMA),
    "cfg5": Workload("cfg5", "bf16", 32768, block=64, window=64, keep_ratio=1.0, seed=4,
                     x_kind="normal", n_layers=32, schedule={8: 0.5, 16: 0.25, 24: 0.125}, **_LLAMA),
    # Second model family of the paper's evaluation (Section 5.1: Qwen2.5-7B-Instruct, pruning at layers
    # 9/18/26 down to 12k/6k/4k tokens).  The layer shapes are not in the paper; they are the public model
    # card's (28 layers, hidden 3584, 28 query / 4 kv heads of 128, FFN 18944, Q/K/V bias, theta 1e6).
    "cfg6": Workload("cfg6", "bf16", 32768, block=64, window=64, keep_ratio=0.375, seed=5,
                     x_kind="zipf", **_QWEN),
    # The schedule the paper uses for LLaMA-3.1-8B (Section 5.1: pruning at layers 10/20/30 down to 8k/4k/2k of a 32k
    # prompt, i.e. 0.25/0.5/0.5 of the incoming blocks), on the same random-init layer shapes as cfg5.
    "cfg8": Workload("cfg8", "bf16", 32768, block=64, window=64, keep_ratio=1.0, seed=7,
                     x_kind="normal", n_layers=32, schedule={10: 0.25, 20: 0.5, 30: 0.5}, **_LLAMA),
    "cfg7": Workload("cfg7", "bf16", 32768, block=64, window=64, keep_ratio=1.0, seed=6,
                     x_kind="normal", n_layers=28, schedule={9: 0.375, 18: 0.5, 26: 0.66666}, **_QWEN),
}


def scaled(wl: Workload, **changes) -> Workload:
    """A smaller or otherwise altered copy of a workload (for tests that span a few tiles)."""
    return replace(wl, **changes)


def _store(a: np.ndarray, dtype: str) -> torch.Tensor:
    t = torch.from_numpy(a)
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def hidden_states(wl: Workload) -> torch.Tensor:
    """x[seq, hidden] for the workload, stored in its dtype."""
    rng = np.random.default_rng(wl.seed)
    x = rng.standard_normal((wl.seq, wl.hidden), dtype=np.float32)
    if wl.x_kind == "planted":
        idx = rng.choice(wl.seq, size=min(wl.planted, wl.seq), replace=False)
        x[idx] *= 4.0
    elif wl.x_kind == "zipf":
        nb = wl.n_blocks
        rank = rng.permutation(nb) + 1
        scale = rank.astype(np.float64) ** -1.1
        x *= np.repeat(scale, wl.block)[: wl.seq, None].astype(np.float32)
    return _store(x, wl.dtype)


WEIGHT_NAMES = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")


def weight_shapes(wl: Workload) -> dict:
    qd, kvd = wl.n_q_heads * wl.head_dim, wl.n_kv_heads * wl.head_dim
    return dict(wq=(qd, wl.hidden), wk=(kvd, wl.hidden), wv=(kvd, wl.hidden), wo=(wl.hidden, qd),
                w_gate=(wl.ffn, wl.hidden), w_up=(wl.ffn, wl.hidden), w_down=(wl.hidden, wl.ffn))


def _one_weight(args):
    seed, layer, idx, shp, dtype = args
    rng = np.random.default_rng([seed, 1000 + layer, idx])
    return _store(0.02 * rng.standard_normal(shp, dtype=np.float32), dtype)


def layer_weights(wl: Workload, layer: int = 0, pool=None) -> dict:
    """Dict of [out, in] weight tensors plus unit gains, stored in the workload's dtype.  Each matrix has
    its own generator seeded with (seed, 1000 + layer, index in WEIGHT_NAMES), so matrices can be drawn
    concurrently (`pool`: a concurrent.futures executor) without changing their values."""
    jobs = [(wl.seed, layer, i, shp, wl.dtype) for i, shp in enumerate(weight_shapes(wl).values())]
    mats = list(pool.map(_one_weight, jobs)) if pool is not None else [_one_weight(j) for j in jobs]
    out = dict(zip(weight_shapes(wl).keys(), mats))
    ones = np.ones(wl.hidden, dtype=np.float32)
    out["g_attn"] = _store(ones, wl.dtype)
    out["g_ffn"] = _store(ones.copy(), wl.dtype)
    if wl.qkv_bias:
        for i, name in enumerate(("q", "k", "v")):
            rng = np.random.default_rng([wl.seed, 1000 + layer, 7 + i])
            out["b" + name] = _store(0.5 * rng.standard_normal(out["w" + name].shape[0], dtype=np.float32), wl.dtype)
    return out


def model_weights(wl: Workload, layers=None, workers: int = 8):
    """Yields (layer, weights dict) for the chosen layers of a multi-layer workload, drawing the
    matrices on a thread pool (NumPy's generators release the GIL while they fill an array)."""
    from concurrent.futures import ThreadPoolExecutor
    layers = range(wl.n_layers) if layers is None else layers
    with ThreadPoolExecutor(max_workers=workers) as pool:
        for l in layers:
            yield l, layer_weights(wl, l, pool)


def positions(wl: Workload) -> torch.Tensor:
    return torch.arange(wl.seq, dtype=torch.int32)


def stage_qk(wl: Workload, skew: bool = True):
    """Direct inputs for the scoring stage alone: a query window q_win[w, Hq, d] and keys
    k[seq, Hkv, d] ~ N(0,1); with `skew`, each block's keys carry a Zipf(1.1) scale so the block
    scores are strongly skewed (the layer-level RMSNorm would cancel such a scale)."""
    rng = np.random.default_rng([wl.seed, 77])
    q = rng.standard_normal((wl.window, wl.n_q_heads, wl.head_dim), dtype=np.float32)
    k = rng.standard_normal((wl.seq, wl.n_kv_heads, wl.head_dim), dtype=np.float32)
    if skew:
        rank = rng.permutation(wl.n_blocks) + 1
        scale = (rank.astype(np.float64) ** -1.1).astype(np.float32)
        k *= np.repeat(scale, wl.block)[: wl.seq, None, None]
    return _store(q, wl.dtype), _store(k, wl.dtype)


def stage_qkv(n: int, n_q_heads: int, n_kv_heads: int, head_dim: int, dtype: str, seed: int):
    """Direct inputs for the attention stage alone: q[n,Hq,d], k,v[n,Hkv,d] ~ N(0,1)."""
    rng = np.random.default_rng([seed, 78])
    q = rng.standard_normal((n, n_q_heads, head_dim), dtype=np.float32)
    k = rng.standard_normal((n, n_kv_heads, head_dim), dtype=np.float32)
    v = rng.standard_normal((n, n_kv_heads, head_dim), dtype=np.float32)
    return _store(q, dtype), _store(k, dtype), _store(v, dtype)
