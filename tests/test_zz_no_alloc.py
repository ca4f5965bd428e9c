"""The entry point that allocates nothing (slim_score_blocks_static: the window query travels through an array
in the library's device image instead of a caller workspace) against slim_score_blocks, through the C ABI.
Two calls in a row, the second with a smaller input, so that what the first call left in the array would show."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import slim_oracle as so

pytestmark = pytest.mark.gpu


def _rand(shape, dtype, seed):
    g = torch.Generator().manual_seed(seed)
    return torch.randn(*shape, generator=g, dtype=torch.float32).to(dtype)


def _raw_static(lib, q, k, block, unit, scores):
    """The raw C call: device pointers and sizes only, the default stream."""
    w, Hq, d = q.shape
    N, Hkv, _ = k.shape
    code = 1 if k.dtype == torch.bfloat16 else 0
    return lib.slim_score_blocks_static(ctypes.c_void_p(q.data_ptr()), ctypes.c_void_p(k.data_ptr()), N, w, Hq, Hkv, d,
                                        block, unit, code, ctypes.c_void_p(scores.data_ptr()), ctypes.c_void_p(0))


def test_static_scratch_scores_equal_workspace_scores_on_two_calls():
    import paper_2508_06447_amd as slim
    lib = slim.load_library()
    dev = torch.device("cuda:0")
    # (N, block, unit, window, Hq, Hkv, d, dtype): a LLaMA-shaped call, then smaller ones whose window query is
    # shorter than what the call before left in the array
    calls = [(4096 + 40, 64, 8, 64, 32, 8, 128, torch.bfloat16),
             (700, 32, 8, 5, 8, 2, 64, torch.bfloat16),
             (130, 32, 1, 3, 4, 1, 16, torch.float32)]
    for n, (N, block, unit, w, Hq, Hkv, d, dtype) in enumerate(calls):
        print(f"static-scratch score call {n}: N={N} B={block} u={unit} w={w} H={Hq}/{Hkv} d={d} {dtype}", flush=True)
        q, k = _rand((w, Hq, d), dtype, 100 + n).to(dev), _rand((N, Hkv, d), dtype, 200 + n).to(dev)
        nb = (N + block - 1) // block
        got = torch.full((nb,), float("nan"), dtype=torch.float32, device=dev)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        rc = _raw_static(lib, q, k, block, unit, got)
        assert rc == 0, (rc, lib.slim_last_hip_error())
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        ref = slim.slim_score_blocks(q, k, block, unit)
        torch.cuda.synchronize()
        assert torch.equal(got, ref), (got - ref).abs().max()          # same kernels: bit for bit
        want = so.block_scores(q.double().cpu().numpy(), k.double().cpu().numpy(), block, unit)
        np.testing.assert_allclose(got.double().cpu().numpy(), want, atol=2e-5 * max(np.abs(want).max(), 1.0), rtol=1e-4)
    # the binding's function of the same name, same result
    N, block, unit, w, Hq, Hkv, d, dtype = calls[1]
    q, k = _rand((w, Hq, d), dtype, 101).to(dev), _rand((N, Hkv, d), dtype, 201).to(dev)
    out = torch.empty((N + block - 1) // block, dtype=torch.float32, device=dev)
    assert torch.equal(slim.slim_score_blocks_static(q, k, block, unit, out), slim.slim_score_blocks(q, k, block, unit))


def test_static_scratch_rejects_sizes_beyond_its_array():
    import paper_2508_06447_amd as slim
    lib = slim.load_library()
    one, null = ctypes.c_void_p(256), ctypes.c_void_p(0)
    # Hkv * d = 8320 > 8192 floats of scratch
    assert lib.slim_score_blocks_static(one, one, 64, 4, 65, 65, 128, 64, 8, 1, one, null) == -2
    assert lib.slim_score_blocks_static(null, one, 64, 4, 8, 8, 128, 64, 8, 1, one, null) == -1
    assert lib.slim_score_blocks_static(one, one, 64, 4, 8, 8, 128, 64, 128, 1, one, null) == -1      # unit > block
