"""Host-side logic that needs no GPU: keep counts, kept-token counts, the schedule walk, workspace sizes."""
import ctypes as C

import pytest
import torch

import paper_2508_06447_amd as slim
from paper_2508_06447_amd import inputs


@pytest.fixture(scope="module")
def lib():
    import os
    if not os.path.exists(slim.LIB_PATH):
        from paper_2508_06447_amd.build import build_lib
        build_lib(verbose=False)
    return slim.load_library()


def test_workload_table_matches_the_stated_shapes():
    w = inputs.WORKLOADS
    assert [(w[k].n_blocks, w[k].n_keep, w[k].n_kept_tokens) for k in ("cfg1", "cfg2", "cfg3", "cfg4")] == \
        [(32, 16, 256), (128, 64, 4096), (512, 154, 9856), (1024, 205, 26240)]
    assert inputs.keep_count(0.0, 10) == 2 and inputs.keep_count(1.0, 10) == 10 and inputs.keep_count(0.5, 1) == 1
    assert inputs.kept_tokens(45, 8, 3) == 21 and inputs.kept_tokens(45, 8, 9) == 45


def test_schedule_keep_counts_and_model_token_walk(lib):
    wl = inputs.WORKLOADS["cfg5"]
    keeps = slim.schedule_keep_counts(wl.seq, wl.block, wl.n_layers, wl.schedule)
    assert len(keeps) == 32 and keeps[8] == 256 and keeps[16] == 64 and keeps[24] == 8 and sum(1 for k in keeps if k) == 3
    shape = slim.make_shape(wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn, wl.block, wl.unit, wl.window,
                            torch.bfloat16)
    arr = (C.c_int * 32)(*keeps)
    assert lib.slim_prefill_model_tokens(C.byref(shape), 32, arr, wl.seq) == 512
    need = lib.slim_prefill_model_workspace_bytes(C.byref(shape), 32, arr, wl.seq)
    layer0 = slim.pruned_layer_workspace_bytes(shape, wl.seq, wl.n_blocks)
    assert need >= layer0 + 2 * wl.seq * wl.hidden * 2
    # a schedule that asks for fewer blocks than are forced is rejected on the host
    bad = (C.c_int * 32)(*([0] * 8 + [1] + [0] * 23))
    assert lib.slim_prefill_model_tokens(C.byref(shape), 32, bad, wl.seq) == 0
    assert lib.slim_prefill_model_workspace_bytes(C.byref(shape), 32, bad, wl.seq) == 0
    # ragged sequence: whole blocks survive plus the short last block
    keeps2 = slim.schedule_keep_counts(2085, 64, 5, {1: 0.5, 3: 0.25})
    assert keeps2 == [0, 17, 0, 5, 0]
    arr2 = (C.c_int * 5)(*keeps2)
    assert lib.slim_prefill_model_tokens(C.byref(shape), 5, arr2, 2085) == 4 * 64 + 37


def test_layer_workspace_grows_with_tokens_and_is_aligned(lib):
    shape = slim.make_shape(4096, 32, 8, 128, 14336, 64, 8, 64, torch.bfloat16)
    a = slim.pruned_layer_workspace_bytes(shape, 8192, 64)
    b = slim.pruned_layer_workspace_bytes(shape, 32768, 154)
    assert 0 < a < b and a % 256 == 0 and b % 256 == 0


def test_generators_are_seeded_and_per_matrix():
    wl = inputs.scaled(inputs.WORKLOADS["cfg2"], seq=64, hidden=64, ffn=128, n_q_heads=2, n_kv_heads=1, head_dim=32)
    a, b = inputs.layer_weights(wl, 3), inputs.layer_weights(wl, 3)
    assert all(torch.equal(a[k], b[k]) for k in a)
    c = inputs.layer_weights(wl, 4)
    assert not torch.equal(a["wq"], c["wq"])
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(4) as pool:
        d = inputs.layer_weights(wl, 3, pool)
    assert all(torch.equal(a[k], d[k]) for k in a)
    x1, x2 = inputs.hidden_states(wl), inputs.hidden_states(wl)
    assert torch.equal(x1, x2) and x1.dtype == torch.bfloat16 and float(a["g_attn"].float().min()) == 1.0


def test_product_and_oracle_do_not_know_each_other():
    """The package never imports the oracle (no CPU fallback can hide in it), the oracle never imports the package,
    and outside tests/ the oracle is imported only inside bench.py's cpu_baseline and __graft_entry__.smoke()."""
    import ast
    import os
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

    def imported(path):
        tree = ast.parse(open(path).read())
        mods = set()
        for node in ast.walk(tree):
            if isinstance(node, ast.Import):
                mods |= {a.name.split(".")[0] for a in node.names}
            elif isinstance(node, ast.ImportFrom) and node.level == 0 and node.module:
                mods.add(node.module.split(".")[0])
        return mods

    pkg = os.path.join(root, "paper_2508_06447_amd")
    for f in os.listdir(pkg):
        if f.endswith(".py"):
            assert "oracle" not in imported(os.path.join(pkg, f)), f
    for f in os.listdir(os.path.join(root, "oracle")):
        if f.endswith(".py"):
            assert "paper_2508_06447_amd" not in imported(os.path.join(root, "oracle", f)), f
    # top-level scripts: the oracle only inside the named functions
    for script, allowed in (("bench.py", {"cpu_baseline"}), ("__graft_entry__.py", {"smoke"})):
        tree = ast.parse(open(os.path.join(root, script)).read())
        for fn in [n for n in ast.walk(tree) if isinstance(n, (ast.FunctionDef, ast.Module))]:
            own = [n for n in (fn.body if isinstance(fn, ast.Module) else ast.walk(fn))
                   if isinstance(n, (ast.Import, ast.ImportFrom))]
            for n in own:
                names = [a.name for a in n.names] if isinstance(n, ast.Import) else [n.module or ""]
                if any(m.split(".")[0] == "oracle" for m in names):
                    assert isinstance(fn, ast.FunctionDef) and fn.name in allowed, (script, getattr(fn, "name", "module"))


def test_binding_fails_loudly_without_the_library(tmp_path):
    from paper_2508_06447_amd import binding
    with pytest.raises(FileNotFoundError):
        binding.load_library(str(tmp_path / "libslim.so"))
    with pytest.raises(ValueError):
        binding._dev(torch.zeros(4), "x")                 # a CPU tensor is refused, not silently computed on
