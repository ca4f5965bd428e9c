"""Host-side checks of the assembly generators (csrc/gen_*.py): the wait-state padding and the order of the
attention loop that the lazily moved softmax reference relies on.  No GPU."""
import importlib.util
import os

import pytest

CSRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2508_06447_amd", "csrc")


def load(name):
    spec = importlib.util.spec_from_file_location(name, os.path.join(CSRC, name + ".py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


@pytest.fixture(scope="module")
def ga():
    return load("gen_attn_asm")


def slots_between(seq, i, j, ga):
    return sum(ga.weight(x) for x in seq[i + 1:j])


def test_padding_between_dependent_instructions(ga):
    mf = ga.Ins("v_mfma_f32_32x32x16_bf16 v[0:15], v[100:103], a[0:3], 0", "mfma", r=ga.vr(100, 4) + ga.ar(0, 4), w=ga.vr(0, 16))
    use = ga.valu("v_exp_f32 v20, v3", r=ga.vr(3), w=ga.vr(20), kind="trans")
    dep = ga.valu("v_add_f32 v21, v21, v20", r=ga.vr(20) + ga.vr(21), w=ga.vr(21))
    other = ga.valu("v_mov_b32 v30, 0", w=ga.vr(30))
    out = ga.fix_hazards([mf, use, dep])
    i, j, k = out.index(mf), out.index(use), out.index(dep)
    assert slots_between(out, i, j, ga) >= 12            # matrix result -> vector ALU
    assert slots_between(out, j, k, ga) >= 1             # transcendental -> use
    # enough independent work in between: nothing is added
    filler = [ga.valu(f"v_mov_b32 v{40 + n}, 0", w=ga.vr(40 + n)) for n in range(12)]
    out = ga.fix_hazards([mf] + filler + [use, other, dep])
    assert not any(x.kind == "nop" for x in out)
    # vector ALU -> matrix operand
    wr = ga.valu("v_cvt_pk_bf16_f32 v100, v50, v51", r=ga.vr(50, 2), w=ga.vr(100))
    out = ga.fix_hazards([wr, mf])
    assert slots_between(out, out.index(wr), out.index(mf), ga) >= 2
    # accumulating on the same registers back to back needs nothing
    acc1 = ga.Ins("v_mfma_f32_32x32x16_bf16 v[0:15], v[100:103], a[0:3], v[0:15]", "mfma",
                  r=ga.vr(100, 4) + ga.ar(0, 4) + ga.vr(0, 16), w=ga.vr(0, 16))
    acc2 = ga.Ins("v_mfma_f32_32x32x16_bf16 v[0:15], v[104:107], a[4:7], v[0:15]", "mfma",
                  r=ga.vr(104, 4) + ga.ar(4, 4) + ga.vr(0, 16), w=ga.vr(0, 16))
    assert [x.kind for x in ga.fix_hazards([acc1, acc2])] == ["mfma", "mfma"]


@pytest.mark.parametrize("masked", [False, True])
def test_attention_loop_shape(ga, masked):
    body = ga.loop_body(masked, "t")
    kinds = [x.kind for x in body]
    assert kinds.count("mfma") == 128 and kinds.count("barrier") == 2 and kinds.count("vmem") == 16
    assert sum(1 for x in body if x.text.startswith("v_exp_f32")) == 128          # one exponential per logit
    checks = [x for x in body if x.text.startswith("s_cbranch_vccnz RARE_")]
    assert len(checks) == 4                                                        # one per 32-key unit
    # the hazard pass leaves the looped stream consistent: a second pass over two copies adds nothing
    assert ga.fix_hazards(body, history=body, verify=True) == 0


@pytest.mark.parametrize("masked", [False, True])
def test_no_probability_is_used_before_its_unit_is_checked(ga, masked):
    """Between two consecutive checks the PV MFMAs may read only bf16 pairs written before the earlier check (the
    unit that check has passed): a pair register written in the segment belongs to the unit whose check is still
    ahead, so no MFMA of the segment may read it afterwards.  The same must hold across the loop's back edge."""
    body = ga.loop_body(masked, "t")
    pb = {f"v{r}" for qt in (0, 1) for r in range(ga.PB[qt], ga.PB[qt] + 8)}
    two = body + body
    cuts = [i for i, x in enumerate(two) if x.text.startswith("s_cbranch_vccnz RARE_")]
    assert len(cuts) == 8
    reads = 0
    for a, b in zip(cuts, cuts[1:]):
        fresh = set()
        for x in two[a + 1:b + 1]:
            if x.kind == "mfma":
                assert not (x.r & fresh), f"{x.text} reads a pair written after the previous check"
                reads += len(x.r & pb)
            fresh |= (x.w & pb)
        assert fresh == pb                       # every pair of the next unit is formed before its check
    assert reads == 7 * 16 * 4                   # 16 PV MFMAs per unit, 4 pair registers each


def test_rare_path_renews_everything_the_check_covers(ga):
    """The path taken when a check fires: the unit's maxima from S (which the common path must have left whole:
    the exponentials write temporaries, never S), the shift of this unit's and the next unit's S, then all eight
    pairs per query sub-tile again with a fresh sum."""
    body = ga.loop_body(False, "t")
    sbuf = {f"v{r}" for r in range(0, 64)}
    for x in body:
        if x.kind in ("trans", "valu", "vcmp", "perm"):
            assert not (x.w & sbuf), f"{x.text} writes an S register on the common path"
    for j in range(4):
        cur, nxt = j & 1, (j + 1) & 1
        rare = ga.rare_block("t", j, 0)
        subs = [x for x in rare if x.text.startswith("v_sub_f32")]
        shifted = set().union(*(x.w for x in subs))
        want = {f"v{ga.S_BUF[b][qt] + v}" for b in (cur, nxt) for qt in (0, 1) for v in range(16)}
        assert shifted == want
        redo = ga.redo_block("t", j)
        pb = {f"v{r}" for qt in (0, 1) for r in range(ga.PB[qt], ga.PB[qt] + 8)}
        assert set().union(*(x.w for x in redo if x.text.startswith("v_cvt_pk_bf16_f32"))) == pb
        exps = [x for x in redo if x.text.startswith("v_exp_f32")]
        assert len(exps) == 32 and set().union(*(x.r for x in exps)) == {f"v{ga.S_BUF[cur][qt] + v}" for qt in (0, 1) for v in range(16)}
        first_sums = [x for x in redo if x.text.startswith("v_add_f32") and not (x.r & x.w)]
        assert len(first_sums) == 2              # each sub-tile's sum starts afresh


def test_gemm_loops_shape():
    gg = load("gen_gemm_asm")
    for cfg in ((4, 4, 1), (2, 4, 2), (4, 2, 1), (2, 2, 2)):
        sh = gg.Shape(*cfg)
        kt = sh.k_tile(0, False)
        kinds = [x.kind for x in kt]
        tw, ta, nw = cfg
        assert kinds.count("mfma") == 4 * tw * ta * nw and kinds.count("barrier") == 1
        assert kinds.count("lds") == 4 * (tw * nw + ta)                # every fragment of a k-step read once
        assert kinds.count("vmem") == sh.NLD                           # the tile two ahead, spread over the k-tile
        assert not any(x.kind in ("valu", "trans") for x in kt)        # no vector ALU work in the loop
