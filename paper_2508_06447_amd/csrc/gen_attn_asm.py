#!/usr/bin/env python3
"""Writes the body of the bf16 prefill-attention kernel ("Attention" stage of Fig. 2) as one block of gfx950
assembly: attn_bf16_body.inc (the instructions, as C string literals) and attn_bf16_clobbers.inc (the registers
the block uses).  csrc/attn.hip includes both inside an asm statement; its C++ part computes the per-lane and
per-workgroup constants that the block takes as operands.  Run `python gen_attn_asm.py` after changing this file;
the two .inc files are committed, so building the library needs no Python step.

Why assembly: a wave owns 64 queries (two 32-query sub-tiles), so every K and V^T fragment read from LDS feeds two
MFMAs.  That takes 128 accumulator registers for O, 64 for the Query fragments and 64 for two S tiles per lane: more
than 256, so a SIMD holds one wave with the O accumulators and the Query fragments in the accumulation registers
(a0-a191) and everything the vector ALU touches in v0-v231.  The compiler does not find that split, and with one
wave per SIMD the order of matrix, vector and LDS instructions inside the wave is the whole schedule, so it is
written out here.

Schedule.  A unit is 32 keys x 64 queries.  For unit u the wave runs
  A(u): 16 MFMAs S(u+1) = K Q^T - reference, dealt between them: P(u) = exp2(S(u)) for 10 of its 16 values per
        query sub-tile (into temporaries: S(u) stays whole), their sum, conversion to bf16; at the end the test
        whether a lane's sum of P(u) exceeds 2^8;
  B(u): 16 MFMAs O += V^T P(u); between the second eight (the first eight still read the registers that the first
        bf16 pairs go to): the first 6 values of P(u+1).
The softmax reference of a query moves only on a path of its own, entered when that test fires, which is before any
P(u) has been used: a sum above 2^8 means that some logit may lie more than 8 above the reference (or that its
exponential overflowed).  There the per-query maximum of S(u) is taken, the reference moves up by it, S(u) and
S(u+1) are shifted, O and the row sums rescaled and P(u) formed again.  Testing the sums, which the row sums need
anyway, instead of the maxima of S saves 17 vector instructions of 100 per unit; every vector instruction between
the MFMAs of this loop costs about 1.8 cycles (measured by leaving groups of them out).
Fragments are read three MFMA pairs ahead into rings of registers.  K/V tiles of 128 keys (4 units) go from global
memory straight into LDS, two stages each; per tile the workgroup meets at two barriers placed in the middle of a
phase: one after which the K stage of the tile just finished is refilled, one for the V stage.  The last three
tiles of a workgroup (where keys can lie above queries) run a second copy of the loop that masks S where needed.
Every wave of a workgroup runs the same number of units (masked keys give P = 0), so the barriers line up.

Wait states between dependent instructions (matrix result -> vector ALU 12, vector ALU -> matrix operand 2,
transcendental -> use 1, compare -> select 2, ...) are checked on the finished instruction list and padded with
s_nop where a pair is too close; the numbers are the ones the compiler inserts for the same pairs on gfx950.
"""
import os
import re
import sys

# ----------------------------------------------------------------------------- register map
S_BUF = [[0, 16], [32, 48]]          # S buffers [buf][qt] -> first vgpr
NEGR = [64, 80]
PB = [96, 104]                       # P as bf16 pairs, 8 regs per qt
VRING, KRING = 112, 200              # 8 slots x 4 regs each
NRING = 8
KOFF, VOFF = 144, 152                # 8 + 4 LDS byte addresses
KOFS, VOFS = 156, 164                # global byte offsets of the tile loads (8 + 8)
REF, LRUN, TMAX = [172, 173], [174, 175], [176, 177]
LUNIT = TMAX                         # a lane's sum of P over the unit in progress (TMAX is free outside the rare path)
EARLY = 3                            # pairs of a unit whose P are formed during the unit before
EXPT = [188, 189, 190, 191]          # P in fp32 on its way to the row sum and the bf16 pair: two items in flight
LIMU = [178, 179]
TMP = 180                            # 180..199 temporaries
LAST_V, LAST_A = 231, 191
O_ACC, Q_ACC = 0, 128                # agprs: oacc[dt][qt] at (dt*2+qt)*16 ; qf[qt][st] at 128 + (qt*8+st)*4

S_T, S_K0N, S_KST, S_VST = 40, 42, 43, 44
S_KPTR, S_VPTR = 46, 48
S_TMP = 50                           # 50..59 scratch
S_RAGK, S_RAGV = 60, 62
S_RET, S_TLK, S_TLV, S_MASKC = 64, 65, 66, 67
S_SAVE = 68
FIRST_S, LAST_S = 40, 69
SUM_LIMIT, NINF, ONES_BF16 = "0x43800000", "0xff800000", "0x3f803f80"      # 2^8
AHEAD = 3


class Ins:
    __slots__ = ("text", "kind", "r", "w")

    def __init__(self, text, kind, r=(), w=()):
        self.text, self.kind, self.r, self.w = text, kind, set(r), set(w)


def vr(b, n=1): return [f"v{b + i}" for i in range(n)]
def ar(b, n=1): return [f"a{b + i}" for i in range(n)]
def sr(b, n=1): return [f"s{b + i}" for i in range(n)]
def V(b, n=1): return f"v{b}" if n == 1 else f"v[{b}:{b + n - 1}]"
def A(b, n=1): return f"a{b}" if n == 1 else f"a[{b}:{b + n - 1}]"
def S(b, n=1): return f"s{b}" if n == 1 else f"s[{b}:{b + n - 1}]"
def valu(t, r=(), w=(), kind="valu"): return Ins(t, kind, r, w)
def salu(t, r=(), w=()): return Ins(t, "salu", r, w)
def nop(n): return Ins(f"s_nop {n - 1}", "nop")
def label(name): return Ins(f"{name}:", "label")
def branch(t): return Ins(t, "branch")
def raw(t, kind="other", r=(), w=()): return Ins(t, kind, r, w)


# ----------------------------------------------------------------------------- building blocks
def mfma_qk(buf, qt, st, kbase, zero_c=False):
    d = S_BUF[buf][qt]
    q = Q_ACC + (qt * 8 + st) * 4
    if st == 0:
        c, cr = ("0", []) if zero_c else (V(NEGR[qt], 16), vr(NEGR[qt], 16))
    else:
        c, cr = V(d, 16), vr(d, 16)
    return Ins(f"v_mfma_f32_32x32x16_bf16 {V(d, 16)}, {V(kbase, 4)}, {A(q, 4)}, {c}", "mfma",
               r=vr(kbase, 4) + ar(q, 4) + cr, w=vr(d, 16))


def mfma_pv(dt, qt, step, vslot):
    o = O_ACC + (dt * 2 + qt) * 16
    p = PB[qt] + step * 4
    v = VRING + vslot * 4
    return Ins(f"v_mfma_f32_32x32x16_bf16 {A(o, 16)}, {V(v, 4)}, {V(p, 4)}, {A(o, 16)}", "mfma",
               r=vr(v, 4) + vr(p, 4) + ar(o, 16), w=ar(o, 16))


def ld_k(st, sub, dst):
    return [Ins(f"ds_read_b128 {V(dst, 4)}, {V(KOFF + st)} offset:{sub * 8192}", "lds", r=vr(KOFF + st), w=vr(dst, 4))]


def ld_v(dt, sub, step, vslot):
    v = VRING + vslot * 4
    off = (sub * 2 + step) * 4096
    return [Ins(f"ds_read_b64_tr_b16 {V(v, 2)}, {V(VOFF + dt)} offset:{off}", "lds", r=vr(VOFF + dt), w=vr(v, 2)),
            Ins(f"ds_read_b64_tr_b16 {V(v + 2, 2)}, {V(VOFF + dt)} offset:{off + 2048}", "lds", r=vr(VOFF + dt),
                w=vr(v + 2, 2))]


def exp_item(buf, qt, pair, slot, first):
    """P for two keys of one query sub-tile: exp2 into temporaries (S stays, for the path that moves the reference),
    their sum into the unit's sum (first: the sum starts with them), the bf16 pair."""
    s = S_BUF[buf][qt] + 2 * pair
    p = PB[qt] + pair
    t = EXPT[2 * slot]
    lu = LUNIT[qt]
    out = [valu(f"v_exp_f32 {V(t)}, {V(s)}", r=vr(s), w=vr(t), kind="trans"),
           valu(f"v_exp_f32 {V(t + 1)}, {V(s + 1)}", r=vr(s + 1), w=vr(t + 1), kind="trans")]
    if first:
        out.append(valu(f"v_add_f32 {V(lu)}, {V(t)}, {V(t + 1)}", r=vr(t, 2), w=vr(lu)))
    else:
        out.append(valu(f"v_add_f32 {V(lu)}, {V(lu)}, {V(t)}", r=vr(t) + vr(lu), w=vr(lu)))
        out.append(valu(f"v_add_f32 {V(lu)}, {V(lu)}, {V(t + 1)}", r=vr(t + 1) + vr(lu), w=vr(lu)))
    out.append(valu(f"v_cvt_pk_bf16_f32 {V(p)}, {V(t)}, {V(t + 1)}", r=vr(t, 2), w=vr(p)))
    return out


def exp_stream(buf, pairs, fresh):
    """The items of `pairs` for both query sub-tiles, the exponentials of an item issued ahead of the previous
    item's sum and conversion.  fresh: the first item of each sub-tile starts the unit's sum."""
    out, prev, started, n = [], None, set(), 0
    for p in pairs:
        for qt in (0, 1):
            sq = exp_item(buf, qt, p, n & 1, fresh and qt not in started)
            started.add(qt)
            n += 1
            out += sq[:2]
            if prev:
                out += prev[2:]
            prev = sq
    return out + prev[2:]


def sum_check():
    """vcc = some lane's part-of-unit sum exceeds 2^8: some logit may lie more than 8 above the reference (or the
    exponential overflowed), and nothing computed from these P has been used yet."""
    return [valu(f"v_max_f32 {V(TMP + 2)}, {V(LUNIT[0])}, {V(LUNIT[1])}", r=vr(LUNIT[0]) + vr(LUNIT[1]), w=vr(TMP + 2)),
            valu(f"v_cmp_lt_f32 vcc, {SUM_LIMIT}, {V(TMP + 2)}", r=vr(TMP + 2), w=["vcc"], kind="vcmp")]


def sum_commit():
    return [valu(f"v_add_f32 {V(LRUN[qt])}, {V(LRUN[qt])}, {V(LUNIT[qt])}", r=vr(LRUN[qt]) + vr(LUNIT[qt]), w=vr(LRUN[qt]))
            for qt in (0, 1)]


def max_local(buf):
    out = []
    for qt in (0, 1):
        s, m = S_BUF[buf][qt], TMAX[qt]
        out.append(valu(f"v_max_f32 {V(m)}, {V(s)}, {V(s + 1)}", r=vr(s, 2), w=vr(m)))
    for i in range(1, 8):
        for qt in (0, 1):
            s, m = S_BUF[buf][qt] + 2 * i, TMAX[qt]
            out.append(valu(f"v_max3_f32 {V(m)}, {V(m)}, {V(s)}, {V(s + 1)}", r=vr(m) + vr(s, 2), w=vr(m)))
    return out


def max_exchange():
    """Both 32-lane halves hold 16 keys of each query: combine the two partial maxima."""
    out = []
    for qt in (0, 1):
        out.append(valu(f"v_mov_b32 {V(TMP + qt)}, {V(TMAX[qt])}", r=vr(TMAX[qt]), w=vr(TMP + qt)))
    for qt in (0, 1):
        out.append(valu(f"v_permlane32_swap_b32 {V(TMAX[qt])}, {V(TMP + qt)}", r=vr(TMAX[qt]) + vr(TMP + qt),
                        w=vr(TMAX[qt]) + vr(TMP + qt), kind="perm"))
    for qt in (0, 1):
        out.append(valu(f"v_max_f32 {V(TMAX[qt])}, {V(TMAX[qt])}, {V(TMP + qt)}", r=vr(TMAX[qt]) + vr(TMP + qt), w=vr(TMAX[qt])))
    return out


def mask_block(buf):
    out = []
    for qt in (0, 1):
        out.append(valu(f"v_subrev_u32 {V(LIMU[qt])}, {S(S_K0N)}, %[limabs{qt}]", r=sr(S_K0N), w=vr(LIMU[qt])))
    out.append(valu(f"v_mov_b32 {V(TMP + 3)}, {NINF}", w=vr(TMP + 3)))
    for qt in (0, 1):
        for v0 in range(0, 16, 4):
            for j in range(4):
                v = v0 + j
                ko = 8 * (v >> 2) + (v & 3)
                sg = S_TMP + 2 * j
                out.append(valu(f"v_cmp_lt_i32 {S(sg, 2)}, {V(LIMU[qt])}, {ko}", r=vr(LIMU[qt]), w=sr(sg, 2), kind="vcmp"))
            for j in range(4):
                sj, sg = S_BUF[buf][qt] + v0 + j, S_TMP + 2 * j
                out.append(valu(f"v_cndmask_b32 {V(sj)}, {V(sj)}, {V(TMP + 3)}, {S(sg, 2)}", r=vr(sj) + vr(TMP + 3) + sr(sg, 2), w=vr(sj)))
    return out


def tile_load_instrs(which):
    ofs = KOFS if which == 0 else VOFS
    st, ptr = (S_KST, S_KPTR) if which == 0 else (S_VST, S_VPTR)
    out = []
    for i in range(8):
        out.append(salu(f"s_add_u32 m0, {S(st)}, {i * 4096}", r=sr(st), w=["m0", "scc"]))
        out.append(Ins(f"global_load_lds_dwordx4 {V(ofs + i)}, {S(ptr, 2)}", "vmem", r=vr(ofs + i) + ["m0"] + sr(ptr, 2)))
    return out


_uid = [0]


def ragged_switch(which):
    """Skippable block: when the tile to load next is the short last one, the lane offsets of the loads are
    recomputed with their rows clamped to the last row (a one-way switch: every later tile is that tile again)."""
    ofs, chunk, tl = (KOFS, "kchunk", S_TLK) if which == 0 else (VOFS, "vchunk", S_TLV)
    _uid[0] += 1
    name = f"RAGSKIP_{_uid[0]}"
    out = [salu(f"s_cmp_eq_u32 {S(tl)}, %[last_ragged]", r=sr(tl), w=["scc"]), branch(f"s_cbranch_scc0 {name}")]
    for i in range(8):
        t = TMP + 12 + (i & 1)
        out.append(valu(f"v_add_u32 {V(t)}, {16 * i}, %[r0]", w=vr(t)))
        out.append(valu(f"v_min_u32 {V(t)}, %[nl1], {V(t)}", r=vr(t), w=vr(t)))
        out.append(valu(f"v_mad_u32_u24 {V(ofs + i)}, {V(t)}, %[rowbytes], %[{chunk}]", r=vr(t), w=vr(ofs + i)))
    out.append(label(name))
    return out


def tile_advance(which):
    """After a tile's loads: next tile index; pointer moves on unless the last tile was reached; stage flips."""
    tl, st, ptr = (S_TLK, S_KST, S_KPTR) if which == 0 else (S_TLV, S_VST, S_VPTR)
    t0 = S_TMP + 8
    return [salu(f"s_add_u32 {S(tl)}, {S(tl)}, 1", r=sr(tl), w=sr(tl) + ["scc"]),
            salu(f"s_cmp_le_u32 {S(tl)}, %[last_tile]", r=sr(tl), w=["scc"]),
            salu(f"s_cselect_b32 {S(t0)}, %[tile_bytes], 0", r=["scc"], w=sr(t0)),
            salu(f"s_add_u32 {S(ptr)}, {S(ptr)}, {S(t0)}", r=sr(ptr) + sr(t0), w=sr(ptr) + ["scc"]),
            salu(f"s_addc_u32 {S(ptr + 1)}, {S(ptr + 1)}, 0", r=sr(ptr + 1) + ["scc"], w=sr(ptr + 1) + ["scc"]),
            salu(f"s_xor_b32 {S(st)}, {S(st)}, 0x10000", r=sr(st), w=sr(st) + ["scc"]),
            ragged_switch(which)]


def barrier_block():
    return [raw("s_waitcnt vmcnt(8)", "wait"), raw("s_barrier", "barrier")]


# ----------------------------------------------------------------------------- hazards
def needed_gap(prod, cons, reg):
    pk, ck = prod.kind, cons.kind
    if pk == "mfma":
        if ck == "mfma":
            return 0 if (reg in cons.w and reg in cons.r and cons.w == prod.w) else 14
        return 12
    if pk in ("valu", "trans", "dot", "perm", "vcmp"):
        if ck == "mfma":
            return 2
        if pk == "trans":
            return 1
        if pk == "dot":
            return 0 if ck == "dot" else 3
        if pk == "vcmp":
            return 2 if ck in ("valu", "trans", "dot", "perm", "vcmp") else 0
        if ck == "perm":
            return 2
        if ck == "vmem" and reg.startswith("s"):
            return 5
        return 0
    if pk == "salu":
        return 1 if (ck == "vmem" and reg == "m0") else 0
    return 0


def weight(ins):
    return int(ins.text.split()[1]) + 1 if ins.kind == "nop" else (0 if ins.kind == "label" else 1)


def fix_hazards(seq, history=(), verify=False):
    """Insert s_nop where a dependent pair is too close (straight-line view of seq, preceded by `history`)."""
    out = list(history)
    start = len(out)
    last_w = {}
    for i, ins in enumerate(out):
        for reg in ins.w:
            last_w[reg] = i
    added = 0
    for ins in seq:
        need = 0
        if ins.kind not in ("label", "branch", "nop", "wait", "barrier"):
            for reg in ins.r | ins.w:
                if reg in last_w:
                    pi = last_w[reg]
                    prod = out[pi]
                    if reg in ins.w and reg not in ins.r and prod.kind != "mfma":
                        continue
                    gap = needed_gap(prod, ins, reg)
                    if gap:
                        have = sum(weight(x) for x in out[pi + 1:])
                        need = max(need, gap - have)
        added += max(need, 0)
        while need > 0:
            k = min(need, 8)
            out.append(nop(k))
            need -= k
        out.append(ins)
        for reg in ins.w:
            last_w[reg] = len(out) - 1
    if verify:
        return added
    return out[start:]


# ----------------------------------------------------------------------------- loop body
def flat(items):
    out = []
    for x in items:
        if isinstance(x, list):
            out += flat(x)
        else:
            out.append(x)
    return out


def deal(groups, fills):
    """Spread fills (instructions, or lists that stay together) over the MFMAs of the groups."""
    n = 2 * len(groups)
    for i, f in enumerate(fills):
        slot = i * n // len(fills)
        groups[slot // 2]["fill"].append((slot & 1, f))


def build_groups(masked, tag):
    """One tile = 4 units.  masked: the version for the diagonal tiles, where each unit checks whether its keys
    can lie above some query of the wave (then S gets -inf there before the maxima)."""
    G = []
    kslot = vslot = 0
    for j in range(4):
        cur, nxt = j & 1, (j + 1) & 1
        sub_k = (j + 1) & 3
        ag = []
        for st in range(8):
            ks = KRING + (kslot % NRING) * 4
            ag.append(dict(frag=ld_k(st, sub_k, ks), mfma=[mfma_qk(nxt, 0, st, ks), mfma_qk(nxt, 1, st, ks)], fill=[], pre=[], post=[]))
            kslot += 1
        deal(ag, exp_stream(cur, range(EARLY, 8), fresh=False) + sum_check())
        ag[7]["post"] += [branch(f"s_cbranch_vccnz RARE_{tag}{j}"), label(f"BACK_{tag}{j}")] + sum_commit()
        if masked:
            ag[0]["pre"] += [salu(f"s_add_u32 {S(S_K0N)}, {S(S_K0N)}, 32", r=sr(S_K0N), w=sr(S_K0N) + ["scc"]),
                             salu(f"s_add_u32 {S(S_TMP)}, {S(S_K0N)}, 31", r=sr(S_K0N), w=sr(S_TMP) + ["scc"]),
                             salu(f"s_cmp_gt_i32 {S(S_TMP)}, %[qw0]", r=sr(S_TMP), w=["scc"]),
                             salu(f"s_cselect_b32 {S(S_MASKC)}, 1, 0", r=["scc"], w=sr(S_MASKC))]
        if j == 0:
            ag[4]["pre"] += barrier_block()
        G += ag
        bg = []
        for step in range(2):
            for dt in range(4):
                bg.append(dict(frag=ld_v(dt, j, step, vslot % NRING), mfma=[mfma_pv(dt, 0, step, vslot % NRING), mfma_pv(dt, 1, step, vslot % NRING)],
                               fill=[], pre=[], post=[]))
                vslot += 1
        deal(bg[4:], exp_stream(nxt, range(0, EARLY), fresh=True))
        if j == 2:
            bg[4]["pre"] += barrier_block()
            bg[4]["pre"] += [valu(f"v_xor_b32 {V(KOFF + st)}, 0x10000, {V(KOFF + st)}", r=vr(KOFF + st), w=vr(KOFF + st)) for st in range(8)]
        if masked:
            bg[4]["pre"] += [salu(f"s_cmp_lg_u32 {S(S_MASKC)}, 0", r=sr(S_MASKC), w=["scc"]), branch(f"s_cbranch_scc0 SKIPM_{tag}{j}"),
                             ("MASKBLOCK", nxt), label(f"SKIPM_{tag}{j}")]
        G += bg
    iy = 4                      # Y barrier sits before group 4 of A(0)
    deal(G[iy:iy + 12], tile_load_instrs(1) + tile_advance(1))
    ix = 2 * 16 + 8 + 4         # X barrier sits before group 4 of B(2)
    deal(G[ix:ix + 12], tile_load_instrs(0) + tile_advance(0))
    return G


def linearise(G, with_mask):
    n = len(G)
    seq = []
    queue = []
    for g in range(AHEAD):
        queue += [g] * len(G[g]["frag"])
    for gi, g in enumerate(G):
        for p in g["pre"]:
            if isinstance(p, tuple):
                if with_mask:
                    seq += mask_block(p[1])
            else:
                seq.append(p)
        seq += G[(gi + AHEAD) % n]["frag"]
        queue += [gi + AHEAD] * len(G[(gi + AHEAD) % n]["frag"])
        own = sum(1 for q in queue if q == gi)
        assert queue[:own] == [gi] * own, (gi, queue)
        if gi % 2 == 0:                     # one wait per two groups: also for the next group's fragment
            both = sum(1 for q in queue if q in (gi, gi + 1))
            after = len(queue) - both
            assert after <= 15
            seq.append(raw(f"s_waitcnt lgkmcnt({after})", "wait"))
        queue = queue[own:]
        for half in (0, 1):
            seq.append(g["mfma"][half])
            seq += flat([f for h, f in g["fill"] if h == half])
        seq += g["post"]
    assert queue == [n + i for i in range(AHEAD) for _ in G[i]["frag"]], queue
    return seq


def loop_body(masked, tag):
    G = build_groups(masked, tag)
    full = linearise(G, True)
    fixed = fix_hazards(full, history=full)          # second copy: wrap-around hazards included
    # the same stream with the skippable blocks (mask, ragged switch) left out must need no further padding
    skippable = {x.text for buf in (0, 1) for x in mask_block(buf)}
    skippable |= {x.text for w in (0, 1) for x in ragged_switch(w) if x.kind == "valu"}
    lean = [x for x in fixed if x.text not in skippable]
    extra = fix_hazards(lean, history=lean, verify=True)
    assert extra == 0, f"skipping a block exposes {extra} wait states"
    return fixed


def loop_tail(name, bound):
    out = [valu(f"v_xor_b32 {V(VOFF + dt)}, 0x10000, {V(VOFF + dt)}", r=vr(VOFF + dt), w=vr(VOFF + dt)) for dt in range(4)]
    out += [salu(f"s_add_u32 {S(S_T)}, {S(S_T)}, 1", r=sr(S_T), w=sr(S_T) + ["scc"]),
            salu(f"s_cmp_lt_u32 {S(S_T)}, {bound}", r=sr(S_T), w=["scc"]), branch(f"s_cbranch_scc1 {name}")]
    return out


# ----------------------------------------------------------------------------- rare path, prologue, epilogue
def rare_block(tag, j, ret):
    """Entered from unit j's check, behind all of its P and before any of them is used.  S of the unit is still whole:
    take its maximum per query, move the reference up by it (if positive), shift S of this unit and of the next (already
    computed against the old reference), rescale the row sums and, on the common path behind this block, O."""
    cur, nxt = j & 1, (j + 1) & 1
    out = [label(f"RARE_{tag}{j}"), nop(8), nop(8)] + max_local(cur) + max_exchange()
    for qt in (0, 1):
        d = TMP + 6 + qt
        out.append(valu(f"v_max_f32 {V(d)}, 0, {V(TMAX[qt])}", r=vr(TMAX[qt]), w=vr(d)))
        out.append(valu(f"v_add_f32 {V(REF[qt])}, {V(REF[qt])}, {V(d)}", r=vr(REF[qt]) + vr(d), w=vr(REF[qt])))
        for buf in (cur, nxt):
            for v in range(16):
                s = S_BUF[buf][qt] + v
                out.append(valu(f"v_sub_f32 {V(s)}, {V(s)}, {V(d)}", r=vr(s) + vr(d), w=vr(s)))
        out.append(valu(f"v_xor_b32 {V(TMP + 3)}, 0x80000000, {V(REF[qt])}", r=vr(REF[qt]), w=vr(TMP + 3)))
        for v in range(16):
            out.append(valu(f"v_mov_b32 {V(NEGR[qt] + v)}, {V(TMP + 3)}", r=vr(TMP + 3), w=vr(NEGR[qt] + v)))
        out.append(valu(f"v_exp_f32_e64 {V(TMP + 4 + qt)}, -{V(d)}", r=vr(d), w=vr(TMP + 4 + qt), kind="trans"))
    out.append(nop(2))
    for qt in (0, 1):
        out.append(valu(f"v_mul_f32 {V(LRUN[qt])}, {V(LRUN[qt])}, {V(TMP + 4 + qt)}", r=vr(LRUN[qt]) + vr(TMP + 4 + qt), w=vr(LRUN[qt])))
    out += [salu(f"s_mov_b32 {S(S_RET)}, {ret}", w=sr(S_RET)), branch("s_branch RESCALE")]
    return out


def redo_block(tag, j):
    """Behind the rescaling: the unit's P and their sum again, from the shifted S."""
    out = [label(f"REDO_{tag}{j}")] + exp_stream(j & 1, range(0, 8), fresh=True)
    out += [nop(4), branch(f"s_branch BACK_{tag}{j}")]
    return out


def rescale_block(returns):
    out = [label("RESCALE")]
    for dt in range(4):
        for qt in (0, 1):
            o = O_ACC + (dt * 2 + qt) * 16
            for v0 in range(0, 16, 4):
                for k in range(4):
                    out.append(valu(f"v_accvgpr_read_b32 {V(TMP + 16 + k)}, {A(o + v0 + k)}", r=ar(o + v0 + k), w=vr(TMP + 16 + k)))
                for k in range(4):
                    out.append(valu(f"v_mul_f32 {V(TMP + 16 + k)}, {V(TMP + 16 + k)}, {V(TMP + 4 + qt)}",
                                    r=vr(TMP + 16 + k) + vr(TMP + 4 + qt), w=vr(TMP + 16 + k)))
                for k in range(4):
                    out.append(valu(f"v_accvgpr_write_b32 {A(o + v0 + k)}, {V(TMP + 16 + k)}", r=vr(TMP + 16 + k), w=ar(o + v0 + k)))
    out += [nop(4)]
    for ret, name in returns:
        out += [salu(f"s_cmp_eq_u32 {S(S_RET)}, {ret}", r=sr(S_RET), w=["scc"]), branch(f"s_cbranch_scc1 {name}")]
    out += [branch("s_endpgm")]
    return out


def prologue():
    out = []
    e = out.append
    # Query rows first (raw, into v0..63), so that their latency passes under the address arithmetic, the tile loads
    # and the clearing of the accumulators; then scaled by scale*log2(e), rounded to bf16 again, into the Q agprs
    for qt in (0, 1):
        for ks in range(8):
            d = (qt * 8 + ks) * 4
            e(Ins(f"global_load_dwordx4 {V(d, 4)}, %[qrow{qt}], off offset:{ks * 32}", "vmem", w=vr(d, 4)))
    for st in range(8):
        e(valu(f"v_xor_b32 {V(KOFF + st)}, {st << 5}, %[koff0]", w=vr(KOFF + st)))
    for dt in range(4):
        e(valu(f"v_xor_b32 {V(VOFF + dt)}, {dt << 6}, %[voff0]", w=vr(VOFF + dt)))
    for i in range(8):
        t = TMP + 12
        e(valu(f"v_add_u32 {V(t)}, {16 * i}, %[r0]", w=vr(t)))
        e(valu(f"v_mad_u32_u24 {V(KOFS + i)}, {V(t)}, %[rowbytes], %[kchunk]", r=vr(t), w=vr(KOFS + i)))
        e(valu(f"v_mad_u32_u24 {V(VOFS + i)}, {V(t)}, %[rowbytes], %[vchunk]", r=vr(t), w=vr(VOFS + i)))
    # tile loads: K(0), V(0), K(1)
    e(salu(f"s_mov_b32 {S(S_KST)}, %[ldsw]", w=sr(S_KST)))
    e(salu(f"s_add_u32 {S(S_VST)}, %[ldsw], 0x8000", w=sr(S_VST) + ["scc"]))
    e(salu(f"s_mov_b32 {S(S_TLK)}, 0", w=sr(S_TLK)))
    e(salu(f"s_mov_b32 {S(S_TLV)}, 0", w=sr(S_TLV)))
    e(salu(f"s_mov_b32 {S(S_KPTR)}, %[kbase_lo]", w=sr(S_KPTR)))
    e(salu(f"s_mov_b32 {S(S_KPTR + 1)}, %[kbase_hi]", w=sr(S_KPTR + 1)))
    e(salu(f"s_mov_b32 {S(S_VPTR)}, %[vbase_lo]", w=sr(S_VPTR)))
    e(salu(f"s_mov_b32 {S(S_VPTR + 1)}, %[vbase_hi]", w=sr(S_VPTR + 1)))
    out += flat([ragged_switch(0), ragged_switch(1)])
    out += flat(tile_load_instrs(0) + tile_advance(0) + tile_load_instrs(1) + tile_advance(1) + tile_load_instrs(0) + tile_advance(0))
    for i in range(128):
        e(valu(f"v_accvgpr_write_b32 {A(O_ACC + i)}, 0", w=ar(O_ACC + i)))
    for qt in (0, 1):
        e(valu(f"v_mov_b32 {V(LRUN[qt])}, 0", w=vr(LRUN[qt])))
    e(salu(f"s_mov_b32 {S(S_T)}, 0", w=sr(S_T)))
    e(salu(f"s_mov_b32 {S(S_K0N)}, 0", w=sr(S_K0N)))
    e(raw("s_waitcnt vmcnt(24)", "wait"))       # the Query rows are there; the 24 tile loads may still be in flight
    for i in range(64):
        lo, hi = TMP + 2 * (i & 3), TMP + 2 * (i & 3) + 1
        e(valu(f"v_lshlrev_b32 {V(lo)}, 16, {V(i)}", r=vr(i), w=vr(lo)))
        e(valu(f"v_and_b32 {V(hi)}, 0xffff0000, {V(i)}", r=vr(i), w=vr(hi)))
        e(valu(f"v_mul_f32 {V(lo)}, %[scale], {V(lo)}", r=vr(lo), w=vr(lo)))
        e(valu(f"v_mul_f32 {V(hi)}, %[scale], {V(hi)}", r=vr(hi), w=vr(hi)))
        e(valu(f"v_cvt_pk_bf16_f32 {V(lo)}, {V(lo)}, {V(hi)}", r=vr(lo) + vr(hi), w=vr(lo)))
        e(valu(f"v_accvgpr_write_b32 {A(Q_ACC + i)}, {V(lo)}", r=vr(lo), w=ar(Q_ACC + i)))
    e(raw("s_waitcnt vmcnt(16)", "wait"))       # K(0) is there; V(0) and K(1) are waited for at the loop's own barriers
    e(raw("s_barrier", "barrier"))
    # S(0): K fragments of unit 0 into the second S buffer's registers (free for now), 16 MFMAs from zero
    for st in range(8):
        out += ld_k(st, 0, S_BUF[1][0] + 4 * st)
    e(raw("s_waitcnt lgkmcnt(0)", "wait"))
    for st in range(8):
        for qt in (0, 1):
            e(mfma_qk(0, qt, st, S_BUF[1][0] + 4 * st, zero_c=True))
    G = build_groups(False, "x")
    for g in range(AHEAD):
        out += G[g]["frag"]
    e(nop(8)); e(nop(8))
    # first tail: mask (unit 0 needs it only for the wave that owns query 0), maxima, reference = maximum
    e(salu(f"s_cmp_gt_i32 %[qw0], 30", w=["scc"]))
    e(branch("s_cbranch_scc1 SKIPM_P"))
    out += mask_block(0)
    e(label("SKIPM_P"))
    out += max_local(0) + max_exchange()
    for qt in (0, 1):
        e(valu(f"v_mov_b32 {V(REF[qt])}, {V(TMAX[qt])}", r=vr(TMAX[qt]), w=vr(REF[qt])))
        for v in range(16):
            s = S_BUF[0][qt] + v
            e(valu(f"v_sub_f32 {V(s)}, {V(s)}, {V(TMAX[qt])}", r=vr(s) + vr(TMAX[qt]), w=vr(s)))
        e(valu(f"v_xor_b32 {V(TMP + 3)}, 0x80000000, {V(TMAX[qt])}", r=vr(TMAX[qt]), w=vr(TMP + 3)))
        for v in range(16):
            e(valu(f"v_mov_b32 {V(NEGR[qt] + v)}, {V(TMP + 3)}", r=vr(TMP + 3), w=vr(NEGR[qt] + v)))
    out += exp_stream(0, range(0, EARLY), fresh=True)
    e(nop(8)); e(nop(8))
    return out


def epilogue():
    out = [raw("s_waitcnt vmcnt(0) lgkmcnt(0)", "wait"), nop(8), nop(8)]
    e = out.append
    for qt in (0, 1):
        l, t, inv = LRUN[qt], TMP + qt, TMP + 4 + qt
        e(valu(f"v_mov_b32 {V(t)}, {V(l)}", r=vr(l), w=vr(t)))
        e(nop(4))
        e(valu(f"v_permlane32_swap_b32 {V(l)}, {V(t)}", r=vr(l) + vr(t), w=vr(l) + vr(t), kind="perm"))
        e(valu(f"v_add_f32 {V(l)}, {V(l)}, {V(t)}", r=vr(l) + vr(t), w=vr(l)))
        e(valu(f"v_rcp_f32 {V(inv)}, {V(l)}", r=vr(l), w=vr(inv), kind="trans"))
    e(nop(2))
    for qt in (0, 1):
        inv = TMP + 4 + qt
        e(valu(f"v_cmp_ne_u32 vcc, 0, %[valid{qt}]", w=["vcc"], kind="vcmp"))
        e(raw(f"s_and_saveexec_b64 {S(S_SAVE, 2)}, vcc", "salu", r=["vcc"], w=sr(S_SAVE, 2) + ["exec"]))
        for dt in range(4):
            o = O_ACC + (dt * 2 + qt) * 16
            for vg in range(4):
                t = TMP + 8 + 4 * (vg & 1)
                for k in range(4):
                    e(valu(f"v_accvgpr_read_b32 {V(t + k)}, {A(o + vg * 4 + k)}", r=ar(o + vg * 4 + k), w=vr(t + k)))
                for k in range(4):
                    e(valu(f"v_mul_f32 {V(t + k)}, {V(t + k)}, {V(inv)}", r=vr(t + k) + vr(inv), w=vr(t + k)))
                e(valu(f"v_cvt_pk_bf16_f32 {V(t)}, {V(t)}, {V(t + 1)}", r=vr(t, 2), w=vr(t)))
                e(valu(f"v_cvt_pk_bf16_f32 {V(t + 1)}, {V(t + 2)}, {V(t + 3)}", r=vr(t + 2, 2), w=vr(t + 1)))
                e(Ins(f"global_store_dwordx2 %[orow{qt}], {V(t, 2)}, off offset:{(dt * 32 + 8 * vg) * 2}", "vmem", r=vr(t, 2)))
        e(raw(f"s_mov_b64 exec, {S(S_SAVE, 2)}", "salu", r=sr(S_SAVE, 2), w=["exec"]))
    return out


def stats(name, body):
    from collections import Counter
    c = Counter()
    for x in body:
        c[x.kind] += weight(x) if x.kind == "nop" else 1
    n_mfma = c["mfma"]
    others = sum(v for k, v in c.items() if k not in ("mfma", "label"))
    print(f"{name}: {n_mfma} MFMAs, {others} other issue slots ({others / n_mfma:.2f} per MFMA): " +
          ", ".join(f"{k} {v}" for k, v in sorted(c.items())), file=sys.stderr)


def main():
    main_body = loop_body(False, "m")
    diag_body = loop_body(True, "d")
    stats("main loop", main_body)
    stats("diagonal loop", diag_body)
    pro = fix_hazards(prologue())
    # main loop over the tiles before the last three, then the masked loop over the rest
    seq = list(pro)
    seq += [salu(f"s_cmp_lt_u32 {S(S_T)}, %[nmain]", r=sr(S_T), w=["scc"]), branch("s_cbranch_scc0 MAIN_DONE"),
            label("LOOP_M")] + main_body + loop_tail("LOOP_M", "%[nmain]") + [label("MAIN_DONE")]
    seq += [salu(f"s_lshl_b32 {S(S_K0N)}, {S(S_T)}, 7", r=sr(S_T), w=sr(S_K0N) + ["scc"]),
            label("LOOP_D")] + diag_body + loop_tail("LOOP_D", "%[nkt]")
    seq += fix_hazards(epilogue()) + [branch("s_branch DONE")]
    returns = []
    for tag in ("m", "d"):
        for j in range(4):
            ret = len(returns)
            returns.append((ret, f"REDO_{tag}{j}"))
            seq += fix_hazards(rare_block(tag, j, ret)) + fix_hazards(redo_block(tag, j))
    seq += fix_hazards(rescale_block(returns)) + [label("DONE")]
    used_v = max(int(r[1:]) for x in seq for r in (x.r | x.w) if r[0] == "v" and r[1:].isdigit())
    used_a = max(int(r[1:]) for x in seq for r in (x.r | x.w) if r[0] == "a" and r[1:].isdigit())
    assert used_v <= LAST_V and used_a <= LAST_A, (used_v, used_a)
    here = sys.argv[1] if len(sys.argv) > 1 else os.path.dirname(os.path.abspath(__file__))   # output directory
    with open(os.path.join(here, "attn_bf16_body.inc"), "w") as f:
        f.write("// generated by gen_attn_asm.py -- do not edit\n")
        # labels get the asm statement's unique number, so that the block can be instantiated more than once
        names = sorted((x.text[:-1] for x in seq if x.kind == "label"), key=len, reverse=True)
        pattern = re.compile(r"\b(" + "|".join(names) + r")\b")
        for x in seq:
            f.write('    "' + pattern.sub(lambda m: m.group(1) + "_%=", x.text) + '\\n"\n')
    clob = ([f'"v{i}"' for i in range(LAST_V + 1)] + [f'"a{i}"' for i in range(LAST_A + 1)] +
            [f'"s{i}"' for i in range(FIRST_S, LAST_S + 1)] + ['"vcc"', '"scc"', '"memory"'])
    with open(os.path.join(here, "attn_bf16_clobbers.inc"), "w") as f:
        f.write(", ".join(clob) + "\n")
    print(f"{len(seq)} lines, vgprs to v{used_v}, agprs to a{used_a}", file=sys.stderr)


if __name__ == "__main__":
    main()
