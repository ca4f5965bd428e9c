#!/usr/bin/env python3
"""Writes gemm_bf16_mainloops.inc: the k-loops of the bf16 projection kernels ("QKV Generation", output projection
and "FFN" of Fig. 2) as gfx950 assembly inside C++ device functions, one per wave-tile shape.  csrc/gemm.hip
includes the file; its C++ part computes the operands and runs the epilogues on the accumulators the functions
return.  Run `python gen_gemm_asm.py` after changing this file (an argument names another output directory); the .inc is
committed and tests/test_generated_sources.py checks that it is current.

Shape of a workgroup: 4 waves, one per SIMD, arranged 2 (features) x 2 (tokens); a wave owns TW x TA MFMA tiles of
32 x 32 (for SwiGLU: of each of the NW = 2 weight matrices), 128 x 128 outputs in the large tiles, so that each
fragment read from LDS feeds four MFMAs.  The 16 accumulators fill the accumulation registers (they are the asm
statement's outputs); fragments are double-buffered in v0..; a lone wave per SIMD means the order of matrix, LDS and
tile-load instructions in the wave is the schedule, so it is written out here.

k-loop: k-tiles of 64, two LDS stages (tile rows of 128 bytes, 16-byte chunks XOR-swizzled as in gemm.hip), operand
tiles global -> LDS directly.  Per k-tile: four k-steps of TW*TA*NW MFMAs; the fragments of step s+1 are read beside
the MFMAs of step s, also across k-tiles.  The one barrier of a k-tile sits before its last k-step, when every wave
holds that step's fragments and its own part of the next tile has landed; from there on the stage is refilled with
the tile two ahead.  Those tile loads are issued over three k-steps (a third beside the last k-step, the rest beside
the first two k-steps of the next tile): issued in one burst right after the barrier they back the wave's
instruction issue up behind the memory pipeline and cost a quarter of the MFMA rate.
"""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
from gen_attn_asm import Ins, vr, sr, V, S, valu, salu, nop, label, branch, raw, fix_hazards, weight   # noqa: E402

SPREAD = 3
N_ACC_IN_VGPRS = 4
S_KPW, S_KPW2, S_KPA, S_CNT, S_LST, S_TMP = 40, 42, 44, 46, 47, 48
FIRST_S, LAST_S = 40, 48


class Shape:
    def __init__(self, TW, TA, NW, resid=False):
        self.TW, self.TA, self.NW = TW, TA, NW
        # resid: out = a . w^T + R.  The loop's prologue requests the wave's part of the residual tile as MFMA B
        # fragments (lane (token, half) takes features 8*half .. 8*half+7 of each group of 16 output features: 16-byte
        # loads), and behind the first k-tile, when they have arrived, adds them to the accumulators with two MFMAs per
        # accumulator whose A operand is a slice of the identity (row f of the 32-row tile has its one at k = f - 16p
        # for the group p): acc += I . R, exact, no vector ALU work, and the epilogue is the plain one.
        self.resid = resid
        self.NWF, self.NAF = NW * TW, TA                       # fragments per k-step
        n = 4 * (self.NWF + self.NAF)
        self.FRAG = [0, n]                                     # two fragment buffers: W frags then A frags
        self.WADR = 2 * n                                      # [stage][ks] LDS addresses of the W fragments
        self.AADR = self.WADR + 8
        self.WOFS = self.AADR + 8                              # lane offsets of the tile loads: <= 8 W, <= 8 A
        self.AOFS = self.WOFS + 8
        self.TMPV = self.AOFS + 8
        self.BN = 32 * TW * 2                                  # features per matrix in a workgroup tile
        self.WROWS = self.BN * NW
        self.AROWS = 32 * TA * 2
        self.STAGE = (self.WROWS + self.AROWS) * 128
        self.NLW = self.WROWS // 32                            # wave-loads per wave and k-tile: weights, then activations
        self.NLD = (self.WROWS + self.AROWS) // 32
        assert self.STAGE <= 65536 and self.NLW <= 8 and self.NLD - self.NLW <= 8
        self.ROFS = self.TMPV + 1                              # byte offsets of the lane's TA residual rows
        self.IDENT = (self.ROFS + TA + 2) & ~1                 # two identity slices, 4 registers each (ROFS + TA stays spare)
        self.RES = self.IDENT + 8                              # residual fragments, 4 registers per (j, i, p)
        self.LAST_V = self.RES + 4 * TA * TW * 2 - 1 if resid else self.TMPV
        assert self.LAST_V < 256
        self.name = f"{TW}_{TA}_{NW}" + ("_resid" if resid else "")

    def acc(self, w, i, j):
        return f"%[c{(w * self.TW + i) * self.TA + j}]"

    def mfma(self, buf, w, i, j, zero):
        wf = self.FRAG[buf] + 4 * (w * self.TW + i)
        af = self.FRAG[buf] + 4 * (self.NWF + j)
        c = self.acc(w, i, j)
        return Ins(f"v_mfma_f32_32x32x16_bf16 {c}, {V(wf, 4)}, {V(af, 4)}, {'0' if zero else c}", "mfma",
                   r=vr(wf, 4) + vr(af, 4) + ([] if zero else [c]), w=[c])

    def res_frag(self, j, i, p):
        return self.RES + 4 * ((j * self.TW + i) * 2 + p)

    def residual_mfmas(self):
        out = []
        for p in range(2):                                     # the two MFMAs of an accumulator 16 apart
            for j in range(self.TA):
                for i in range(self.TW):
                    c, a, b = self.acc(0, i, j), self.IDENT + 4 * p, self.res_frag(j, i, p)
                    out.append(Ins(f"v_mfma_f32_32x32x16_bf16 {c}, {V(a, 4)}, {V(b, 4)}, {c}", "mfma",
                                   r=vr(a, 4) + vr(b, 4) + [c], w=[c]))
        return out

    def frag_reads(self, buf, stage, ks):
        out = []
        for w in range(self.NW):
            for i in range(self.TW):
                d = self.FRAG[buf] + 4 * (w * self.TW + i)
                off = (w * self.BN + i * 32) * 128
                out.append(Ins(f"ds_read_b128 {V(d, 4)}, {V(self.WADR + stage * 4 + ks)} offset:{off}", "lds",
                               r=vr(self.WADR + stage * 4 + ks), w=vr(d, 4)))
        for j in range(self.TA):
            d = self.FRAG[buf] + 4 * (self.NWF + j)
            out.append(Ins(f"ds_read_b128 {V(d, 4)}, {V(self.AADR + stage * 4 + ks)} offset:{j * 32 * 128}", "lds",
                           r=vr(self.AADR + stage * 4 + ks), w=vr(d, 4)))
        return out

    def tile_loads(self, stage):
        """The wave's wave-loads of the k-tile at the pending pointers into `stage`; then the pointers move on
        (they stay on the last k-tile once it is reached: later loads re-read it into a stage nobody reads)."""
        out = []
        for i in range(self.NLD):
            if i < self.NLW:
                ofs, ptr = self.WOFS + i, (S_KPW2 if (self.NW == 2 and i * 32 >= self.BN) else S_KPW)
            else:
                ofs, ptr = self.AOFS + i - self.NLW, S_KPA
            out.append(salu(f"s_add_u32 m0, %[ldsw], {stage * self.STAGE + i * 4096}", w=["m0", "scc"]))
            out.append(Ins(f"global_load_lds_dwordx4 {V(ofs)}, {S(ptr, 2)}", "vmem", r=vr(ofs) + ["m0"] + sr(ptr, 2)))
        out += [salu(f"s_sub_u32 {S(S_LST)}, {S(S_LST)}, 1", r=sr(S_LST), w=sr(S_LST) + ["scc"]),
                salu(f"s_cmp_gt_i32 {S(S_LST)}, 0", r=sr(S_LST), w=["scc"]),
                salu(f"s_cselect_b32 {S(S_TMP)}, 128, 0", r=["scc"], w=sr(S_TMP))]
        for p in (S_KPW, S_KPW2, S_KPA) if self.NW == 2 else (S_KPW, S_KPA):
            out += [salu(f"s_add_u32 {S(p)}, {S(p)}, {S(S_TMP)}", r=sr(p) + sr(S_TMP), w=sr(p) + ["scc"]),
                    salu(f"s_addc_u32 {S(p + 1)}, {S(p + 1)}, 0", r=sr(p + 1) + ["scc"], w=sr(p + 1) + ["scc"])]
        return out

    @staticmethod
    def deal(mf, fills):
        out, k = [], 0
        for i, m in enumerate(mf):
            out.append(m)
            want = (i + 1) * len(fills) // len(mf)
            out += fills[k:want]
            k = want
        return out

    def k_tile(self, stage, first):
        """One k-tile from `stage`; the fragments of its k-step 0 are in buffer 0 (already requested)."""
        seq = []
        order = [(w, i, j) for w in range(self.NW) for i in range(self.TW) for j in range(self.TA)]
        share = lambda loads, k: loads[k * len(loads) // SPREAD:(k + 1) * len(loads) // SPREAD]
        for ks in range(4):
            buf = ks & 1
            seq.append(raw("s_waitcnt lgkmcnt(0)", "wait"))
            mf = [self.mfma(buf, w, i, j, first and ks == 0) for (w, i, j) in order]
            if ks < 3:
                carry = share(self.tile_loads(stage ^ 1), ks + 1) if (not first and ks + 1 < SPREAD) else []
                seq += self.deal(mf, self.frag_reads(buf ^ 1, stage, ks + 1) + carry)
            else:
                seq += [raw("s_waitcnt vmcnt(0)", "wait"), raw("s_barrier", "barrier")]
                seq += self.deal(mf, self.frag_reads(buf ^ 1, stage ^ 1, 0) + share(self.tile_loads(stage), 0))
        return seq

    def body(self):
        pro = []
        e = pro.append
        for st in range(2):
            for ks in range(4):
                for adr, src in ((self.WADR, "wfrag0"), (self.AADR, "afrag0")):
                    r = adr + st * 4 + ks
                    e(valu(f"v_xor_b32 {V(r)}, {ks << 5}, %[{src}]", w=vr(r)))
                    if st:
                        e(valu(f"v_add_u32 {V(r)}, {self.STAGE}, {V(r)}", r=vr(r), w=vr(r)))
        # tile-load lane offsets: row 32 i + r0 of its matrix, clamped to the last valid row
        for i in range(self.NLD):
            is_w = i < self.NLW
            ofs = (self.WOFS + i) if is_w else (self.AOFS + i - self.NLW)
            row = (32 * i) % self.BN if is_w else 32 * (i - self.NLW)
            lim, stride = ("%[wlim]", "%[wstride]") if is_w else ("%[alim]", "%[astride]")
            e(valu(f"v_add_u32 {V(self.TMPV)}, {row}, %[r0]", w=vr(self.TMPV)))
            e(valu(f"v_min_i32 {V(self.TMPV)}, {lim}, {V(self.TMPV)}", r=vr(self.TMPV), w=vr(self.TMPV)))
            e(valu(f"v_mad_u32_u24 {V(ofs)}, {V(self.TMPV)}, {stride}, %[chunk]", r=vr(self.TMPV), w=vr(ofs)))
        ptrs = [(S_KPW, "w0base"), (S_KPA, "abase")] + ([(S_KPW2, "w1base")] if self.NW == 2 else [])
        for p, name in ptrs:
            e(salu(f"s_mov_b32 {S(p)}, %[{name}_lo]", w=sr(p)))
            e(salu(f"s_mov_b32 {S(p + 1)}, %[{name}_hi]", w=sr(p + 1)))
        e(salu(f"s_mov_b32 {S(S_CNT)}, %[kt]", w=sr(S_CNT)))
        e(salu(f"s_mov_b32 {S(S_LST)}, %[kt]", w=sr(S_LST)))
        pro += self.tile_loads(0) + self.tile_loads(1)
        n_res = 0
        if self.resid:
            for j in range(self.TA):                           # row = min(rrow0 + 32 j, alim) of the workgroup tile
                e(valu(f"v_add_u32 {V(self.TMPV)}, {32 * j}, %[rrow0]", w=vr(self.TMPV)))
                e(valu(f"v_min_i32 {V(self.TMPV)}, %[alim], {V(self.TMPV)}", r=vr(self.TMPV), w=vr(self.TMPV)))
                e(valu(f"v_mad_u32_u24 {V(self.ROFS + j)}, {V(self.TMPV)}, %[rstride], %[rcol0]", r=vr(self.TMPV), w=vr(self.ROFS + j)))
            for j in range(self.TA):
                for i in range(self.TW):
                    for p in range(2):
                        d = self.res_frag(j, i, p)
                        e(Ins(f"global_load_dwordx4 {V(d, 4)}, {V(self.ROFS + j)}, %[rbase] offset:{i * 64 + p * 32}", "vmem",
                              r=vr(self.ROFS + j), w=vr(d, 4)))
                        n_res += 1
            # identity slices: t = f - 8*half - 16p with f = rrow0 & 31 and half = bit 4 of rcol0; the lane's one is
            # bf16 element t of its 8 (if 0 <= t < 8): dword t >> 1, upper half if t is odd
            t, val, idx = self.TMPV, self.ROFS + self.TA, self.TMPV      # ROFS + TA is a spare register below IDENT
            for p in range(2):
                e(valu(f"v_and_b32 {V(t)}, 31, %[rrow0]", w=vr(t)))
                e(valu(f"v_bfe_u32 {V(val)}, %[rcol0], 4, 1", w=vr(val)))
                e(valu(f"v_lshlrev_b32 {V(val)}, 3, {V(val)}", r=vr(val), w=vr(val)))
                e(valu(f"v_sub_u32 {V(t)}, {V(t)}, {V(val)}", r=vr(t) + vr(val), w=vr(t)))
                e(valu(f"v_subrev_u32 {V(t)}, {16 * p}, {V(t)}", r=vr(t), w=vr(t)))
                sh = self.IDENT + 7                            # free until the last select of p = 1 writes it
                e(valu(f"v_and_b32 {V(sh)}, 1, {V(t)}", r=vr(t), w=vr(sh)))
                e(valu(f"v_lshlrev_b32 {V(sh)}, 4, {V(sh)}", r=vr(sh), w=vr(sh)))
                e(valu(f"v_mov_b32 {V(val)}, 0x3f80", w=vr(val)))                  # bf16 1.0
                e(valu(f"v_lshlrev_b32 {V(val)}, {V(sh)}, {V(val)}", r=vr(sh) + vr(val), w=vr(val)))
                e(valu(f"v_ashrrev_i32 {V(idx)}, 1, {V(t)}", r=vr(t), w=vr(idx)))
                for dw in range(4):
                    e(valu(f"v_cmp_eq_u32 vcc, {dw}, {V(idx)}", r=vr(idx), w=["vcc"], kind="vcmp"))
                    e(valu(f"v_cndmask_b32 {V(self.IDENT + 4 * p + dw)}, 0, {V(val)}, vcc", r=vr(val) + ["vcc"], w=vr(self.IDENT + 4 * p + dw)))
        # only the first k-tile has to be there: the second one (and the residual fragments) may stay in flight
        # until the first k-tile's own wait before its barrier
        e(raw(f"s_waitcnt vmcnt({self.NLD + n_res})", "wait"))
        e(raw("s_barrier", "barrier"))
        pro += self.frag_reads(0, 0, 0)
        body0f, body0, body1 = self.k_tile(0, True), self.k_tile(0, False), self.k_tile(1, False)
        if self.resid:
            body0f = body0f + self.residual_mfmas()            # behind the first k-tile's wait for every load
        dec = lambda: [salu(f"s_sub_u32 {S(S_CNT)}, {S(S_CNT)}, 1", r=sr(S_CNT), w=sr(S_CNT) + ["scc"]),
                       salu(f"s_cmp_eq_u32 {S(S_CNT)}, 0", r=sr(S_CNT), w=["scc"]), branch("s_cbranch_scc1 GDONE_%=")]
        seq = fix_hazards(pro + body0f) + dec() + [label("GLOOP_%=")]
        loop = body1 + dec() + body0 + dec() + [branch("s_branch GLOOP_%=")]
        seq += fix_hazards(loop, history=body0 + body1)
        # drain the trailing loads; the accumulators are read by the compiler's code next: pad past the MFMA latency
        seq += [label("GDONE_%="), raw("s_waitcnt vmcnt(0) lgkmcnt(0)", "wait"), nop(8), nop(8)]
        n_mfma = sum(1 for x in body0 if x.kind == "mfma")
        n_oth = sum(weight(x) for x in body0 if x.kind not in ("mfma", "label"))
        print(f"wave tile {self.name}: k-tile of {n_mfma} MFMAs and {n_oth} other instructions, vgprs to v{self.LAST_V}", file=sys.stderr)
        return seq

    def function(self):
        n = self.NW * self.TW * self.TA
        seq = self.body()
        out = [f"// wave tile of {self.TW} x {self.TA} MFMA tiles, {self.NW} weight matri{'x' if self.NW == 1 else 'ces'}"
               + ("; adds the residual tile to the accumulators" if self.resid else ""),
               f"__device__ __forceinline__ void gemm_mainloop_{self.name}(unsigned wfrag0, unsigned afrag0, unsigned r0, unsigned chunk,",
               "        int wlim, int alim, unsigned wstride, unsigned astride, unsigned kt, unsigned ldsw, uint64_t w0base,",
               f"        uint64_t w1base, uint64_t abase, f32x16 (&acc)[{self.NW}][{self.TW}][{self.TA}]"
               + (", unsigned rrow0, unsigned rcol0, unsigned rstride, const void* rbase" if self.resid else "") + ") {",
               "    f32x16 " + ", ".join(f"c{k}" for k in range(n)) + ";",
               "    const unsigned w0base_lo = (unsigned)w0base, w0base_hi = (unsigned)(w0base >> 32);",
               "    const unsigned w1base_lo = (unsigned)w1base, w1base_hi = (unsigned)(w1base >> 32);",
               "    const unsigned abase_lo = (unsigned)abase, abase_hi = (unsigned)(abase >> 32);",
               "    asm volatile("]
        out += ['        "' + x.text + '\\n"' for x in seq]
        # the last accumulators live in VGPRs: with all 256 accumulation registers taken by the outputs the compiler
        # spills some of them to scratch memory behind the loop (the residual form has no VGPRs to spare for that)
        in_vgprs = 0 if self.resid else N_ACC_IN_VGPRS
        out.append("        : " + ", ".join(f'[c{k}] "=&{"a" if k < n - in_vgprs else "v"}"(c{k})' for k in range(n)))
        ins = ['[wfrag0] "v"(wfrag0)', '[afrag0] "v"(afrag0)', '[r0] "v"(r0)', '[chunk] "v"(chunk)', '[wlim] "s"(wlim)',
               '[alim] "s"(alim)', '[wstride] "s"(wstride)', '[astride] "s"(astride)', '[kt] "s"(kt)', '[ldsw] "s"(ldsw)',
               '[w0base_lo] "s"(w0base_lo)', '[w0base_hi] "s"(w0base_hi)', '[abase_lo] "s"(abase_lo)', '[abase_hi] "s"(abase_hi)']
        if self.NW == 2:
            ins += ['[w1base_lo] "s"(w1base_lo)', '[w1base_hi] "s"(w1base_hi)']
        if self.resid:
            ins += ['[rrow0] "v"(rrow0)', '[rcol0] "v"(rcol0)', '[rstride] "s"(rstride)', '[rbase] "s"(rbase)']
        out.append("        : " + ", ".join(ins))
        clob = [f'"v{i}"' for i in range(self.LAST_V + 1)] + [f'"s{i}"' for i in range(FIRST_S, LAST_S + 1)] + ['"vcc"', '"scc"', '"memory"']
        out.append("        : " + ", ".join(clob) + ");")
        if self.NW == 1:
            out.append("    (void)w1base_lo; (void)w1base_hi;")
        k = 0
        for w in range(self.NW):
            for i in range(self.TW):
                for j in range(self.TA):
                    out.append(f"    acc[{w}][{i}][{j}] = c{k};")
                    k += 1
        out.append("}")
        return "\n".join(out) + "\n"


def main():
    here = sys.argv[1] if len(sys.argv) > 1 else os.path.dirname(os.path.abspath(__file__))   # output directory
    with open(os.path.join(here, "gemm_bf16_mainloops.inc"), "w") as f:
        f.write("// generated by gen_gemm_asm.py -- do not edit\n")
        for cfg in ((4, 4, 1), (2, 4, 2), (4, 2, 1), (2, 2, 2), (4, 4, 1, True), (4, 2, 1, True)):
            f.write("\n" + Shape(*cfg).function())


if __name__ == "__main__":
    main()
