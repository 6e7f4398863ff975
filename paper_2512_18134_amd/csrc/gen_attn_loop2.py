#!/usr/bin/env python3
"""Emit the hand-scheduled main loop of the one-wave-per-SIMD attention kernels.

Same three-stage modulo schedule as gen_attn_loop.py (the paper's Fig. 1a loop,
Section 3.1 vocabulary: iteration j issues P(j-1)V(j-1) and K(j+1)Q^T on the
matrix pipe while the softmax of S(j) runs on the VALU), for the tilings in
which a wave owns the whole 512-entry register file of its SIMD:

    d128a  D=128: 4 waves x 64 query rows (two 32-row blocks per wave, BM=256),
           32-key tiles.  Every K / V^T fragment read from LDS feeds two MFMAs,
           which halves the LDS operand traffic of the 8-wave kernel.
    d256a  D=256: 4 waves x 32 query rows (BM=128), 32-key tiles; K Q^T is
           accumulated in two interleaved accumulators (even / odd k-step) so
           that consecutive MFMAs are independent, and summed on the VALU.

The O accumulators and the Q fragments live in AGPRs (MFMA reads and writes
them directly); everything the VALU touches (S, P, addresses, state) is in
VGPRs.  K/V tiles: direct global->LDS loads, 4-stage rings, one barrier per tile.

The softmax runs without a per-tile row maximum, as in gen_attn_loop.py: P is
taken against the reference the row already has, the tile's row sum is tested
against a bound, and a failed test (rare) sends the wave through an out-of-line
pass that finds the exact maximum, moves the reference and redoes the tile's P
from its intact scores.

usage: gen_attn_loop2.py <d128a|d256a> <out.inc> [bf16|f16]
"""
import struct
import sys

CONFIGS = {
    "d128a": dict(D=128, QB=2, NACC=1),
    "d256a": dict(D=256, QB=1, NACC=2),
}


class Gen:
    def __init__(self, name, NF=4, PFD=3, dtype="bf16"):
        cfg = CONFIGS[name]
        self.name = name
        assert dtype in ("bf16", "f16")
        self.dtype = dtype                       # element type of Q, K, V and of the rounded P
        self.D, self.QB, self.NACC = cfg["D"], cfg["QB"], cfg["NACC"]
        D, QB, NACC = self.D, self.QB, self.NACC
        self.NW = 4
        self.BN = 32
        self.KS = D // 16
        self.DB = D // 32
        self.ROWB = 2 * D
        self.TB = self.BN * self.ROWB
        self.NLD = self.TB // (self.NW * 1024)
        self.NF, self.PFD = NF, PFD
        self.NG = 2 * self.DB + self.KS          # fragment groups per iteration
        self.NM = self.NG * QB                   # MFMA slots per iteration
        assert self.NG % NF == 0 and PFD < NF
        # ---- AGPR map
        self.O = 0                               # O[qb][db]: 16 each
        self.Q = 16 * QB * self.DB               # Q[qb][ks]: 4 each
        self.NA = self.Q + 4 * QB * self.KS
        assert self.NA <= 256
        # ---- VGPR map
        r = 0
        def take(n):
            nonlocal r
            b = r
            r += n
            return b
        self.SA = take(16 * QB * NACC)
        self.SB = take(16 * QB * NACC)
        self.PA = take(8 * QB)
        self.PB = take(8 * QB)
        self.FR = take(4 * NF)
        self.KOFF = take(self.KS)
        self.VOFF = take(2 * self.DB)
        self.DVOFF = take(self.NLD)
        self.DROW = take(self.NLD)
        self.DCH = take(self.NLD)
        self.MREF = take(QB)
        self.MRC = take(QB)
        self.L = take(QB)                        # running row sums
        self.TLA = take(QB)                      # row sums of the current tile, two partial sums each
        self.TLB = take(QB)
        self.TP = take(6)                        # exponent / exp temporaries of three element pairs in flight
        self.ALPHA = take(QB)
        self.THRB = take(QB)
        self.THR = take(QB)
        self.T = take(QB)
        self.TMP2 = take(QB)
        self.DD = take(QB)
        self.MX = take(2 * QB)
        self.NEGINF = take(1)
        self.DT = take(2 * self.NLD)
        self.AT = take(4)                        # temporaries of the accumulator rescale
        self.NV = r
        assert r <= 256, r
        # ---- SGPR map
        self.s_kbase, self.s_vbase = 32, 34
        self.s_c, self.s_ntiles, self.s_jmask, self.s_tfull, self.s_skvm1 = 36, 37, 38, 39, 40
        self.s_ldsk, self.s_ldsv = 41, 42
        self.s_j, self.s_resc, self.s_tau = 43, 44, 45
        self.s_kptr, self.s_vptr = 46, 48
        self.s_tk, self.s_tv = 50, 51
        self.s_t0 = 52                           # s[52:53], s[54:55]: compare masks
        self.s_t2 = 56
        self.s_m0 = 57            # m0 of the surrounding code (reserved register: saved and restored here)
        self.lines = []

    # ------------------------------------------------------------------ helpers
    def e(self, s):
        self.lines.append(s)

    def lab(self, name):
        return "%s%%=" % name

    @staticmethod
    def rg(cls, base, n=1):
        return "%s%d" % (cls, base) if n == 1 else "%s[%d:%d]" % (cls, base, base + n - 1)

    def vr(self, base, n=1):
        return self.rg("v", base, n)

    def ar(self, base, n=1):
        return self.rg("a", base, n)

    def sr(self, base, n=1):
        return self.rg("s", base, n)

    def s_reg(self, S, qb, acc, r=0):
        return S + (qb * self.NACC + acc) * 16 + r

    # ------------------------------------------------------------ MFMA programs
    def groups(self):
        """Fragment groups in issue order: ('pv', kc, db) / ('qk', ks); each feeds QB MFMAs."""
        pv0 = [("pv", 0, db) for db in range(self.DB)]
        pv1 = [("pv", 1, db) for db in range(self.DB)]
        qk = [("qk", ks, 0) for ks in range(self.KS)]
        return pv0 + qk + pv1

    def frag_loads(self, grp, buf, kst, vst):
        f = self.FR + 4 * buf
        kind, a, b = grp
        if kind == "pv":
            kc, db = a, b
            off = vst * self.TB + kc * 16 * self.ROWB
            assert off < 65536
            return ["ds_read_b64_tr_b16 %s, %s offset:%d" % (self.vr(f, 2), self.vr(self.VOFF + 2 * db), off),
                    "ds_read_b64_tr_b16 %s, %s offset:%d" % (self.vr(f + 2, 2), self.vr(self.VOFF + 2 * db + 1), off)]
        ks = a
        off = kst * self.TB
        assert off < 65536
        return ["ds_read_b128 %s, %s offset:%d" % (self.vr(f, 4), self.vr(self.KOFF + ks), off)]

    def mfma_text(self, grp, qb, buf, P_prev, S_nxt):
        f = self.vr(self.FR + 4 * buf, 4)
        kind, a, b = grp
        if kind == "pv":
            kc, db = a, b
            o = self.ar(self.O + 16 * (qb * self.DB + db), 16)
            return "v_mfma_f32_32x32x16_%s %s, %s, %s, %s" % (self.dtype, o, f, self.vr(P_prev + qb * 8 + kc * 4, 4), o)
        ks = a
        acc = ks % self.NACC
        s = self.vr(self.s_reg(S_nxt, qb, acc), 16)
        q = self.ar(self.Q + 4 * (qb * self.KS + ks), 4)
        return "v_mfma_f32_32x32x16_%s %s, %s, %s, %s" % (self.dtype, s, f, q, "0" if ks < self.NACC else s)

    # ---------------------------------------------------------- softmax programs
    def max_ops(self, S_cur):
        chains = []
        for qb in range(self.QB):
            for c in range(2):
                mx = self.MX + 2 * qb + c
                s = [self.s_reg(S_cur, qb, 0, 8 * c + i) for i in range(8)]
                ch = ["v_max3_f32 v%d, v%d, v%d, v%d" % (mx, s[0], s[1], s[2]),
                      "v_max3_f32 v%d, v%d, v%d, v%d" % (mx, mx, s[3], s[4]),
                      "v_max3_f32 v%d, v%d, v%d, v%d" % (mx, mx, s[5], s[6]),
                      "v_max_f32 v%d, v%d, v%d" % (mx, mx, s[7])]
                chains.append(ch)
        ops = []
        for step in range(4):
            for ch in chains:
                ops.append(ch[step])
        for qb in range(self.QB):
            ops.append("v_max_f32 v%d, v%d, v%d" % (self.T + qb, self.MX + 2 * qb, self.MX + 2 * qb + 1))
        return ops

    def pairmax_ops(self):
        """Lane-pair max and the new reference maximum into T, for every query block."""
        seqs = []
        for qb in range(self.QB):
            T, TMP2 = self.T + qb, self.TMP2 + qb
            seqs.append([
                "v_mov_b32 v%d, v%d" % (TMP2, T),
                "s_nop 1",
                "v_permlane32_swap_b32 v%d, v%d" % (T, TMP2),
                "s_nop 1",
                "v_max_f32 v%d, v%d, v%d" % (T, T, TMP2),
                "v_max_f32 v%d, v%d, v%d" % (T, T, self.MREF + qb),
            ])
        return [seqs[qb][i] for i in range(len(seqs[0])) for qb in range(self.QB)]

    def pair_ops(self, S_cur, P_new):
        """fma -> exp2 -> row-sum add -> pack over the element pairs, software pipelined three deep; the
        exponent arguments go to the temporaries TP, S_cur stays intact for the out-of-line pass."""
        pairs = [(qb, k) for qb in range(self.QB) for k in range(8)]
        def regs(p):
            qb, k = p
            return self.s_reg(S_cur, qb, 0, 2 * k), self.s_reg(S_cur, qb, 0, 2 * k + 1)
        def tp(t, i):
            return self.TP + 2 * (t % 3) + i
        def F(t):
            p = pairs[t]
            return ["v_fma_f32 v%d, v%d, s%d, -v%d" % (tp(t, i), x, self.s_c, self.MRC + p[0])
                    for i, x in enumerate(regs(p))]
        def E(t):
            return ["v_exp_f32 v%d, v%d" % (tp(t, i), tp(t, i)) for i in (0, 1)]
        def A(t):
            qb, k = pairs[t]
            if k == 0:   # the first pair of a query block starts its two partial sums
                acc = ["v_mov_b32 v%d, v%d" % (self.TLA + qb, tp(t, 0)), "v_mov_b32 v%d, v%d" % (self.TLB + qb, tp(t, 1))]
            else:
                acc = ["v_add_f32 v%d, v%d, v%d" % (self.TLA + qb, self.TLA + qb, tp(t, 0)),
                       "v_add_f32 v%d, v%d, v%d" % (self.TLB + qb, self.TLB + qb, tp(t, 1))]
            return acc + ["v_cvt_pk_%s_f32 v%d, v%d, v%d" % (self.dtype, P_new + qb * 8 + k, tp(t, 0), tp(t, 1))]
        ops = []
        n = len(pairs)
        for t in range(n + 2):
            if t < n:
                ops += F(t)
            if 0 <= t - 1 < n:
                ops += E(t - 1)
            if 0 <= t - 2 < n:
                ops += A(t - 2)
        for qb in range(self.QB):
            ops.append("v_add_f32 v%d, v%d, v%d" % (self.TLA + qb, self.TLA + qb, self.TLB + qb))
        return ops

    def check_ops(self, b):
        """Tile row sums below the bound?  Otherwise (too large, inf or NaN) take the out-of-line pass."""
        ops = []
        for qb in range(self.QB):
            ops.append("v_cmp_ngt_f32 %s, s%d, v%d" % (self.sr(self.s_t0 + 2 * qb, 2), self.s_tau, self.TLA + qb))
        t0 = self.sr(self.s_t0, 2)
        if self.QB == 2:
            ops.append("s_or_b64 %s, %s, %s" % (t0, t0, self.sr(self.s_t0 + 2, 2)))
        ops += ["s_cmp_lg_u64 %s, 0" % t0,
                "s_cbranch_scc1 %s" % self.lab("SLOW%d_" % b),
                "%s:" % self.lab("SLOWRET%d_" % b)]
        for qb in range(self.QB):
            ops.append("v_add_f32 v%d, v%d, v%d" % (self.L + qb, self.L + qb, self.TLA + qb))
        return ops

    def combine_ops(self, S_nxt):
        """Sum the even / odd k-step accumulators of K(j+1)Q^T (NACC == 2)."""
        ops = []
        if self.NACC == 2:
            for qb in range(self.QB):
                for r in range(16):
                    a0, a1 = self.s_reg(S_nxt, qb, 0, r), self.s_reg(S_nxt, qb, 1, r)
                    ops.append("v_add_f32 v%d, v%d, v%d" % (a0, a0, a1))
        return ops

    # ------------------------------------------------------------------- DMA
    def dma_fast(self, which, stage):
        lds = self.s_ldsk if which == "k" else self.s_ldsv
        ptr = self.s_kptr if which == "k" else self.s_vptr
        out = []
        for i in range(self.NLD):
            out += ["s_add_u32 m0, s%d, %d" % (lds, stage * self.TB + i * self.NW * 1024),
                    "s_nop 0",
                    "global_load_lds_dwordx4 v%d, %s" % (self.DVOFF + i, self.sr(ptr, 2))]
        return out

    def dma_slow(self, which, stage, label, ret):
        lds = self.s_ldsk if which == "k" else self.s_ldsv
        base = self.s_kbase if which == "k" else self.s_vbase
        st = self.s_tk if which == "k" else self.s_tv
        sh = {256: 8, 512: 9}[self.ROWB]
        self.e("%s:" % label)
        self.e("s_lshl_b32 s%d, s%d, 5" % (self.s_t2, st))          # first key of the tile (BN = 32)
        for i in range(self.NLD):
            t = self.DT + (0 if which == "k" else self.NLD) + i
            self.e("v_add_u32 v%d, s%d, v%d" % (t, self.s_t2, self.DROW + i))
            self.e("v_min_i32 v%d, s%d, v%d" % (t, self.s_skvm1, t))
            self.e("v_lshlrev_b32 v%d, %d, v%d" % (t, sh, t))
            self.e("v_add_u32 v%d, v%d, v%d" % (t, t, self.DCH + i))
            self.e("s_add_u32 m0, s%d, %d" % (lds, stage * self.TB + i * self.NW * 1024))
            self.e("s_nop 0")
            self.e("global_load_lds_dwordx4 v%d, %s" % (t, self.sr(base, 2)))
        self.e("s_branch %s" % ret)

    # ------------------------------------------------------- one MFMA stream
    def stream(self, grps, P_prev, S_nxt, kst, vst, valu_by_slot, extra_by_slot, prefetched, nxt):
        NF, PFD, QB = self.NF, self.PFD, self.QB
        n = len(grps)
        def issue(idx, grp, k, v):
            for ins in self.frag_loads(grp, idx % NF, k, v):
                self.e(ins)
                self.outstanding.append(idx)
        for i in range(prefetched, min(PFD, n)):
            issue(i, grps[i], kst, vst)
        slot = 0
        for i, grp in enumerate(grps):
            last = max(p for p, x in enumerate(self.outstanding) if x == i)
            after = len(self.outstanding) - 1 - last
            self.e("s_waitcnt lgkmcnt(%d)" % after)
            self.outstanding = self.outstanding[last + 1:]
            for qb in range(QB):
                self.e(self.mfma_text(grp, qb, i % NF, P_prev, S_nxt))
                if qb == QB - 1:
                    # the fragment buffer of group i+PFD was last read by group i+PFD-NF <= i-1
                    j = i + PFD
                    if j < n:
                        issue(j, grps[j], kst, vst)
                    elif nxt is not None:
                        ng, nk, nv = nxt
                        issue(j - n + 1000, ng[j - n], nk, nv)
                for ins in extra_by_slot.get(slot, []):
                    self.e(ins)
                for ins in valu_by_slot.get(slot, []):
                    self.e(ins)
                slot += 1
        self.outstanding = [x - 1000 for x in self.outstanding]
        assert all(0 <= x < PFD for x in self.outstanding), self.outstanding

    # --------------------------------------------------------------- the loop
    def body(self, b):
        NM, NLD = self.NM, self.NLD
        S_cur, S_nxt = (self.SA, self.SB) if b % 2 == 0 else (self.SB, self.SA)
        P_prev, P_new = (self.PA, self.PB) if b % 2 == 0 else (self.PB, self.PA)
        kst, vst = (b + 1) % 4, (b + 3) % 4
        nb = (b + 1) % 4
        nxt = (self.groups(), (nb + 1) % 4, (nb + 3) % 4)
        L = self.lab
        self.e("%s:" % L("BODY%d_" % b))
        self.e("s_cmp_ge_i32 s%d, s%d" % (self.s_j, self.s_ntiles))
        self.e("s_cbranch_scc1 %s" % L("EXIT%d_" % b))
        self.e("s_cmp_ge_i32 s%d, s%d" % (self.s_j, self.s_jmask))
        self.e("s_cbranch_scc1 %s" % L("MASK%d_" % b))
        self.e("%s:" % L("MASKRET%d_" % b))
        self.e("s_waitcnt vmcnt(%d)" % (2 * NLD))
        self.e("s_barrier")
        b_ops = self.pair_ops(S_cur, P_new)
        c_ops = self.combine_ops(S_nxt)
        nc = 4 if c_ops else 0                       # slots reserved at the end for the combine
        valu = {}
        nbs = NM - nc
        for i in range(nbs):
            valu[i] = b_ops[i * len(b_ops) // nbs:(i + 1) * len(b_ops) // nbs]
        for i in range(nc):
            valu[NM - nc + i] = c_ops[i * len(c_ops) // nc:(i + 1) * len(c_ops) // nc]
        valu[NM - 1] = valu[NM - 1] + self.check_ops(b)     # the row-sum test closes the last slot
        # the last K Q^T MFMA must be >= 11 wait states before the combine
        assert not c_ops or (self.DB + self.KS) * self.QB <= NM - nc - 3
        extra = {}
        extra[0] = ["s_cmp_ge_i32 s%d, s%d" % (self.s_tk, self.s_tfull),
                    "s_cbranch_scc1 %s" % L("KSLOW%d_" % b)] + self.dma_fast("k", b) + ["%s:" % L("KRET%d_" % b)]
        extra[1] = ["s_cmp_ge_i32 s%d, s%d" % (self.s_tv, self.s_tfull),
                    "s_cbranch_scc1 %s" % L("VSLOW%d_" % b)] + self.dma_fast("v", (b + 2) % 4) + ["%s:" % L("VRET%d_" % b)]
        extra[2] = [
            "s_add_u32 s%d, s%d, %d" % (self.s_kptr, self.s_kptr, self.TB),
            "s_addc_u32 s%d, s%d, 0" % (self.s_kptr + 1, self.s_kptr + 1),
            "s_add_u32 s%d, s%d, %d" % (self.s_vptr, self.s_vptr, self.TB),
            "s_addc_u32 s%d, s%d, 0" % (self.s_vptr + 1, self.s_vptr + 1),
            "s_add_i32 s%d, s%d, 1" % (self.s_tk, self.s_tk),
            "s_add_i32 s%d, s%d, 1" % (self.s_tv, self.s_tv),
            "s_add_i32 s%d, s%d, 1" % (self.s_j, self.s_j)]
        self.stream(self.groups(), P_prev, S_nxt, kst, vst, valu, extra, self.PFD, nxt)
        self.e("s_cmp_lg_u32 s%d, 0" % self.s_resc)
        self.e("s_cbranch_scc1 %s" % L("RESCO%d_" % b))
        self.e("%s:" % L("RESCORET%d_" % b))
        if b == 3:
            self.e("s_branch %s" % L("BODY0_"))

    def out_of_line(self, b):
        L = self.lab
        S_cur = self.SA if b % 2 == 0 else self.SB
        QB = self.QB
        # ---- mask pre-pass
        self.e("%s:" % L("MASK%d_" % b))
        self.e("s_lshl_b32 s%d, s%d, 5" % (self.s_t2, self.s_j))
        self.e("v_mov_b32 v%d, 0xff800000" % self.NEGINF)
        for qb in range(QB):
            self.e("v_subrev_u32 v%d, s%d, v%d" % (self.THR + qb, self.s_t2, self.THRB + qb))
        for qb in range(QB):
            for r in range(16):
                const = 8 * (r >> 2) + (r & 3)
                x = self.s_reg(S_cur, qb, 0, r)
                self.e("v_cmp_gt_i32 vcc, %d, v%d" % (const, self.THR + qb))
                self.e("v_cndmask_b32 v%d, v%d, v%d, vcc" % (x, x, self.NEGINF))
        self.e("s_branch %s" % L("MASKRET%d_" % b))
        # ---- a tile row sum failed the test: exact row maxima of the (intact) scores, move the references
        # there (alpha = exp2((m_ref - m_new) c); 0 when m_ref was still -inf), redo the tile's P
        P_new = self.PB if b % 2 == 0 else self.PA
        self.e("%s:" % L("SLOW%d_" % b))
        for ins in self.max_ops(S_cur) + self.pairmax_ops():
            self.e(ins)
        for qb in range(QB):
            self.e("v_sub_f32 v%d, v%d, v%d" % (self.DD + qb, self.MREF + qb, self.T + qb))
            self.e("v_mul_f32 v%d, s%d, v%d" % (self.DD + qb, self.s_c, self.DD + qb))
            self.e("v_exp_f32 v%d, v%d" % (self.ALPHA + qb, self.DD + qb))
            self.e("v_mov_b32 v%d, v%d" % (self.MREF + qb, self.T + qb))
            self.e("v_mul_f32 v%d, s%d, v%d" % (self.MRC + qb, self.s_c, self.T + qb))
        self.e("s_nop 1")
        for qb in range(QB):
            self.e("v_mul_f32 v%d, v%d, v%d" % (self.L + qb, self.L + qb, self.ALPHA + qb))
        self.e("s_mov_b32 s%d, 1" % self.s_resc)
        for ins in self.pair_ops(S_cur, P_new):
            self.e(ins)
        self.e("s_nop 7")
        self.e("s_branch %s" % L("SLOWRET%d_" % b))
        # ---- O *= alpha (accumulators live in AGPRs: read, scale, write back)
        self.e("%s:" % L("RESCO%d_" % b))
        self.e("s_nop 15")
        self.e("s_nop 7")
        for qb in range(QB):
            regs = [self.O + 16 * (qb * self.DB + db) + r for db in range(self.DB) for r in range(16)]
            for i in range(0, len(regs), 4):
                for t in range(4):
                    self.e("v_accvgpr_read_b32 v%d, a%d" % (self.AT + t, regs[i + t]))
                self.e("s_nop 1")
                for t in range(4):
                    self.e("v_mul_f32 v%d, v%d, v%d" % (self.AT + t, self.ALPHA + qb, self.AT + t))
                self.e("s_nop 1")
                for t in range(4):
                    self.e("v_accvgpr_write_b32 a%d, v%d" % (regs[i + t], self.AT + t))
        self.e("s_mov_b32 s%d, 0" % self.s_resc)
        self.e("s_nop 7")
        self.e("s_branch %s" % L("RESCORET%d_" % b))
        self.dma_slow("k", b, L("KSLOW%d_" % b), L("KRET%d_" % b))
        self.dma_slow("v", (b + 2) % 4, L("VSLOW%d_" % b), L("VRET%d_" % b))

    def drain(self, b):
        L = self.lab
        P_prev = self.PA if b % 2 == 0 else self.PB
        vst = (b + 3) % 4
        pv = [("pv", kc, db) for kc in range(2) for db in range(self.DB)]
        self.e("%s:" % L("EXIT%d_" % b))
        self.outstanding = [i for i in range(self.PFD) for _ in range(2)]
        self.stream(pv, P_prev, 0, 0, vst, {}, {}, self.PFD, None)
        self.e("s_branch %s" % L("DONE_"))

    def generate(self):
        L = self.lab
        e = self.e
        QB = self.QB
        e("s_nop 15")
        e("s_nop 7")
        e("s_mov_b32 s%d, m0" % self.s_m0)
        e("s_mov_b32 s%d, 0" % self.s_j)
        e("s_mov_b32 s%d, 0" % self.s_resc)
        # bound on a lane's row sum over one tile (every P of the tile is then below it); small, so that a
        # key that outgrows the reference by more than a few bits moves the reference onto itself and its
        # P is exactly 1 (see gen_attn_loop.py)
        tau = 2.0 ** 8
        e("s_mov_b32 s%d, 0x%08x" % (self.s_tau, struct.unpack("<I", struct.pack("<f", tau))[0]))
        e("s_add_u32 s%d, s%d, %d" % (self.s_kptr, self.s_kbase, 4 * self.TB))
        e("s_addc_u32 s%d, s%d, 0" % (self.s_kptr + 1, self.s_kbase + 1))
        e("s_add_u32 s%d, s%d, %d" % (self.s_vptr, self.s_vbase, 2 * self.TB))
        e("s_addc_u32 s%d, s%d, 0" % (self.s_vptr + 1, self.s_vbase + 1))
        e("s_mov_b32 s%d, 4" % self.s_tk)
        e("s_mov_b32 s%d, 2" % self.s_tv)
        for i in range(8 * QB):
            e("v_mov_b32 v%d, 0" % (self.PA + i))
        for qb in range(QB):
            e("v_mov_b32 v%d, 0xff800000" % (self.MREF + qb))      # no reference yet: the first tile's test fails
            e("v_mov_b32 v%d, 0xff800000" % (self.MRC + qb))
            e("v_mov_b32 v%d, 0" % (self.L + qb))
            e("v_mov_b32 v%d, 1.0" % (self.ALPHA + qb))
        self.outstanding = []
        g0 = self.groups()
        assert all(g[0] == "pv" for g in g0[:self.PFD])
        for i in range(self.PFD):
            for ins in self.frag_loads(g0[i], i % self.NF, 1, 3):
                e(ins)
                self.outstanding.append(i)
        for b in range(4):
            self.body(b)
        for b in range(4):
            self.out_of_line(b)
        for b in range(4):
            self.drain(b)
        e("%s:" % L("DONE_"))
        e("s_waitcnt vmcnt(0) lgkmcnt(0)")
        e("s_mov_b32 m0, s%d" % self.s_m0)
        e("s_nop 15")
        e("s_nop 7")

    # ----------------------------------------------------------- C++ wrapper
    def emit_inc(self):
        self.generate()
        D, DB, KS, QB = self.D, self.DB, self.KS, self.QB
        out = []
        out.append("// Generated by gen_attn_loop2.py %s -- do not edit.  Main loop of attn_fwd_asm2_kernel<%d, %d, *>." % (self.name, D, QB))
        out.append("// VGPRs used: %d, AGPRs used: %d.  MFMA slots per iteration: %d." % (self.NV, self.NA, self.NM))
        out.append("asm volatile(")
        for ln in self.lines:
            out.append('    "%s\\n\\t"' % ln)
        outs, ins = [], []
        for i in range(QB * DB):
            outs.append('"+{%s}"(o_acc[%d])' % (self.ar(self.O + 16 * i, 16), i))
        for qb in range(QB):
            outs.append('"+{%s}"(s_init[%d])' % (self.vr(self.s_reg(self.SA, qb, 0), 16), qb))
        outs.append('"={%s}"(m_ref_v)' % self.vr(self.MREF, QB))
        outs.append('"={%s}"(l_run_v)' % self.vr(self.L, QB))
        for i in range(4 * QB * KS // 16):
            ins.append('"{%s}"(q_pack[%d])' % (self.ar(self.Q + 16 * i, 16), i))
        ins.append('"{%s}"(koff_v)' % self.vr(self.KOFF, KS))
        ins.append('"{%s}"(voff_v)' % self.vr(self.VOFF, 2 * DB))
        ins.append('"{%s}"(dma_voff_v)' % self.vr(self.DVOFF, self.NLD))
        ins.append('"{%s}"(dma_row_v)' % self.vr(self.DROW, self.NLD))
        ins.append('"{%s}"(dma_choff_v)' % self.vr(self.DCH, self.NLD))
        ins.append('"{%s}"(thr_base_v)' % self.vr(self.THRB, QB))
        ins.append('"{%s}"(k_head)' % self.sr(self.s_kbase, 2))
        ins.append('"{%s}"(v_head)' % self.sr(self.s_vbase, 2))
        ins.append('"{s%d}"(c_log2e)' % self.s_c)
        ins.append('"{s%d}"(n_tiles)' % self.s_ntiles)
        ins.append('"{s%d}"(j_mask)' % self.s_jmask)
        ins.append('"{s%d}"(t_full)' % self.s_tfull)
        ins.append('"{s%d}"(skv_m1)' % self.s_skvm1)
        ins.append('"{s%d}"(lds_k_wave)' % self.s_ldsk)
        ins.append('"{s%d}"(lds_v_wave)' % self.s_ldsv)
        pinned = set()
        for qb in range(QB):
            pinned.update(range(self.s_reg(self.SA, qb, 0), self.s_reg(self.SA, qb, 0) + 16))
        for base, n in ((self.MREF, QB), (self.L, QB), (self.THRB, QB), (self.KOFF, KS),
                        (self.VOFF, 2 * DB), (self.DVOFF, self.NLD), (self.DROW, self.NLD), (self.DCH, self.NLD)):
            pinned.update(range(base, base + n))
        clob = ['"memory"', '"vcc"', '"scc"']
        clob += ['"v%d"' % i for i in range(self.NV) if i not in pinned]
        clob += ['"s%d"' % i for i in range(self.s_j, self.s_m0 + 1)]
        out.append("    : " + ", ".join(outs))
        out.append("    : " + ", ".join(ins))
        out.append("    : " + ", ".join(clob) + ");")
        return "\n".join(out) + "\n"


if __name__ == "__main__":
    text = Gen(sys.argv[1], dtype=sys.argv[3] if len(sys.argv) > 3 else "bf16").emit_inc()
    with open(sys.argv[2], "w") as f:
        f.write(text)
