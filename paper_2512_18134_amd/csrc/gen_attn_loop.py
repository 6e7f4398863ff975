#!/usr/bin/env python3
"""Emit the hand-scheduled main loop of the gfx950 attention-forward kernel.

The loop is the paper's Fig. 1a, modulo-scheduled by hand for CDNA4 (Section 3.1
vocabulary: initiation interval I = one K/V tile = NM MFMA slots per wave,
schedule length L = 3 I).  Iteration j of the steady state issues, from one
in-order instruction stream per wave,

    slot i:  [s_waitcnt for the operand of MFMA i]
             MFMA i            -- first half of P(j-1) V(j-1), then K(j+1) Q^T,
                                  then the second half of P(j-1) V(j-1)
             LDS reads for MFMA i+PFD (K fragment: ds_read_b128, V^T fragment:
                                  2 x ds_read_b64_tr_b16), a ring of NF buffers
             ~VPS VALU/transcendental ops of softmax(S(j)): fma -> exp2 -> row-sum
                                  add -> bf16 pack, software pipelined over element
                                  pairs (no row maximum on this path, see below)

so that the matrix pipe (32 cycles per MFMA) and the VALU run side by side; the
same stream runs on two waves per SIMD, which fills the remaining bubbles.
K/V tiles arrive by direct global->LDS loads into 4-stage rings, two tiles
ahead, with one workgroup barrier per tile.

Online softmax without a per-tile row maximum.  P = exp2(c s - c m_ref) is
taken against the reference m_ref the row already has; floating point is scale
invariant, so a reference that lags the true maximum costs no accuracy as long
as nothing overflows.  The only per-tile test is therefore on the tile's row
sum (which is needed anyway): if it is not below 2^8 (an element has grown
too large, has overflowed, or m_ref is still -inf in the first tile) the wave
leaves the interleaved stream for an out-of-line pass that finds the exact row
maximum of the tile, moves m_ref there, scales the running sum (and, deferred
to the end of the iteration, the accumulator) by alpha = exp2(c (m_old - m_new))
and recomputes the tile's P from its scores, which the fast path leaves intact
(the exponent arguments go to temporaries).  On N(0,1) inputs this pass runs
once per workgroup; it replaces 29 of the 140 VALU operations per tile.

The compiler cannot be made to hold this schedule inside 256 VGPRs (it spills),
so registers are assigned here and the loop is emitted as ONE inline-asm
statement with operands pinned to physical registers.  Everything around the
loop (addressing, Q load, S(0), normalisation, stores) stays in HIP C++.

Hazards handled by construction (the assembler inserts no wait states):
  * MFMA result -> VALU read needs 11 wait states for an 8-pass MFMA: the
    K Q^T MFMAs sit in the middle of the iteration, S is first read in the next;
    explicit s_nop before the accumulator rescale and at loop exit.
  * transcendental result -> VALU use needs 1 wait state: the element-pair
    pipeline keeps >= 4 instructions between producer and consumer.
  * LDS reads return in order: every s_waitcnt lgkmcnt(N) is computed by
    replaying the instruction stream (including the reads prefetched for the
    next iteration).

usage: gen_attn_loop.py <D> <out.inc> [bf16|f16] [waves per workgroup: 8|4] [--pfd N] [--drop part,part]
(--pfd and --drop exist for timing experiments; a library build passes neither)
"""
import struct
import sys


class Gen:
    def __init__(self, D, NF=4, PFD=3, dtype="bf16", NW=8, drop=()):
        assert D in (64, 128) and dtype in ("bf16", "f16") and NW in (4, 8)
        self.NW = NW                      # waves per workgroup: every wave loads 1/NW of each K/V tile
        self.D = D
        self.dtype = dtype
        # the two element types differ only in the MFMA and in the pack instruction (both round to nearest even)
        self.mfma = "v_mfma_f32_32x32x16_" + dtype
        self.cvt = "v_cvt_pk_%s_f32" % dtype
        self.KS = D // 16
        self.DB = D // 32
        self.ROWB = 2 * D
        self.TB = 64 * self.ROWB
        self.NLD = self.TB // (NW * 1024)
        self.NSTG = 4
        self.NF, self.PFD = NF, PFD
        self.NPV = 4 * self.DB
        self.NQK = 2 * self.KS
        self.NM = self.NPV + self.NQK
        assert self.NM % NF == 0 and PFD < NF
        # ---- VGPR map
        r = 0
        def take(n):
            nonlocal r
            b = r
            r += n
            return b
        self.O = take(16 * self.DB)
        self.Q = take(4 * self.KS)
        self.SA = take(32)
        self.SB = take(32)
        self.PA = take(16)
        self.PB = take(16)
        self.FR = take(4 * NF)
        self.KOFF = take(self.KS)
        self.VOFF = take(2 * self.DB)
        self.DVOFF = take(self.NLD)
        self.DROW = take(self.NLD)
        self.DCH = take(self.NLD)
        self.MREF = take(1)
        self.MRC = take(1)
        self.L = take(1)                  # running row sum (this lane's half of the keys)
        self.TLA = take(1)                # row sum of the current tile, two partial sums
        self.TLB = take(1)
        self.TP = take(6)                 # exponent / exp temporaries of three element pairs in flight
        self.ALPHA = take(1)
        self.THRB = take(1)
        self.MX0 = take(1)
        self.MX1 = take(1)
        self.T = take(1)
        self.TMP2 = take(1)
        self.DD = take(1)
        self.NEGINF = take(1)
        self.THR = take(1)
        self.DT = take(2 * self.NLD)  # address temporaries of the ragged-tile loads
        self.NV = r
        assert r <= 256, r
        # ---- SGPR map (inputs pinned by the asm constraints, the rest clobbered)
        self.s_kbase, self.s_vbase = 32, 34
        self.s_c, self.s_ntiles, self.s_jmask, self.s_tfull, self.s_skvm1 = 36, 37, 38, 39, 40
        self.s_ldsk, self.s_ldsv = 41, 42
        self.s_j, self.s_resc, self.s_tau = 43, 44, 45
        self.s_kptr, self.s_vptr = 46, 48
        self.s_tk, self.s_tv = 50, 51
        self.s_t0 = 52            # s[52:53] scratch pair
        self.s_t2 = 54
        self.s_m0 = 55            # m0 of the surrounding code (reserved register: saved and restored here)
        self.lines = []
        # timing experiments only (results are wrong with any of these set): parts of the loop to leave out
        self.exp = set(drop)

    def tau_bits(self):
        """Bound on a lane's row sum over one tile, as fp32 bits: 2^8, so every P of a tile that passes is
        below 2^8 (inside fp16's range too).  The bound could be far larger without overflow (bf16 has
        fp32's exponent range), but a small one keeps one-hot rows exact: a key that outgrows the reference
        by more than a few bits moves the reference onto itself, its P is then exactly 1 and O is exactly
        its V row; with a lagging reference its P = 2^x would be rounded to bf16 (2^-9 relative)."""
        return struct.unpack("<I", struct.pack("<f", 2.0 ** 8))[0]

    # ------------------------------------------------------------------ helpers
    def e(self, s):
        self.lines.append(s)

    def lab(self, name):
        return "%s%%=" % name   # unique per expansion of the asm statement

    def vr(self, base, n=1):
        return "v%d" % base if n == 1 else "v[%d:%d]" % (base, base + n - 1)

    def sr(self, base, n=1):
        return "s%d" % base if n == 1 else "s[%d:%d]" % (base, base + n - 1)

    # ------------------------------------------------------------ MFMA programs
    def mfma_list(self):
        """[(kind, a, b)] in issue order: ('pv', kc, db) and ('qk', ks, sb)."""
        DB, KS = self.DB, self.KS
        pv = [("pv", kc, db) for kc in range(4) for db in range(DB)]
        qk = [("qk", ks, sb) for ks in range(KS) for sb in range(2)]
        return pv[:2 * DB] + qk + pv[2 * DB:]

    def frag_loads(self, op, buf, kst, vst):
        """LDS reads that bring the A operand of `op` into fragment buffer `buf`."""
        f = self.FR + 4 * buf
        kind, a, b = op
        if "nolds" in self.exp:
            return []
        if kind == "pv":
            kc, db = a, b
            off = vst * self.TB + kc * 16 * self.ROWB
            assert off < 65536
            return ["ds_read_b64_tr_b16 %s, %s offset:%d" % (self.vr(f, 2), self.vr(self.VOFF + 2 * db), off),
                    "ds_read_b64_tr_b16 %s, %s offset:%d" % (self.vr(f + 2, 2), self.vr(self.VOFF + 2 * db + 1), off)]
        ks, sb = a, b
        off = kst * self.TB + sb * 32 * self.ROWB
        assert off < 65536
        return ["ds_read_b128 %s, %s offset:%d" % (self.vr(f, 4), self.vr(self.KOFF + ks), off)]

    def mfma_text(self, op, buf, P_prev, S_nxt):
        f = self.vr(self.FR + 4 * buf, 4)
        kind, a, b = op
        if kind == "pv":
            kc, db = a, b
            o = self.vr(self.O + 16 * db, 16)
            return "%s %s, %s, %s, %s" % (self.mfma, o, f, self.vr(P_prev + 4 * kc, 4), o)
        ks, sb = a, b
        s = self.vr(S_nxt + 16 * sb, 16)
        return "%s %s, %s, %s, %s" % (self.mfma, s, f, self.vr(self.Q + 4 * ks, 4), "0" if ks == 0 else s)

    # ---------------------------------------------------------- softmax programs
    def max_ops(self, S_cur):
        """Row max of the lane's 32 scores into T, two interleaved max3 chains."""
        ops = []
        if "nomax" in self.exp:
            return []
        ch = [[], []]
        for c, mx in enumerate((self.MX0, self.MX1)):
            s = [S_cur + 16 * c + i for i in range(16)]
            ch[c].append("v_max3_f32 v%d, v%d, v%d, v%d" % (mx, s[0], s[1], s[2]))
            for i in range(3, 15, 2):
                ch[c].append("v_max3_f32 v%d, v%d, v%d, v%d" % (mx, mx, s[i], s[i + 1]))
            ch[c].append("v_max_f32 v%d, v%d, v%d" % (mx, mx, s[15]))
        for a, b in zip(ch[0], ch[1]):
            ops += [a, b]
        ops.append("v_max_f32 v%d, v%d, v%d" % (self.T, self.MX0, self.MX1))
        return ops

    def pairmax_ops(self):
        """Lane-pair max (the two lanes that hold one query's keys) and the new reference maximum into T."""
        T, TMP2 = self.T, self.TMP2
        return [
            "v_mov_b32 v%d, v%d" % (TMP2, T),
            "s_nop 1",
            "v_permlane32_swap_b32 v%d, v%d" % (T, TMP2),   # T = {lo,lo}, TMP2 = {hi,hi}
            "s_nop 1",
            "v_max_f32 v%d, v%d, v%d" % (T, T, TMP2),
            "v_max_f32 v%d, v%d, v%d" % (T, T, self.MREF),  # m_new
        ]

    def pair_ops(self, S_cur, P_new):
        """fma -> exp2 -> row-sum add -> bf16 pack over the 16 element pairs, software pipelined three deep.
        The exponent arguments go to the temporaries TP: S_cur stays intact for the out-of-line pass."""
        ops = []
        def tp(k, i):
            return self.TP + 2 * (k % 3) + i
        def F(k):
            return ["v_fma_f32 v%d, v%d, s%d, -v%d" % (tp(k, i), S_cur + 2 * k + i, self.s_c, self.MRC) for i in (0, 1)]
        def E(k):
            return ["v_exp_f32 v%d, v%d" % (tp(k, i), tp(k, i)) for i in (0, 1)]
        def A(k):
            if k == 0:   # the first pair starts the tile's two partial sums
                acc = ["v_mov_b32 v%d, v%d" % (self.TLA, tp(k, 0)), "v_mov_b32 v%d, v%d" % (self.TLB, tp(k, 1))]
            else:
                acc = ["v_add_f32 v%d, v%d, v%d" % (self.TLA, self.TLA, tp(k, 0)),
                       "v_add_f32 v%d, v%d, v%d" % (self.TLB, self.TLB, tp(k, 1))]
            return acc + ["%s v%d, v%d, v%d" % (self.cvt, P_new + k, tp(k, 0), tp(k, 1))]
        if "novalu" in self.exp:
            return []
        for t in range(16 + 2):
            if t < 16:
                ops += F(t)
            if 0 <= t - 1 < 16:
                ops += E(t - 1)
            if 0 <= t - 2 < 16:
                ops += A(t - 2)
        ops.append("v_add_f32 v%d, v%d, v%d" % (self.TLA, self.TLA, self.TLB))
        return ops

    def check_ops(self, b):
        """Tile row sum below the bound?  Otherwise (too large, inf or NaN) take the out-of-line pass."""
        t0 = self.sr(self.s_t0, 2)
        if "novalu" in self.exp:
            return []
        return [
            "v_cmp_ngt_f32 %s, s%d, v%d" % (t0, self.s_tau, self.TLA),   # not (bound > sum)
            "s_cmp_lg_u64 %s, 0" % t0,
            "s_cbranch_scc1 %s" % self.lab("SLOW%d_" % b),
            "%s:" % self.lab("SLOWRET%d_" % b),
            "v_add_f32 v%d, v%d, v%d" % (self.L, self.L, self.TLA),
        ]

    # ------------------------------------------------------------------- DMA
    def dma_fast(self, which, stage):
        """Issue one K or V tile: NLD direct loads, scalar base already points at the tile."""
        lds = self.s_ldsk if which == "k" else self.s_ldsv
        ptr = self.s_kptr if which == "k" else self.s_vptr
        out = []
        for i in range(self.NLD):
            if "nodma" in self.exp:
                out.append([])
                continue
            out.append(["s_add_u32 m0, s%d, %d" % (lds, stage * self.TB + i * self.NW * 1024),
                        "s_nop 0",
                        "global_load_lds_dwordx4 v%d, %s" % (self.DVOFF + i, self.sr(ptr, 2))])
        return out

    def dma_slow(self, which, stage, label, ret):
        """Ragged / past-the-end tile: clamp the row index, read through the head's base pointer."""
        lds = self.s_ldsk if which == "k" else self.s_ldsv
        base = self.s_kbase if which == "k" else self.s_vbase
        st = self.s_tk if which == "k" else self.s_tv
        sh = {128: 7, 256: 8}[self.ROWB]
        self.e("%s:" % label)
        self.e("s_lshl_b32 s%d, s%d, 6" % (self.s_t2, st))
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
    def stream(self, mfmas, P_prev, S_nxt, kst, vst, valu_by_slot, extra_by_slot, prefetched, nxt):
        """Emit the slots of one iteration.

        mfmas: list of ops; prefetched: how many leading operands are already in flight
        (ids in self.outstanding); nxt: (mfma list, kst, vst) of the following iteration whose
        first PFD operands are prefetched at the tail, or None.
        """
        NF, PFD = self.NF, self.PFD
        n = len(mfmas)
        def issue(idx, op, k, v):
            if "halflds" in self.exp and idx % 2 == 1:
                return
            for ins in self.frag_loads(op, idx % NF, k, v):
                self.e(ins)
                self.outstanding.append(idx)
        for i in range(prefetched, min(PFD, n)):
            issue(i, mfmas[i], kst, vst)
        for i, op in enumerate(mfmas):
            # wait until every read of operand i has returned (reads return in order)
            if "nolds" not in self.exp and any(x == i for x in self.outstanding):
                last = max(p for p, x in enumerate(self.outstanding) if x == i)
                after = len(self.outstanding) - 1 - last
                self.e("s_waitcnt lgkmcnt(%d)" % after)
                self.outstanding = self.outstanding[last + 1:]
            self.e(self.mfma_text(op, i % NF, P_prev, S_nxt))
            j = i + PFD
            if j < n:
                issue(j, mfmas[j], kst, vst)
            elif nxt is not None:
                nm, nk, nv = nxt
                issue(j - n + 1000, nm[j - n], nk, nv)   # ids >= 1000: next iteration's operands
            for ins in extra_by_slot.get(i, []):
                self.e(ins)
            for ins in valu_by_slot.get(i, []):
                self.e(ins)
        # rename the next iteration's prefetches to its own numbering
        self.outstanding = [x - 1000 for x in self.outstanding]
        assert "nolds" in self.exp or all(0 <= x < PFD for x in self.outstanding), self.outstanding

    # --------------------------------------------------------------- the loop
    def body(self, b):
        NM, NLD = self.NM, self.NLD
        S_cur, S_nxt = (self.SA, self.SB) if b % 2 == 0 else (self.SB, self.SA)
        P_prev, P_new = (self.PA, self.PB) if b % 2 == 0 else (self.PB, self.PA)
        kst, vst = (b + 1) % 4, (b + 3) % 4           # stages of K(j+1), V(j-1)
        nb = (b + 1) % 4
        nxt = (self.mfma_list(), (nb + 1) % 4, (nb + 3) % 4)
        L = self.lab
        self.e("%s:" % L("BODY%d_" % b))
        self.e("s_cmp_ge_i32 s%d, s%d" % (self.s_j, self.s_ntiles))
        self.e("s_cbranch_scc1 %s" % L("EXIT%d_" % b))
        self.e("s_cmp_ge_i32 s%d, s%d" % (self.s_j, self.s_jmask))
        self.e("s_cbranch_scc1 %s" % L("MASK%d_" % b))
        self.e("%s:" % L("MASKRET%d_" % b))
        # loads of the previous iteration may stay in flight; everything older has landed
        if "nobar" not in self.exp:
            self.e("s_waitcnt vmcnt(%d)" % (2 * NLD))
            self.e("s_barrier")
        # ---- VALU program, dealt out evenly over the slots; the row-sum test closes the last slot
        b_ops = self.pair_ops(S_cur, P_new)
        valu = {}
        for i in range(NM):
            valu[i] = b_ops[i * len(b_ops) // NM:(i + 1) * len(b_ops) // NM]
        valu[NM - 1] = valu[NM - 1] + self.check_ops(b)
        # ---- K(j+4) -> K stage b, V(j+2) -> V stage (b+2)%4, spread over the first slots
        # (a fast/slow choice must not jump over other slots' work: each tensor's issue is contiguous)
        extra = {}
        extra[0] = ["s_cmp_ge_i32 s%d, s%d" % (self.s_tk, self.s_tfull),
                    "s_cbranch_scc1 %s" % L("KSLOW%d_" % b)]
        for grp in self.dma_fast("k", b):
            extra[0].extend(grp)
        extra[0].append("%s:" % L("KRET%d_" % b))
        extra[1] = ["s_cmp_ge_i32 s%d, s%d" % (self.s_tv, self.s_tfull),
                    "s_cbranch_scc1 %s" % L("VSLOW%d_" % b)]
        for grp in self.dma_fast("v", (b + 2) % 4):
            extra[1].extend(grp)
        extra[1].append("%s:" % L("VRET%d_" % b))
        extra[2] = [
            "s_add_u32 s%d, s%d, %d" % (self.s_kptr, self.s_kptr, self.TB),
            "s_addc_u32 s%d, s%d, 0" % (self.s_kptr + 1, self.s_kptr + 1),
            "s_add_u32 s%d, s%d, %d" % (self.s_vptr, self.s_vptr, self.TB),
            "s_addc_u32 s%d, s%d, 0" % (self.s_vptr + 1, self.s_vptr + 1),
            "s_add_i32 s%d, s%d, 1" % (self.s_tk, self.s_tk),
            "s_add_i32 s%d, s%d, 1" % (self.s_tv, self.s_tv),
            "s_add_i32 s%d, s%d, 1" % (self.s_j, self.s_j)]
        self.stream(self.mfma_list(), P_prev, S_nxt, kst, vst, valu, extra, self.PFD, nxt)
        # ---- deferred accumulator rescale (rare)
        self.e("s_cmp_lg_u32 s%d, 0" % self.s_resc)
        self.e("s_cbranch_scc1 %s" % L("RESCO%d_" % b))
        self.e("%s:" % L("RESCORET%d_" % b))
        if b == 3:
            self.e("s_branch %s" % L("BODY0_"))

    def out_of_line(self, b):
        L = self.lab
        S_cur = self.SA if b % 2 == 0 else self.SB
        # ---- mask pre-pass: keys past the causal diagonal / past S_kv become -inf
        self.e("%s:" % L("MASK%d_" % b))
        self.e("s_lshl_b32 s%d, s%d, 6" % (self.s_t2, self.s_j))
        self.e("v_subrev_u32 v%d, s%d, v%d" % (self.THR, self.s_t2, self.THRB))  # limit - 4g - 64 j
        self.e("v_mov_b32 v%d, 0xff800000" % self.NEGINF)
        for el in range(32):
            sb, r = el // 16, el % 16
            const = 32 * sb + 8 * (r >> 2) + (r & 3)
            self.e("v_cmp_gt_i32 vcc, %d, v%d" % (const, self.THR))       # key index > limit ?
            self.e("v_cndmask_b32 v%d, v%d, v%d, vcc" % (S_cur + el, S_cur + el, self.NEGINF))
        self.e("s_branch %s" % L("MASKRET%d_" % b))
        # ---- the tile's row sum failed the test: exact row maximum of the (intact) scores, move the
        # reference there (alpha = exp2((m_ref - m_new) c); 0 when m_ref was still -inf), redo the tile's P
        P_new = self.PB if b % 2 == 0 else self.PA
        self.e("%s:" % L("SLOW%d_" % b))
        for ins in self.max_ops(S_cur) + self.pairmax_ops():
            self.e(ins)
        self.e("v_sub_f32 v%d, v%d, v%d" % (self.DD, self.MREF, self.T))
        self.e("v_mul_f32 v%d, s%d, v%d" % (self.DD, self.s_c, self.DD))
        self.e("v_exp_f32 v%d, v%d" % (self.ALPHA, self.DD))
        self.e("v_mov_b32 v%d, v%d" % (self.MREF, self.T))
        self.e("v_mul_f32 v%d, s%d, v%d" % (self.MRC, self.s_c, self.T))
        self.e("s_nop 1")
        self.e("v_mul_f32 v%d, v%d, v%d" % (self.L, self.L, self.ALPHA))
        self.e("s_mov_b32 s%d, 1" % self.s_resc)
        for ins in self.pair_ops(S_cur, P_new):
            self.e(ins)
        self.e("s_nop 7")
        self.e("s_branch %s" % L("SLOWRET%d_" % b))
        # ---- O *= alpha once every MFMA of P(j-1) V(j-1) has been issued and has retired
        self.e("%s:" % L("RESCO%d_" % b))
        self.e("s_nop 15")
        self.e("s_nop 7")
        for i in range(16 * self.DB):
            self.e("v_mul_f32 v%d, v%d, v%d" % (self.O + i, self.ALPHA, self.O + i))
        self.e("s_mov_b32 s%d, 0" % self.s_resc)
        self.e("s_nop 7")
        self.e("s_branch %s" % L("RESCORET%d_" % b))
        # ---- ragged-tile loads
        self.dma_slow("k", b, L("KSLOW%d_" % b), L("KRET%d_" % b))
        self.dma_slow("v", (b + 2) % 4, L("VSLOW%d_" % b), L("VRET%d_" % b))

    def drain(self, b):
        """Loop exit taken at the top of iteration b: O += P(n-1) V(n-1), operands of the first
        PFD MFMAs were prefetched by the previous iteration."""
        L = self.lab
        P_prev = self.PA if b % 2 == 0 else self.PB
        vst = (b + 3) % 4
        pv = [("pv", kc, db) for kc in range(4) for db in range(self.DB)]
        self.e("%s:" % L("EXIT%d_" % b))
        # the prefetched operands belong to the interleaved order (first half of PV only): same ops
        self.outstanding = [i for i in range(self.PFD) for _ in range(2) if not ("halflds" in self.exp and i % 2 == 1)]
        self.stream(pv, P_prev, 0, 0, vst, {}, {}, self.PFD, None)
        self.e("s_branch %s" % L("DONE_"))

    def generate(self):
        L = self.lab
        e = self.e
        e("s_nop 15")
        e("s_nop 7")
        e("s_mov_b32 s%d, m0" % self.s_m0)
        e("s_mov_b32 s%d, 0" % self.s_j)
        e("s_mov_b32 s%d, 0" % self.s_resc)
        e("s_mov_b32 s%d, 0x%08x" % (self.s_tau, self.tau_bits()))   # bound on a tile's row sum
        e("s_add_u32 s%d, s%d, %d" % (self.s_kptr, self.s_kbase, 4 * self.TB))
        e("s_addc_u32 s%d, s%d, 0" % (self.s_kptr + 1, self.s_kbase + 1))
        e("s_add_u32 s%d, s%d, %d" % (self.s_vptr, self.s_vbase, 2 * self.TB))
        e("s_addc_u32 s%d, s%d, 0" % (self.s_vptr + 1, self.s_vbase + 1))
        e("s_mov_b32 s%d, 4" % self.s_tk)
        e("s_mov_b32 s%d, 2" % self.s_tv)
        for i in range(16):
            e("v_mov_b32 v%d, 0" % (self.PA + i))                # P(-1) = 0
        e("v_mov_b32 v%d, 0xff800000" % self.MREF)              # no reference yet: the first tile's test fails
        e("v_mov_b32 v%d, 0xff800000" % self.MRC)
        e("v_mov_b32 v%d, 0" % self.L)
        e("v_mov_b32 v%d, 1.0" % self.ALPHA)
        # operands of the first PFD MFMAs of iteration 0 ("V(-1)" lives in stage 3)
        self.outstanding = []
        m0 = self.mfma_list()
        for i in range(self.PFD):
            for ins in self.frag_loads(m0[i], i % self.NF, 1, 3):
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
        D, DB, KS = self.D, self.DB, self.KS
        out = []
        out.append("// Generated by gen_attn_loop.py %d %s -- do not edit.  Main loop of attn_fwd_asm_kernel<%d, *> (%s)." % (D, self.dtype, D, self.dtype))
        out.append("// VGPRs used: %d.  MFMA slots per iteration: %d." % (self.NV, self.NM))
        out.append("asm volatile(")
        for ln in self.lines:
            out.append('    "%s\\n\\t"' % ln)
        # outputs
        outs = []
        for db in range(DB):
            outs.append('"+{%s}"(o_acc[%d])' % (self.vr(self.O + 16 * db, 16), db))
        outs.append('"+{%s}"(s_init[0])' % self.vr(self.SA, 16))
        outs.append('"+{%s}"(s_init[1])' % self.vr(self.SA + 16, 16))
        outs.append('"={%s}"(m_ref)' % self.vr(self.MREF))
        outs.append('"={%s}"(l_run)' % self.vr(self.L))
        ins = []
        nq = 4 * KS // 16
        for i in range(nq):
            ins.append('"{%s}"(q_pack[%d])' % (self.vr(self.Q + 16 * i, 16), i))
        ins.append('"{%s}"(koff_v)' % self.vr(self.KOFF, KS))
        ins.append('"{%s}"(voff_v)' % self.vr(self.VOFF, 2 * DB))
        ins.append('"{%s}"(dma_voff_v)' % self.vr(self.DVOFF, self.NLD))
        ins.append('"{%s}"(dma_row_v)' % self.vr(self.DROW, self.NLD))
        ins.append('"{%s}"(dma_choff_v)' % self.vr(self.DCH, self.NLD))
        ins.append('"{%s}"(thr_base)' % self.vr(self.THRB))
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
        for db in range(DB):
            pinned.update(range(self.O + 16 * db, self.O + 16 * db + 16))
        pinned.update(range(self.SA, self.SA + 32))
        pinned.update([self.MREF, self.L, self.THRB])
        pinned.update(range(self.Q, self.Q + 4 * KS))
        pinned.update(range(self.KOFF, self.KOFF + KS))
        pinned.update(range(self.VOFF, self.VOFF + 2 * DB))
        pinned.update(range(self.DVOFF, self.DVOFF + self.NLD))
        pinned.update(range(self.DROW, self.DROW + self.NLD))
        pinned.update(range(self.DCH, self.DCH + self.NLD))
        clob = ['"memory"', '"vcc"', '"scc"']
        clob += ['"v%d"' % i for i in range(self.NV) if i not in pinned]
        clob += ['"s%d"' % i for i in range(self.s_j, self.s_m0 + 1)]
        out.append("    : " + ", ".join(outs))
        out.append("    : " + ", ".join(ins))
        out.append("    : " + ", ".join(clob) + ");")
        return "\n".join(out) + "\n"


if __name__ == "__main__":
    args = sys.argv[1:]
    pfd, drop = 3, ()
    while len(args) > 2 and args[-2] in ("--pfd", "--drop"):
        if args[-2] == "--pfd":
            pfd = int(args[-1])
        else:
            drop = tuple(filter(None, args[-1].split(",")))
        args = args[:-2]
    D = int(args[0])
    dtype = args[2] if len(args) > 2 else "bf16"
    nw = int(args[3]) if len(args) > 3 else 8
    text = Gen(D, PFD=pfd, dtype=dtype, NW=nw, drop=drop).emit_inc()
    with open(args[1], "w") as f:
        f.write(text)
