#!/usr/bin/env python3
"""Emit the hand-scheduled main loop of the gfx950 attention-forward kernels.

The loop is the paper's Fig. 1a, modulo-scheduled by hand for CDNA4 (Section 3.1
vocabulary: initiation interval I = one K/V tile = NM MFMA slots per wave,
schedule length L = 3 I).  Iteration j of the steady state issues, from one
in-order instruction stream per wave,

    slot i:  [s_waitcnt for the operand of MFMA i]
             MFMA i            -- first half of P(j-1) V(j-1), then K(j+1) Q^T,
                                  then the second half of P(j-1) V(j-1)
             LDS reads for a later MFMA (K fragment: ds_read_b128, V^T fragment:
                                  2 x ds_read_b64_tr_b16), a ring of NF buffers
             this slot's share of softmax(S(j)): fma -> exp2 -> row-sum add ->
                                  16-bit pack, software pipelined over element pairs

so that the matrix pipe (32 cycles per MFMA) and the VALU run side by side.
K/V tiles arrive by direct global->LDS loads into 4-stage rings, two tiles
ahead, with one workgroup barrier per tile.

Tilings (CONFIGS): a wave owns QB blocks of 32 query rows; a K/V tile holds SB
blocks of 32 keys; a fragment read from LDS feeds QB MFMAs.
  * two waves per SIMD (8 waves x 32 rows): all 256 VGPRs of a wave are assigned
    here, O and Q included; the hardware arbiter interleaves the two streams;
  * one wave per SIMD (4 waves x 64 rows at D = 128, 4 x 32 at D = 256): the wave
    owns the SIMD's 512 registers, O and Q sit in AGPRs (the MFMA reads and writes
    them directly), everything the VALU touches in VGPRs.  Half the LDS operand
    reads per MFMA at D = 128; the stream has to keep the matrix pipe fed alone,
    so the instruction count per MFMA is what bounds it (see asm_emit.spread).

Online softmax without a per-tile row maximum.  P = exp2(c s - c m_ref) is
taken against the reference m_ref the row already has; floating point is scale
invariant, so a reference that lags the true maximum costs no accuracy as long
as nothing overflows.  The only per-tile test is on the tile's row sum (needed
anyway): if it is not below 2^8 (an element has grown large, has overflowed, or
m_ref is still -inf in the first tile) the wave leaves the interleaved stream
for an out-of-line pass that finds the exact row maximum of the tile, moves
m_ref there, scales the running sum and the accumulator by
alpha = exp2(c (m_old - m_new)) and recomputes the tile's P from its scores,
which the fast path leaves intact (the exponent arguments go to temporaries).
On N(0,1) inputs this pass runs once per workgroup.

Rare events share one test per iteration: j >= s_special (last tile, tiles that
need a mask, tiles whose loads reach past S_kv) branches out of line and comes
back with SCC saying whether this iteration's loads need their rows clamped,
which the two load slots test.

The ramp of the schedule is peeled, so no MFMA runs on operands that do not
exist: the first iteration holds K(1) Q^T and softmax(S(0)) only (there is no
P(-1) V(-1)), and the last tile has a body of its own per ring phase:
P(n-2) V(n-2) beside softmax(S(n-1)), then P(n-1) V(n-1), no K Q^T, no loads.
A launch with one tile leaves after the first iteration through P(0) V(0).

The compiler cannot be made to hold this schedule (it spills), so registers are
assigned here and the loop is emitted as ONE inline-asm statement with operands
pinned to physical registers.  Everything around the loop (addressing, Q load,
S(0), normalisation, stores) stays in HIP C++ (attn_fwd_asm.h).

Hazards handled by construction (the assembler inserts no wait states; the rules
are re-checked on the emitted text by asm_emit.check_stream in the tests):
  * MFMA result -> VALU read needs 11 wait states for an 8-pass MFMA: the
    K Q^T MFMAs sit in the middle of the iteration, S is first read in the next;
    explicit s_nop before the accumulator rescale and at loop exit.
  * transcendental result -> VALU use needs 1 wait state: the element-pair
    pipeline keeps >= 4 instructions between producer and consumer.
  * LDS reads return in order: every s_waitcnt lgkmcnt(N) is computed by
    replaying the instruction stream (including the reads prefetched for the
    next iteration).
  * scalar write of m0 -> direct load needs 1 wait state: an s_nop goes between
    them.

usage: gen_attn_loop.py <config> <out.inc> [bf16|f16] [--pfd N] [--nf N] [--w N] [--dep N] [--ls N] [--drop part,part]
(--pfd, --nf, --w, --dep, --ls and --drop exist for timing experiments; a library build passes none.
 --drop parts, results are wrong with any of them: novalu, noexp, nobar, nodma, nolds (fragments zeroed),
 ldsonce (fragments filled once from K(0)))
"""
import os
import struct
import sys

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
from asm_emit import Emitter, spread  # noqa: E402

CONFIGS = {
    # D: head dimension; QB: 32-row query blocks per wave; SB: 32-key blocks per K/V tile; NW: waves per
    # workgroup; AG: O and Q in AGPRs (one wave per SIMD); NACC: K Q^T accumulators per score block;
    # NF: fragment buffers; PFD: groups between a fragment's LDS read and its MFMA; W: groups per s_waitcnt
    "d64":    dict(D=64,  QB=1, SB=2, NW=8, AG=False, NACC=1, NF=8, PFD=6, W=2),
    "d64_w4": dict(D=64,  QB=1, SB=2, NW=4, AG=False, NACC=1, NF=8, PFD=6, W=2),
    "d128":   dict(D=128, QB=1, SB=2, NW=8, AG=False, NACC=1, NF=4, PFD=3, W=1),
    "d128a":  dict(D=128, QB=2, SB=1, NW=4, AG=True,  NACC=1, NF=8, PFD=7, W=4),
    "d256a":  dict(D=256, QB=1, SB=1, NW=4, AG=True,  NACC=2, NF=8, PFD=7, W=4, LS=2),
}


class Gen(Emitter):
    def __init__(self, name, dtype="bf16", NF=None, PFD=None, W=None, drop=(), DEP=None, LS=None):
        Emitter.__init__(self)
        cfg = CONFIGS[name]
        # direct loads of an iteration: LS = 0: K's in slot 0, V's in slot 1; LS > 0: one load per slot, LS slots apart
        self.LS = cfg.get("LS", 0) if LS is None else LS
        NF = cfg["NF"] if NF is None else NF
        PFD = cfg["PFD"] if PFD is None else PFD
        self.W = cfg["W"] if W is None else W
        assert dtype in ("bf16", "f16")
        self.name, self.dtype = name, dtype
        # the two element types differ only in the MFMA and in the pack instruction (both round to nearest even)
        self.mfma = "v_mfma_f32_32x32x16_" + dtype
        self.cvt = "v_cvt_pk_%s_f32" % dtype
        D, QB, SB, NW = cfg["D"], cfg["QB"], cfg["SB"], cfg["NW"]
        self.D, self.QB, self.SB, self.NW, self.AG, self.NACC = D, QB, SB, NW, cfg["AG"], cfg["NACC"]
        self.BN = 32 * SB
        self.KS = D // 16                         # k-steps of K Q^T
        self.DB = D // 32                         # 32-wide blocks of the head dimension
        self.ROWB = 2 * D
        self.TB = self.BN * self.ROWB             # bytes of one K (or V) tile
        self.NLD = self.TB // (NW * 1024)         # direct loads per wave, tile and tensor
        assert self.NLD >= 1 and self.TB % (NW * 1024) == 0
        self.NF, self.PFD = NF, PFD
        self.NPVG = 2 * SB * self.DB              # fragment groups of P V
        self.NQKG = self.KS * SB                  # fragment groups of K Q^T
        self.NG = self.NPVG + self.NQKG
        self.NM = self.NG * QB                    # MFMA slots per iteration
        assert self.NG % NF == 0 and self.W <= PFD < NF and self.NG % self.W == 0
        # timing experiments only (results are wrong with any of these set): parts of the loop to leave out
        self.exp = set(drop)
        # ---- register map
        v = [0]
        a = [0]
        def take(n, agpr=False, operand=False):
            c = a if agpr else v
            if operand and n > 1:
                c[0] += c[0] & 1      # a register tuple bound to a C++ operand starts at an even register
            b = c[0]
            c[0] += n
            return b
        self.O = take(16 * QB * self.DB, self.AG)            # O[qb][db]
        self.Q = take(4 * QB * self.KS, self.AG)             # Q[qb][ks]
        self.SA = take(16 * QB * SB * self.NACC)             # S double buffer: [qb][sb][acc]
        self.SBUF = take(16 * QB * SB * self.NACC)
        self.PA = take(8 * QB * SB)                          # P double buffer: [qb][pair]
        self.PB = take(8 * QB * SB)
        self.FR = take(4 * NF)
        self.KOFF = take(self.KS)
        self.VOFF = take(2 * self.DB)
        self.DVOFF = take(self.NLD)
        self.DROW = take(self.NLD)
        self.DCH = take(self.NLD)
        self.MREF = take(QB, operand=True)
        self.MRC = take(QB)
        self.L = take(QB, operand=True)   # running row sums (this lane's half of the keys)
        self.TLA = take(QB)               # row sums of the current tile, two partial sums each
        self.TLB = take(QB)
        self.DEP = cfg.get("DEP", 1) if DEP is None else DEP   # element pairs between fma, exp2 and the add / pack
        self.TP = take(2 * (2 * self.DEP + 2))   # exponent / exp temporaries: 2 DEP + 1 element pairs in flight, one kept
        self.ALPHA = take(QB)
        self.THRB = take(QB, operand=True)
        self.THR = take(QB)
        self.T = take(QB)
        self.TMP2 = take(QB)
        self.DD = take(QB)
        self.MX = take(2 * QB)
        self.TS = take(1) if QB == 2 else None   # sum of the tile row sums of the two query blocks
        self.NEGINF = take(1)
        self.DT = take(2 * self.NLD)      # address temporaries of the ragged-tile loads
        self.AT = take(4) if self.AG else None   # temporaries of the accumulator rescale
        self.NV, self.NA = v[0], a[0]
        assert self.NV <= 256 and self.NA <= 256, (self.NV, self.NA)
        # ---- SGPR map (inputs pinned by the asm constraints, the rest clobbered)
        self.s_kbase, self.s_vbase = 32, 34
        self.s_c, self.s_ntiles, self.s_jmask, self.s_tfull, self.s_skvm1 = 36, 37, 38, 39, 40
        self.s_ldsk, self.s_ldsv = 41, 42
        self.s_j, self.s_special, self.s_tau = 43, 44, 45
        self.s_kptr, self.s_vptr = 46, 48
        self.s_t2 = 50
        self.s_m0 = 51            # m0 of the surrounding code (reserved register: saved and restored here)
        self.s_nm1 = 52           # index of this wave's last tile
        self.s_tload = 53         # first iteration whose K load (four tiles ahead) reaches past S_kv
        self.s_lk = 54            # LDS addresses of this wave's K loads, [stage] (load i: + i KB, an immediate)
        self.s_lv = self.s_lk + 4
        self.s_wgnm1 = self.s_lv + 4      # index of the workgroup's last tile
        self.s_t3 = self.s_wgnm1 + 1
        self.s_last = self.s_t3
        self.s_nw = self.s_last + 1       # input: tiles this wave has rows for (causal: fewer than the workgroup's)
        assert self.NLD <= 4      # the immediate offset of a load ends at 4095
        assert self.s_last < 100

    # ------------------------------------------------------------------ helpers
    def acc(self, base, n):
        return self.ar(base, n) if self.AG else self.vr(base, n)

    def s_reg(self, S, qb, sb, acc=0, r=0):
        return S + ((qb * self.SB + sb) * self.NACC + acc) * 16 + r

    def bufs(self, b):
        """(S_cur, S_nxt, P_prev, P_new) of body b."""
        S = (self.SA, self.SBUF) if b % 2 == 0 else (self.SBUF, self.SA)
        P = (self.PA, self.PB) if b % 2 == 0 else (self.PB, self.PA)
        return S[0], S[1], P[0], P[1]

    def tau_bits(self):
        """Bound on a lane's row sum over one tile, as fp32 bits: 2^8, so every P of a tile that passes is
        below 2^8 (inside fp16's range too).  The bound could be far larger without overflow (bf16 has
        fp32's exponent range), but a small one keeps one-hot rows exact: a key that outgrows the reference
        by more than a few bits moves the reference onto itself, its P is then exactly 1 and O is exactly
        its V row; with a lagging reference its P = 2^x would be rounded to 16 bits (2^-9 relative)."""
        return struct.unpack("<I", struct.pack("<f", 2.0 ** 8))[0]

    # ------------------------------------------------------------ MFMA programs
    def groups(self):
        """Fragment groups in issue order: ('pv', kc, db) and ('qk', ks, sb); each feeds QB MFMAs."""
        pv = [("pv", kc, db) for kc in range(2 * self.SB) for db in range(self.DB)]
        qk = [("qk", ks, sb) for ks in range(self.KS) for sb in range(self.SB)]
        return pv[:self.NPVG // 2] + qk + pv[self.NPVG // 2:]

    def frag_loads(self, grp, buf, kst, vst):
        """LDS reads that bring the A operand of group `grp` into fragment buffer `buf`."""
        f = self.FR + 4 * buf
        kind, a, b = grp
        if "nolds" in self.exp or "ldsonce" in self.exp:
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

    def mfma_texts(self, grp, buf, P_prev, S_nxt):
        f = self.vr(self.FR + 4 * buf, 4)
        kind, a, b = grp
        out = []
        for qb in range(self.QB):
            if kind == "pv":
                kc, db = a, b
                o = self.acc(self.O + 16 * (qb * self.DB + db), 16)
                out.append("%s %s, %s, %s, %s" % (self.mfma, o, f, self.vr(P_prev + qb * 8 * self.SB + 4 * kc, 4), o))
            else:
                ks, sb = a, b
                s = self.vr(self.s_reg(S_nxt, qb, sb, ks % self.NACC), 16)
                q = self.acc(self.Q + 4 * (qb * self.KS + ks), 4)
                out.append("%s %s, %s, %s, %s" % (self.mfma, s, f, q, "0" if ks < self.NACC else s))
        return out

    # ---------------------------------------------------------- softmax programs
    def pairs(self):
        return [(qb, k) for qb in range(self.QB) for k in range(8 * self.SB)]

    def pair_regs(self, S_cur, p):
        qb, k = p
        r = self.s_reg(S_cur, qb, k // 8, 0, 2 * (k % 8))
        return r, r + 1

    def pair_ops(self, S_cur, P_new):
        """fma -> exp2 -> row-sum add -> 16-bit pack over the element pairs, software pipelined three deep.
        The exponent arguments go to the temporaries TP: S_cur stays intact for the out-of-line pass."""
        pairs = self.pairs()
        def tp(t, i):
            return self.TP + 2 * (t % (2 * self.DEP + 2)) + i
        def F(t):
            qb = pairs[t][0]
            return ["v_fma_f32 v%d, v%d, s%d, -v%d" % (tp(t, i), x, self.s_c, self.MRC + qb)
                    for i, x in enumerate(self.pair_regs(S_cur, pairs[t]))]
        def E(t):
            op = "v_mov_b32" if "noexp" in self.exp else "v_exp_f32"     # timing experiment: a full-rate stand-in
            return ["%s v%d, v%d" % (op, tp(t, i), tp(t, i)) for i in (0, 1)]
        def A(t):
            qb, k = pairs[t]
            if k == 0:     # the partial sums of a query block start with its first two pairs (next step)
                acc = []
            elif k == 1:   # the temporaries of pair t-1 are still intact: four sets, three pairs in flight
                acc = ["v_add_f32 v%d, v%d, v%d" % (self.TLA + qb, tp(t - 1, 0), tp(t, 0)),
                       "v_add_f32 v%d, v%d, v%d" % (self.TLB + qb, tp(t - 1, 1), tp(t, 1))]
            else:
                acc = ["v_add_f32 v%d, v%d, v%d" % (self.TLA + qb, self.TLA + qb, tp(t, 0)),
                       "v_add_f32 v%d, v%d, v%d" % (self.TLB + qb, self.TLB + qb, tp(t, 1))]
            return acc + ["%s v%d, v%d, v%d" % (self.cvt, P_new + qb * 8 * self.SB + k, tp(t, 0), tp(t, 1))]
        if "novalu" in self.exp:
            return []
        ops = []
        n = len(pairs)
        for t in range(n + 2 * self.DEP):
            if t < n:
                ops += F(t)
            if 0 <= t - self.DEP < n:
                ops += E(t - self.DEP)
            if 0 <= t - 2 * self.DEP < n:
                ops += A(t - 2 * self.DEP)
        for qb in range(self.QB):
            ops.append("v_add_f32 v%d, v%d, v%d" % (self.TLA + qb, self.TLA + qb, self.TLB + qb))
        if self.QB == 2:   # the sum of two positive sums is below the bound only if both are; inf / NaN carry over
            ops.append("v_add_f32 v%d, v%d, v%d" % (self.TS, self.TLA, self.TLA + 1))
        return ops

    def check_ops(self, tag):
        """Tile row sums below the bound?  Otherwise (too large, inf or NaN) take the out-of-line pass."""
        if "novalu" in self.exp:
            return ["%s:" % self.lab("SLOWRET%s_" % tag)]
        ts = self.TS if self.QB == 2 else self.TLA
        ops = ["v_cmp_ngt_f32 vcc, s%d, v%d" % (self.s_tau, ts),     # not (bound > sum)
               "s_cbranch_vccnz %s" % self.lab("SLOW%s_" % tag),
               "%s:" % self.lab("SLOWRET%s_" % tag)]
        if "sgprcheck" in self.exp:
            ops = ["v_cmp_ngt_f32 s[96:97], s%d, v%d" % (self.s_tau, ts), "s_cmp_lg_u64 s[96:97], 0",
                   "s_cbranch_scc1 %s" % self.lab("SLOW%s_" % tag), "%s:" % self.lab("SLOWRET%s_" % tag)]
        for qb in range(self.QB):
            ops.append("v_add_f32 v%d, v%d, v%d" % (self.L + qb, self.L + qb, self.TLA + qb))
        return ops

    def combine_ops(self, S_nxt):
        """Sum the even / odd k-step accumulators of K(j+1) Q^T (NACC == 2)."""
        ops = []
        if self.NACC == 2:
            for qb in range(self.QB):
                for sb in range(self.SB):
                    for r in range(16):
                        a0, a1 = self.s_reg(S_nxt, qb, sb, 0, r), self.s_reg(S_nxt, qb, sb, 1, r)
                        ops.append("v_add_f32 v%d, v%d, v%d" % (a0, a0, a1))
        return ops

    def max_ops(self, S_cur):
        """Row maxima of the lane's scores into T[qb]: two interleaved max3 chains per query block."""
        chains = []
        for qb in range(self.QB):
            els = [self.s_reg(S_cur, qb, sb, 0, r) for sb in range(self.SB) for r in range(16)]
            half = len(els) // 2
            for c in range(2):
                mx, s = self.MX + 2 * qb + c, els[c * half:(c + 1) * half]
                ch = ["v_max3_f32 v%d, v%d, v%d, v%d" % (mx, s[0], s[1], s[2])]
                i = 3
                while i + 1 < len(s):
                    ch.append("v_max3_f32 v%d, v%d, v%d, v%d" % (mx, mx, s[i], s[i + 1]))
                    i += 2
                if i < len(s):
                    ch.append("v_max_f32 v%d, v%d, v%d" % (mx, mx, s[i]))
                chains.append(ch)
        ops = []
        for step in range(len(chains[0])):
            for ch in chains:
                ops.append(ch[step])
        for qb in range(self.QB):
            ops.append("v_max_f32 v%d, v%d, v%d" % (self.T + qb, self.MX + 2 * qb, self.MX + 2 * qb + 1))
        return ops

    def pairmax_ops(self):
        """Max over the two lanes that hold one query's keys, and the new reference maximum, into T[qb]."""
        seqs = []
        for qb in range(self.QB):
            T, TMP2 = self.T + qb, self.TMP2 + qb
            seqs.append([
                "v_mov_b32 v%d, v%d" % (TMP2, T),
                "s_nop 1",
                "v_permlane32_swap_b32 v%d, v%d" % (T, TMP2),   # T = {lo,lo}, TMP2 = {hi,hi}
                "s_nop 1",
                "v_max_f32 v%d, v%d, v%d" % (T, T, TMP2),
                "v_max_f32 v%d, v%d, v%d" % (T, T, self.MREF + qb),  # m_new
            ])
        return [seqs[qb][i] for i in range(len(seqs[0])) for qb in range(self.QB)]

    def rescale_o_ops(self):
        """O *= alpha per query block (accumulators in VGPRs: in place; in AGPRs: read, scale, write back)."""
        ops = []
        for qb in range(self.QB):
            regs = [self.O + 16 * (qb * self.DB + db) + r for db in range(self.DB) for r in range(16)]
            if not self.AG:
                ops += ["v_mul_f32 v%d, v%d, v%d" % (x, self.ALPHA + qb, x) for x in regs]
                continue
            for i in range(0, len(regs), 4):
                ops += ["v_accvgpr_read_b32 v%d, a%d" % (self.AT + t, regs[i + t]) for t in range(4)]
                ops.append("s_nop 1")
                ops += ["v_mul_f32 v%d, v%d, v%d" % (self.AT + t, self.ALPHA + qb, self.AT + t) for t in range(4)]
                ops.append("s_nop 1")
                ops += ["v_accvgpr_write_b32 a%d, v%d" % (regs[i + t], self.AT + t) for t in range(4)]
        return ops

    # ------------------------------------------------------------------- DMA
    def dma_fast(self, which, stage):
        """One K or V tile, as a list of NLD instruction groups (one direct load each): m0 <- LDS address of
        the wave's NLD KB of the stage, s_nop, then load i with the immediate offset i KB, which the hardware
        adds to the LDS address and to the global address alike (the offset register of load i holds i KB
        less to make up for it); the scalar base already points at the tile.  The wait state between the m0
        write and the first load has to be an s_nop: with a VALU instruction of the softmax program in its
        place that instruction's result came out wrong on the MI355X (measured; every other use of the slot
        stayed correct).  Nothing else in the loop writes m0 between the loads of a tile."""
        tab = self.s_lk if which == "k" else self.s_lv
        ptr = self.s_kptr if which == "k" else self.s_vptr
        if "nodma" in self.exp:
            return [[] for _ in range(self.NLD)]
        out = []
        for i in range(self.NLD):
            head = ["s_mov_b32 m0, s%d" % (tab + stage), "s_nop 0"] if i == 0 else []
            out.append(head + ["global_load_lds_dwordx4 v%d, %s%s" % (self.DVOFF + i, self.sr(ptr, 2),
                                                                     " offset:%d" % (1024 * i) if i else "")])
        return out

    def dma_slow(self, which, stage, ahead):
        """Ragged / past-the-end tile j + ahead: clamp the row index, read through the head's base pointer."""
        tab = self.s_lk if which == "k" else self.s_lv
        base = self.s_kbase if which == "k" else self.s_vbase
        sh = {128: 7, 256: 8, 512: 9}[self.ROWB]
        self.e("s_add_i32 s%d, s%d, %d" % (self.s_t2, self.s_j, ahead))
        self.e("s_lshl_b32 s%d, s%d, %d" % (self.s_t2, self.s_t2, {32: 5, 64: 6}[self.BN]))
        for i in range(self.NLD):
            t = self.DT + (0 if which == "k" else self.NLD) + i
            self.e("v_add_u32 v%d, s%d, v%d" % (t, self.s_t2, self.DROW + i))
            self.e("v_min_i32 v%d, s%d, v%d" % (t, self.s_skvm1, t))
            self.e("v_lshlrev_b32 v%d, %d, v%d" % (t, sh, t))
            self.e(("s_add_u32 m0, s%d, %d" % (tab + stage, 1024 * i)) if i else ("s_mov_b32 m0, s%d" % (tab + stage)))
            self.e("v_add_u32 v%d, v%d, v%d" % (t, t, self.DCH + i))
            self.e("s_nop 0")
            self.e("global_load_lds_dwordx4 v%d, %s" % (t, self.sr(base, 2)))

    # --------------------------------------------------------------- the loop
    def entry_reads(self, vst, pv_only):
        """State of the LDS queue where an iteration starts: the iteration before it (or the set-up code) has
        issued the reads of the first PFD groups of the interleaved order.  A P V-only iteration uses the
        leading P V groups among them; the K Q^T reads behind those are never used (id -1)."""
        groups = self.groups()
        lead = min(self.PFD, self.NPVG // 2) if pv_only else self.PFD
        self.outstanding = []
        for i in range(self.PFD):
            self.outstanding += [i if i < lead else -1] * len(self.frag_loads(groups[i], i % self.NF, 0, vst))
        return lead

    def body(self, b, kind="loop"):
        """One iteration, for ring phase b (iteration j = b mod 4).
        kind "loop":  P(j-1)V(j-1) and K(j+1)Q^T around softmax(S(j)), loads of K(j+4), V(j+2).
        kind "first": iteration 0 (b = 0): there is no P(-1): K(1)Q^T and softmax(S(0)) only.
        kind "last":  iteration n-1 (n > 1): there is no tile n: P(n-2)V(n-2) next to softmax(S(n-1)), then
                      P(n-1)V(n-1), and the loop is done; no loads."""
        tag = {"loop": "%d" % b, "first": "F", "last": "L%d" % b}[kind]
        S_cur, S_nxt, P_prev, P_new = self.bufs(b)
        kst, vst = (b + 1) % 4, (b + 3) % 4           # stages of K(j+1), V(j-1)
        nb = (b + 1) % 4
        nkst, nvst = (nb + 1) % 4, (nb + 3) % 4
        all_groups = self.groups()
        pv = [g for g in all_groups if g[0] == "pv"]
        qk = [g for g in all_groups if g[0] == "qk"]
        # the groups next to the softmax of S(j), and the groups after it
        groups = {"loop": all_groups, "first": qk, "last": [("a",) + g for g in pv]}[kind]
        tail = [("b",) + g for g in pv] if kind == "last" else []
        n_soft = len(groups) * self.QB                 # slots that carry the softmax
        L = self.lab
        if kind != "last":
            self.e("%s:" % L({"loop": "BODY%d_" % b, "first": "FIRST_"}[kind]))
            # one test for everything rare: last iteration, masked tiles, loads that reach past S_kv
            self.e("s_cmp_ge_i32 s%d, s%d" % (self.s_j, self.s_special))
            self.e("s_cbranch_scc1 %s" % L("SPECIAL%s_" % tag))
        self.e("%s:" % L("TOP%s_" % tag))              # SCC: this iteration's loads reach past S_kv (kept up to the load slots)
        # loads of the previous iteration may stay in flight; everything older has landed
        if "nobar" not in self.exp:
            self.e("s_waitcnt vmcnt(%d)" % (0 if kind == "last" else 2 * self.NLD))
            self.e("s_barrier")
        if kind == "last":
            # a wave whose rows end before the workgroup's tiles do (causal) still owes the others its share of
            # this iteration's loads: issued here, out of line, before its last products
            self.e("s_cmp_lt_i32 s%d, s%d" % (self.s_j, self.s_wgnm1))
            self.e("s_cbranch_scc1 %s" % L("OWED%d_" % b))
            self.e("%s:" % L("OWEDRET%d_" % b))
        # ---- scalar work of the slots: K(j+4) -> K stage b in slot 0, V(j+2) -> V stage (b+2)%4 in slot 1
        # (nothing between the test above and these two branches writes SCC), pointer bumps in slot 2
        extra = {}
        if kind != "last":
            bumps = [
                "s_add_u32 s%d, s%d, %d" % (self.s_kptr, self.s_kptr, self.TB),
                "s_addc_u32 s%d, s%d, 0" % (self.s_kptr + 1, self.s_kptr + 1),
                "s_add_u32 s%d, s%d, %d" % (self.s_vptr, self.s_vptr, self.TB),
                "s_addc_u32 s%d, s%d, 0" % (self.s_vptr + 1, self.s_vptr + 1),
                "s_add_i32 s%d, s%d, 1" % (self.s_j, self.s_j)]
            if self.LS == 0:
                extra[0] = ["s_cbranch_scc1 %s" % L("KSLOW%s_" % tag)] + sum(self.dma_fast("k", b), []) + ["%s:" % L("KRET%s_" % tag)]
                extra[1] = ["s_cbranch_scc1 %s" % L("VSLOW%s_" % tag)] + sum(self.dma_fast("v", (b + 2) % 4), []) + ["%s:" % L("VRET%s_" % tag)]
                extra[2] = bumps
            else:
                # one load per slot: a wave that issues several in a row waits for the address unit to take
                # them.  The out-of-line clamped loads (all of K and V at once, from the first load slot) come
                # back with SCC still set, which sends the other slots past their loads.
                one = self.dma_fast("k", b) + self.dma_fast("v", (b + 2) % 4)
                ls = min(self.LS, (n_soft - 2) // (len(one) - 1))      # the first iteration has fewer slots
                assert ls >= 1
                for n, ld in enumerate(one):
                    lab = L(("KRET%s_" if n == 0 else "LD%d_%%s_" % n) % tag)
                    to = L("KSLOW%s_" % tag) if n == 0 else lab
                    extra[n * ls] = ["s_cbranch_scc1 %s" % to] + ld + ["%s:" % lab]
                extra[(len(one) - 1) * ls + 1] = bumps
            if "nodma" in self.exp:
                assert self.LS == 0
                extra[0], extra[1] = ["%s:" % L("KRET%s_" % tag)], ["%s:" % L("VRET%s_" % tag)]
        # ---- VALU program: dealt out so that every slot carries about the same issue cost
        b_ops = self.pair_ops(S_cur, P_new)
        # sum of the K Q^T partial accumulators: in the last slots of a loop iteration (its K Q^T ends in the
        # middle); after the first iteration, whose K Q^T fills every slot
        c_ops = self.combine_ops(S_nxt) if kind != "last" else []
        nc = 4 if c_ops and kind == "loop" else 0
        fixed = {}
        for slot in range(n_soft):
            last_of_group = slot % self.QB == self.QB - 1
            cost = 1.0 + (1.0 if slot % (self.QB * self.W) == 0 else 0.0)   # MFMA (+ an s_waitcnt)
            if last_of_group:
                nxt_g = (groups + tail + all_groups)[slot // self.QB + self.PFD]
                cost += 2.0 if "pv" in nxt_g else 1.0                    # LDS reads issued here
            cost += len([x for x in extra.get(slot, []) if not x.endswith(":")])
            fixed[slot] = cost
        valu = spread(b_ops, fixed, n_soft - nc)
        for i in range(nc):
            valu[n_soft - nc + i] = c_ops[i * len(c_ops) // nc:(i + 1) * len(c_ops) // nc]
        # the last K Q^T MFMA must be >= 11 wait states before the combine
        assert nc == 0 or (self.NPVG // 2 + self.NQKG) * self.QB <= n_soft - nc - 3
        valu[n_soft - 1] = valu.get(n_soft - 1, []) + self.check_ops(tag)   # the row-sum test closes the softmax
        if kind == "last":
            # reads in flight: the previous iteration's prefetches.  V(n-1) lies in V stage b
            lead = self.entry_reads(vst, pv_only=True)
            self.stream(groups + tail,
                        lambda g, buf: self.mfma_texts(g[1:], buf, P_prev if g[0] == "a" else P_new, 0),
                        lambda g, buf: self.frag_loads(g[1:], buf, 0, vst if g[0] == "a" else b % 4),
                        self.NF, self.PFD, valu, extra, None, prefetched=lead, wait_every=self.W)
            self.e("s_branch %s" % L("AFTERLAST_"))
            return
        if kind == "first":
            self.outstanding = []
        else:
            self.entry_reads(vst, pv_only=False)
        self.stream(groups,
                    lambda g, buf: self.mfma_texts(g, buf, P_prev, S_nxt),
                    lambda g, buf: self.frag_loads(g, buf, kst, vst),
                    self.NF, self.PFD, valu, extra,
                    lambda i, buf: self.frag_loads(all_groups[i], buf, nkst, nvst),
                    prefetched=0 if kind == "first" else None, wait_every=self.W)
        if kind == "first":
            if c_ops:
                self.e("s_nop 15")
                for ins in c_ops:
                    self.e(ins)
            self.e("s_branch %s" % L("BODY1_"))
        elif b == 3:
            self.e("s_branch %s" % L("BODY0_"))

    def out_of_line(self, b, kind="loop"):
        L = self.lab
        tag = {"loop": "%d" % b, "first": "F", "last": "L%d" % b}[kind]
        S_cur, S_nxt, P_prev, P_new = self.bufs(b)
        QB = self.QB
        if kind != "last":
            # ---- rare iterations: past the last tile (only ever seen by BODY1, when there is a single
            # tile)?  a tile that needs a mask?  the last tile?  (its loads: KSLOW / VSLOW)
            self.e("%s:" % L("SPECIAL%s_" % tag))
            if kind == "loop" and b == 1:
                self.e("s_cmp_ge_i32 s%d, s%d" % (self.s_j, self.s_nw))
                self.e("s_cbranch_scc1 %s" % L("EXIT1_"))
            self.e("s_cmp_lt_i32 s%d, s%d" % (self.s_j, self.s_jmask))
            self.e("s_cbranch_scc1 %s" % L("NOMASK%s_" % tag))
            # mask pre-pass: keys past the causal diagonal / past S_kv become -inf
            self.e("s_lshl_b32 s%d, s%d, %d" % (self.s_t2, self.s_j, {32: 5, 64: 6}[self.BN]))
            self.e("v_mov_b32 v%d, 0xff800000" % self.NEGINF)
            for qb in range(QB):
                self.e("v_subrev_u32 v%d, s%d, v%d" % (self.THR + qb, self.s_t2, self.THRB + qb))  # limit - 4g - BN j
            for qb in range(QB):
                for sb in range(self.SB):
                    for r in range(16):
                        const = 32 * sb + 8 * (r >> 2) + (r & 3)
                        x = self.s_reg(S_cur, qb, sb, 0, r)
                        self.e("v_cmp_gt_i32 vcc, %d, v%d" % (const, self.THR + qb))       # key index > limit ?
                        self.e("v_cndmask_b32 v%d, v%d, v%d, vcc" % (x, x, self.NEGINF))
            self.e("%s:" % L("NOMASK%s_" % tag))
            if kind == "loop":
                self.e("s_cmp_ge_i32 s%d, s%d" % (self.s_j, self.s_nm1))                   # the last tile?
                self.e("s_cbranch_scc1 %s" % L("TOPL%d_" % b))
            self.e("s_cmp_ge_i32 s%d, s%d" % (self.s_j, self.s_tload))     # SCC: do this iteration's loads need clamping?
            self.e("s_branch %s" % L("TOP%s_" % tag))
        # ---- a tile row sum failed the test: exact row maxima of the (intact) scores, move the references
        # there (alpha = exp2((m_ref - m_new) c); 0 when m_ref was still -inf), redo the tile's P, and scale
        # the accumulators (every MFMA that uses the old reference has been issued; wait for the last to retire)
        self.e("%s:" % L("SLOW%s_" % tag))
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
        for ins in self.pair_ops(S_cur, P_new):
            self.e(ins)
        if kind == "first":      # nothing has been accumulated yet
            self.e("s_nop 1")
        else:
            self.e("s_nop 15")
            for ins in self.rescale_o_ops():
                self.e(ins)
            self.e("s_nop 7")
        self.e("s_branch %s" % L("SLOWRET%s_" % tag))
        if kind == "last":
            self.e("%s:" % L("OWED%d_" % b))
            if "nodma" not in self.exp:
                self.dma_slow("k", b, 4)
                self.dma_slow("v", (b + 2) % 4, 2)
            self.e("s_branch %s" % L("OWEDRET%d_" % b))
            return
        # ---- ragged-tile loads
        self.e("%s:" % L("KSLOW%s_" % tag))
        if "nodma" not in self.exp:
            self.dma_slow("k", b, 4)
        if self.LS:
            self.dma_slow("v", (b + 2) % 4, 2)
        self.e("s_cmp_ge_i32 s%d, s%d" % (self.s_j, self.s_tload))     # SCC = 1 for the load slots that follow
        self.e("s_branch %s" % L("KRET%s_" % tag))
        if self.LS:
            return
        self.e("%s:" % L("VSLOW%s_" % tag))
        if "nodma" not in self.exp:
            self.dma_slow("v", (b + 2) % 4, 2)
        self.e("s_branch %s" % L("VRET%s_" % tag))

    def drain(self, b):
        """Loop exit at the top of iteration b (b = 1: a launch with a single tile, whose only iteration was
        the first one): O += P(0) V(0); the operands of the first PFD groups were prefetched by that iteration."""
        L = self.lab
        S_cur, S_nxt, P_prev, P_new = self.bufs(b)
        vst = (b + 3) % 4
        pv = [("pv", kc, db) for kc in range(2 * self.SB) for db in range(self.DB)]
        self.e("%s:" % L("EXIT%d_" % b))
        lead = self.entry_reads(vst, pv_only=True)
        self.stream(pv, lambda g, buf: self.mfma_texts(g, buf, P_prev, 0),
                    lambda g, buf: self.frag_loads(g, buf, 0, vst), self.NF, self.PFD, {}, {}, None,
                    prefetched=lead, wait_every=self.W)
        self.e("s_branch %s" % L("STANDBY_"))

    def standby(self):
        """A wave that has no rows for the workgroup's remaining tiles (causal: its rows end before the
        diagonal tile's keys do) keeps step with the others without computing: one barrier per remaining
        iteration, and its share of every iteration's loads (the ring stage follows from the iteration number).
        AFTERLAST: the last iteration's counter has not moved on; STANDBY: s_j = this wave's tile count."""
        L, e = self.lab, self.e
        sh = {128: 7, 256: 8, 512: 9}[self.ROWB]
        tb = {4096: 12, 8192: 13, 16384: 14}[self.TB]
        e("%s:" % L("AFTERLAST_"))
        e("s_add_i32 s%d, s%d, 1" % (self.s_j, self.s_j))
        e("%s:" % L("STANDBY_"))
        e("s_cmp_ge_i32 s%d, s%d" % (self.s_j, self.s_ntiles))
        e("s_cbranch_scc1 %s" % L("DONE_"))
        e("s_waitcnt vmcnt(%d)" % (2 * self.NLD))
        e("s_barrier")
        e("s_cmp_ge_i32 s%d, s%d" % (self.s_j, self.s_wgnm1))        # the workgroup's last iteration has no loads
        e("s_cbranch_scc1 %s" % L("STANDBYNEXT_"))
        for which, ahead in (("k", 4), ("v", 2)):
            base = self.s_kbase if which == "k" else self.s_vbase
            lds = self.s_ldsk if which == "k" else self.s_ldsv
            e("s_add_i32 s%d, s%d, %d" % (self.s_t2, self.s_j, ahead))              # tile index
            e("s_and_b32 s%d, s%d, 3" % (self.s_t3, self.s_t2 if which == "v" else self.s_j))   # ring stage
            e("s_lshl_b32 s%d, s%d, %d" % (self.s_t3, self.s_t3, tb))
            e("s_add_u32 s%d, s%d, s%d" % (self.s_t3, self.s_t3, lds))
            e("s_lshl_b32 s%d, s%d, %d" % (self.s_t2, self.s_t2, {32: 5, 64: 6}[self.BN]))
            for i in range(self.NLD):
                t = self.DT + (0 if which == "k" else self.NLD) + i
                e("v_add_u32 v%d, s%d, v%d" % (t, self.s_t2, self.DROW + i))
                e("v_min_i32 v%d, s%d, v%d" % (t, self.s_skvm1, t))
                e("v_lshlrev_b32 v%d, %d, v%d" % (t, sh, t))
                e(("s_add_u32 m0, s%d, %d" % (self.s_t3, 1024 * i)) if i else ("s_mov_b32 m0, s%d" % self.s_t3))
                e("v_add_u32 v%d, v%d, v%d" % (t, t, self.DCH + i))
                e("s_nop 0")
                e("global_load_lds_dwordx4 v%d, %s" % (t, self.sr(base, 2)))
        e("%s:" % L("STANDBYNEXT_"))
        e("s_add_i32 s%d, s%d, 1" % (self.s_j, self.s_j))
        e("s_branch %s" % L("STANDBY_"))

    def generate(self):
        L = self.lab
        e = self.e
        QB = self.QB
        e("s_nop 15")
        e("s_nop 7")
        self.save_m0(self.s_m0)
        e("s_mov_b32 s%d, 0" % self.s_j)
        e("s_mov_b32 s%d, 0x%08x" % (self.s_tau, self.tau_bits()))   # bound on a tile's row sum
        # first iteration that is not plain: min(first masked tile, first tile whose K load (4 tiles ahead)
        # reaches past S_kv, last tile)
        e("s_sub_i32 s%d, s%d, 1" % (self.s_nm1, self.s_nw))
        e("s_sub_i32 s%d, s%d, 1" % (self.s_wgnm1, self.s_ntiles))
        e("s_sub_i32 s%d, s%d, 4" % (self.s_tload, self.s_tfull))
        e("s_min_i32 s%d, s%d, s%d" % (self.s_special, self.s_tload, self.s_jmask))
        e("s_min_i32 s%d, s%d, s%d" % (self.s_special, self.s_special, self.s_nm1))
        e("s_add_u32 s%d, s%d, %d" % (self.s_kptr, self.s_kbase, 4 * self.TB))
        e("s_addc_u32 s%d, s%d, 0" % (self.s_kptr + 1, self.s_kbase + 1))
        e("s_add_u32 s%d, s%d, %d" % (self.s_vptr, self.s_vbase, 2 * self.TB))
        e("s_addc_u32 s%d, s%d, 0" % (self.s_vptr + 1, self.s_vbase + 1))
        for st in range(4):
            e("s_add_u32 s%d, s%d, %d" % (self.s_lk + st, self.s_ldsk, st * self.TB))
            e("s_add_u32 s%d, s%d, %d" % (self.s_lv + st, self.s_ldsv, st * self.TB))
        for qb in range(QB):
            e("v_mov_b32 v%d, 0xff800000" % (self.MREF + qb))        # no reference yet: the first tile's test fails
            e("v_mov_b32 v%d, 0xff800000" % (self.MRC + qb))
            e("v_mov_b32 v%d, 0" % (self.L + qb))
        if "nolds" in self.exp:      # timing experiment: the fragments are never read; keep them finite
            for r in range(4 * self.NF):
                e("v_mov_b32 v%d, 0" % (self.FR + r))
        if "ldsonce" in self.exp:    # timing experiment: the fragment buffers are filled once, from K(0), and never again
            for buf in range(self.NF):
                e("ds_read_b128 %s, %s" % (self.vr(self.FR + 4 * buf, 4), self.vr(self.KOFF + buf % self.KS)))
            e("s_waitcnt lgkmcnt(0)")
        self.body(0, "first")
        for b in range(4):
            self.body(b)
        for b in range(4):
            self.body(b, "last")
        self.out_of_line(0, "first")
        for b in range(4):
            self.out_of_line(b)
        for b in range(4):
            self.out_of_line(b, "last")
        self.drain(1)
        self.standby()
        e("%s:" % L("DONE_"))
        e("s_waitcnt vmcnt(0) lgkmcnt(0)")
        self.restore_m0(self.s_m0)
        e("s_nop 15")
        e("s_nop 7")

    # ----------------------------------------------------------- C++ wrapper
    def emit_inc(self):
        self.generate()
        D, DB, KS, QB, SB = self.D, self.DB, self.KS, self.QB, self.SB
        out = []
        out.append("// Generated by gen_attn_loop.py %s %s -- do not edit.  Main loop of attn_fwd_asm_kernel (D = %d, %d waves x %d rows, %d-key tiles)."
                   % (self.name, self.dtype, D, self.NW, 32 * QB, self.BN))
        out.append("// VGPRs used: %d, AGPRs used: %d.  MFMA slots per iteration: %d." % (self.NV, self.NA, self.NM))
        out.append("asm volatile(")
        for ln in self.lines:
            out.append('    "%s\\n\\t"' % ln)
        outs, ins = [], []
        for i in range(QB * DB):
            outs.append('"+{%s}"(o_acc[%d])' % (self.acc(self.O + 16 * i, 16), i))
        for qb in range(QB):
            for sb in range(SB):
                outs.append('"+{%s}"(s_init[%d])' % (self.vr(self.s_reg(self.SA, qb, sb), 16), qb * SB + sb))
        outs.append('"={%s}"(m_ref_v)' % self.vr(self.MREF, QB))
        outs.append('"={%s}"(l_run_v)' % self.vr(self.L, QB))
        for i in range(4 * QB * KS // 16):
            ins.append('"{%s}"(q_pack[%d])' % (self.acc(self.Q + 16 * i, 16), i))
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
        ins.append('"{s%d}"(n_tiles_wave)' % self.s_nw)
        ins.append('"{s%d}"(j_mask)' % self.s_jmask)
        ins.append('"{s%d}"(t_full)' % self.s_tfull)
        ins.append('"{s%d}"(skv_m1)' % self.s_skvm1)
        ins.append('"{s%d}"(lds_k_wave)' % self.s_ldsk)
        ins.append('"{s%d}"(lds_v_wave)' % self.s_ldsv)
        pinned = set()
        if not self.AG:
            pinned.update(range(self.O, self.O + 16 * QB * DB))
            pinned.update(range(self.Q, self.Q + 4 * QB * KS))
        for qb in range(QB):
            for sb in range(SB):
                pinned.update(range(self.s_reg(self.SA, qb, sb), self.s_reg(self.SA, qb, sb) + 16))
        for base, n in ((self.MREF, QB), (self.L, QB), (self.THRB, QB), (self.KOFF, KS), (self.VOFF, 2 * DB),
                        (self.DVOFF, self.NLD), (self.DROW, self.NLD), (self.DCH, self.NLD)):
            pinned.update(range(base, base + n))
        clob = ['"memory"', '"vcc"', '"scc"']
        clob += ['"v%d"' % i for i in range(self.NV) if i not in pinned]
        clob += ['"s%d"' % i for i in range(self.s_j, self.s_last + 1)]
        if "sgprcheck" in self.exp:
            clob += ['"s96"', '"s97"']
        out.append("    : " + ", ".join(outs))
        out.append("    : " + ", ".join(ins))
        out.append("    : " + ", ".join(clob) + ");")
        return "\n".join(out) + "\n"


def main(argv):
    args = list(argv)
    kw = {}
    while len(args) > 2 and args[-2] in ("--pfd", "--nf", "--w", "--drop", "--dep", "--ls"):
        if args[-2] == "--pfd":
            kw["PFD"] = int(args[-1])
        elif args[-2] == "--nf":
            kw["NF"] = int(args[-1])
        elif args[-2] == "--w":
            kw["W"] = int(args[-1])
        elif args[-2] == "--dep":
            kw["DEP"] = int(args[-1])
        elif args[-2] == "--ls":
            kw["LS"] = int(args[-1])
        else:
            kw["drop"] = tuple(filter(None, args[-1].split(",")))
        args = args[:-2]
    dtype = args[2] if len(args) > 2 else "bf16"
    text = Gen(args[0], dtype=dtype, **kw).emit_inc()
    with open(args[1], "w") as f:
        f.write(text)


if __name__ == "__main__":
    main(sys.argv[1:])
