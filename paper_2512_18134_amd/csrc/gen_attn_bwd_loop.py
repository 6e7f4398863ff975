#!/usr/bin/env python3
"""Emit the hand-scheduled main loop of the attention-backward sweeps (gfx950, one wave per SIMD).

The backward pass of the paper's Section 6.3 is split into two sweeps (see attn_bwd_kernels.h):
a key-owner sweep (a wave owns 32 keys and streams query tiles: S = Q K^T, dP = dO V^T,
P = exp(S - LSE), dS = P (dP - Delta), dV^T += dO^T P, dK^T += Q^T dS) and a query-owner sweep
(a wave owns 32 queries and streams key tiles: dQ^T += K^T dS^T).  Both have the shape of the
forward loop of Fig. 1a -- product, element-wise work with one exponential, product -- and get the
same three-stage modulo schedule (Section 3.1 vocabulary: initiation interval I = one streamed
tile of 32 rows = NM MFMA slots, schedule length 3 I): iteration j issues, from one in-order stream,

    contraction MFMAs of tile j-1, first half     (dK^T/dV^T or dQ^T  +=  T^T x dS/P of tile j-1)
    S and dP MFMAs of tile j+1
    contraction MFMAs of tile j-1, second half
    next to:  the VALU work of tile j  (x = S c - LSE', t = dP - Delta, p = exp2 x, ds = p t,
              bf16 packs), dealt out over the MFMA slots so that every slot carries about the same
              issue cost (asm_emit.spread); LDS operand reads PFD slots ahead.

Registers are assigned here: the accumulators and the owner's K/V (or Q/dO) rows, which only the
matrix pipe touches, live in AGPRs; S, dP, P, dS and all addresses in VGPRs.  Streamed tiles
arrive by direct global->LDS loads into two 6-stage rings, four tiles ahead, one barrier per tile;
the key-owner sweep also streams 32 LSE' and 32 Delta values per tile into a small ring.

Hazards handled by construction (the assembler inserts no wait states):
  * MFMA result -> VALU read (11 wait states for an 8-pass MFMA): S and dP of tile j+1 are written
    in the middle of iteration j and first read in iteration j+1, eight MFMAs later.
  * transcendental result -> VALU use: the element-pair pipeline keeps >= 4 instructions between.
  * LDS reads return in order: every s_waitcnt lgkmcnt(N) is computed by replaying the stream.
  * back-to-back MFMAs never share an accumulator (S and dP alternate; the contraction walks its
    2*DB or DB accumulators round robin).

The emitter, the replay of the LDS-read counter and the slot stream are shared with the forward
generator (asm_emit.py); the tests re-check the hazard rules on the emitted text (asm_emit.check_stream).

usage: gen_attn_bwd_loop.py <kv|q> <D> <out.inc> [bf16|f16]
"""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
from asm_emit import Emitter, spread  # noqa: E402


# (key owner?, D) -> NF: fragment buffers; PFD: MFMA slots between a fragment's LDS read and its use;
# W: fragment groups per s_waitcnt
DEFAULTS = {
    (True, 128):  dict(NF=8, PFD=6, W=2),
    (False, 128): dict(NF=8, PFD=4, W=2),
    (True, 64):   dict(NF=8, PFD=4, W=2),
    (False, 64):  dict(NF=4, PFD=2, W=1),
}


class Gen(Emitter):
    def __init__(self, key_owner, D, NF=None, PFD=None, dtype="bf16", drop=(), W=None, balance=True):
        self.balance = balance
        Emitter.__init__(self)
        assert D in (64, 128) and dtype in ("bf16", "f16")
        dflt = DEFAULTS[(bool(key_owner), D)]
        NF = dflt["NF"] if NF is None else NF
        PFD = dflt["PFD"] if PFD is None else PFD
        W = dflt["W"] if W is None else W
        self.KO = key_owner
        # the two element types differ only in the MFMA and in the pack instruction (both round to nearest even)
        self.dtype = dtype
        self.mfma = "v_mfma_f32_32x32x16_" + dtype
        self.cvt = "v_cvt_pk_%s_f32" % dtype
        self.D = D
        self.NW = 4
        self.BN = 32
        self.NST = 6
        self.KS = D // 16
        self.DB = D // 32
        self.ROWB = 2 * D
        self.TB = self.BN * self.ROWB
        self.NLD = self.TB // (self.NW * 1024)
        assert self.NLD >= 1
        self.NSET = 2 if key_owner else 1            # accumulator sets: (dK, dV) or (dQ)
        self.NC = self.NSET * self.DB                # contraction MFMAs per 16-row chunk
        PFD = min(PFD, self.NC)                      # the prefetched operands belong to the first chunk (see drain)
        self.NF, self.PFD, self.W = NF, PFD, W           # W: fragment groups per s_waitcnt
        self.NM = 2 * self.NC + 2 * self.KS          # MFMA slots per iteration
        self.NGRP = 2 * self.NLD + (1 if key_owner else 0)  # direct loads per wave and tile
        assert self.NM % NF == 0 and PFD < NF
        # ---- AGPR map
        self.ACC = 0
        self.B1 = 16 * self.NSET * self.DB
        self.B2 = self.B1 + 4 * self.KS
        self.NA = self.B2 + 4 * self.KS
        assert self.NA <= 256
        # ---- VGPR map
        r = 0
        def take(n):
            nonlocal r
            b = r
            r += n
            return b
        self.SA = take(16)
        self.DPA = take(16)
        self.SB = take(16)
        self.DPB = take(16)
        self.PA = take(8)
        self.DSA = take(8)
        self.PB = take(8)
        self.DSB = take(8)
        self.NAUX = 16 if key_owner else 1
        self.AUXL = take(self.NAUX)
        self.AUXD = take(self.NAUX)
        self.FR = take(4 * NF)
        self.ROFF1 = take(self.KS)
        self.ROFF2 = take(self.KS)
        self.TOFF1 = take(2 * self.DB)
        self.TOFF2 = take(2 * self.DB)
        self.DVOFF = take(self.NLD)
        self.DROW = take(self.NLD)
        self.DCH = take(self.NLD)
        self.DT = take(self.NLD)
        self.AOFF = take(1)
        self.AUXROW = take(1)
        self.AUXSEL = take(1)
        self.AT = take(1)
        self.THRLOB = take(1)
        self.THRHIB = take(1)
        self.THR = take(1)
        self.NEGINF = take(1)
        self.NV = r
        assert r <= 256, r
        # ---- SGPR map (inputs pinned by the asm constraints, the rest clobbered)
        self.s_t1base, self.s_t2base, self.s_auxbase = 32, 34, 36
        self.s_c, self.s_ntiles, self.s_jlo, self.s_jhi = 38, 39, 40, 41
        self.s_tfull, self.s_strm1, self.s_tbeg = 42, 43, 44
        self.s_lds1, self.s_lds2, self.s_ldsaux = 45, 46, 47
        self.s_j, self.s_tk = 48, 49
        self.s_ptr1, self.s_ptr2 = 50, 52
        self.s_t2, self.s_t3 = 54, 55
        self.s_m0 = 56            # m0 of the surrounding code (reserved register: saved and restored here)
        # timing experiments only (results are wrong with any of these set): parts of the loop to leave out
        self.exp = set(drop)

    # ------------------------------------------------------------------ helpers
    def bufs(self, b):
        """(S_cur, dP_cur, S_nxt, dP_nxt, P_prev, dS_prev, P_new, dS_new) of body b."""
        if b % 2 == 0:
            return self.SA, self.DPA, self.SB, self.DPB, self.PA, self.DSA, self.PB, self.DSB
        return self.SB, self.DPB, self.SA, self.DPA, self.PB, self.DSB, self.PA, self.DSA

    # ------------------------------------------------------------ MFMA programs
    def chunk_groups(self, ch):
        return [("c", ch, db, st) for db in range(self.DB) for st in range(self.NSET)]

    def groups(self):
        sdp = [("r", ks, t, 0) for ks in range(self.KS) for t in range(2)]
        return self.chunk_groups(0) + sdp + self.chunk_groups(1)

    def frag_loads(self, grp, buf, rst, tst):
        """LDS reads of one MFMA's A operand; rst / tst: ring stages of the row / transposed reads."""
        f = self.FR + 4 * buf
        kind, a, b, c = grp
        if kind == "c":
            ch, db, st = a, b, c
            toff = self.TOFF1 if st == 0 else self.TOFF2
            off = tst * self.TB + ch * 16 * self.ROWB
            assert off < 65536
            return ["ds_read_b64_tr_b16 %s, %s offset:%d" % (self.vr(f, 2), self.vr(toff + 2 * db), off),
                    "ds_read_b64_tr_b16 %s, %s offset:%d" % (self.vr(f + 2, 2), self.vr(toff + 2 * db + 1), off)]
        ks, t = a, b
        roff = self.ROFF1 if t == 0 else self.ROFF2
        off = rst * self.TB
        assert off < 65536
        return ["ds_read_b128 %s, %s offset:%d" % (self.vr(f, 4), self.vr(roff + ks), off)]

    def mfma_text(self, grp, buf, bf):
        S_cur, DP_cur, S_nxt, DP_nxt, P_prev, DS_prev, P_new, DS_new = bf
        f = self.vr(self.FR + 4 * buf, 4)
        kind, a, b, c = grp
        if kind == "c":
            ch, db, st = a, b, c
            acc = self.ar(self.ACC + 16 * (st * self.DB + db), 16)
            src = DS_prev if st == 0 else P_prev      # set 0: dK^T (or dQ^T) from dS; set 1: dV^T from P
            return "%s %s, %s, %s, %s" % (self.mfma, acc, f, self.vr(src + 4 * ch, 4), acc)
        ks, t = a, b
        dst = self.vr(S_nxt if t == 0 else DP_nxt, 16)
        own = self.ar((self.B1 if t == 0 else self.B2) + 4 * ks, 4)
        return "%s %s, %s, %s, %s" % (self.mfma, dst, f, own, "0" if ks == 0 else dst)

    # ------------------------------------------------------------ VALU programs
    def aux(self, base, r):
        return base + (r if self.KO else 0)

    def phase1_ops(self, bf):
        """x = S c - LSE', t = dP - Delta, in place; frees the LSE'/Delta registers of this tile."""
        S_cur, DP_cur = bf[0], bf[1]
        ops = []
        for r in range(16):
            ops.append("v_fma_f32 v%d, v%d, s%d, -v%d" % (S_cur + r, S_cur + r, self.s_c, self.aux(self.AUXL, r)))
            ops.append("v_sub_f32 v%d, v%d, v%d" % (DP_cur + r, DP_cur + r, self.aux(self.AUXD, r)))
        return ops

    def phase2_ops(self, bf):
        """p = exp2 x, ds = p t, bf16 packs; pipelined over element pairs."""
        S_cur, DP_cur, P_new, DS_new = bf[0], bf[1], bf[6], bf[7]
        def E(k):
            return ["v_exp_f32 v%d, v%d" % (S_cur + 2 * k + i, S_cur + 2 * k + i) for i in range(2)]
        def M(k):
            return ["v_mul_f32 v%d, v%d, v%d" % (DP_cur + 2 * k + i, S_cur + 2 * k + i, DP_cur + 2 * k + i)
                    for i in range(2)]
        def C(k):
            return ["%s v%d, v%d, v%d" % (self.cvt, P_new + k, S_cur + 2 * k, S_cur + 2 * k + 1),
                    "%s v%d, v%d, v%d" % (self.cvt, DS_new + k, DP_cur + 2 * k, DP_cur + 2 * k + 1)]
        ops = []
        for t in range(8 + 2):
            if t < 8:
                ops += E(t)
            if 0 <= t - 1 < 8:
                ops += M(t - 1)
            if 0 <= t - 2 < 8:
                ops += C(t - 2)
        return ops

    def aux_reads(self, stage):
        """LSE' and Delta of the next tile -> AUXL / AUXD (key-owner sweep): rows 8a + 4g + 0..3."""
        out = []
        for a in range(4):
            out.append("ds_read_b128 %s, %s offset:%d" % (self.vr(self.AUXL + 4 * a, 4), self.vr(self.AOFF),
                                                          stage * 256 + 32 * a))
        for a in range(4):
            out.append("ds_read_b128 %s, %s offset:%d" % (self.vr(self.AUXD + 4 * a, 4), self.vr(self.AOFF),
                                                          stage * 256 + 128 + 32 * a))
        return out

    # ------------------------------------------------------------------- DMA
    def dma_fast(self, stage):
        out = []
        for i in range(self.NLD):
            off = stage * self.TB + i * self.NW * 1024
            out += ["s_add_u32 m0, s%d, %d" % (self.s_lds1, off),
                    "s_nop 0",
                    "global_load_lds_dwordx4 v%d, %s" % (self.DVOFF + i, self.sr(self.s_ptr1, 2)),
                    "s_add_u32 m0, s%d, %d" % (self.s_lds2, off),
                    "s_nop 0",
                    "global_load_lds_dwordx4 v%d, %s" % (self.DVOFF + i, self.sr(self.s_ptr2, 2))]
        return out

    def dma_slow(self, stage, label, ret):
        """Tile that reaches past the end of the streamed tensor: rows are clamped to the last one."""
        sh = {128: 7, 256: 8}[self.ROWB]
        self.e("%s:" % label)
        self.e("s_lshl_b32 s%d, s%d, 5" % (self.s_t2, self.s_tk))
        for i in range(self.NLD):
            t = self.DT + i
            off = stage * self.TB + i * self.NW * 1024
            self.e("v_add_u32 v%d, s%d, v%d" % (t, self.s_t2, self.DROW + i))
            self.e("v_min_i32 v%d, s%d, v%d" % (t, self.s_strm1, t))
            self.e("v_lshlrev_b32 v%d, %d, v%d" % (t, sh, t))
            self.e("v_add_u32 v%d, v%d, v%d" % (t, t, self.DCH + i))
            self.e("s_add_u32 m0, s%d, %d" % (self.s_lds1, off))
            self.e("s_nop 0")
            self.e("global_load_lds_dwordx4 v%d, %s" % (t, self.sr(self.s_t1base, 2)))
            self.e("s_add_u32 m0, s%d, %d" % (self.s_lds2, off))
            self.e("s_nop 0")
            self.e("global_load_lds_dwordx4 v%d, %s" % (t, self.sr(self.s_t2base, 2)))
        self.e("s_branch %s" % ret)

    def dma_aux(self, stage):
        """32 LSE' (lanes 0-31) and 32 Delta (lanes 32-63) values of tile s_tk, rows clamped."""
        return ["s_lshl_b32 s%d, s%d, 5" % (self.s_t3, self.s_tk),
                "v_add_u32 v%d, s%d, v%d" % (self.AT, self.s_t3, self.AUXROW),
                "v_min_i32 v%d, s%d, v%d" % (self.AT, self.s_strm1, self.AT),
                "v_lshl_add_u32 v%d, v%d, 2, v%d" % (self.AT, self.AT, self.AUXSEL),
                "s_add_u32 m0, s%d, %d" % (self.s_ldsaux, stage * 256),
                "s_nop 0",
                "global_load_lds_dword v%d, %s" % (self.AT, self.sr(self.s_auxbase, 2))]

    # ------------------------------------------------------- one MFMA stream
    def run_stream(self, grps, bf, rst, tst, valu_by_slot, extra_by_slot, lds_by_slot, nxt):
        """One iteration's slots through the shared stream: one MFMA per fragment group."""
        loads = lambda g, buf, r, t: [] if "nolds" in self.exp else self.frag_loads(g, buf, r, t)
        nxt_loads = None
        if nxt is not None:
            ng, nr, nt = nxt
            nxt_loads = lambda i, buf: loads(ng[i], buf, nr, nt)
        if "nolds" in self.exp:
            lds_by_slot = {}
        self.stream(grps, lambda g, buf: [self.mfma_text(g, buf, bf)], lambda g, buf: loads(g, buf, rst, tst),
                    self.NF, self.PFD, valu_by_slot, extra_by_slot, nxt_loads, lds_by_slot=lds_by_slot,
                    wait_every=self.W)

    # --------------------------------------------------------------- the loop
    def body(self, b):
        NM, NST = self.NM, self.NST
        bf = self.bufs(b)
        S_cur = bf[0]
        rst, tst = (b + 1) % NST, (b + NST - 1) % NST       # stages of tile j+1 (rows), tile j-1 (transposed)
        dst = (b + 4) % NST                                  # stage that receives tile j+4
        nb = (b + 1) % NST
        nxt = (self.groups(), (nb + 1) % NST, (nb + NST - 1) % NST)
        L = self.lab
        self.e("%s:" % L("BODY%d_" % b))
        self.e("s_cmp_ge_i32 s%d, s%d" % (self.s_j, self.s_ntiles))
        self.e("s_cbranch_scc1 %s" % L("EXIT%d_" % b))
        self.e("s_cmp_lt_i32 s%d, s%d" % (self.s_j, self.s_jlo))
        self.e("s_cbranch_scc1 %s" % L("MASKLO%d_" % b))
        self.e("%s:" % L("MASKLORET%d_" % b))
        self.e("s_cmp_ge_i32 s%d, s%d" % (self.s_j, self.s_jhi))
        self.e("s_cbranch_scc1 %s" % L("MASKHI%d_" % b))
        self.e("%s:" % L("MASKHIRET%d_" % b))
        # the loads of the two previous iterations may stay in flight; tile j+1 has landed
        if "nobar" not in self.exp:
            self.e("s_waitcnt vmcnt(%d)" % (2 * self.NGRP))
            self.e("s_barrier")
        p1, p2 = self.phase1_ops(bf), self.phase2_ops(bf)
        quota = -(-(len(p1) + len(p2)) // NM)
        n1 = -(-len(p1) // quota)
        valu = {}
        for i in range(n1):
            valu[i] = p1[i * len(p1) // n1:(i + 1) * len(p1) // n1]
        n2 = NM - n1
        for i in range(n2):
            valu[n1 + i] = p2[i * len(p2) // n2:(i + 1) * len(p2) // n2]
        if self.balance:
            # deal the two phases out by issue cost instead of by count: a slot's MFMA, its s_waitcnt, the LDS
            # reads and scalar work it carries count against its share of the VALU program
            grps = self.groups()
            def fixed_of(lo, hi):
                out = {}
                for slot in range(lo, hi):
                    c = 1.0 + (1.0 if slot % self.W == 0 else 0.0)
                    c += len(self.frag_loads(grps[(slot + self.PFD) % NM], 0, 0, 0))
                    c += {0: 2 + 6 * self.NLD, 1: 7 if self.KO else 0, 2: 6}.get(slot, 0)
                    if self.KO and slot == n1:
                        c += 8
                    out[slot - lo] = c
                return out
            a = spread(p1, fixed_of(0, n1), n1)
            b2 = spread(p2, fixed_of(n1, NM), n2)
            valu = {i: a[i] for i in range(n1)}
            valu.update({n1 + i: b2[i] for i in range(n2)})
        lds = {}
        if self.KO:
            lds[n1] = self.aux_reads(rst)       # after the last use of this tile's values
            assert n1 + self.PFD + 1 < NM
        extra = {}
        extra[0] = ["s_cmp_ge_i32 s%d, s%d" % (self.s_tk, self.s_tfull),
                    "s_cbranch_scc1 %s" % L("SLOW%d_" % b)] + self.dma_fast(dst) + ["%s:" % L("SLOWRET%d_" % b)]
        if self.KO:
            extra[1] = self.dma_aux(dst)
        extra[2] = [
            "s_add_u32 s%d, s%d, %d" % (self.s_ptr1, self.s_ptr1, self.TB),
            "s_addc_u32 s%d, s%d, 0" % (self.s_ptr1 + 1, self.s_ptr1 + 1),
            "s_add_u32 s%d, s%d, %d" % (self.s_ptr2, self.s_ptr2, self.TB),
            "s_addc_u32 s%d, s%d, 0" % (self.s_ptr2 + 1, self.s_ptr2 + 1),
            "s_add_i32 s%d, s%d, 1" % (self.s_tk, self.s_tk),
            "s_add_i32 s%d, s%d, 1" % (self.s_j, self.s_j)]
        if "novalu" in self.exp:
            valu = {}
        if "nodma" in self.exp:
            extra = {0: ["%s:" % L("SLOWRET%d_" % b)], 2: extra[2]}
        self.run_stream(self.groups(), bf, rst, tst, valu, extra, lds, nxt)
        if b == NST - 1:
            self.e("s_branch %s" % L("BODY0_"))

    def out_of_line(self, b):
        L = self.lab
        S_cur = self.bufs(b)[0]
        # ---- mask pre-passes on S(j): invalid elements become -inf, so p = 0 and ds = 0.
        # Element r of a lane is streamed row 32*(t_begin + j) + 8*(r/4) + 4*g + r%4.
        for kind, base, cmp in (("LO", self.THRLOB, "v_cmp_lt_i32"), ("HI", self.THRHIB, "v_cmp_gt_i32")):
            self.e("%s:" % L("MASK%s%d_" % (kind, b)))
            self.e("s_lshl_b32 s%d, s%d, 5" % (self.s_t2, self.s_j))
            self.e("v_subrev_u32 v%d, s%d, v%d" % (self.THR, self.s_t2, base))
            self.e("v_mov_b32 v%d, 0xff800000" % self.NEGINF)
            for r in range(16):
                const = 8 * (r >> 2) + (r & 3)
                self.e("%s vcc, %d, v%d" % (cmp, const, self.THR))
                self.e("v_cndmask_b32 v%d, v%d, v%d, vcc" % (S_cur + r, S_cur + r, self.NEGINF))
            self.e("s_branch %s" % L("MASK%sRET%d_" % (kind, b)))
        self.dma_slow((b + 4) % self.NST, L("SLOW%d_" % b), L("SLOWRET%d_" % b))

    def drain(self, b):
        """Loop exit taken at the top of iteration b: the contraction of the last tile."""
        L = self.lab
        bf = self.bufs(b)
        tst = (b + self.NST - 1) % self.NST
        grps = self.chunk_groups(0) + self.chunk_groups(1)
        self.e("%s:" % L("EXIT%d_" % b))
        g0 = self.groups()
        self.outstanding = [] if "nolds" in self.exp else [i for i in range(self.PFD) for _ in self.frag_loads(g0[i], 0, 0, 0)]
        assert grps[:self.PFD] == g0[:self.PFD]
        self.run_stream(grps, bf, 0, tst, {}, {}, {}, None)
        self.e("s_branch %s" % L("DONE_"))

    def generate(self):
        L = self.lab
        e = self.e
        e("s_nop 15")
        e("s_nop 7")
        self.save_m0(self.s_m0)
        e("s_mov_b32 s%d, 0" % self.s_j)
        # tiles 0..3 were issued by the prologue: the loop's first load is tile 4 (absolute t_begin + 4)
        e("s_add_i32 s%d, s%d, 4" % (self.s_tk, self.s_tbeg))
        e("s_mul_i32 s%d, s%d, %d" % (self.s_t2, self.s_tk, self.TB))
        e("s_add_u32 s%d, s%d, s%d" % (self.s_ptr1, self.s_t1base, self.s_t2))
        e("s_addc_u32 s%d, s%d, 0" % (self.s_ptr1 + 1, self.s_t1base + 1))
        e("s_add_u32 s%d, s%d, s%d" % (self.s_ptr2, self.s_t2base, self.s_t2))
        e("s_addc_u32 s%d, s%d, 0" % (self.s_ptr2 + 1, self.s_t2base + 1))
        for i in range(8):
            e("v_mov_b32 v%d, 0" % (self.PA + i))                # P(-1) = dS(-1) = 0
            e("v_mov_b32 v%d, 0" % (self.DSA + i))
        self.outstanding = []
        g0 = self.groups()
        assert all(g[0] == "c" for g in g0[:self.PFD])
        for i in range(self.PFD):
            if "nolds" not in self.exp:
                self.lds_issue(i, self.frag_loads(g0[i], i % self.NF, 1, self.NST - 1))   # "tile -1": last stage
        for b in range(self.NST):
            self.body(b)
        for b in range(self.NST):
            self.out_of_line(b)
        for b in range(self.NST):
            self.drain(b)
        e("%s:" % L("DONE_"))
        e("s_waitcnt vmcnt(0) lgkmcnt(0)")
        self.restore_m0(self.s_m0)
        e("s_nop 15")
        e("s_nop 7")

    # ----------------------------------------------------------- C++ wrapper
    def emit_inc(self):
        self.generate()
        KS, DB = self.KS, self.DB
        out = []
        out.append("// Generated by gen_attn_bwd_loop.py %s %d %s -- do not edit.  Main loop of attn_bwd_asm_kernel<%d, *, %s, %s>."
                   % ("kv" if self.KO else "q", self.D, self.dtype, self.D, "true" if self.KO else "false",
                      "true" if self.dtype == "f16" else "false"))
        out.append("// VGPRs used: %d, AGPRs used: %d.  MFMA slots per iteration: %d." % (self.NV, self.NA, self.NM))
        out.append("asm volatile(")
        for ln in self.lines:
            out.append('    "%s\\n\\t"' % ln)
        outs, ins = [], []
        for i in range(self.NSET * DB):
            outs.append('"+{%s}"(acc[%d])' % (self.ar(self.ACC + 16 * i, 16), i))
        outs.append('"+{%s}"(s_init)' % self.vr(self.SA, 16))
        outs.append('"+{%s}"(dp_init)' % self.vr(self.DPA, 16))
        outs.append('"+{%s}"(aux_l)' % self.vr(self.AUXL, self.NAUX))
        outs.append('"+{%s}"(aux_d)' % self.vr(self.AUXD, self.NAUX))
        for i in range(4 * KS // 16):
            ins.append('"{%s}"(b1_pack[%d])' % (self.ar(self.B1 + 16 * i, 16), i))
        for i in range(4 * KS // 16):
            ins.append('"{%s}"(b2_pack[%d])' % (self.ar(self.B2 + 16 * i, 16), i))
        ins.append('"{%s}"(roff1_v)' % self.vr(self.ROFF1, KS))
        ins.append('"{%s}"(roff2_v)' % self.vr(self.ROFF2, KS))
        ins.append('"{%s}"(toff1_v)' % self.vr(self.TOFF1, 2 * DB))
        ins.append('"{%s}"(toff2_v)' % self.vr(self.TOFF2, 2 * DB))
        ins.append('"{%s}"(dma_voff_v)' % self.vr(self.DVOFF, self.NLD))
        ins.append('"{%s}"(dma_row_v)' % self.vr(self.DROW, self.NLD))
        ins.append('"{%s}"(dma_choff_v)' % self.vr(self.DCH, self.NLD))
        ins.append('"{v%d}"(aux_off)' % self.AOFF)
        ins.append('"{v%d}"(aux_row)' % self.AUXROW)
        ins.append('"{v%d}"(aux_sel)' % self.AUXSEL)
        ins.append('"{v%d}"(thr_lo_base)' % self.THRLOB)
        ins.append('"{v%d}"(thr_hi_base)' % self.THRHIB)
        ins.append('"{%s}"(t1_head)' % self.sr(self.s_t1base, 2))
        ins.append('"{%s}"(t2_head)' % self.sr(self.s_t2base, 2))
        ins.append('"{%s}"(aux_head)' % self.sr(self.s_auxbase, 2))
        ins.append('"{s%d}"(c_log2e)' % self.s_c)
        ins.append('"{s%d}"(n_tiles)' % self.s_ntiles)
        ins.append('"{s%d}"(j_lo)' % self.s_jlo)
        ins.append('"{s%d}"(j_hi)' % self.s_jhi)
        ins.append('"{s%d}"(t_full)' % self.s_tfull)
        ins.append('"{s%d}"(str_m1)' % self.s_strm1)
        ins.append('"{s%d}"(t_begin)' % self.s_tbeg)
        ins.append('"{s%d}"(lds_1_wave)' % self.s_lds1)
        ins.append('"{s%d}"(lds_2_wave)' % self.s_lds2)
        ins.append('"{s%d}"(lds_aux)' % self.s_ldsaux)
        pinned = set()
        for base, n in ((self.SA, 16), (self.DPA, 16), (self.AUXL, self.NAUX), (self.AUXD, self.NAUX),
                        (self.ROFF1, KS), (self.ROFF2, KS), (self.TOFF1, 2 * DB), (self.TOFF2, 2 * DB),
                        (self.DVOFF, self.NLD), (self.DROW, self.NLD), (self.DCH, self.NLD), (self.AOFF, 1),
                        (self.AUXROW, 1), (self.AUXSEL, 1), (self.THRLOB, 1), (self.THRHIB, 1)):
            pinned.update(range(base, base + n))
        clob = ['"memory"', '"vcc"', '"scc"']
        clob += ['"v%d"' % i for i in range(self.NV) if i not in pinned]
        clob += ['"s%d"' % i for i in range(self.s_j, self.s_m0 + 1)]
        out.append("    : " + ", ".join(outs))
        out.append("    : " + ", ".join(ins))
        out.append("    : " + ", ".join(clob) + ");")
        return "\n".join(out) + "\n"


if __name__ == "__main__":
    # --nf / --pfd / --w / --balance / --drop: timing experiments (fragment buffers, prefetch distance, groups per wait,
    # VALU program dealt out by count instead of by cost, parts left out);
    # a library build passes none of them
    args = sys.argv[1:]
    nf, pfd, w, drop, balance = None, None, None, (), True
    while len(args) > 3 and args[-2] in ("--nf", "--pfd", "--w", "--drop", "--balance"):
        if args[-2] == "--nf":
            nf = int(args[-1])
        elif args[-2] == "--pfd":
            pfd = int(args[-1])
        elif args[-2] == "--w":
            w = int(args[-1])
        elif args[-2] == "--balance":
            balance = bool(int(args[-1]))
        else:
            drop = tuple(filter(None, args[-1].split(",")))
        args = args[:-2]
    dtype = args[3] if len(args) > 3 else "bf16"
    text = Gen(args[0] == "kv", int(args[1]), NF=nf, PFD=pfd, dtype=dtype, drop=drop, W=w, balance=balance).emit_inc()
    with open(args[2], "w") as f:
        f.write(text)
