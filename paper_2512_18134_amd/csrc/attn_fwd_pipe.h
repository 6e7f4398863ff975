// attn_fwd_pipe.h -- software-pipelined attention-forward kernel for gfx950.
//
// This is the loop of the paper's Fig. 1a, modulo-scheduled for CDNA4 in the
// sense of Section 3.1: the paper's Hopper schedule (Fig. 1f) overlaps
// S = gemm(Q, K[i]) with P = exp(S[i-1]) and issues O += gemm(P, V[i-1]) after
// it.  On gfx950 one wavefront issues MFMA and VALU instructions from a single
// in-order stream, an MFMA occupies the matrix pipe for 32 cycles and the
// softmax of one score element costs about as much VALU time as its two
// MFMAs cost matrix time (measured), so the schedule here goes one stage
// deeper: iteration j of the steady state runs
//       QK^T of tile j+1   (MFMA)
//       softmax of tile j  (VALU + transcendental)
//       P V of tile j-1    (MFMA)
// which are mutually independent, and interleaves them instruction by
// instruction: one MFMA, then about four VALU operations, then the LDS reads
// for a later MFMA.  In the paper's terms the initiation interval I is one
// K/V tile (32 MFMAs per wave) and the schedule length L spans three of them.
// K/V tiles reach LDS through direct global->LDS loads that run two tiles
// ahead (the "streaming" loads of Section 5.3), three ring stages each.
//
// The accumulator rescale of the online softmax is lazy: the reference maximum
// m_ref of a row only moves when the running maximum has grown by more than
// kLazyLog2 in the base-2 domain, so P = exp2(c*s - c*m_ref) may reach
// 2^kLazyLog2.  This is an exact re-association (O and the row sum l share the
// reference, and O/l does not depend on it); it makes the 64-register
// accumulator rescale a rare, wave-uniform branch.
#pragma once
#include "attn_common.h"

namespace attn {

constexpr float kLazyLog2 = 8.0f;

// direct global -> LDS load of 16 bytes per lane: LDS address = m0 + lane*16
__device__ __forceinline__ void dma16(uint32_t lds_addr, const void *base, uint32_t voff)
{
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(base)
                 : "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

__device__ __forceinline__ float lane_pair_max(float x)
{
    // max over the two lanes (l, l^32) that share a query column
    return fmaxf(x, xor32(x));
}

// Template parameters:
//   D      head dimension (64 or 128)
//   BN     keys per K/V tile (32 or 64)
//   NW     wavefronts per workgroup
//   QB     32-row query blocks per wavefront (a K or V^T fragment read from LDS
//          feeds QB MFMAs); the workgroup owns BM = 32*QB*NW query rows
//   PIPE   3: three-stage schedule (QK^T of tile j+1 || softmax of tile j ||
//          PV of tile j-1); 2: two-stage (QK^T of tile j runs on its own, then
//          softmax of tile j || PV of tile j-1), 16*QB*BN/32 fewer registers;
//          1: no overlap inside a wave (QK^T, softmax, PV of tile j in order)
template <int D, int BN, int NW, int QB, int PIPE, bool CAUSAL>
__global__ __launch_bounds__(NW * 64) void attn_fwd_pipe_kernel(const Params p)
{
    static_assert(D == 64 || D == 128, "pipelined kernel: D = 64 or 128");
    static_assert(BN == 32 || BN == 64, "BN = 32 or 64");
    constexpr int BM = NW * 32 * QB, NST = 3;
    constexpr int SB = BN / 32;                // 32-key blocks per tile
    constexpr int CPR = D / 8;                 // 16-byte chunks per row
    constexpr int KS = D / 16;                 // k-steps of QK^T
    constexpr int DB = D / 32;                 // 32-wide blocks of the head dimension
    constexpr int ROWB = D * 2;                // bytes per K/V row
    constexpr int TB = BN * ROWB;              // bytes per K (or V) tile
    constexpr int NLD = TB / (NW * 1024);      // direct loads per wave per tile and tensor
    constexpr int RPG = 1024 / ROWB;           // rows covered by one wave-wide direct load
    static_assert(NLD >= 1 && TB % (NW * 1024) == 0, "tile must split over the waves");
    constexpr bool PIPE3 = (PIPE == 3);
    constexpr bool SEQ = (PIPE == 1);          // no overlap inside a wave: QK^T, softmax, PV of tile j in order
    constexpr int KLEAD = PIPE3 ? 1 : 0;       // iteration j multiplies K(j + KLEAD)
    constexpr int NPV = 2 * SB * DB * QB;      // MFMAs of one P V product per wave
    constexpr int NQK = KS * SB * QB;          // MFMAs of one Q K^T product per wave
    constexpr int NPV1 = PIPE3 ? NPV / 2 : 0;  // P V MFMAs issued next to the row-max reduction
    constexpr int NP = QB * SB * 8;            // score-element pairs per lane and tile

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // K ring [3][TB], V ring [3][TB]
    constexpr uint32_t KRING = 0, VRING = NST * TB;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(ATTN_LDS_PTR(unsigned char))smem;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lq = lane & 31;
    const int g = lane >> 5;

    int bh, qt;
    wg_to_tile<CAUSAL>(blockIdx.x, p, D, bh, qt);
    const int q0 = qt * BM;
    const int q0w = q0 + wave * 32 * QB;
    auto qcol = [&](int qb) { return q0w + 32 * qb + lq; };  // query row of this lane in block qb

    const bf16_t *qg = p.q + (size_t)bh * p.S_q * D;
    const bf16_t *kg = p.k + (size_t)bh * p.S_kv * D;
    const bf16_t *vg = p.v + (size_t)bh * p.S_kv * D;

    int kv_end = p.S_kv;
    if (CAUSAL)
        kv_end = min(kv_end, min(q0 + BM, p.S_q));
    const int n_tiles = (kv_end + BN - 1) / BN;
    // first tile whose softmax needs a mask (ragged key tail / causal diagonal)
    const int j_tail = (n_tiles * BN > p.S_kv) ? n_tiles - 1 : n_tiles;
    const int j_mask = CAUSAL ? min(q0 / BN, j_tail) : j_tail;

    // ---- direct-load addressing: lane -> (row in tile, 16-byte chunk) -------
    // A wave-wide load fills 1 KB of LDS linearly (lane*16), i.e. RPG rows; the
    // XOR swizzle is applied on the global side: the lane that fills physical
    // chunk pc of a row fetches logical chunk pc ^ swz(row).
    // Full tiles use a per-lane constant offset and a scalar base that advances
    // by one tile; a tile that reaches past S_kv re-reads the last row instead
    // (those keys are masked later).
    int dma_row[NLD];
    uint32_t dma_choff[NLD], dma_voff[NLD];
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
        const int gi = i * NW + wave;
        dma_row[i] = RPG * gi + lane / CPR;
        dma_choff[i] = (uint32_t)(((lane % CPR) ^ swz<D>(dma_row[i])) * 16);
        dma_voff[i] = (uint32_t)dma_row[i] * ROWB + dma_choff[i];
    }
    const int t_full = p.S_kv / BN;  // tiles below this index lie entirely inside [0, S_kv)
    auto issue_tile = [&](const bf16_t *base, uint32_t ring_off, int stage, int t) {
        if (t < t_full) {
            const unsigned char *tb = reinterpret_cast<const unsigned char *>(base) + (size_t)t * TB;
#pragma unroll
            for (int i = 0; i < NLD; ++i)
                dma16(lds0 + ring_off + stage * TB + (i * NW + wave) * 1024, tb, dma_voff[i]);
        } else {
#pragma unroll
            for (int i = 0; i < NLD; ++i) {
                const int r = min(t * BN + dma_row[i], p.S_kv - 1);
                dma16(lds0 + ring_off + stage * TB + (i * NW + wave) * 1024, base, (uint32_t)r * ROWB + dma_choff[i]);
            }
        }
    };

    // ---- operand addressing inside a tile ------------------------------------
    // K as A operand: lane reads row 32*sb + lq, logical chunk 2*ks + g.
    uint32_t koff[KS];
    {
        const int sw = swz<D>(lq);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            koff[ks] = lds0 + KRING + (uint32_t)(lq * ROWB + (((2 * ks + g) ^ sw) * 16));
    }
    // V^T as A operand through ds_read_b64_tr_b16: in a 16-lane block, source
    // lane i supplies the 8-byte piece i%4 of row i/4; lane L receives column L
    // of those four rows.  Contraction slot s of lane group g in chunk c of
    // block sb is key 32*sb + 16*c + 8*(s/4) + 4*g + s%4.
    uint32_t voff[DB][2];
    {
        const int i16 = lane & 15, dh = (lane >> 4) & 1;
        const int rho = i16 >> 2, pi = i16 & 3;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int hlf = 0; hlf < 2; ++hlf) {
                const int row = 4 * g + 8 * hlf + rho;
                const int ch = 4 * db + 2 * dh + (pi >> 1);
                voff[db][hlf] = lds0 + VRING + (uint32_t)(row * ROWB + ((ch ^ swz<D>(row)) * 16) + (pi & 1) * 8);
            }
    }
    // `kst` / `vst` are byte offsets of the stage inside its ring (compile-time
    // constants at every call site, so they fold into the instruction's offset field)
    auto k_frag = [&](uint32_t kst, int sb, int ks) {
        return *(ATTN_LDS_PTR(const bf16x8))(uintptr_t)(koff[ks] + (kst + sb * 32 * ROWB));
    };
    auto v_frag = [&](uint32_t vst, int sbc, int db) {
        bf16x8 a;
#pragma unroll
        for (int hlf = 0; hlf < 2; ++hlf) {
            const bf16x4 t = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                (ATTN_LDS_PTR(bf16x4))(uintptr_t)(voff[db][hlf] + (vst + sbc * 16 * ROWB)));
            a[4 * hlf + 0] = t[0];
            a[4 * hlf + 1] = t[1];
            a[4 * hlf + 2] = t[2];
            a[4 * hlf + 3] = t[3];
        }
        return a;
    };

    // ---- prologue: start the K/V stream, load Q ---------------------------------
    issue_tile(kg, KRING, 0, 0);
    if (PIPE3)
        issue_tile(kg, KRING, 1, 1);
    if (SEQ) {
        issue_tile(vg, VRING, 0, 0);
        issue_tile(kg, KRING, 1, 1);
        issue_tile(vg, VRING, 1, 1);
    } else {
        issue_tile(vg, VRING, 2, 0);  // stands in for "V(-1)": multiplied by P(-1) = 0 in iteration 0
        issue_tile(kg, KRING, KLEAD + 1, KLEAD + 1);
        issue_tile(vg, VRING, 0, 0);
    }

    bf16x8 bq[QB][KS];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const bf16_t *src = qg + (size_t)min(qcol(qb), p.S_q - 1) * D + 8 * g;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            bq[qb][ks] = *reinterpret_cast<const bf16x8 *>(src + 16 * ks);
    }

    f32x16 oacc[QB][DB];
    f32x16 s_cur[QB][SB];   // S(j): raw scores of the tile whose softmax runs in this iteration
    bf16x8 pb[QB][SB][2];   // P(j-1), already in B-operand form
    float m_ref[QB];        // reference maximum (raw score units) that the stored P, l, O are relative to
    float mrc[QB];          // m_ref * c
    float l_run[QB];        // this lane's partial row sum
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                oacc[qb][db][r] = 0.f;
#pragma unroll
        for (int sb = 0; sb < SB; ++sb)
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    pb[qb][sb][c][e] = (bf16_t)0.f;
        m_ref[qb] = -INFINITY;
        mrc[qb] = 0.f;
        l_run[qb] = 0.f;
    }

    // S = K(t) Q^T, not overlapped with anything
    auto qk_plain = [&](uint32_t kst, f32x16(&s)[QB][SB]) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int sb = 0; sb < SB; ++sb)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    s[qb][sb][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int sb = 0; sb < SB; ++sb) {
                const bf16x8 a = k_frag(kst, sb, ks);
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
                    s[qb][sb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bq[qb][ks], s[qb][sb], 0, 0, 0);
            }
    };

    if (PIPE3) {
        // S(0) = K(0) Q^T.  Issued so far by this wave: 5*NLD direct loads, then QB*KS
        // loads of Q; s_waitcnt counts from the newest: everything but K(0) may be in flight.
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(QB * KS + 4 * NLD) : "memory");
        __syncthreads();
        qk_plain(0, s_cur);
    }

    // ---- one steady-state iteration ----------------------------------------------
    auto step = [&](int j, auto st_tag, auto mask_tag) {
        constexpr int ST = decltype(st_tag)::value;  // j % 3
        constexpr bool MASK = decltype(mask_tag)::value;
        constexpr int KST = (ST + KLEAD) % NST;  // stage of K(j + KLEAD)
        constexpr int VST = SEQ ? ST : (ST + 2) % NST;  // stage of V(j-1) (of V(j) when SEQ)
        constexpr uint32_t kst = KST * TB, vst = VST * TB;
        const int j0 = j * BN;

        // K(j+KLEAD) and V(j-1) were issued two iterations ago; the loads of the
        // previous iteration (K(j+KLEAD+1), V(j)) may still be in flight.
        wait_vmcnt<2 * NLD>();
        __syncthreads();
        // Every wave has finished iteration j-1: the stages of K(j+KLEAD-1) and V(j-2) are free.
        issue_tile(kg, KRING, (ST + KLEAD + 2) % NST, j + KLEAD + 2);
        issue_tile(vg, VRING, (ST + (SEQ ? 2 : 1)) % NST, j + (SEQ ? 2 : 1));

        if (!PIPE3)
            qk_plain(kst, s_cur);

        auto dead = [&](int qb, int sb, int r) {
            const int kv = j0 + 32 * sb + acc_row(r, g);
            return (kv >= p.S_kv) || (CAUSAL && kv > qcol(qb));
        };
        // the n-th MFMA of P(j-1) V(j-1): A fragment shared by the QB query blocks
        bf16x8 va;
        auto pv_mfma = [&](int n) {
            const int qb = n % QB, db = (n / QB) % DB, sbc = n / (QB * DB);
            if (qb == 0)
                va = v_frag(vst, sbc, db);
            oacc[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[qb][sbc >> 1][sbc & 1], oacc[qb][db], 0, 0, 0);
        };

        // -- part 1: first MFMAs of P(j-1) V(j-1)  ||  row max of S(j)
        float mx[QB][4];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                mx[qb][i] = -INFINITY;
        constexpr int NMX = QB * SB * 8;  // max3 operations
#pragma unroll
        for (int n = 0; n < (NPV1 > 0 ? NPV1 : 1); ++n) {
            if (NPV1 > 0)
                pv_mfma(n);
            const int lo = n * NMX / (NPV1 > 0 ? NPV1 : 1), hi = (n + 1) * NMX / (NPV1 > 0 ? NPV1 : 1);
#pragma unroll
            for (int e = lo; e < hi; ++e) {
                const int qb = e / (SB * 8), sb = (e / 8) % SB, r = (e % 8) * 2;
                const float a0 = (MASK && dead(qb, sb, r)) ? -INFINITY : s_cur[qb][sb][r];
                const float a1 = (MASK && dead(qb, sb, r + 1)) ? -INFINITY : s_cur[qb][sb][r + 1];
                mx[qb][e & 3] = fmaxf(fmaxf(mx[qb][e & 3], a0), a1);
            }
        }
        float m_new[QB];
        bool need = false;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const float mloc = lane_pair_max(fmaxf(fmaxf(mx[qb][0], mx[qb][1]), fmaxf(mx[qb][2], mx[qb][3])));
            m_new[qb] = fmaxf(m_ref[qb], mloc);
            // move the reference only when it is far off (or unset)
            need = need || (m_ref[qb] == -INFINITY) || ((m_new[qb] - m_ref[qb]) * p.c > kLazyLog2);
        }
        const bool resc = __any(need);
        float alpha[QB];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
            alpha[qb] = 1.f;
        if (resc) {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                alpha[qb] = (m_ref[qb] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((m_ref[qb] - m_new[qb]) * p.c);
                m_ref[qb] = m_new[qb];
                mrc[qb] = m_new[qb] * p.c;
                l_run[qb] *= alpha[qb];
            }
        }

        // -- part 2: remaining MFMAs of P(j-1) V(j-1) [, then K(j+1) Q^T]  ||  exp2, row sum, P(j) -> bf16
        f32x16 s_nxt[QB][SB];
        if (PIPE3) {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                for (int sb = 0; sb < SB; ++sb)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        s_nxt[qb][sb][r] = 0.f;
        }
        bf16x8 pn[QB][SB][2];
        float psum[QB];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
            psum[qb] = 0.f;
        auto softmax_pair = [&](int e) {
            const int qb = e / (SB * 8), sb = (e / 8) % SB, r = (e % 8) * 2;
            float t0 = fmaf(s_cur[qb][sb][r], p.c, -mrc[qb]);
            float t1 = fmaf(s_cur[qb][sb][r + 1], p.c, -mrc[qb]);
            if (MASK) {
                t0 = dead(qb, sb, r) ? -INFINITY : t0;
                t1 = dead(qb, sb, r + 1) ? -INFINITY : t1;
            }
            const float p0 = __builtin_amdgcn_exp2f(t0);
            const float p1 = __builtin_amdgcn_exp2f(t1);
            psum[qb] += p0 + p1;
            const f32x2 pp = {p0, p1};
            const bf16x2 pk = __builtin_convertvector(pp, bf16x2);  // round to nearest even
            pn[qb][sb][r >> 3][r & 7] = pk[0];
            pn[qb][sb][r >> 3][(r & 7) + 1] = pk[1];
        };
        constexpr int NSLOT = SEQ ? 1 : (NPV - NPV1) + (PIPE3 ? NQK : 0);
        bf16x8 ka;
#pragma unroll
        for (int slot = 0; slot < NSLOT; ++slot) {
            if (SEQ) {
            } else if (slot < NPV - NPV1) {
                pv_mfma(NPV1 + slot);
            } else {
                const int n = slot - (NPV - NPV1);
                const int qb = n % QB, sb = (n / QB) % SB, ks = n / (QB * SB);
                if (qb == 0)
                    ka = k_frag(kst, sb, ks);
                s_nxt[qb][sb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, bq[qb][ks], s_nxt[qb][sb], 0, 0, 0);
            }
            const int e_lo = slot * NP / NSLOT, e_hi = (slot + 1) * NP / NSLOT;
#pragma unroll
            for (int e = e_lo; e < e_hi; ++e)
                softmax_pair(e);
        }
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
            l_run[qb] += psum[qb];

        // deferred accumulator rescale: after every MFMA of P(j-1) V(j-1) has been issued
        if (resc) {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        oacc[qb][db][r] *= alpha[qb];
        }
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int sb = 0; sb < SB; ++sb) {
                if (PIPE3)
                    s_cur[qb][sb] = s_nxt[qb][sb];
#pragma unroll
                for (int c = 0; c < 2; ++c)
                    pb[qb][sb][c] = pn[qb][sb][c];
            }
        if (SEQ) {
#pragma unroll
            for (int n = 0; n < NPV; ++n)
                pv_mfma(n);
        }
    };

    auto step_m = [&](int j, auto st_tag) {
        if (j >= j_mask)
            step(j, st_tag, std::true_type{});
        else
            step(j, st_tag, std::false_type{});
    };
    {
        int j = 0;
        while (true) {
            if (j >= n_tiles) break;
            step_m(j, std::integral_constant<int, 0>{});
            ++j;
            if (j >= n_tiles) break;
            step_m(j, std::integral_constant<int, 1>{});
            ++j;
            if (j >= n_tiles) break;
            step_m(j, std::integral_constant<int, 2>{});
            ++j;
        }
    }

    // ---- drain: O += P(n-1) V(n-1) -----------------------------------------------
    wait_vmcnt<0>();
    __syncthreads();
    if (!SEQ) {
        const uint32_t vst = ((n_tiles - 1) % NST) * TB;
#pragma unroll
        for (int sbc = 0; sbc < 2 * SB; ++sbc)
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                const bf16x8 a = v_frag(vst, sbc, db);
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
                    oacc[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[qb][sbc >> 1][sbc & 1], oacc[qb][db], 0, 0, 0);
            }
    }

    // ---- epilogue: normalise, write O (bf16) and the log-sum-exp (fp32) ----------
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const float l_tot = l_run[qb] + xor32(l_run[qb]);
        const float inv = 1.f / l_tot;
        const int qrow = qcol(qb);
        if (qrow < p.S_q) {
            bf16_t *orow = p.o + ((size_t)bh * p.S_q + qrow) * D;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int rb = 0; rb < 4; ++rb) {
                    const f32x2 lo = {oacc[qb][db][4 * rb + 0] * inv, oacc[qb][db][4 * rb + 1] * inv};
                    const f32x2 hi = {oacc[qb][db][4 * rb + 2] * inv, oacc[qb][db][4 * rb + 3] * inv};
                    const bf16x2 blo = __builtin_convertvector(lo, bf16x2);
                    const bf16x2 bhi = __builtin_convertvector(hi, bf16x2);
                    const bf16x4 out = {blo[0], blo[1], bhi[0], bhi[1]};
                    *reinterpret_cast<bf16x4 *>(orow + 32 * db + 8 * rb + 4 * g) = out;
                }
            if (g == 0)
                p.lse[(size_t)bh * p.S_q + qrow] =
                    m_ref[qb] * p.scale + __builtin_amdgcn_logf(l_tot) * 0.69314718055994530942f;
        }
    }
}

}  // namespace attn
