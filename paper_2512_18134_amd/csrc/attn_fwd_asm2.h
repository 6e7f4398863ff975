// attn_fwd_asm2.h -- hand-scheduled attention-forward kernels with one wave per SIMD.
//
// Same mathematics, LDS layout and three-stage modulo schedule as attn_fwd_asm.h
// (the paper's Fig. 1a loop; see gen_attn_loop2.py), for tilings in which a wave
// owns all 512 registers of its SIMD lane: the O accumulators and the Q fragments
// sit in AGPRs, S/P and everything the VALU touches in VGPRs.
//   <D=128, QB=2>: 4 waves x 64 query rows (BM = 256); each K / V^T fragment read
//                  from LDS feeds two MFMAs (half the LDS operand traffic).
//   <D=256, QB=1>: 4 waves x 32 query rows (BM = 128).
// K/V tiles of 32 keys in two 4-stage LDS rings (8 * 32 * D * 2 bytes).
// Requires scale > 0 and S_kv * D * 2 < 2^31.
#pragma once
#include "attn_common.h"
#include "attn_fwd_asm.h"   // U32Vec
#include "attn_dma.h"       // dma16, wait_vmcnt

namespace attn {

template <int N>
struct F32Vec {
    typedef float type __attribute__((ext_vector_type(N)));
    static __device__ __forceinline__ float get(const type &v, int i) { return v[i]; }
};
template <>
struct F32Vec<1> {
    typedef float type;
    static __device__ __forceinline__ float get(const type &v, int) { return v; }
};

template <int D, int QB, bool CAUSAL, bool F16 = false>
__global__ __launch_bounds__(256) void attn_fwd_asm2_kernel(const Params p)
{
    static_assert((D == 128 && QB == 2 && !F16) || (D == 256 && QB == 1), "supported tilings");
    typedef typename std::conditional<F16, ElemF16, ElemBF16>::type E;
    typedef typename E::t elem_t;
    typedef typename E::x2 ex2;
    typedef typename E::x4 ex4;
    typedef typename E::x8 ex8;
    constexpr int BN = 32, NW = 4, BM = NW * 32 * QB, NST = 4;
    constexpr int CPR = D / 8;
    constexpr int KS = D / 16;
    constexpr int DB = D / 32;
    constexpr int ROWB = D * 2;
    constexpr int TB = BN * ROWB;
    constexpr int NLD = TB / (NW * 1024);
    constexpr int NQP = 4 * QB * KS / 16;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // K ring [4][TB], V ring [4][TB]
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
    auto qcol = [&](int qb) { return q0 + (wave * QB + qb) * 32 + lq; };

    const elem_t *qg = reinterpret_cast<const elem_t *>(p.q) + (size_t)bh * p.S_q * D;
    const elem_t *k_head = reinterpret_cast<const elem_t *>(p.k) + (size_t)bh * p.S_kv * D;
    const elem_t *v_head = reinterpret_cast<const elem_t *>(p.v) + (size_t)bh * p.S_kv * D;

    int kv_end = p.S_kv;
    if (CAUSAL)
        kv_end = min(kv_end, min(q0 + BM, p.S_q));
    const int n_tiles = (kv_end + BN - 1) / BN;
    const int j_tail = (n_tiles * BN > p.S_kv) ? n_tiles - 1 : n_tiles;
    const int j_mask = CAUSAL ? min(q0 / BN, j_tail) : j_tail;
    const int t_full = p.S_kv / BN;
    const int skv_m1 = p.S_kv - 1;

    // ---- direct-load addressing: a wave-wide load fills 1 KB of LDS linearly
    typename U32Vec<NLD>::type dma_row_v, dma_choff_v, dma_voff_v;
    uint32_t dma_row[NLD], dma_choff[NLD];
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
        const int gi = i * NW + wave;
        dma_row[i] = (1024 / ROWB) * gi + lane / CPR;
        const int ch = lane % CPR;
        dma_choff[i] = (uint32_t)(((ch & ~15) | ((ch & 15) ^ swz<D>(dma_row[i]))) * 16);
        U32Vec<NLD>::set(dma_row_v, i, dma_row[i]);
        U32Vec<NLD>::set(dma_choff_v, i, dma_choff[i]);
        U32Vec<NLD>::set(dma_voff_v, i, dma_row[i] * ROWB + dma_choff[i]);
    }
    auto issue_tile = [&](const elem_t *base, uint32_t ring_off, int stage, int t) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int r = min(t * BN + (int)dma_row[i], p.S_kv - 1);
            dma16(lds0 + ring_off + stage * TB + (i * NW + wave) * 1024, base, (uint32_t)r * ROWB + dma_choff[i]);
        }
    };
    const uint32_t lds_k_wave = lds0 + KRING + wave * 1024;
    const uint32_t lds_v_wave = lds0 + VRING + wave * 1024;

    // ---- operand addressing inside a tile
    uint32_t koff[KS];
    typename U32Vec<KS>::type koff_v;
    {
        const int sw = swz<D>(lq);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int ch = 2 * ks + g;
            koff[ks] = lds0 + KRING + (uint32_t)(lq * ROWB + (((ch & ~15) | ((ch & 15) ^ sw)) * 16));
            koff_v[ks] = koff[ks];
        }
    }
    typename U32Vec<2 * DB>::type voff_v;
    {
        const int i16 = lane & 15, dh = (lane >> 4) & 1;
        const int rho = i16 >> 2, pi = i16 & 3;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int hlf = 0; hlf < 2; ++hlf) {
                const int row = 4 * g + 8 * hlf + rho;
                const int ch = 4 * db + 2 * dh + (pi >> 1);
                voff_v[2 * db + hlf] = lds0 + VRING +
                    (uint32_t)(row * ROWB + (((ch & ~15) | ((ch & 15) ^ swz<D>(row))) * 16) + (pi & 1) * 8);
            }
    }

    // ---- prologue: K(0..3), V(0), V(1) and a stand-in for "V(-1)" (multiplied by P(-1) = 0)
#pragma unroll
    for (int t = 0; t < 4; ++t)
        issue_tile(k_head, KRING, t, t);
    issue_tile(v_head, VRING, 3, 0);
    issue_tile(v_head, VRING, 0, 0);
    issue_tile(v_head, VRING, 1, 1);

    ex8 bq[QB][KS];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const elem_t *src = qg + (size_t)min(qcol(qb), p.S_q - 1) * D + 8 * g;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            bq[qb][ks] = *reinterpret_cast<const ex8 *>(src + 16 * ks);
    }
    f32x16 o_acc[QB * DB];
#pragma unroll
    for (int i = 0; i < QB * DB; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            o_acc[i][r] = 0.f;

    wait_vmcnt<0>();
    __syncthreads();

    // S(0) = K(0) Q^T
    f32x16 s_init[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            s_init[qb][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        const ex8 a = *(ATTN_LDS_PTR(const ex8))(uintptr_t)(koff[ks]);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
            s_init[qb] = E::mfma(a, bq[qb][ks], s_init[qb]);
    }

    typedef uint32_t u32x16 __attribute__((ext_vector_type(16)));
    u32x16 q_pack[NQP];
#pragma unroll
    for (int i = 0; i < NQP; ++i) {
        struct Four {
            ex8 a[4];
        } f;
#pragma unroll
        for (int t = 0; t < 4; ++t)
            f.a[t] = bq[(4 * i + t) / KS][(4 * i + t) % KS];
        q_pack[i] = __builtin_bit_cast(u32x16, f);
    }
    typename U32Vec<QB>::type thr_base_v;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
        U32Vec<QB>::set(thr_base_v, qb, (uint32_t)((CAUSAL ? min(qcol(qb), skv_m1) : skv_m1) - 4 * g));
    const float c_log2e = p.c;
    typename F32Vec<QB>::type m_ref_v, l_run_v;

    if constexpr (D == 128) {
#include "generated/attn_loop_d128a.inc"
    } else if constexpr (!F16) {
#include "generated/attn_loop_d256a.inc"
    } else {
#include "generated/attn_loop_d256a_f16.inc"
    }

    // ---- epilogue
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const float l_lane = F32Vec<QB>::get(l_run_v, qb);
        const float l_tot = l_lane + xor32(l_lane);
        const float inv = 1.f / l_tot;
        const int qrow = qcol(qb);
        if (qrow < p.S_q) {
            elem_t *orow = reinterpret_cast<elem_t *>(p.o) + ((size_t)bh * p.S_q + qrow) * D;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int rb = 0; rb < 4; ++rb) {
                    const f32x16 &oa = o_acc[qb * DB + db];
                    const f32x2 lo = {oa[4 * rb + 0] * inv, oa[4 * rb + 1] * inv};
                    const f32x2 hi = {oa[4 * rb + 2] * inv, oa[4 * rb + 3] * inv};
                    const ex2 blo = __builtin_convertvector(lo, ex2);  // round to nearest even
                    const ex2 bhi = __builtin_convertvector(hi, ex2);
                    const ex4 out = {blo[0], blo[1], bhi[0], bhi[1]};
                    *reinterpret_cast<ex4 *>(orow + 32 * db + 8 * rb + 4 * g) = out;
                }
            if (g == 0)
                p.lse[(size_t)bh * p.S_q + qrow] =
                    F32Vec<QB>::get(m_ref_v, qb) * p.scale + __builtin_amdgcn_logf(l_tot) * 0.69314718055994530942f;
        }
    }
}

}  // namespace attn
