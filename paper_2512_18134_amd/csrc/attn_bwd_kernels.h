// attn_bwd_kernels.h -- attention backward for gfx950 (the pass of the paper's Section 6.3).
//
// The paper's single-pass form (Section 6.3) runs five matrix products per (query tile, key tile)
// pair and reduces dQ into global memory with atomics; the paper itself finds that reduction to
// be the bound once the tensor cores are fast enough, and measured alone on this chip it takes
// longer than the whole pass below.  Here the work is split into two sweeps that need no atomics
// and no cross-workgroup reduction, so the results are bitwise reproducible:
//
//   KEY_OWNER = true   a workgroup owns 128 keys and streams query tiles:
//                      S = Q K^T, dP = dO V^T, P = exp(S - LSE), dS = P o (dP - Delta),
//                      dV += P^T dO,  dK += dS^T Q                       (4 GEMMs)
//   KEY_OWNER = false  a workgroup owns 128 queries and streams key tiles:
//                      S, dP, P, dS as above,  dQ += dS K                 (3 GEMMs)
//
// Delta_i = sum_d dO_id O_id comes from a small kernel that runs first (attn_bwd_delta_kernel).
//
// Both sweeps are one kernel template.  As in the forward kernels every product is arranged
// so that the "owner" index (key or query) is the lane: S is computed as a 32x32 MFMA tile
// whose columns are owner indices, its accumulator registers then already have the layout of
// the B operand of the products that contract over the streamed index, and the transposed A
// operands of those products (Q^T, dO^T, K^T) come out of LDS through ds_read_b64_tr_b16.
// The owner's rows of Q/dO (or K/V) stay in registers as B operands for the whole kernel.
// Streamed tiles (64 rows) arrive by direct global->LDS loads, three ring stages, one
// barrier per tile.  Instruction scheduling inside a tile is left to the compiler.
#pragma once
#include <type_traits>

#include "attn_common.h"
#include "attn_dma.h"       // dma16, wait_vmcnt

namespace attn {

struct BwdParams {
    const bf16_t *q, *k, *v, *o, *d_o;
    const float *lse;
    float *lse2;   // workspace, [B][H][S_q]: LSE * log2(e), written by the delta kernel, read by the sweeps
    float *delta;  // workspace, [B][H][S_q], directly behind lse2: Delta
    bf16_t *dq, *dk, *dv;
    int S_q, S_kv;
    int n_t;       // owner tiles per (b,h) of the launched sweep
    int total_wg;  // B*H*n_t
    long long n_rows;  // B*H*S_q (delta kernel)
    float c;       // scale * log2(e)
    float scale;
};

// Delta[r] = sum_d dO[r][d] * O[r][d] (fp32) and LSE'[r] = LSE[r] * log2(e).  D/8 lanes per row, 16 bytes per lane.
template <int D, typename ELEM = bf16_t>
__global__ __launch_bounds__(256) void attn_bwd_delta_kernel(const BwdParams p)
{
    typedef ELEM ex8 __attribute__((ext_vector_type(8)));
    constexpr int LPR = D / 8;        // lanes per row
    constexpr int RPB = 256 / LPR;    // rows per block and step
    const int tid = threadIdx.x;
    const int sub = tid % LPR;
    for (long long r = (long long)blockIdx.x * RPB + tid / LPR; r < p.n_rows; r += (long long)gridDim.x * RPB) {
        const ex8 a = *reinterpret_cast<const ex8 *>(reinterpret_cast<const ELEM *>(p.d_o) + r * D + 8 * sub);
        const ex8 b = *reinterpret_cast<const ex8 *>(reinterpret_cast<const ELEM *>(p.o) + r * D + 8 * sub);
        float acc = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e)
            acc = fmaf((float)a[e], (float)b[e], acc);
#pragma unroll
        for (int m = LPR / 2; m >= 1; m >>= 1)
            acc += __shfl_xor(acc, m, 64);
        if (sub == 0) {
            p.delta[r] = acc;
            p.lse2[r] = p.lse[r] * 1.44269504088896340736f;
        }
    }
}

// NW = waves per workgroup: 4 (one per SIMD, up to 512 registers: the key-owner sweep needs them) or
// 8 (two per SIMD, 256 registers: the query-owner sweep fits, and the second wave hides latencies).
template <int D, bool CAUSAL, bool KEY_OWNER, int NW>
__global__ __launch_bounds__(NW * 64) void attn_bwd_sweep_kernel(const BwdParams p)
{
    static_assert(D == 64 || D == 128, "backward sweeps: D = 64 or 128");
    static_assert(NW == 4 || NW == 8, "4 or 8 waves: one or two per SIMD");
    constexpr int BN = 64, BO = NW * 32, NST = 3;
    constexpr int CPR = D / 8;
    constexpr int KS = D / 16;
    constexpr int DB = D / 32;
    constexpr int ROWB = D * 2;
    constexpr int TB = BN * ROWB;
    constexpr int NLD = TB / (NW * 1024);
    constexpr int RPG = 1024 / ROWB;
    constexpr int NGRP = 2 * NLD + (KEY_OWNER ? 1 : 0);  // direct loads per wave and streamed tile
    constexpr float kLog2e = 1.44269504088896340736f;

    // T1 ring [3][TB] (K, or Q), T2 ring [3][TB] (V, or dO), aux ring [3][NW][64] floats (LSE, Delta rows)
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr uint32_t RING1 = 0, RING2 = NST * TB, AUX = 2 * NST * TB;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(ATTN_LDS_PTR(unsigned char))smem;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lq = lane & 31;
    const int g = lane >> 5;

    // ---- workgroup -> (head, owner tile).  Causal: a query tile streams more keys the later it is,
    // a key tile streams more queries the earlier it is; heaviest first either way.
    int bh, ot;
    // a head's sweeps stream Q, dO, K and V between them
    wg_to_tile_n<CAUSAL>(blockIdx.x, p.total_wg, p.n_t, 4ll * (p.S_q + p.S_kv) * D, bh, ot);
    if (CAUSAL && KEY_OWNER)
        ot = p.n_t - 1 - ot;
    const int S_own = KEY_OWNER ? p.S_kv : p.S_q;
    const int S_str = KEY_OWNER ? p.S_q : p.S_kv;
    const int o0 = ot * BO;
    const int o0w = o0 + wave * 32;
    const int own = o0w + lq;                 // this lane's key (or query)
    const int own_c = min(own, S_own - 1);    // clamped for loads; lanes past the end never store

    const size_t q_head = (size_t)bh * p.S_q * D, k_head = (size_t)bh * p.S_kv * D;
    const bf16_t *x1 = KEY_OWNER ? p.k + k_head : p.q + q_head;    // owner rows, pairs with T1 in S
    const bf16_t *x2 = KEY_OWNER ? p.v + k_head : p.d_o + q_head;  // owner rows, pairs with T2 in dP
    const bf16_t *t1 = KEY_OWNER ? p.q + q_head : p.k + k_head;    // streamed
    const bf16_t *t2 = KEY_OWNER ? p.d_o + q_head : p.v + k_head;  // streamed
    const float *lse_head = p.lse + (size_t)bh * p.S_q;
    const float *delta_head = p.delta + (size_t)bh * p.S_q;

    // ---- streamed tile range
    int t_begin = 0, t_end;
    if (KEY_OWNER) {
        t_end = (p.S_q + BN - 1) / BN;
        if (CAUSAL)
            t_begin = min(o0 / BN, t_end);  // queries before the first owned key see none of them
    } else {
        int kv_end = p.S_kv;
        if (CAUSAL)
            kv_end = min(kv_end, min(o0 + BO, p.S_q));
        t_end = (kv_end + BN - 1) / BN;
    }

    // ---- direct-load addressing (lane -> row in tile, swizzled 16-byte chunk)
    int dma_row[NLD];
    uint32_t dma_choff[NLD];
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
        const int gi = i * NW + wave;
        dma_row[i] = RPG * gi + lane / CPR;
        dma_choff[i] = (uint32_t)(((lane % CPR) ^ swz<D>(dma_row[i])) * 16);
    }
    // rows past the end of the streamed tensor re-read its last row (masked later)
    auto issue_tile = [&](int stage, int t) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int r = min(t * BN + dma_row[i], S_str - 1);
            const uint32_t voff = (uint32_t)r * ROWB + dma_choff[i];
            dma16(lds0 + RING1 + stage * TB + (i * NW + wave) * 1024, t1, voff);
            dma16(lds0 + RING2 + stage * TB + (i * NW + wave) * 1024, t2, voff);
        }
        if (KEY_OWNER) {
            // even waves: LSE of the tile's 64 queries, odd waves: Delta; waves past the first two fill spare slots so that
            // every wave has the same number of loads in flight
            const int r = min(t * BN + lane, p.S_q - 1);
            dma4(lds0 + AUX + (stage * NW + wave) * 256, (wave & 1) ? delta_head : lse_head, (uint32_t)r * 4);
        }
    };

    // ---- operand addressing inside a tile (ring base added at the use)
    uint32_t roff[KS];   // rows of a tile as A operand: row 32*blk + lq, chunk 2*ks + g
    {
        const int sw = swz<D>(lq);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            roff[ks] = lds0 + (uint32_t)(lq * ROWB + (((2 * ks + g) ^ sw) * 16));
    }
    uint32_t toff[DB][2];  // transposed tile as A operand (ds_read_b64_tr_b16), see attn_fwd_pipe.h
    {
        const int i16 = lane & 15, dh = (lane >> 4) & 1;
        const int rho = i16 >> 2, pi = i16 & 3;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int hlf = 0; hlf < 2; ++hlf) {
                const int row = 4 * g + 8 * hlf + rho;
                const int ch = 4 * db + 2 * dh + (pi >> 1);
                toff[db][hlf] = lds0 + (uint32_t)(row * ROWB + ((ch ^ swz<D>(row)) * 16) + (pi & 1) * 8);
            }
    }
    auto row_frag = [&](uint32_t ring_stage, int blk, int ks) {
        return *(ATTN_LDS_PTR(const bf16x8))(uintptr_t)(roff[ks] + (ring_stage + blk * 32 * ROWB));
    };
    auto tr_frag = [&](uint32_t ring_stage, int chunk, int db) {
        bf16x8 a;
#pragma unroll
        for (int hlf = 0; hlf < 2; ++hlf) {
            const bf16x4 t = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                (ATTN_LDS_PTR(bf16x4))(uintptr_t)(toff[db][hlf] + (ring_stage + chunk * 16 * ROWB)));
            a[4 * hlf + 0] = t[0];
            a[4 * hlf + 1] = t[1];
            a[4 * hlf + 2] = t[2];
            a[4 * hlf + 3] = t[3];
        }
        return a;
    };

    // ---- prologue: start the stream, load the owner's rows as B operands
    issue_tile(0, t_begin);
    issue_tile(1, t_begin + 1);

    bf16x8 b1[KS], b2[KS];
    {
        const bf16_t *s1 = x1 + (size_t)own_c * D + 8 * g;
        const bf16_t *s2 = x2 + (size_t)own_c * D + 8 * g;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            b1[ks] = *reinterpret_cast<const bf16x8 *>(s1 + 16 * ks);
            b2[ks] = *reinterpret_cast<const bf16x8 *>(s2 + 16 * ks);
        }
    }
    float lse2_own = 0.f, delta_own = 0.f;
    if (!KEY_OWNER) {
        lse2_own = lse_head[own_c] * kLog2e;
        delta_own = delta_head[own_c];
    }

    f32x16 acc1[DB], acc2[DB];  // dK^T (or dQ^T), dV^T: rows = head dimension, column = owner
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            acc1[db][r] = 0.f;
            acc2[db][r] = 0.f;
        }

    // Streamed tiles.  With two waves per SIMD the loop is unrolled by the ring depth so that the stage
    // offsets of the LDS reads are instruction immediates; with one wave per SIMD the rolled loop
    // (stage offset in a register) is what the compiler schedules best.
    if constexpr (NW == 8) {
        auto tile = [&](int t, auto st_tag) {
            constexpr int st = decltype(st_tag)::value;
            const uint32_t s1 = RING1 + st * TB, s2 = RING2 + st * TB;
            // tile t was issued two iterations ago; the loads of tile t+1 may still be in flight
            wait_vmcnt<NGRP>();
            __syncthreads();
            // every wave has finished tile t-1: its stage is free
            issue_tile((st + 2) % NST, t + 2);

            // S (owner columns) and dP
            f32x16 s[2], dp[2];
#pragma unroll
            for (int blk = 0; blk < 2; ++blk)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    s[blk][r] = 0.f;
                    dp[blk][r] = 0.f;
                }
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int blk = 0; blk < 2; ++blk)
                    s[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag(s1, blk, ks), b1[ks], s[blk], 0, 0, 0);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int blk = 0; blk < 2; ++blk)
                    dp[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag(s2, blk, ks), b2[ks], dp[blk], 0, 0, 0);

            // does this wave's part of the tile touch the ragged end or the causal diagonal?
            const int r0 = t * BN;  // first streamed row of the tile
            bool need_mask = r0 + BN > S_str;
            if (CAUSAL)
                need_mask = need_mask || (KEY_OWNER ? (r0 < o0w + 31) : (r0 + BN - 1 > o0w));

            // P = exp(S*scale - LSE), dS = P (dP - Delta), both rounded to bf16 as B operands
            bf16x8 pb[2][2], dsb[2][2];
#pragma unroll
            for (int blk = 0; blk < 2; ++blk)
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    float lse2[4], dl[4];
                    if (KEY_OWNER) {
                        const uint32_t aux = lds0 + AUX + st * (NW * 256) + (32 * blk + 8 * a + 4 * g) * 4;
                        const f32x4 l4 = *(ATTN_LDS_PTR(const f32x4))(uintptr_t)aux;
                        const f32x4 d4 = *(ATTN_LDS_PTR(const f32x4))(uintptr_t)(aux + 256);
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            lse2[i] = l4[i] * kLog2e;
                            dl[i] = d4[i];
                        }
                    } else {
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            lse2[i] = lse2_own;
                            dl[i] = delta_own;
                        }
                    }
                    float pv[4], dsv[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int r = 4 * a + i;
                        float pe = __builtin_amdgcn_exp2f(fmaf(s[blk][r], p.c, -lse2[i]));
                        if (need_mask) {
                            const int sr = r0 + 32 * blk + 8 * a + 4 * g + i;  // streamed row of this element
                            bool ok = sr < S_str;
                            if (CAUSAL)
                                ok = ok && (KEY_OWNER ? (sr >= own) : (sr <= own));
                            pe = ok ? pe : 0.f;
                        }
                        pv[i] = pe;
                        dsv[i] = pe * (dp[blk][r] - dl[i]);
                    }
                    const f32x2 p01 = {pv[0], pv[1]}, p23 = {pv[2], pv[3]};
                    const f32x2 d01 = {dsv[0], dsv[1]}, d23 = {dsv[2], dsv[3]};
                    const bf16x2 pa = __builtin_convertvector(p01, bf16x2), pc = __builtin_convertvector(p23, bf16x2);
                    const bf16x2 da = __builtin_convertvector(d01, bf16x2), dc = __builtin_convertvector(d23, bf16x2);
                    const int e0 = 4 * (a & 1);
                    pb[blk][a >> 1][e0 + 0] = pa[0], pb[blk][a >> 1][e0 + 1] = pa[1];
                    pb[blk][a >> 1][e0 + 2] = pc[0], pb[blk][a >> 1][e0 + 3] = pc[1];
                    dsb[blk][a >> 1][e0 + 0] = da[0], dsb[blk][a >> 1][e0 + 1] = da[1];
                    dsb[blk][a >> 1][e0 + 2] = dc[0], dsb[blk][a >> 1][e0 + 3] = dc[1];
                }

            // contractions over the streamed index: dK^T += Q^T dS (or dQ^T += K^T dS^T), dV^T += dO^T P
#pragma unroll
            for (int ch = 0; ch < 4; ++ch)
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    acc1[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tr_frag(s1, ch, db), dsb[ch >> 1][ch & 1], acc1[db], 0, 0, 0);
                    if (KEY_OWNER)
                        acc2[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tr_frag(s2, ch, db), pb[ch >> 1][ch & 1], acc2[db], 0, 0, 0);
                }
        };
        int t = t_begin;
        for (; t + 3 <= t_end; t += 3) {
            tile(t, std::integral_constant<int, 0>{});
            tile(t + 1, std::integral_constant<int, 1>{});
            tile(t + 2, std::integral_constant<int, 2>{});
        }
        if (t < t_end)
            tile(t, std::integral_constant<int, 0>{});
        if (t + 1 < t_end)
            tile(t + 1, std::integral_constant<int, 1>{});
    } else {
        for (int t = t_begin; t < t_end; ++t) {
            const int st = (t - t_begin) % NST;
        const uint32_t s1 = RING1 + st * TB, s2 = RING2 + st * TB;
        // tile t was issued two iterations ago; the loads of tile t+1 may still be in flight
        wait_vmcnt<NGRP>();
        __syncthreads();
        // every wave has finished tile t-1: its stage is free
        issue_tile((st + 2) % NST, t + 2);

        // S (owner columns) and dP
        f32x16 s[2], dp[2];
#pragma unroll
        for (int blk = 0; blk < 2; ++blk)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                s[blk][r] = 0.f;
                dp[blk][r] = 0.f;
            }
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int blk = 0; blk < 2; ++blk)
                s[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag(s1, blk, ks), b1[ks], s[blk], 0, 0, 0);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int blk = 0; blk < 2; ++blk)
                dp[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag(s2, blk, ks), b2[ks], dp[blk], 0, 0, 0);

        // does this wave's part of the tile touch the ragged end or the causal diagonal?
        const int r0 = t * BN;  // first streamed row of the tile
        bool need_mask = r0 + BN > S_str;
        if (CAUSAL)
            need_mask = need_mask || (KEY_OWNER ? (r0 < o0w + 31) : (r0 + BN - 1 > o0w));

        // P = exp(S*scale - LSE), dS = P (dP - Delta), both rounded to bf16 as B operands
        bf16x8 pb[2][2], dsb[2][2];
#pragma unroll
        for (int blk = 0; blk < 2; ++blk)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                float lse2[4], dl[4];
                if (KEY_OWNER) {
                    const uint32_t aux = lds0 + AUX + st * (NW * 256) + (32 * blk + 8 * a + 4 * g) * 4;
                    const f32x4 l4 = *(ATTN_LDS_PTR(const f32x4))(uintptr_t)aux;
                    const f32x4 d4 = *(ATTN_LDS_PTR(const f32x4))(uintptr_t)(aux + 256);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        lse2[i] = l4[i] * kLog2e;
                        dl[i] = d4[i];
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        lse2[i] = lse2_own;
                        dl[i] = delta_own;
                    }
                }
                float pv[4], dsv[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int r = 4 * a + i;
                    float pe = __builtin_amdgcn_exp2f(fmaf(s[blk][r], p.c, -lse2[i]));
                    if (need_mask) {
                        const int sr = r0 + 32 * blk + 8 * a + 4 * g + i;  // streamed row of this element
                        bool ok = sr < S_str;
                        if (CAUSAL)
                            ok = ok && (KEY_OWNER ? (sr >= own) : (sr <= own));
                        pe = ok ? pe : 0.f;
                    }
                    pv[i] = pe;
                    dsv[i] = pe * (dp[blk][r] - dl[i]);
                }
                const f32x2 p01 = {pv[0], pv[1]}, p23 = {pv[2], pv[3]};
                const f32x2 d01 = {dsv[0], dsv[1]}, d23 = {dsv[2], dsv[3]};
                const bf16x2 pa = __builtin_convertvector(p01, bf16x2), pc = __builtin_convertvector(p23, bf16x2);
                const bf16x2 da = __builtin_convertvector(d01, bf16x2), dc = __builtin_convertvector(d23, bf16x2);
                const int e0 = 4 * (a & 1);
                pb[blk][a >> 1][e0 + 0] = pa[0], pb[blk][a >> 1][e0 + 1] = pa[1];
                pb[blk][a >> 1][e0 + 2] = pc[0], pb[blk][a >> 1][e0 + 3] = pc[1];
                dsb[blk][a >> 1][e0 + 0] = da[0], dsb[blk][a >> 1][e0 + 1] = da[1];
                dsb[blk][a >> 1][e0 + 2] = dc[0], dsb[blk][a >> 1][e0 + 3] = dc[1];
            }

        // contractions over the streamed index: dK^T += Q^T dS (or dQ^T += K^T dS^T), dV^T += dO^T P
#pragma unroll
        for (int ch = 0; ch < 4; ++ch)
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                acc1[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tr_frag(s1, ch, db), dsb[ch >> 1][ch & 1], acc1[db], 0, 0, 0);
                if (KEY_OWNER)
                    acc2[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tr_frag(s2, ch, db), pb[ch >> 1][ch & 1], acc2[db], 0, 0, 0);
            }
        }
    }
    // no direct load may still be writing LDS when the workgroup retires
    wait_vmcnt<0>();

    // ---- epilogue: dK = scale * acc1, dV = acc2 (or dQ = scale * acc1), bf16, row = owner
    if (own < S_own) {
        bf16_t *out1 = (KEY_OWNER ? p.dk + k_head : p.dq + q_head) + (size_t)own * D;
        bf16_t *out2 = p.dv + k_head + (size_t)own * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int rb = 0; rb < 4; ++rb) {
                const f32x2 lo = {acc1[db][4 * rb + 0] * p.scale, acc1[db][4 * rb + 1] * p.scale};
                const f32x2 hi = {acc1[db][4 * rb + 2] * p.scale, acc1[db][4 * rb + 3] * p.scale};
                const bf16x2 blo = __builtin_convertvector(lo, bf16x2), bhi = __builtin_convertvector(hi, bf16x2);
                const bf16x4 w = {blo[0], blo[1], bhi[0], bhi[1]};
                *reinterpret_cast<bf16x4 *>(out1 + 32 * db + 8 * rb + 4 * g) = w;
                if (KEY_OWNER) {
                    const f32x2 lo2 = {acc2[db][4 * rb + 0], acc2[db][4 * rb + 1]};
                    const f32x2 hi2 = {acc2[db][4 * rb + 2], acc2[db][4 * rb + 3]};
                    const bf16x2 b2lo = __builtin_convertvector(lo2, bf16x2), b2hi = __builtin_convertvector(hi2, bf16x2);
                    const bf16x4 w2 = {b2lo[0], b2lo[1], b2hi[0], b2hi[1]};
                    *reinterpret_cast<bf16x4 *>(out2 + 32 * db + 8 * rb + 4 * g) = w2;
                }
            }
    }
}

}  // namespace attn
