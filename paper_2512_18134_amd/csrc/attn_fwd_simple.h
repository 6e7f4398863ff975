// attn_fwd_simple.h -- generic attention-forward kernel: any S_q/S_kv, D in
// {64,128,256}, causal or not.  It runs the loop of the paper's Fig. 1a in
// program order (S = QK^T, softmax, O += PV per K/V tile, no software
// pipelining inside a wave); two wavefronts per SIMD give the hardware
// something to overlap.  The hand-scheduled kernels (attn_fwd_asm.h,
// attn_fwd_asm2.h) take over for the shapes they support; this one covers
// everything else (scale == 0, heads of K/V of 2 GiB or more) and is the
// program-order reference of the schedule-equivalence test.
//
// Formulation: S^T = K Q^T and O^T = V^T P^T with v_mfma_f32_32x32x16_bf16, so
// that a lane owns one query column: row max / row sum are in-lane reductions
// plus one exchange with lane^32, and the S^T accumulators are already the B
// operand of the second MFMA up to a permutation of the contraction index that
// is absorbed by fetching V^T in the same permuted key order.
#pragma once
#include "attn_common.h"

namespace attn {

template <int D, int BN, int NW, bool CAUSAL>
__global__ __launch_bounds__(NW * 64) void attn_fwd_simple_kernel(const Params p)
{
    constexpr int BM = NW * 32;
    constexpr int NT = NW * 64;
    constexpr int CPR = D / 8;   // 16-byte chunks per row
    constexpr int KS = D / 16;   // k-steps of QK^T
    constexpr int DB = D / 32;   // 32-wide blocks of the head dimension
    constexpr int SB = BN / 32;  // 32-key blocks per tile
    constexpr int TILE_CHUNKS = BN * CPR;
    constexpr int LD_ITERS = TILE_CHUNKS / NT;
    static_assert(TILE_CHUNKS % NT == 0, "tile must split evenly over the threads");
    constexpr int TILE_BYTES = BN * D * 2;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // [K0][K1][V0][V1]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int lq = lane & 31;  // query column owned by this lane
    const int g = lane >> 5;   // which half of the keys of a 32-key block

    // ---- workgroup -> (b*H+h, query tile), XCD-aware, heaviest causal tiles first
    int bh, qt;
    wg_to_tile<CAUSAL>(blockIdx.x, p, D, bh, qt);

    const int q0 = qt * BM;
    const int q0w = q0 + wave * 32;
    const int qrow = q0w + lq;  // may be >= S_q in a ragged tile

    const bf16_t *qg = p.q + (size_t)bh * p.S_q * D;
    const bf16_t *kg = p.k + (size_t)bh * p.S_kv * D;
    const bf16_t *vg = p.v + (size_t)bh * p.S_kv * D;

    int kv_end = p.S_kv;
    if (CAUSAL)
        kv_end = min(kv_end, min(q0 + BM, p.S_q));
    const int n_tiles = (kv_end + BN - 1) / BN;

    // ---- Q tile -> B-operand registers
    bf16x8 bq[KS];
    {
        const bf16_t *src = qg + (size_t)min(qrow, p.S_q - 1) * D + 8 * g;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            bq[ks] = *reinterpret_cast<const bf16x8 *>(src + 16 * ks);
    }

    // ---- K/V tile: global -> registers -> LDS (swizzled)
    u32x4 kreg[LD_ITERS], vreg[LD_ITERS];
    auto load_tile = [&](int j) {
#pragma unroll
        for (int it = 0; it < LD_ITERS; ++it) {
            const int cid = it * NT + tid;
            const int row = cid / CPR, ch = cid % CPR;
            const int grow = min(j * BN + row, p.S_kv - 1);  // ragged tail: re-read the last row, masked later
            const size_t off = (size_t)grow * D + ch * 8;
            kreg[it] = *reinterpret_cast<const u32x4 *>(kg + off);
            vreg[it] = *reinterpret_cast<const u32x4 *>(vg + off);
        }
    };
    auto store_tile = [&](int buf) {
#pragma unroll
        for (int it = 0; it < LD_ITERS; ++it) {
            const int cid = it * NT + tid;
            const int row = cid / CPR, ch = cid % CPR;
            const int boff = row * (D * 2) + ((ch & ~15) | ((ch & 15) ^ swz<D>(row))) * 16;
            *reinterpret_cast<u32x4 *>(smem + buf * TILE_BYTES + boff) = kreg[it];
            *reinterpret_cast<u32x4 *>(smem + (2 + buf) * TILE_BYTES + boff) = vreg[it];
        }
    };

    f32x16 oacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            oacc[db][r] = 0.f;
    float m_run = -INFINITY;  // running max of the raw scores of this lane's query
    float l_run = 0.f;        // this lane's partial row sum (its 16 of every 32 keys)

    // one K/V tile; MASK: apply the ragged-tail / causal masks
    auto tile_body = [&](const unsigned char *ks_, const unsigned char *vs_, int j0, auto mask_tag) {
        constexpr bool MASK = decltype(mask_tag)::value;
        f32x16 s[SB];
#pragma unroll
        for (int sb = 0; sb < SB; ++sb)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                s[sb][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int sb = 0; sb < SB; ++sb) {
                const int row = 32 * sb + lq;
                const int ch = 2 * ks + g;
                const int pc = (ch & ~15) | ((ch & 15) ^ swz<D>(row));
                const bf16x8 a = *reinterpret_cast<const bf16x8 *>(ks_ + row * (D * 2) + pc * 16);
                s[sb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bq[ks], s[sb], 0, 0, 0);
            }

        auto dead = [&](int sb, int r) {
            const int kv = j0 + 32 * sb + acc_row(r, g);
            return (kv >= p.S_kv) || (CAUSAL && kv > qrow);
        };
        float mloc = -INFINITY;
#pragma unroll
        for (int sb = 0; sb < SB; ++sb)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                mloc = fmaxf(mloc, (MASK && dead(sb, r)) ? -INFINITY : s[sb][r]);
        mloc = fmaxf(mloc, xor32(mloc));
        const float m_new = fmaxf(m_run, mloc);
        // m_new is finite from tile 0 on: key 0 is visible to every query.
        const float alpha = (m_run == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((m_run - m_new) * p.c);
        const float mc = m_new * p.c;
        m_run = m_new;

        bf16x8 pb[SB][2];
        float psum = 0.f;
#pragma unroll
        for (int sb = 0; sb < SB; ++sb)
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                float t0 = fmaf(s[sb][r], p.c, -mc);
                float t1 = fmaf(s[sb][r + 1], p.c, -mc);
                if (MASK) {
                    t0 = dead(sb, r) ? -INFINITY : t0;
                    t1 = dead(sb, r + 1) ? -INFINITY : t1;
                }
                const float p0 = __builtin_amdgcn_exp2f(t0);
                const float p1 = __builtin_amdgcn_exp2f(t1);
                psum += p0 + p1;
                const f32x2 pp = {p0, p1};
                const bf16x2 pk = __builtin_convertvector(pp, bf16x2);  // round to nearest even
                pb[sb][r >> 3][r & 7] = pk[0];
                pb[sb][r >> 3][(r & 7) + 1] = pk[1];
            }
        l_run = l_run * alpha + psum;

        if (__any(alpha != 1.f)) {  // skipped when no lane's max moved (alpha == 1 exactly)
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    oacc[db][r] *= alpha;
        }

        // O^T += V^T P^T.  Contraction slot s of lane group g in chunk c of block sb
        // is key 32*sb + 16*c + 8*(s/4) + 4*g + s%4 (the accumulator row order of S^T).
        // ds_read_b64_tr_b16: inside a 16-lane block, source lane i supplies the
        // 8-byte piece i%4 of row i/4, and lane L receives column L of those 4 rows.
        const int i16 = lane & 15, dh = (lane >> 4) & 1;
        const int rho = i16 >> 2, pi = i16 & 3;
#pragma unroll
        for (int sb = 0; sb < SB; ++sb)
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    bf16x8 a;
                    const int ch = 4 * db + 2 * dh + (pi >> 1);
#pragma unroll
                    for (int hlf = 0; hlf < 2; ++hlf) {
                        const int row = 32 * sb + 16 * c + 4 * g + 8 * hlf + rho;
                        const int pc = (ch & ~15) | ((ch & 15) ^ swz<D>(row));
                        const bf16x4 t = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                            (ATTN_LDS_PTR(bf16x4))(vs_ + row * (D * 2) + pc * 16 + (pi & 1) * 8));
                        a[4 * hlf + 0] = t[0];
                        a[4 * hlf + 1] = t[1];
                        a[4 * hlf + 2] = t[2];
                        a[4 * hlf + 3] = t[3];
                    }
                    oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[sb][c], oacc[db], 0, 0, 0);
                }
    };

    load_tile(0);
    store_tile(0);
    __syncthreads();

    for (int j = 0; j < n_tiles; ++j) {
        const int buf = j & 1;
        const int j0 = j * BN;
        const bool has_next = (j + 1 < n_tiles);
        if (has_next)
            load_tile(j + 1);  // in flight while this tile is computed

        const unsigned char *ks_ = smem + buf * TILE_BYTES;
        const unsigned char *vs_ = smem + (2 + buf) * TILE_BYTES;
        // causal: a wave whose rows all precede this tile has nothing to add
        if (!CAUSAL || j0 <= q0w + 31) {
            const bool need_mask = (j0 + BN > p.S_kv) || (CAUSAL && (j0 + BN - 1 > q0w));
            if (need_mask)
                tile_body(ks_, vs_, j0, std::true_type{});
            else
                tile_body(ks_, vs_, j0, std::false_type{});
        }
        if (has_next)
            store_tile(buf ^ 1);  // buffer buf^1 was last read in iteration j-1
        __syncthreads();
    }

    // ---- epilogue: normalise, write O (bf16) and the log-sum-exp (fp32)
    const float l_tot = l_run + xor32(l_run);
    const float inv = 1.f / l_tot;
    if (qrow < p.S_q) {
        bf16_t *orow = p.o + ((size_t)bh * p.S_q + qrow) * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int rb = 0; rb < 4; ++rb) {
                const f32x2 lo = {oacc[db][4 * rb + 0] * inv, oacc[db][4 * rb + 1] * inv};
                const f32x2 hi = {oacc[db][4 * rb + 2] * inv, oacc[db][4 * rb + 3] * inv};
                const bf16x2 blo = __builtin_convertvector(lo, bf16x2);
                const bf16x2 bhi = __builtin_convertvector(hi, bf16x2);
                const bf16x4 out = {blo[0], blo[1], bhi[0], bhi[1]};
                *reinterpret_cast<bf16x4 *>(orow + 32 * db + 8 * rb + 4 * g) = out;
            }
        if (g == 0)
            p.lse[(size_t)bh * p.S_q + qrow] = m_run * p.scale + __builtin_amdgcn_logf(l_tot) * 0.69314718055994530942f;
    }
}

}  // namespace attn
