// attn_fwd.hip -- Flash-Attention forward for MI355X (gfx950 / CDNA4) and its C ABI.
//
// The loop is the paper's Section 3 running example (Fig. 1a), in its full
// online-softmax form: per query tile, stream K/V tiles, S = Q K^T on MFMA,
// running row max / exp2 / row sum / accumulator rescale on the VALU,
// O += P V on MFMA, then normalise and write O and the log-sum-exp.
//
// Register-level formulation (why everything is "transposed"):
//   The kernel computes S^T = K Q^T and O^T = V^T P^T with
//   v_mfma_f32_32x32x16_bf16.  In the 32x32 accumulator layout a lane owns one
//   column, so with the transposed product a lane owns one *query*: lane l
//   holds query (l & 31) and, per 32-key block, the 16 keys
//       key(r) = 8*(r/4) + 4*(l/32) + r%4,   r = 0..15.
//   Row max and row sum are therefore in-lane reductions plus one exchange
//   with lane l^32, and the accumulator registers of S^T are already the
//   B operand of the second MFMA up to a fixed permutation of the contraction
//   index, which is absorbed by fetching V^T (the A operand) in the same
//   permuted key order: a contraction is invariant under a common permutation
//   of its index in both operands.
//
// One workgroup = NW wavefronts, each owning 32 query rows (BM = 32*NW);
// K/V tiles of BN keys are double-buffered in LDS.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

#include "attn_fwd.h"

namespace {

typedef __bf16 bf16_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

#define LDS_PTR(T) __attribute__((address_space(3))) T *

constexpr int kNumXcd = 8;  // MI355X: 8 XCDs, workgroups are dealt to them round-robin

// 16-byte-chunk XOR swizzle of a K/V tile row in LDS.  `row` is the key index
// inside the tile.  Requirements it meets:
//   * ds_read_b128 of one chunk column over 16 consecutive rows touches 16
//     different 16-byte bank groups (K as MFMA A operand);
//   * the transposing 8-byte reads of V touch rows r..r+3 in four different
//     64-byte bank groups.
template <int D>
__device__ __forceinline__ int swz(int row)
{
    const int x = (D == 64) ? (row >> 1) : row;
    if (D == 64)
        return ((x & 1) << 2) | ((x >> 1) & 3);
    return ((x & 3) << 2) | ((x >> 2) & 3);
}

__device__ __forceinline__ float xor32(float x)
{
    // exchange with the lane that holds the other 16 keys of the same query
    return __shfl_xor(x, 32, 64);
}

// Kernel parameters (plain struct, passed by value).
struct Params {
    const bf16_t *q, *k, *v;
    bf16_t *o;
    float *lse;
    int S_q, S_kv;
    int n_qt;       // query tiles per (b,h)
    int total_wg;   // B*H*n_qt
    float c;        // scale * log2(e): scores are handled in the base-2 domain
    float scale;
};

// VMODE selects how the V^T operand is fetched from the row-major V tile:
//   0: eight 16-bit LDS reads per operand (slow; layout-independent reference)
//   1: ds_read_b64_tr_b16, source lane i of a 16-lane block addresses (row i/4, 8-byte piece i%4)
//   2: ds_read_b64_tr_b16, source lane i addresses (row i%4, piece i/4)
template <int D, int BN, int NW, bool CAUSAL, int VMODE>
__global__ __launch_bounds__(NW * 64) void attn_fwd_kernel(const Params p)
{
    constexpr int BM = NW * 32;
    constexpr int NT = NW * 64;
    constexpr int CPR = D / 8;              // 16-byte chunks per row
    constexpr int KS = D / 16;              // k-steps of QK^T
    constexpr int DB = D / 32;              // 32-wide blocks of the head dimension
    constexpr int SB = BN / 32;             // 32-key blocks per tile
    constexpr int TILE_CHUNKS = BN * CPR;
    constexpr int LD_ITERS = TILE_CHUNKS / NT;
    static_assert(TILE_CHUNKS % NT == 0, "tile must split evenly over the threads");
    constexpr int TILE_BYTES = BN * D * 2;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    // [K buf0][K buf1][V buf0][V buf1]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int lq = lane & 31;   // query column owned by this lane
    const int g = lane >> 5;    // which half of the keys of a 32-key block

    // ---- a0: workgroup -> (b*H+h, query tile), XCD-aware ------------------
    // Workgroup ids are dealt round-robin to the 8 XCDs; give each XCD a
    // contiguous range of logical ids so that all query tiles of a head share
    // one XCD's L2 while they stream the same K/V.
    int logical;
    {
        const int wid = blockIdx.x;
        const int per = p.total_wg / kNumXcd, rem = p.total_wg % kNumXcd;
        const int xcd = wid % kNumXcd, slot = wid / kNumXcd;
        logical = (xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per) + slot;
    }
    const int bh = logical / p.n_qt;
    int qt = logical % p.n_qt;
    if (CAUSAL)
        qt = p.n_qt - 1 - qt;  // heaviest tiles first

    const int q0 = qt * BM;           // first query row of the workgroup
    const int q0w = q0 + wave * 32;   // first query row of this wave
    const int qrow = q0w + lq;        // this lane's query row (may be >= S_q in a ragged tile)

    const bf16_t *qg = p.q + (size_t)bh * p.S_q * D;
    const bf16_t *kg = p.k + (size_t)bh * p.S_kv * D;
    const bf16_t *vg = p.v + (size_t)bh * p.S_kv * D;

    // number of K/V tiles this workgroup visits
    int kv_end = p.S_kv;
    if (CAUSAL) {
        const int last_q = min(q0 + BM, p.S_q) - 1;
        kv_end = min(kv_end, last_q + 1);
    }
    const int n_tiles = (kv_end + BN - 1) / BN;

    // ---- a1: Q tile -> B-operand registers --------------------------------
    bf16x8 bq[KS];
    {
        const int r = min(qrow, p.S_q - 1);
        const bf16_t *src = qg + (size_t)r * D + 8 * g;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            bq[ks] = *reinterpret_cast<const bf16x8 *>(src + 16 * ks);
    }

    // ---- a2: K/V tile loads (global -> registers -> LDS) -------------------
    u32x4 kreg[LD_ITERS], vreg[LD_ITERS];
    auto load_tile = [&](int j) {
        const int j0 = j * BN;
#pragma unroll
        for (int it = 0; it < LD_ITERS; ++it) {
            const int cid = it * NT + tid;
            const int row = cid / CPR, ch = cid % CPR;
            const int grow = min(j0 + row, p.S_kv - 1);  // ragged tail: re-read the last row, masked later
            const size_t off = (size_t)grow * D + ch * 8;
            kreg[it] = *reinterpret_cast<const u32x4 *>(kg + off);
            vreg[it] = *reinterpret_cast<const u32x4 *>(vg + off);
        }
    };
    auto store_tile = [&](int buf) {
        unsigned char *ks = smem + buf * TILE_BYTES;
        unsigned char *vs = smem + (2 + buf) * TILE_BYTES;
#pragma unroll
        for (int it = 0; it < LD_ITERS; ++it) {
            const int cid = it * NT + tid;
            const int row = cid / CPR, ch = cid % CPR;
            const int pc = (ch & ~15) | ((ch & 15) ^ swz<D>(row));
            const int boff = row * (D * 2) + pc * 16;
            *reinterpret_cast<u32x4 *>(ks + boff) = kreg[it];
            *reinterpret_cast<u32x4 *>(vs + boff) = vreg[it];
        }
    };

    f32x16 oacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            oacc[db][r] = 0.f;
    float m_run = -INFINITY;  // running max of the raw (unscaled) scores of this lane's query
    float l_run = 0.f;        // this lane's partial row sum (its 16 of every 32 keys)

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
        const bool wave_active = !CAUSAL || (j0 <= q0w + 31);
        if (wave_active) {
            // ---- a3: S^T = K Q^T ------------------------------------------
            f32x16 s[SB];
#pragma unroll
            for (int sb = 0; sb < SB; ++sb) {
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    s[sb][r] = 0.f;
                const int row = 32 * sb + lq;
                const unsigned char *rowp = ks_ + row * (D * 2);
                const int sw = swz<D>(row);
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const int ch = 2 * ks + g;
                    const int pc = (ch & ~15) | ((ch & 15) ^ sw);
                    const bf16x8 a = *reinterpret_cast<const bf16x8 *>(rowp + pc * 16);
                    s[sb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bq[ks], s[sb], 0, 0, 0);
                }
            }

            // ---- a4: masks (ragged key tail, causal diagonal) ---------------
            const bool need_mask = (j0 + BN > p.S_kv) || (CAUSAL && (j0 + BN - 1 > q0w));
            // ---- a5: running row max ---------------------------------------
            float mloc = -INFINITY;
            if (need_mask) {
#pragma unroll
                for (int sb = 0; sb < SB; ++sb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int kv = j0 + 32 * sb + 8 * (r >> 2) + 4 * g + (r & 3);
                        const bool dead = (kv >= p.S_kv) || (CAUSAL && kv > qrow);
                        mloc = fmaxf(mloc, dead ? -INFINITY : s[sb][r]);
                    }
            } else {
#pragma unroll
                for (int sb = 0; sb < SB; ++sb)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        mloc = fmaxf(mloc, s[sb][r]);
            }
            mloc = fmaxf(mloc, xor32(mloc));
            const float m_new = fmaxf(m_run, mloc);
            // m_new stays -inf only for a row with no visible key so far, which
            // cannot happen for tile 0 (key 0 is visible to every query).
            const float alpha = (m_run == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((m_run - m_new) * p.c);
            const float mc = m_new * p.c;
            m_run = m_new;

            // ---- a6/a7/a9: exponentials, row sum, P -> bf16 -----------------
            bf16x8 pb[SB][2];
            float psum = 0.f;
#pragma unroll
            for (int sb = 0; sb < SB; ++sb)
#pragma unroll
                for (int r = 0; r < 16; r += 2) {
                    float t0 = fmaf(s[sb][r], p.c, -mc);
                    float t1 = fmaf(s[sb][r + 1], p.c, -mc);
                    if (need_mask) {
                        const int kv = j0 + 32 * sb + 8 * (r >> 2) + 4 * g + (r & 3);
                        if ((kv >= p.S_kv) || (CAUSAL && kv > qrow))
                            t0 = -INFINITY;
                        if ((kv + 1 >= p.S_kv) || (CAUSAL && kv + 1 > qrow))
                            t1 = -INFINITY;
                    }
                    const float p0 = __builtin_amdgcn_exp2f(t0);
                    const float p1 = __builtin_amdgcn_exp2f(t1);
                    psum += p0 + p1;
                    const f32x2 pp = {p0, p1};
                    const bf16x2 pk = __builtin_convertvector(pp, bf16x2);  // RNE
                    pb[sb][r >> 3][r & 7] = pk[0];
                    pb[sb][r >> 3][(r & 7) + 1] = pk[1];
                }
            l_run = l_run * alpha + psum;

            // ---- a8: accumulator rescale (skipped when no lane's max moved) --
            if (__any(alpha != 1.f)) {
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        oacc[db][r] *= alpha;
            }

            // ---- a10: O^T += V^T P^T ----------------------------------------
#pragma unroll
            for (int sb = 0; sb < SB; ++sb)
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    const int rowbase = 32 * sb + 16 * c + 4 * g;  // keys of slots 0..3; slots 4..7 are +8
#pragma unroll
                    for (int db = 0; db < DB; ++db) {
                        bf16x8 a;
                        if (VMODE == 0) {
                            const int d = 32 * db + lq;
#pragma unroll
                            for (int sl = 0; sl < 8; ++sl) {
                                const int row = rowbase + (sl & 3) + 8 * (sl >> 2);
                                const int ch = d >> 3;
                                const int pc = (ch & ~15) | ((ch & 15) ^ swz<D>(row));
                                a[sl] = *reinterpret_cast<const bf16_t *>(vs_ + row * (D * 2) + pc * 16 + (d & 7) * 2);
                            }
                        } else {
                            const int i = lane & 15;
                            const int dh = (lane >> 4) & 1;
                            const int rho = (VMODE == 1) ? (i >> 2) : (i & 3);
                            const int pi = (VMODE == 1) ? (i & 3) : (i >> 2);
                            const int ch = 4 * db + 2 * dh + (pi >> 1);
#pragma unroll
                            for (int hlf = 0; hlf < 2; ++hlf) {
                                const int row = rowbase + 8 * hlf + rho;
                                const int pc = (ch & ~15) | ((ch & 15) ^ swz<D>(row));
                                const unsigned char *src = vs_ + row * (D * 2) + pc * 16 + (pi & 1) * 8;
                                const bf16x4 t = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
                                    (LDS_PTR(bf16x4))(uintptr_t)(src - smem + (uintptr_t)(LDS_PTR(unsigned char))smem));
                                a[4 * hlf + 0] = t[0];
                                a[4 * hlf + 1] = t[1];
                                a[4 * hlf + 2] = t[2];
                                a[4 * hlf + 3] = t[3];
                            }
                        }
                        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[sb][c], oacc[db], 0, 0, 0);
                    }
                }
        }

        if (has_next) {
            store_tile(buf ^ 1);  // buffer buf^1 was last read in iteration j-1, fenced by the barrier below
        }
        __syncthreads();
    }

    // ---- a11: epilogue ------------------------------------------------------
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
                bf16x4 out = {blo[0], blo[1], bhi[0], bhi[1]};
                *reinterpret_cast<bf16x4 *>(orow + 32 * db + 8 * rb + 4 * g) = out;
            }
        if (g == 0)
            p.lse[(size_t)bh * p.S_q + qrow] = m_run * p.scale + __builtin_amdgcn_logf(l_tot) * 0.69314718055994530942f;
    }
}

template <int D, int BN, int NW, bool CAUSAL, int VMODE>
int launch(const Params &prm, int BH, hipStream_t stream)
{
    constexpr int BM = NW * 32;
    constexpr int LDS_BYTES = 4 * BN * D * 2;
    Params p = prm;
    p.n_qt = (p.S_q + BM - 1) / BM;
    const long long total = (long long)BH * p.n_qt;
    if (total > 0x7fffffffLL)
        return ATTN_ERR_SHAPE;
    p.total_wg = (int)total;
    auto kern = attn_fwd_kernel<D, BN, NW, CAUSAL, VMODE>;
    if (LDS_BYTES > 64 * 1024) {
        // opt in to more than 64 KB of dynamic LDS (gfx950 has 160 KB per CU)
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                LDS_BYTES) != hipSuccess) {
            (void)hipGetLastError();
            return ATTN_ERR_LAUNCH;
        }
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)p.total_wg), dim3(NW * 64), LDS_BYTES, stream, p);
    return hipGetLastError() == hipSuccess ? ATTN_OK : ATTN_ERR_LAUNCH;
}

template <int D, int BN, int NW, int VMODE>
int launch_c(const Params &prm, int BH, int causal, hipStream_t stream)
{
    return causal ? launch<D, BN, NW, true, VMODE>(prm, BH, stream) : launch<D, BN, NW, false, VMODE>(prm, BH, stream);
}

template <int VMODE>
int launch_d(const Params &prm, int BH, int D, int causal, hipStream_t stream)
{
    switch (D) {
    case 64:
        return launch_c<64, 64, 8, VMODE>(prm, BH, causal, stream);
    case 128:
        return launch_c<128, 64, 8, VMODE>(prm, BH, causal, stream);
    case 256:
        return launch_c<256, 32, 4, VMODE>(prm, BH, causal, stream);
    }
    return ATTN_ERR_UNSUPPORTED_D;
}

}  // namespace

extern "C" int attn_fwd(const void *q, const void *k, const void *v, void *o, float *lse, int B, int H, int S_q,
                        int S_kv, int D, int causal, float scale, void *stream)
{
    if (!q || !k || !v || !o || !lse)
        return ATTN_ERR_NULL;
    if (B < 1 || H < 1 || S_q < 1 || S_kv < 1)
        return ATTN_ERR_SHAPE;
    if (D != 64 && D != 128 && D != 256)
        return ATTN_ERR_UNSUPPORTED_D;
    const long long BH = (long long)B * H;
    if (BH > 0x7fffffffLL || BH * (long long)(S_q > S_kv ? S_q : S_kv) > (1LL << 40) / D)
        return ATTN_ERR_SHAPE;
    if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)o) & 15)
        return ATTN_ERR_ALIGN;
    if ((uintptr_t)lse & 3)
        return ATTN_ERR_ALIGN;
    if (!(scale >= 0.f) || isinf(scale))
        return ATTN_ERR_SCALE;

    Params p;
    p.q = static_cast<const bf16_t *>(q);
    p.k = static_cast<const bf16_t *>(k);
    p.v = static_cast<const bf16_t *>(v);
    p.o = static_cast<bf16_t *>(o);
    p.lse = lse;
    p.S_q = S_q;
    p.S_kv = S_kv;
    p.n_qt = 0;
    p.total_wg = 0;
    p.c = scale * 1.44269504088896340736f;
    p.scale = scale;

    // Debug only: ATTN_FWD_VMODE picks how V^T is fetched from LDS (see the kernel).
    static const int vmode = [] {
        const char *e = getenv("ATTN_FWD_VMODE");
        return e ? atoi(e) : 1;
    }();
    hipStream_t st = static_cast<hipStream_t>(stream);
    switch (vmode) {
    case 0:
        return launch_d<0>(p, (int)BH, D, causal, st);
    case 2:
        return launch_d<2>(p, (int)BH, D, causal, st);
    default:
        return launch_d<1>(p, (int)BH, D, causal, st);
    }
}

extern "C" const char *attn_strerror(int status)
{
    switch (status) {
    case ATTN_OK:
        return "ok";
    case ATTN_ERR_NULL:
        return "a required pointer is NULL";
    case ATTN_ERR_SHAPE:
        return "B, H, S_q, S_kv must be >= 1 and the tensors must not exceed 2^40 elements";
    case ATTN_ERR_UNSUPPORTED_D:
        return "head dimension D must be 64, 128 or 256";
    case ATTN_ERR_ALIGN:
        return "q, k, v, o must be 16-byte aligned and lse 4-byte aligned";
    case ATTN_ERR_SCALE:
        return "scale must be finite and >= 0";
    case ATTN_ERR_LAUNCH:
        return "the HIP runtime rejected the kernel launch";
    }
    return "unknown attn_status";
}

extern "C" int attn_version(void) { return 100; }
