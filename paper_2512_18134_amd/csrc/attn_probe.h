// attn_probe.h -- measurement kernels of the debug build (libmi355attn_debug.so), not part of the product
// path: what the matrix pipe sustains when nothing else is issued, as the ceiling the attention kernels are
// set against, and what the fp32 atomic reduction of dQ in the paper's single-pass backward (Section 6.3) costs
// on its own.
#pragma once
#include "attn_common.h"

namespace attn {

// Every wave keeps 4 A and 4 B fragments in registers (read once from `operands`: 2 x 4 x 64 lanes x 16
// bytes) and issues `iters` rounds of 8 independent v_mfma_f32_32x32x16_bf16 (8 accumulators, so that no MFMA
// waits for another).  No LDS, no VALU work, no memory traffic inside the loop.
template <int NW>
__global__ __launch_bounds__(NW * 64) void attn_probe_mfma_kernel(const bf16x8 *operands, float *out, int iters)
{
    const int lane = threadIdx.x & 63;
    bf16x8 a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i] = operands[i * 64 + lane];
        b[i] = operands[(4 + i) * 64 + lane];
    }
    f32x16 acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            acc[j][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 8; ++j)
            acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j & 3], b[(j + (j >> 2)) & 3], acc[j], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            s += acc[j][r];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// The same loop with the operand pattern as a parameter, to see what the matrix pipe's power depends on
// (one wave per SIMD).  PATTERN 0: consecutive MFMAs differ in both operands (the loop above); 1: pairs share A
// (what the attention loops do with a K or V fragment); 2: A fixed, B changes; 3: both fixed (only the
// accumulator changes); 4: v_mfma_f32_16x16x32_bf16 instead of 32x32x16, both operands change; 5: 32x32x16 on
// fp16 operands (`operands` then holds IEEE binary16), both change.
template <int PATTERN>
__global__ __launch_bounds__(256) void attn_probe_mfma_pattern_kernel(const bf16x8 *operands, float *out, int iters)
{
    typedef __attribute__((ext_vector_type(4))) float f32x4;
    typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
    const int lane = threadIdx.x & 63;
    bf16x8 a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i] = operands[i * 64 + lane];
        b[i] = operands[(4 + i) * 64 + lane];
    }
    float s = 0.f;
    if constexpr (PATTERN == 4) {
        f32x4 acc[16];
#pragma unroll
        for (int j = 0; j < 16; ++j)
            acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int j = 0; j < 16; ++j)
                acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[j & 3], b[(j + (j >> 2)) & 3], acc[j], 0, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < 16; ++j)
            s += acc[j][0] + acc[j][1] + acc[j][2] + acc[j][3];
    } else {
        f32x16 acc[8];
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                acc[j][r] = 0.f;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int ia = PATTERN == 1 ? (j >> 1) & 3 : (PATTERN == 2 || PATTERN == 3) ? 0 : j & 3;
                const int ib = PATTERN == 1 || PATTERN == 2 ? j & 3 : PATTERN == 3 ? 0 : (j + (j >> 2)) & 3;
                if constexpr (PATTERN == 5)
                    acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a[ia]),
                                                                     __builtin_bit_cast(f16x8, b[ib]), acc[j], 0, 0, 0);
                else
                    acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ia], b[ib], acc[j], 0, 0, 0);
            }
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                s += acc[j][r];
    }
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// The dQ reduction of the single-pass backward, alone.  A workgroup stands for one 128-key tile of one head
// (D = 128) and adds, for every 64-query tile it would visit (causal: from the tile that holds its first key),
// a 64 x 128 fp32 block of ones to dq[head][S_q][128] with hardware float atomics.  The access shape is the one
// a kernel whose dQ accumulators have lane = head-dimension column would produce: wave w owns columns 32 w ..,
// one instruction covers two query rows x 32 consecutive floats.  Afterwards dq[h][i][d] = number of key tiles
// query i sees.
__global__ __launch_bounds__(256) void attn_probe_dq_atomics_kernel(float *dq, int S_q, int n_kt, int causal)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int bh = blockIdx.x / n_kt, kt = blockIdx.x % n_kt;
    const int n_qt = S_q / 64;
    const int t_begin = causal ? min(kt * 2, n_qt) : 0;
    float *head = dq + (size_t)bh * S_q * 128 + 32 * wave + (lane & 31);
    for (int qt = t_begin; qt < n_qt; ++qt)
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = qt * 64 + 32 * qb + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                unsafeAtomicAdd(head + (size_t)row * 128, 1.0f);
            }
}

}  // namespace attn
