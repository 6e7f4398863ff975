// attn_probe.h -- measurement kernels of the debug build (libmi355attn_debug.so), not part of the product
// path: what the matrix pipe sustains when nothing else is issued, as the ceiling the attention kernels are
// set against.
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

}  // namespace attn
