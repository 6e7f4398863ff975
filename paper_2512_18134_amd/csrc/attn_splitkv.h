// attn_splitkv.h -- merge kernel of the split-KV forward launch.
//
// A split-KV launch runs the forward kernel once per key range; range s leaves a normalised partial
// output O_s (fp32) and its log-sum-exp LSE_s.  Softmax attention over the union of the ranges is
//     LSE = ln sum_s exp(LSE_s),    O = sum_s exp(LSE_s - LSE) O_s
// (the same rescaling that the online softmax applies tile by tile inside one workgroup).
#pragma once
#include "attn_common.h"

namespace attn {

// One row = D/4 threads, 4 head-dimension elements each.  HBM-bound: reads n_split * (D + 1) floats per row.
// OUT: bf16_t or _Float16, the element type of o.
template <int D, typename OUT>
__global__ __launch_bounds__(256) void attn_splitkv_merge_kernel(const float *__restrict__ o_part,
                                                                 const float *__restrict__ lse_part,
                                                                 OUT *__restrict__ o, float *__restrict__ lse,
                                                                 long long n_rows, int n_split)
{
    constexpr int TPR = D / 4;
    constexpr int RPB = 256 / TPR;
    const int sub = threadIdx.x % TPR;
    for (long long r = (long long)blockIdx.x * RPB + threadIdx.x / TPR; r < n_rows; r += (long long)gridDim.x * RPB) {
        float m = -INFINITY;
#pragma unroll 8
        for (int s = 0; s < n_split; ++s)
            m = fmaxf(m, lse_part[(long long)s * n_rows + r]);
        // unnormalised weights first, one division at the end: the loads do not wait for the sum
        float sum = 0.f;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
        for (int s = 0; s < n_split; ++s) {
            const float w = expf(lse_part[(long long)s * n_rows + r] - m);
            const f32x4 x = *reinterpret_cast<const f32x4 *>(o_part + ((long long)s * n_rows + r) * D + 4 * sub);
            sum += w;
            acc += w * x;
        }
        const float total = m + logf(sum);
        acc *= 1.f / sum;
        const f32x2 lo = {acc[0], acc[1]}, hi = {acc[2], acc[3]};
        typedef OUT out2 __attribute__((ext_vector_type(2)));
        typedef OUT out4 __attribute__((ext_vector_type(4)));
        const out2 blo = __builtin_convertvector(lo, out2), bhi = __builtin_convertvector(hi, out2);  // RNE
        const out4 out = {blo[0], blo[1], bhi[0], bhi[1]};
        *reinterpret_cast<out4 *>(o + r * D + 4 * sub) = out;
        if (sub == 0)
            lse[r] = total;
    }
}

}  // namespace attn
