// attn_common.h -- vector types, the LDS swizzle and the kernel parameter block
// shared by the attention-forward kernels of this library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

namespace attn {

typedef __bf16 bf16_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

#define ATTN_LDS_PTR(T) __attribute__((address_space(3))) T *

constexpr int kNumXcd = 8;  // MI355X: 8 XCDs; workgroup ids are dealt to them round-robin

// 16-byte-chunk XOR swizzle of a K/V tile row in LDS (`row` = key index inside
// the tile; the value is XORed into the low 4 bits of the chunk index).
//   * ds_read_b128 of one chunk column over 16 consecutive rows (K as MFMA A
//     operand) touches 16 different 16-byte bank groups;
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

// max / sum partner: the lane that holds the other 16 keys of the same query
__device__ __forceinline__ float xor32(float x) { return __shfl_xor(x, 32, 64); }

// MFMA 32x32x16 bf16 accumulator layout: register r of lane l is
// row 8*(r/4) + 4*(l/32) + r%4, column l%32.
__device__ __forceinline__ int acc_row(int r, int g) { return 8 * (r >> 2) + 4 * g + (r & 3); }

// workgroup id -> logical id such that every XCD owns a contiguous range of
// logical ids (all query tiles of a head then share one XCD's L2 while they
// stream the same K/V).
__host__ __device__ __forceinline__ int xcd_remap(int wid, int total)
{
    const int per = total / kNumXcd, rem = total % kNumXcd;
    const int xcd = wid % kNumXcd, slot = wid / kNumXcd;
    return (xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per) + slot;
}

// Causal launches: workgroups per XCD that are handed out as one heaviest-first group (2 per CU).
constexpr int kCausalGroupWgs = 64;

// Kernel parameters (plain struct, passed by value).
struct Params {
    const bf16_t *q, *k, *v;
    bf16_t *o;
    float *lse;
    int S_q, S_kv;
    int n_qt;      // query tiles per (b,h)
    int total_wg;  // B*H*n_qt
    float c;       // scale * log2(e): the softmax runs in the base-2 domain
    float scale;
    // split-KV launches only: the keys are cut into n_split ranges of split_len keys (a multiple of
    // the K/V tile), every range is a workgroup of its own and writes a normalised partial result
    int n_split, split_len;
    float *o_part;    // [n_split][B*H*S_q][D] fp32
    float *lse_part;  // [n_split][B*H*S_q] fp32
};

// Workgroup id -> (batch*head, query tile).
//  * not causal: all tiles cost the same; every XCD takes a contiguous range of (bh, qt) pairs.
//  * causal: query tile qt streams ~(qt + 1) times as many K/V tiles as tile 0, and a CU holds one
//    workgroup at a time, so the dispatch order decides the balance: tiles are handed out heaviest
//    first (a CU that finishes a light tile of the first batch then picks up the heaviest one left).
//    With B*H a multiple of the XCD count every XCD owns whole heads (K/V stay in one L2) and works
//    through them in groups of just enough heads for 64 workgroups -- two per CU of the XCD, so that
//    heavy and light tiles pair up -- heaviest first across the heads of a group: the workgroups in
//    flight on an XCD then stream the K/V of one or two heads, not of every head the XCD owns, and
//    keep hitting its L2.  Otherwise the tiles of a head go to all XCDs and the order is heaviest
//    first over the whole grid (chip-wide groups of heads measured no better there).
template <bool CAUSAL>
__host__ __device__ __forceinline__ void wg_to_tile_n(int wid, int total_wg, int n_t, int &bh, int &t)
{
    if (!CAUSAL) {
        const int logical = xcd_remap(wid, total_wg);
        bh = logical / n_t;
        t = logical % n_t;
        return;
    }
    const int n_bh = total_wg / n_t;
    if (n_bh % kNumXcd == 0) {
        const int nh = n_bh / kNumXcd, xcd = wid % kNumXcd, i = wid / kNumXcd;
        const int want = (kCausalGroupWgs + n_t - 1) / n_t;
        const int gsz = want < nh ? want : nh;  // heads per group
        const int grp = i / (gsz * n_t), j = i % (gsz * n_t);
        const int left = nh - grp * gsz;
        const int gh = left < gsz ? left : gsz;  // the last group may be short
        t = n_t - 1 - j / gh;
        bh = xcd * nh + grp * gsz + j % gh;
    } else {
        t = n_t - 1 - wid / n_bh;
        bh = wid % n_bh;
    }
}

template <bool CAUSAL>
__device__ __forceinline__ void wg_to_tile(int wid, const Params &p, int &bh, int &qt)
{
    wg_to_tile_n<CAUSAL>(wid, p.total_wg, p.n_qt, bh, qt);
}

}  // namespace attn
