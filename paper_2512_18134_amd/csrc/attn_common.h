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

// Persistent launches: n_slots workgroups (a multiple of the XCD count) share a queue of n_entries tiles, which
// workgroup ids map to as above (entry e belongs to XCD e % 8).  Workgroup `wg` walks the queue of its XCD:
// pass k takes the XCD's entry k*S + m (S = n_slots / 8 slots per XCD, m = wg / 8), odd passes in reverse
// (k*S + S-1-m): with entries queued heaviest first a slot then pairs heavy with light, like a dispatcher
// that hands the next entry to the workgroup that finishes first.  Returns the entry, or -1 when pass k has
// none for this workgroup (only the last pass can be short).  n_slots == n_entries: one entry each.
__host__ __device__ __forceinline__ int persistent_entry(int wg, int n_slots, int n_entries, int k)
{
    if (n_slots >= n_entries)
        return k == 0 && wg < n_entries ? wg : -1;
    const int xcd = wg % kNumXcd, m = wg / kNumXcd, S = n_slots / kNumXcd;
    const int n_x = (n_entries - xcd + kNumXcd - 1) / kNumXcd;  // queue length of this XCD
    const int idx = k * S + ((k & 1) ? S - 1 - m : m);
    return idx < n_x ? idx * kNumXcd + xcd : -1;
}

// Causal launches hand out an XCD's workgroups in heaviest-first groups of whole heads: between 32
// workgroups (one per CU of the XCD) and 128, as many heads as stream no more than one L2 (4 MB) of
// operands between them; heads whose operands do not fit an L2 twice over share it by streaming in step
// instead, and get the large groups (better pairing of heavy and light tiles).
constexpr int kCausalGroupMinWgs = 32, kCausalGroupMaxWgs = 128;
constexpr long long kXcdL2Bytes = 4ll << 20;

// heads per group for tiles of n_t per head whose workgroups stream head_bytes of operands per head
__host__ __device__ __forceinline__ int causal_group_heads(int n_t, long long head_bytes)
{
    const int lo = (kCausalGroupMinWgs + n_t - 1) / n_t, hi = (kCausalGroupMaxWgs + n_t - 1) / n_t;
    const long long fit = head_bytes > 0 ? kXcdL2Bytes / head_bytes : hi;
    if (fit < 2)
        return hi;
    return fit < lo ? lo : (fit > hi ? hi : (int)fit);
}

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
#ifdef ATTN_DEBUG_ENTRY_POINTS
    // debug build only (attn_fwd_trace): per workgroup 8 values -- the 100 MHz clock at six points of the kernel,
    // then the hardware id and XCC id registers of the workgroup's first wave; NULL = no trace
    unsigned long long *trace;
    long long trace_entries;
#endif
};

// ATTN_TRACE(p, wg, slot): in the debug build, every lane of a workgroup stores the constant-rate clock (or
// `value`) into the trace record of tile `wg` (its index in the tile queue) (uniform control flow; the last writer's value stays); nothing in
// the product build.
#ifdef ATTN_DEBUG_ENTRY_POINTS
#define ATTN_TRACE_VALUE(p, wg, slot, value)                                                   \
    do {                                                                                       \
        if ((p).trace && ((long long)(wg) + 1) * 8 <= (p).trace_entries)                       \
            (p).trace[(size_t)(wg) * 8 + (slot)] = (unsigned long long)(value);                \
    } while (0)
#define ATTN_TRACE(p, wg, slot) ATTN_TRACE_VALUE(p, wg, slot, __builtin_amdgcn_s_memrealtime())
#else
#define ATTN_TRACE_VALUE(p, wg, slot, value) ((void)0)
#define ATTN_TRACE(p, wg, slot) ((void)0)
#endif

// Workgroup id -> (batch*head, query tile).
//  * not causal: all tiles cost the same; every XCD takes a contiguous range of (bh, qt) pairs.
//  * causal: query tile qt streams ~(qt + 1) times as many K/V tiles as tile 0, and a CU holds one
//    workgroup at a time, so the dispatch order decides the balance: tiles are handed out heaviest
//    first (a CU that finishes a light tile of the first batch then picks up the heaviest one left).
//    Every XCD owns whole heads (K/V stay in one L2) and works through them in groups of heads
//    (causal_group_heads: sized so that the operands of the heads in flight fit the L2, and so that
//    heavy and light tiles pair up), heaviest first across the heads of a group.  When B*H is not a
//    multiple of the XCD count, the heads left over are shared out tile by tile first.
//    head_bytes: operand bytes one head's workgroups stream (forward: K and V).
template <bool CAUSAL>
__host__ __device__ __forceinline__ void wg_to_tile_n(int wid, int total_wg, int n_t, long long head_bytes, int &bh,
                                                      int &t)
{
    if (!CAUSAL) {
        const int logical = xcd_remap(wid, total_wg);
        bh = logical / n_t;
        t = logical % n_t;
        return;
    }
    // XCD x owns `a` whole heads (x*a .. x*a + a - 1); the r = n_bh % 8 heads left over are dealt
    // to the XCDs tile by tile, heaviest first in alternating direction (so that every XCD gets the
    // same weight), and head the XCD's queue.
    const int n_bh = total_wg / n_t;
    const int a = n_bh / kNumXcd, r = n_bh % kNumXcd;
    const int xcd = wid % kNumXcd;
    int i = wid / kNumXcd;
    const int n_left = r * n_t;                                  // tiles of the left-over heads
    const int m_x = (n_left - xcd + kNumXcd - 1) / kNumXcd;      // ... that reach this XCD
    if (i < m_x) {
        const bool back = (i & 1) && kNumXcd * (i + 1) <= n_left;  // odd full rows run 7..0
        const int e = kNumXcd * i + (back ? kNumXcd - 1 - xcd : xcd);
        t = n_t - 1 - e / r;
        bh = kNumXcd * a + e % r;
        return;
    }
    i -= m_x;
    // groups of at least `want` heads, sizes as even as possible, larger ones first: a short group at
    // the end of the queue would leave its heavy tiles without light partners
    const int want = causal_group_heads(n_t, head_bytes);
    const int ng = a > want ? a / want : 1;
    const int base = a / ng, extra = a % ng;     // `extra` groups of base + 1 heads, then groups of base
    const int big = extra * (base + 1) * n_t;
    int gh, head0, j;
    if (i < big) {
        gh = base + 1;
        head0 = i / (gh * n_t) * gh;
        j = i % (gh * n_t);
    } else {
        gh = base;
        head0 = extra * (base + 1) + (i - big) / (gh * n_t) * gh;
        j = (i - big) % (gh * n_t);
    }
    t = n_t - 1 - j / gh;
    bh = xcd * a + head0 + j % gh;
}

template <bool CAUSAL>
__device__ __forceinline__ void wg_to_tile(int wid, const Params &p, int D, int &bh, int &qt)
{
    // one head's workgroups stream its K and V: 2 tensors x S_kv rows x D 16-bit elements
    wg_to_tile_n<CAUSAL>(wid, p.total_wg, p.n_qt, 4ll * p.S_kv * D, bh, qt);
}

}  // namespace attn
