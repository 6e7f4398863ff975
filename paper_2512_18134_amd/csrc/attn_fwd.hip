// attn_fwd.hip -- C ABI of libmi355attn.so (see include/attn_fwd.h) and kernel dispatch.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include <type_traits>

#include "attn_fwd.h"
#include "attn_fwd_asm.h"
#include "attn_fwd_simple.h"
#include "attn_launch.h"
#ifdef ATTN_DEBUG_ENTRY_POINTS
#include "attn_probe.h"
#endif
#include "attn_splitkv.h"

namespace {

using attn::Params;

constexpr int kW4MaxKeys = 4096;  // D = 64, causal: up to this many keys the 4-wave workgroups win (measured)

using attn::allow_lds;

// persistent: as many workgroups as the chip holds at once, each walking the tile queue of its XCD
// (attn_fwd_asm_kernel); otherwise one workgroup per tile
template <typename K>
int launch(K kern, Params p, int BH, int BM, int threads, int lds_bytes, hipStream_t stream, bool persistent = false)
{
    p.n_qt = (p.S_q + BM - 1) / BM;
    const long long total = (long long)BH * p.n_qt;
    if (total > 0x7fffffffLL)
        return ATTN_ERR_SHAPE;
    p.total_wg = (int)total;
    if (!allow_lds(reinterpret_cast<const void *>(kern), lds_bytes))
        return ATTN_ERR_LAUNCH;
    int grid = p.total_wg;
    if (persistent) {
        // (a runtime that cannot tell the occupancy gets one workgroup per tile: the kernel takes either)
        const int slots = attn::persistent_slots(reinterpret_cast<const void *>(kern), threads, lds_bytes, attn::kNumXcd);
        if (slots >= attn::kNumXcd && slots < grid)
            grid = slots;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(threads), lds_bytes, stream, p);
    return hipGetLastError() == hipSuccess ? ATTN_OK : ATTN_ERR_LAUNCH;
}

template <int D, int BN, int NW>
int launch_simple(const Params &p, int BH, int causal, hipStream_t stream)
{
    constexpr int LDS = 4 * BN * D * 2;
    if (causal)
        return launch(attn::attn_fwd_simple_kernel<D, BN, NW, true>, p, BH, NW * 32, NW * 64, LDS, stream);
    return launch(attn::attn_fwd_simple_kernel<D, BN, NW, false>, p, BH, NW * 32, NW * 64, LDS, stream);
}

// one hand-scheduled tiling: QB 32-row query blocks per wave, SB 32-key blocks per K/V tile, NW waves; persistent
// workgroups where the tiling has them
template <int D, int QB, int SB, int NW, bool F16 = false>
int launch_asm(const Params &p, int BH, int causal, hipStream_t stream)
{
    typedef attn::FwdTiling<D, QB, SB, NW, false> T;
    if (causal)
        return launch(attn::attn_fwd_asm_kernel<D, QB, SB, NW, true, F16>, p, BH, T::BM, NW * 64, T::LDS_BYTES, stream,
                      T::PERSIST);
    return launch(attn::attn_fwd_asm_kernel<D, QB, SB, NW, false, F16>, p, BH, T::BM, NW * 64, T::LDS_BYTES, stream,
                  T::PERSIST);
}

// D = 64.  tiling: -1 = choose, 0 = 8 waves x 32 rows (two waves per SIMD), 1 = 4 waves x 32 rows (two workgroups
// per CU).
// Measured: two 4-wave workgroups per CU instead of one 8-wave one change little when every workgroup
// streams the same number of tiles (-3 % at long S, +-2 % at short S); with a causal mask and few tiles
// the finer query tiles balance better (+13 % at S = 1024, +4 % at S = 4096).
template <bool F16>
int launch_d64(const Params &p, int BH, int causal, hipStream_t stream, int tiling = -1)
{
    if (tiling < 0)
        tiling = (!F16 && causal && p.S_kv <= kW4MaxKeys) ? 1 : 0;
    if (tiling == 1 && !F16)
        return launch_asm<64, 1, 2, 4>(p, BH, causal, stream);
    return launch_asm<64, 1, 2, 8, F16>(p, BH, causal, stream);
}

// D = 128.  wide: -1 = choose, 0 = 8 waves x 32 rows (two waves per SIMD), 1 = 4 waves x 64 rows (one wave
// per SIMD, half the LDS operand reads per MFMA).
template <bool F16>
int launch_d128(const Params &p, int BH, int causal, hipStream_t stream, int wide = -1)
{
    const bool use_wide = wide >= 0 ? wide != 0 : true;
    return use_wide ? launch_asm<128, 2, 1, 4, F16>(p, BH, causal, stream)
                    : launch_asm<128, 1, 2, 8, F16>(p, BH, causal, stream);
}

// the generic kernel: any scale, heads of any size, program order
int launch_generic(const Params &p, int BH, int D, int causal, hipStream_t st)
{
    switch (D) {
    case 64:
        return launch_simple<64, 64, 8>(p, BH, causal, st);
    case 128:
        return launch_simple<128, 64, 8>(p, BH, causal, st);
    default:
        return launch_simple<256, 32, 4>(p, BH, causal, st);
    }
}

// bf16 dispatch.  The hand-scheduled loops set masked scores to -inf before the multiply by
// scale*log2e (they need scale > 0) and address K/V of one head with 32-bit byte offsets.
int dispatch_fwd(const Params &p, int BH, int D, int causal, hipStream_t st)
{
    const bool asm_ok = p.scale > 0.f && (long long)p.S_kv * D * 2 < (1LL << 31);
    if (!asm_ok)
        return launch_generic(p, BH, D, causal, st);
    switch (D) {
    case 64:
        return launch_d64<false>(p, BH, causal, st);
    case 128:
        return launch_d128<false>(p, BH, causal, st);
    default:
        return launch_asm<256, 1, 1, 4>(p, BH, causal, st);
    }
}

}  // namespace

// host-side validation shared by the entry points; fills `p` on success
static int validate(const void *q, const void *k, const void *v, void *o, float *lse, int B, int H, int S_q, int S_kv,
                    int D, float scale, Params &p)
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
    p.q = static_cast<const attn::bf16_t *>(q);
    p.k = static_cast<const attn::bf16_t *>(k);
    p.v = static_cast<const attn::bf16_t *>(v);
    p.o = static_cast<attn::bf16_t *>(o);
    p.lse = lse;
    p.S_q = S_q;
    p.S_kv = S_kv;
    p.n_qt = 0;
    p.total_wg = 0;
    p.c = scale * 1.44269504088896340736f;
    p.scale = scale;
    p.n_split = 1;
#ifdef ATTN_DEBUG_ENTRY_POINTS
    p.trace = nullptr;
    p.trace_entries = 0;
#endif
    p.split_len = 0;
    p.o_part = nullptr;
    p.lse_part = nullptr;
    return ATTN_OK;
}

// key range of one split: a multiple of the 64-key tile; returns the number of non-empty ranges
static int split_plan(int S_kv, int n_split, int &split_len)
{
    const int per = (S_kv + n_split - 1) / n_split;
    split_len = (per + 63) / 64 * 64;
    return (S_kv + split_len - 1) / split_len;
}

extern "C" long long attn_fwd_splitkv_workspace_bytes(int B, int H, int S_q, int D, int n_split)
{
    if (B < 1 || H < 1 || S_q < 1 || n_split < 1 || n_split > 256 || (D != 64 && D != 128))
        return -1;
    return (long long)n_split * B * H * S_q * (D + 1) * 4;
}

template <int D, bool F16>
static int launch_splitkv(Params &p, int BH, int n_eff, void *o, float *lse, hipStream_t st)
{
    typedef typename std::conditional<F16, _Float16, attn::bf16_t>::type out_t;
    const long long n_rows = (long long)BH * p.S_q;
    constexpr int BM = 256;
    p.n_qt = (p.S_q + BM - 1) / BM;
    const long long total = (long long)BH * p.n_qt * n_eff;
    if (total > 0x7fffffffLL)
        return ATTN_ERR_SHAPE;
    p.total_wg = (int)total;
    const int lds = attn::FwdTiling<D, 1, 2, 8, true>::LDS_BYTES;
    auto kern = attn::attn_fwd_asm_kernel<D, 1, 2, 8, false, F16, true>;   // one workgroup per (tile, key range)
    if (!allow_lds(reinterpret_cast<const void *>(kern), lds))
        return ATTN_ERR_LAUNCH;
    hipLaunchKernelGGL(kern, dim3((unsigned)p.total_wg), dim3(512), lds, st, p);
    if (hipGetLastError() != hipSuccess)
        return ATTN_ERR_LAUNCH;
    const int rpb = 256 / (D / 4);
    const long long blocks = (n_rows + rpb - 1) / rpb;
    const unsigned grid = (unsigned)(blocks < 8192 ? blocks : 8192);
    hipLaunchKernelGGL((attn::attn_splitkv_merge_kernel<D, out_t>), dim3(grid), dim3(256), 0, st, p.o_part, p.lse_part,
                       static_cast<out_t *>(o), lse, n_rows, n_eff);
    return hipGetLastError() == hipSuccess ? ATTN_OK : ATTN_ERR_LAUNCH;
}

template <bool F16>
static int splitkv_entry(const void *q, const void *k, const void *v, void *o, float *lse, void *workspace,
                         long long workspace_bytes, int n_split, int B, int H, int S_q, int S_kv, int D, int causal,
                         float scale, void *stream)
{
    Params p;
    const int rc = validate(q, k, v, o, lse, B, H, S_q, S_kv, D, scale, p);
    if (rc != ATTN_OK)
        return rc;
    if (D == 256)
        return ATTN_ERR_UNSUPPORTED_D;
    if (causal)
        return ATTN_ERR_UNSUPPORTED;
    if (!(scale > 0.f))
        return ATTN_ERR_SCALE;
    if (n_split < 1 || n_split > 256 || (long long)S_kv * D * 2 >= (1LL << 31))
        return ATTN_ERR_SHAPE;
    if (!workspace)
        return ATTN_ERR_NULL;
    if ((uintptr_t)workspace & 15)
        return ATTN_ERR_ALIGN;
    if (workspace_bytes < attn_fwd_splitkv_workspace_bytes(B, H, S_q, D, n_split))
        return ATTN_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int n_eff = split_plan(S_kv, n_split, p.split_len);
    if (n_eff == 1) {  // one range: the plain kernel writes o and lse itself
        if (F16)
            return D == 64 ? launch_d64<true>(p, B * H, 0, st) : launch_d128<true>(p, B * H, 0, st);
        return D == 64 ? launch_d64<false>(p, B * H, 0, st) : launch_d128<false>(p, B * H, 0, st);
    }
    const long long n_rows = (long long)B * H * S_q;
    p.n_split = n_eff;
    p.o_part = static_cast<float *>(workspace);
    p.lse_part = p.o_part + (long long)n_eff * n_rows * D;
    return D == 64 ? launch_splitkv<64, F16>(p, B * H, n_eff, o, lse, st)
                   : launch_splitkv<128, F16>(p, B * H, n_eff, o, lse, st);
}

extern "C" int attn_fwd_splitkv(const void *q, const void *k, const void *v, void *o, float *lse, void *workspace,
                                long long workspace_bytes, int n_split, int B, int H, int S_q, int S_kv, int D,
                                int causal, float scale, void *stream)
{
    return splitkv_entry<false>(q, k, v, o, lse, workspace, workspace_bytes, n_split, B, H, S_q, S_kv, D, causal,
                                scale, stream);
}

extern "C" int attn_fwd_splitkv_f16(const void *q, const void *k, const void *v, void *o, float *lse, void *workspace,
                                    long long workspace_bytes, int n_split, int B, int H, int S_q, int S_kv, int D,
                                    int causal, float scale, void *stream)
{
    return splitkv_entry<true>(q, k, v, o, lse, workspace, workspace_bytes, n_split, B, H, S_q, S_kv, D, causal,
                               scale, stream);
}

extern "C" int attn_fwd_f16(const void *q, const void *k, const void *v, void *o, float *lse, int B, int H, int S_q,
                            int S_kv, int D, int causal, float scale, void *stream)
{
    Params p;
    const int rc = validate(q, k, v, o, lse, B, H, S_q, S_kv, D, scale, p);
    if (rc != ATTN_OK)
        return rc;
    // fp16 runs on the hand-scheduled kernels only
    if ((long long)S_kv * D * 2 >= (1LL << 31))
        return ATTN_ERR_SHAPE;
    if (!(scale > 0.f))
        return ATTN_ERR_SCALE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (D == 256)
        return launch_asm<256, 1, 1, 4, true>(p, B * H, causal, st);
    return D == 64 ? launch_d64<true>(p, B * H, causal, st) : launch_d128<true>(p, B * H, causal, st);
}

extern "C" int attn_fwd(const void *q, const void *k, const void *v, void *o, float *lse, int B, int H, int S_q,
                        int S_kv, int D, int causal, float scale, void *stream)
{
    Params p;
    const int rc = validate(q, k, v, o, lse, B, H, S_q, S_kv, D, scale, p);
    if (rc != ATTN_OK)
        return rc;
    return dispatch_fwd(p, B * H, D, causal, static_cast<hipStream_t>(stream));
}

#ifdef ATTN_DEBUG_ENTRY_POINTS
// Test-only entry point of the debug build of the library (libmi355attn_debug.so): attn_fwd with the
// kernel chosen by the caller.  variant 0: as attn_fwd; 1: the generic program-order kernel;
// 2 / 5: D = 128 on the one-wave-per-SIMD tiling (4 waves x 64 query rows) / on the two-waves-per-SIMD
// tiling (8 waves x 32 rows); 3 / 4: D = 64 with 8-wave / 4-wave workgroups.  A variant that does not
// apply to the arguments returns ATTN_ERR_UNSUPPORTED.
extern "C" int attn_fwd_variant(const void *q, const void *k, const void *v, void *o, float *lse, int B, int H,
                                int S_q, int S_kv, int D, int causal, float scale, void *stream, int variant)
{
    Params p;
    const int rc = validate(q, k, v, o, lse, B, H, S_q, S_kv, D, scale, p);
    if (rc != ATTN_OK)
        return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool asm_ok = p.scale > 0.f && (long long)p.S_kv * D * 2 < (1LL << 31);
    switch (variant) {
    case 0:
        return dispatch_fwd(p, B * H, D, causal, st);
    case 1:
        return launch_generic(p, B * H, D, causal, st);
    case 2:
        return D == 128 && asm_ok ? launch_d128<false>(p, B * H, causal, st, 1) : ATTN_ERR_UNSUPPORTED;
    case 5:
        return D == 128 && asm_ok ? launch_d128<false>(p, B * H, causal, st, 0) : ATTN_ERR_UNSUPPORTED;
    case 3:
    case 4:
        return D == 64 && asm_ok ? launch_d64<false>(p, B * H, causal, st, variant - 3) : ATTN_ERR_UNSUPPORTED;
    }
    return ATTN_ERR_UNSUPPORTED;
}
#endif

#ifdef ATTN_DEBUG_ENTRY_POINTS
// Measurement entry point of the debug build: attn_fwd (hand-scheduled kernels) that also records, per
// tile w of the launch's queue, trace[8 w + 0..5] = the 100 MHz constant clock when the tile is taken up, after
// K(0) and Q have landed, before the main loop, after it, after O is staged in LDS, and when O is stored;
// trace[8 w + 6] = the clock when the tile's first loads are all issued; trace[8 w + 7] = XCC_ID << 32 | HW_ID
// (CU, SE, ...) of a wave of the workgroup.  trace: device,
// trace_entries 64-bit values; workgroups whose record would not fit write nothing.
extern "C" int attn_fwd_trace(const void *q, const void *k, const void *v, void *o, float *lse, int B, int H, int S_q,
                              int S_kv, int D, int causal, float scale, void *stream, unsigned long long *trace,
                              long long trace_entries)
{
    Params p;
    const int rc = validate(q, k, v, o, lse, B, H, S_q, S_kv, D, scale, p);
    if (rc != ATTN_OK)
        return rc;
    if (!trace || trace_entries < 8)
        return ATTN_ERR_NULL;
    p.trace = trace;
    p.trace_entries = trace_entries;
    return dispatch_fwd(p, B * H, D, causal, static_cast<hipStream_t>(stream));
}

// Measurement entry point of the debug build: n_wg workgroups of waves_per_wg (4 or 8) waves, each wave
// `iters` x 8 MFMAs (32768 FLOP each) on the 8 fragments at `operands` (device, 8 * 64 * 16 bytes: 4 A then 4 B
// fragments, 16 bytes per lane); `out` (device, n_wg * waves_per_wg * 64 floats) receives one value per lane.
extern "C" int attn_probe_mfma(const void *operands, float *out, int n_wg, int waves_per_wg, int iters, void *stream)
{
    if (!operands || !out)
        return ATTN_ERR_NULL;
    if (n_wg < 1 || iters < 1 || (waves_per_wg != 4 && waves_per_wg != 8))
        return ATTN_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const attn::bf16x8 *ops = static_cast<const attn::bf16x8 *>(operands);
    if (waves_per_wg == 4)
        hipLaunchKernelGGL(attn::attn_probe_mfma_kernel<4>, dim3(n_wg), dim3(256), 0, st, ops, out, iters);
    else
        hipLaunchKernelGGL(attn::attn_probe_mfma_kernel<8>, dim3(n_wg), dim3(512), 0, st, ops, out, iters);
    return hipGetLastError() == hipSuccess ? ATTN_OK : ATTN_ERR_LAUNCH;
}
#endif

#ifdef ATTN_DEBUG_ENTRY_POINTS
// Measurement entry point of the debug build: attn_probe_mfma with four waves per workgroup and the operand
// pattern of attn_probe_mfma_pattern_kernel (0 .. 5; 5 reads `operands` as IEEE binary16).  Patterns 0-3 and 5
// issue iters x 8 MFMAs of 32768 FLOP per wave, pattern 4 iters x 16 of 16384 FLOP.
extern "C" int attn_probe_mfma_pattern(const void *operands, float *out, int n_wg, int pattern, int iters, void *stream)
{
    if (!operands || !out)
        return ATTN_ERR_NULL;
    if (n_wg < 1 || iters < 1 || pattern < 0 || pattern > 5)
        return ATTN_ERR_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const attn::bf16x8 *ops = static_cast<const attn::bf16x8 *>(operands);
    switch (pattern) {
    case 0: hipLaunchKernelGGL(attn::attn_probe_mfma_pattern_kernel<0>, dim3(n_wg), dim3(256), 0, st, ops, out, iters); break;
    case 1: hipLaunchKernelGGL(attn::attn_probe_mfma_pattern_kernel<1>, dim3(n_wg), dim3(256), 0, st, ops, out, iters); break;
    case 2: hipLaunchKernelGGL(attn::attn_probe_mfma_pattern_kernel<2>, dim3(n_wg), dim3(256), 0, st, ops, out, iters); break;
    case 3: hipLaunchKernelGGL(attn::attn_probe_mfma_pattern_kernel<3>, dim3(n_wg), dim3(256), 0, st, ops, out, iters); break;
    case 4: hipLaunchKernelGGL(attn::attn_probe_mfma_pattern_kernel<4>, dim3(n_wg), dim3(256), 0, st, ops, out, iters); break;
    default: hipLaunchKernelGGL(attn::attn_probe_mfma_pattern_kernel<5>, dim3(n_wg), dim3(256), 0, st, ops, out, iters); break;
    }
    return hipGetLastError() == hipSuccess ? ATTN_OK : ATTN_ERR_LAUNCH;
}
#endif

#ifdef ATTN_DEBUG_ENTRY_POINTS
// Measurement entry point of the debug build: the atomic traffic of a single-pass backward's dQ reduction for
// n_heads heads of S_q queries and S_kv keys (D = 128; S_q a multiple of 64, S_kv of 128) into dq (device,
// n_heads * S_q * 128 floats, zeroed by the caller).
extern "C" int attn_probe_dq_atomics(float *dq, int n_heads, int S_q, int S_kv, int causal, void *stream)
{
    if (!dq)
        return ATTN_ERR_NULL;
    if (n_heads < 1 || S_q < 64 || S_kv < 128 || S_q % 64 || S_kv % 128 || (long long)n_heads * (S_kv / 128) > 0x7fffffffLL)
        return ATTN_ERR_SHAPE;
    const int n_kt = S_kv / 128;
    hipLaunchKernelGGL(attn::attn_probe_dq_atomics_kernel, dim3(n_heads * n_kt), dim3(256), 0, static_cast<hipStream_t>(stream),
                       dq, S_q, n_kt, causal);
    return hipGetLastError() == hipSuccess ? ATTN_OK : ATTN_ERR_LAUNCH;
}
#endif

extern "C" int attn_workgroup_tile(int causal, int workgroup, int n_heads, int n_tiles, long long head_bytes, int *head,
                                   int *tile)
{
    if (!head || !tile)
        return ATTN_ERR_NULL;
    if (n_heads < 1 || n_tiles < 1 || head_bytes < 0 || (long long)n_heads * n_tiles > 0x7fffffffLL || workgroup < 0 ||
        workgroup >= n_heads * n_tiles)
        return ATTN_ERR_SHAPE;
    if (causal)
        attn::wg_to_tile_n<true>(workgroup, n_heads * n_tiles, n_tiles, head_bytes, *head, *tile);
    else
        attn::wg_to_tile_n<false>(workgroup, n_heads * n_tiles, n_tiles, head_bytes, *head, *tile);
    return ATTN_OK;
}

extern "C" int attn_workgroup_queue_entry(int workgroup, int n_workgroups, int n_entries, int pass, int *entry)
{
    if (!entry)
        return ATTN_ERR_NULL;
    if (n_workgroups < 1 || n_entries < 1 || pass < 0 || workgroup < 0 || workgroup >= n_workgroups ||
        (n_workgroups < n_entries && n_workgroups % attn::kNumXcd))
        return ATTN_ERR_SHAPE;
    *entry = attn::persistent_entry(workgroup, n_workgroups, n_entries, pass);
    return ATTN_OK;
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
    case ATTN_ERR_UNSUPPORTED:
        return "this entry point does not implement the requested combination (e.g. causal split-KV)";
    case ATTN_ERR_WORKSPACE:
        return "the workspace is too small: smaller than attn_fwd_splitkv_workspace_bytes() asks for, or the shape exceeds "
               "the built-in workspace of attn_bwd_noalloc (B*H*S_q <= 2^21)";
    }
    return "unknown attn_status";
}

extern "C" int attn_version(void) { return 600; }
