// attn_bwd.hip -- C ABI entry point attn_bwd (see include/attn_bwd.h): validation and launches.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include <mutex>

#include "attn_bwd.h"  // the C declaration (include/)
#include "attn_bwd_asm.h"
#include "attn_bwd_kernels.h"
#include "attn_fwd.h"  // attn_status
#include "attn_launch.h"

// Workspace of attn_bwd_noalloc: one copy per GPU that the library runs on, held until the process ends.
// In host code this name is only a handle for hipGetSymbolAddress; the device address it yields (one per
// device) is what is passed to kernels.
#define ATTN_BWD_NOALLOC_MAX_ROWS (1 << 21)
static __device__ __align__(256) float scratch[2 * ATTN_BWD_NOALLOC_MAX_ROWS];

namespace {

using attn::BwdParams;

// persistent: as many workgroups as the chip holds at once, each walking the queue of owner tiles of its XCD
// (the hand-scheduled sweeps); otherwise one workgroup per owner tile
template <typename K>
int launch_sweep(K kern, BwdParams p, int BH, int S_own, int NW, int lds_bytes, hipStream_t stream, bool persistent = false)
{
    p.n_t = (S_own + NW * 32 - 1) / (NW * 32);
    const long long total = (long long)BH * p.n_t;
    if (total > 0x7fffffffLL)
        return ATTN_ERR_SHAPE;
    p.total_wg = (int)total;
    if (!attn::allow_lds(reinterpret_cast<const void *>(kern), lds_bytes))
        return ATTN_ERR_LAUNCH;
    int grid = p.total_wg;
    if (persistent) {
        // (a runtime that cannot tell the occupancy gets one workgroup per owner tile: the kernel takes either)
        const int slots = attn::persistent_slots(reinterpret_cast<const void *>(kern), NW * 64, lds_bytes, attn::kNumXcd);
        if (slots >= attn::kNumXcd && slots < grid)
            grid = slots;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(NW * 64), lds_bytes, stream, p);
    return hipGetLastError() == hipSuccess ? ATTN_OK : ATTN_ERR_LAUNCH;
}

// plain: run the compiler-scheduled sweeps (always when scale == 0, which the hand-scheduled loops exclude)
template <int D>
int launch_bwd(const BwdParams &p, int BH, int causal, hipStream_t stream, bool plain)
{
    constexpr int NWK = 4, NWQ = 8;  // waves per workgroup of the key-owner / query-owner sweep
    constexpr int LDSK = 2 * 3 * 64 * D * 2 + 3 * NWK * 256, LDSQ = 2 * 3 * 64 * D * 2 + 3 * NWQ * 256;
    {
        const long long blocks = (p.n_rows + (256 / (D / 8)) - 1) / (256 / (D / 8));
        const unsigned grid = (unsigned)(blocks < 4096 ? blocks : 4096);
        hipLaunchKernelGGL(attn::attn_bwd_delta_kernel<D>, dim3(grid), dim3(256), 0, stream, p);
        if (hipGetLastError() != hipSuccess)
            return ATTN_ERR_LAUNCH;
    }
    // hand-scheduled sweeps (they need scale > 0), else the compiler-scheduled ones: key owners first
    const bool hand = !plain && p.scale > 0.f;
    constexpr int LDSA = 2 * 6 * 32 * D * 2 + 6 * 256;
    int rc;
    if (hand)
        rc = causal ? launch_sweep(attn::attn_bwd_asm_kernel<D, true, true>, p, BH, p.S_kv, 4, LDSA, stream, true)
                    : launch_sweep(attn::attn_bwd_asm_kernel<D, false, true>, p, BH, p.S_kv, 4, LDSA, stream, true);
    else
        rc = causal ? launch_sweep(attn::attn_bwd_sweep_kernel<D, true, true, NWK>, p, BH, p.S_kv, NWK, LDSK, stream)
                    : launch_sweep(attn::attn_bwd_sweep_kernel<D, false, true, NWK>, p, BH, p.S_kv, NWK, LDSK, stream);
    if (rc != ATTN_OK)
        return rc;
    if (hand)
        return causal ? launch_sweep(attn::attn_bwd_asm_kernel<D, true, false>, p, BH, p.S_q, 4, LDSA, stream, true)
                      : launch_sweep(attn::attn_bwd_asm_kernel<D, false, false>, p, BH, p.S_q, 4, LDSA, stream, true);
    return causal ? launch_sweep(attn::attn_bwd_sweep_kernel<D, true, false, NWQ>, p, BH, p.S_q, NWQ, LDSQ, stream)
                  : launch_sweep(attn::attn_bwd_sweep_kernel<D, false, false, NWQ>, p, BH, p.S_q, NWQ, LDSQ, stream);
}

}  // namespace

// host-side validation shared by the entry points; fills `p` on success
static int validate_bwd(const void *q, const void *k, const void *v, const void *o, const void *d_o, const float *lse,
                        void *dq, void *dk, void *dv, float *delta_ws, int B, int H, int S_q, int S_kv, int D,
                        float scale, BwdParams &p)
{
    if (!q || !k || !v || !o || !d_o || !lse || !dq || !dk || !dv || !delta_ws)
        return ATTN_ERR_NULL;
    if (B < 1 || H < 1 || S_q < 1 || S_kv < 1)
        return ATTN_ERR_SHAPE;
    if (D != 64 && D != 128)
        return ATTN_ERR_UNSUPPORTED_D;
    const long long BH = (long long)B * H;
    if (BH > 0x7fffffffLL || BH * (long long)(S_q > S_kv ? S_q : S_kv) > (1LL << 40) / D)
        return ATTN_ERR_SHAPE;
    // one head of any tensor, and the workspace, are addressed with 32-bit byte offsets
    if ((long long)(S_q > S_kv ? S_q : S_kv) * D * 2 >= (1LL << 31) || BH * S_q * 8 >= (1LL << 31))
        return ATTN_ERR_SHAPE;
    if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)o | (uintptr_t)d_o | (uintptr_t)dq | (uintptr_t)dk |
         (uintptr_t)dv) & 15)
        return ATTN_ERR_ALIGN;
    if (((uintptr_t)lse | (uintptr_t)delta_ws) & 3)
        return ATTN_ERR_ALIGN;
    if (!(scale >= 0.f) || isinf(scale))
        return ATTN_ERR_SCALE;
    p.q = static_cast<const attn::bf16_t *>(q);
    p.k = static_cast<const attn::bf16_t *>(k);
    p.v = static_cast<const attn::bf16_t *>(v);
    p.o = static_cast<const attn::bf16_t *>(o);
    p.d_o = static_cast<const attn::bf16_t *>(d_o);
    p.lse = lse;
    p.lse2 = delta_ws;
    p.delta = delta_ws + BH * S_q;
    p.dq = static_cast<attn::bf16_t *>(dq);
    p.dk = static_cast<attn::bf16_t *>(dk);
    p.dv = static_cast<attn::bf16_t *>(dv);
    p.S_q = S_q;
    p.S_kv = S_kv;
    p.n_t = 0;
    p.total_wg = 0;
    p.n_rows = BH * S_q;
    p.c = scale * 1.44269504088896340736f;
    p.scale = scale;
    return ATTN_OK;
}

extern "C" int attn_bwd(const void *q, const void *k, const void *v, const void *o, const void *d_o, const float *lse,
                        void *dq, void *dk, void *dv, float *delta_ws, int B, int H, int S_q, int S_kv, int D,
                        int causal, float scale, void *stream)
{
    BwdParams p;
    const int rc = validate_bwd(q, k, v, o, d_o, lse, dq, dk, dv, delta_ws, B, H, S_q, S_kv, D, scale, p);
    if (rc != ATTN_OK)
        return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    return D == 64 ? launch_bwd<64>(p, B * H, causal, st, false) : launch_bwd<128>(p, B * H, causal, st, false);
}

// device address of `scratch` on the current device; resolved on the first call on that device
static float *scratch_on_current_device()
{
    constexpr int kMaxDev = 64;
    static std::mutex mu;
    static float *ptr[kMaxDev] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDev) {
        (void)hipGetLastError();
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void *addr = nullptr;
        if (hipGetSymbolAddress(&addr, HIP_SYMBOL(scratch)) != hipSuccess || !addr) {
            (void)hipGetLastError();
            return nullptr;
        }
        ptr[dev] = static_cast<float *>(addr);
    }
    return ptr[dev];
}

extern "C" int attn_bwd_noalloc(const void *q, const void *k, const void *v, const void *o, const void *d_o,
                                const float *lse, void *dq, void *dk, void *dv, int B, int H, int S_q, int S_kv,
                                int D, int causal, float scale, void *stream)
{
    // size check on the host first: the rows must fit the library's own workspace
    if (B >= 1 && H >= 1 && S_q >= 1 && (long long)B * H * S_q > ATTN_BWD_NOALLOC_MAX_ROWS)
        return ATTN_ERR_WORKSPACE;
    BwdParams p;
    float dummy_ws = 0.f;  // validate_bwd only looks at the address
    const int rc = validate_bwd(q, k, v, o, d_o, lse, dq, dk, dv, &dummy_ws, B, H, S_q, S_kv, D, scale, p);
    if (rc != ATTN_OK)
        return rc;
    float *ws = scratch_on_current_device();
    if (!ws)
        return ATTN_ERR_LAUNCH;
    // every word of the workspace that the sweeps read is written by the Delta kernel of this call:
    // nothing has to start at zero
    p.lse2 = ws;
    p.delta = ws + (long long)B * H * S_q;
    hipStream_t st = static_cast<hipStream_t>(stream);
    return D == 64 ? launch_bwd<64>(p, B * H, causal, st, false) : launch_bwd<128>(p, B * H, causal, st, false);
}

#ifdef ATTN_DEBUG_ENTRY_POINTS
// Test-only entry point of the debug build of the library: attn_bwd on the compiler-scheduled sweeps
// (the reference of the schedule-equivalence test).
extern "C" int attn_bwd_plain(const void *q, const void *k, const void *v, const void *o, const void *d_o,
                              const float *lse, void *dq, void *dk, void *dv, float *delta_ws, int B, int H, int S_q,
                              int S_kv, int D, int causal, float scale, void *stream)
{
    BwdParams p;
    const int rc = validate_bwd(q, k, v, o, d_o, lse, dq, dk, dv, delta_ws, B, H, S_q, S_kv, D, scale, p);
    if (rc != ATTN_OK)
        return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    return D == 64 ? launch_bwd<64>(p, B * H, causal, st, true) : launch_bwd<128>(p, B * H, causal, st, true);
}
#endif

template <int D>
static int launch_bwd_f16(const BwdParams &p, int BH, int causal, hipStream_t st)
{
    {
        const long long blocks = (p.n_rows + 15) / 16;
        const unsigned grid = (unsigned)(blocks < 4096 ? blocks : 4096);
        hipLaunchKernelGGL((attn::attn_bwd_delta_kernel<D, _Float16>), dim3(grid), dim3(256), 0, st, p);
        if (hipGetLastError() != hipSuccess)
            return ATTN_ERR_LAUNCH;
    }
    constexpr int LDSA = 2 * 6 * 32 * D * 2 + 6 * 256;
    const int rk = causal ? launch_sweep(attn::attn_bwd_asm_kernel<D, true, true, true>, p, BH, p.S_kv, 4, LDSA, st, true)
                          : launch_sweep(attn::attn_bwd_asm_kernel<D, false, true, true>, p, BH, p.S_kv, 4, LDSA, st, true);
    if (rk != ATTN_OK)
        return rk;
    return causal ? launch_sweep(attn::attn_bwd_asm_kernel<D, true, false, true>, p, BH, p.S_q, 4, LDSA, st, true)
                  : launch_sweep(attn::attn_bwd_asm_kernel<D, false, false, true>, p, BH, p.S_q, 4, LDSA, st, true);
}

extern "C" int attn_bwd_f16(const void *q, const void *k, const void *v, const void *o, const void *d_o,
                            const float *lse, void *dq, void *dk, void *dv, float *delta_ws, int B, int H, int S_q,
                            int S_kv, int D, int causal, float scale, void *stream)
{
    BwdParams p;
    const int rc = validate_bwd(q, k, v, o, d_o, lse, dq, dk, dv, delta_ws, B, H, S_q, S_kv, D, scale, p);
    if (rc != ATTN_OK)
        return rc;
    // fp16 runs on the hand-scheduled sweeps only
    if (!(scale > 0.f))
        return ATTN_ERR_SCALE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    return D == 64 ? launch_bwd_f16<64>(p, B * H, causal, st) : launch_bwd_f16<128>(p, B * H, causal, st);
}
