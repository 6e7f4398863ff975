/*
 * attn_bwd.h -- C ABI of libmi355attn.so: attention backward for MI355X (gfx950).
 *
 * The operation is the backward pass that the paper's Section 6.3 evaluates: given the
 * inputs q, k, v of attn_fwd (see attn_fwd.h), its outputs o and lse, and the gradient
 * d_o of a scalar loss with respect to o, compute the gradients with respect to q, k, v.
 * With J(i), s_ij as in attn_fwd.h and p_ij = exp(s_ij - lse_i):
 *
 *     Delta_i = sum_d d_o[i,d] * o[i,d]
 *     dp_ij   = sum_d d_o[i,d] * v[j,d]
 *     ds_ij   = p_ij * (dp_ij - Delta_i)
 *     dq[i,:] = scale * sum_{j in J(i)} ds_ij * k[j,:]
 *     dk[j,:] = scale * sum_{i : j in J(i)} ds_ij * q[i,:]
 *     dv[j,:] =         sum_{i : j in J(i)} p_ij  * d_o[i,:]
 *
 * (the single-pass form of that section has five matrix products per tile pair; here two of
 * the five are computed twice, once per sweep, so that no atomic reduction of dq is needed and
 * results are bitwise reproducible).  All contractions run on bf16 MFMA with fp32 accumulation; p and ds are
 * rounded to bf16 (nearest even) before the products that consume them.
 */
#ifndef MI355_ATTN_BWD_H
#define MI355_ATTN_BWD_H

#ifdef __cplusplus
extern "C" {
#endif

/*
 * attn_bwd -- enqueue one backward pass on `stream` and return (asynchronous).
 *
 *   q, o, d_o  device pointers, bf16, contiguous row-major [B][H][S_q][D]     (read only)
 *   k, v       device pointers, bf16, contiguous row-major [B][H][S_kv][D]    (read only)
 *   lse        device pointer, fp32, [B][H][S_q]: what attn_fwd wrote for (q, k, v)  (read only)
 *   dq         device pointer, bf16, [B][H][S_q][D]; every element is overwritten
 *   dk, dv     device pointers, bf16, [B][H][S_kv][D]; every element is overwritten
 *              (keys that no query sees get zeros)
 *   delta_ws   device pointer, fp32, 2 * B * H * S_q elements: workspace owned by the caller; the
 *              call overwrites it (first half: lse * log2(e), second half: Delta) and reads it
 *              back on the same stream
 *   B, H, S_q, S_kv   >= 1; S_q * D and S_kv * D below 2^30, B * H * S_q below 2^28
 *   D          64 or 128 (256 returns ATTN_ERR_UNSUPPORTED_D)
 *   causal, scale, stream   as in attn_fwd; they must be the values the forward call used
 *
 * Ownership: the caller owns all ten buffers and keeps them alive until the work
 * enqueued on `stream` has completed.  The library allocates nothing and keeps no state that changes a result.
 * Outputs and the workspace must not overlap the inputs or each other.
 *
 * Errors: as attn_fwd -- arguments are validated on the host before any HIP call, a
 * negative attn_status (attn_fwd.h) is returned and nothing is launched; a launch the
 * runtime rejects returns ATTN_ERR_LAUNCH (earlier kernels of the same call may then have
 * been enqueued; the outputs are unspecified).  Results are bitwise reproducible (no atomics).
 */
int attn_bwd(const void *q, const void *k, const void *v, const void *o, const void *d_o,
             const float *lse, void *dq, void *dk, void *dv, float *delta_ws,
             int B, int H, int S_q, int S_kv, int D, int causal, float scale,
             void *stream);

/*
 * attn_bwd_f16 -- the same operation on IEEE fp16 tensors (q, k, v, o, d_o, dq, dk, dv), the element
 * type of the paper's Section 6.3 backward figures; pairs with attn_fwd_f16.  Arguments, layout,
 * ownership and error behaviour are those of attn_bwd (D 64 or 128), except: scale must be > 0
 * (0 returns ATTN_ERR_SCALE).  p and ds are rounded to fp16 before the products that consume them.
 */
int attn_bwd_f16(const void *q, const void *k, const void *v, const void *o, const void *d_o,
                 const float *lse, void *dq, void *dk, void *dv, float *delta_ws,
                 int B, int H, int S_q, int S_kv, int D, int causal, float scale,
                 void *stream);

/*
 * attn_bwd_noalloc -- attn_bwd for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same operation, same kernels and
 * bitwise the same results as attn_bwd (bf16), without the delta_ws argument: the workspace is a
 * 16 MiB array inside the library, one copy per GPU the library runs on, held until the process
 * ends.  The call allocates nothing on the device.
 *
 *   limit      B * H * S_q <= 2^21 rows (2 fp32 words per row); more returns ATTN_ERR_WORKSPACE
 *              before anything is launched.  All other arguments, layouts, ownership rules and
 *              error codes are those of attn_bwd.
 *   set-up     the first call on a device resolves that device's copy of the array (one runtime
 *              query, no allocation); make that first call outside a graph capture, with the
 *              device of `stream` current.  Every call must be made with the device of `stream`
 *              current.
 *   sharing    every call on a GPU uses that GPU's one array.  A call overwrites the part it uses
 *              before reading it, so nothing has to be cleared and calls may follow each other on
 *              one stream in any mix of sizes; calls that overlap in time on the same GPU (two
 *              streams, or two graphs replayed concurrently) race on it and give undefined results.
 */
int attn_bwd_noalloc(const void *q, const void *k, const void *v, const void *o, const void *d_o,
                     const float *lse, void *dq, void *dk, void *dv,
                     int B, int H, int S_q, int S_kv, int D, int causal, float scale,
                     void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MI355_ATTN_BWD_H */
