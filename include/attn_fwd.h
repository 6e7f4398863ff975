/*
 * attn_fwd.h -- C ABI of libmi355attn.so: Flash-Attention forward for MI355X (gfx950).
 *
 * The operation is the per-SM loop of the paper's Section 3 running example
 * (Fig. 1a; its software-pipelined form is Fig. 1f):
 *     O = 0;  for each K/V tile i:  S = gemm(Q, K[i]);  P = exp(S);  O += gemm(P, V[i])
 * in its complete online-softmax form, i.e. with the max subtraction, the
 * accumulator rescale and the final normalisation that the figure leaves out
 * and Section 6.2 counts among the loop's work, plus the log-sum-exp of every
 * row.  For b in [0,B), h in [0,H), i in [0,S_q):
 *
 *     J(i)   = { j : 0 <= j < S_kv }                  causal == 0
 *            = { j : 0 <= j < S_kv, j <= i }          causal != 0 (top-left aligned)
 *     s_ij   = scale * sum_d q[b,h,i,d] * k[b,h,j,d]
 *     lse[b,h,i] = ln sum_{j in J(i)} exp(s_ij)
 *     o[b,h,i,:] = sum_{j in J(i)} exp(s_ij - lse[b,h,i]) * v[b,h,j,:]
 *
 * Both contractions run on bf16 MFMA with fp32 accumulation; P is rounded to
 * bf16 (round to nearest even) before the second contraction; the row sum is
 * taken over the unrounded fp32 P.
 *
 * No C++ types, no exceptions and no torch types cross this boundary.
 */
#ifndef MI355_ATTN_FWD_H
#define MI355_ATTN_FWD_H

#ifdef __cplusplus
extern "C" {
#endif

typedef enum attn_status {
    ATTN_OK = 0,
    ATTN_ERR_NULL = -1,          /* a required pointer is NULL */
    ATTN_ERR_SHAPE = -2,         /* B, H, S_q or S_kv < 1, or a tensor exceeds 2^31-1 rows / 2^40 elements */
    ATTN_ERR_UNSUPPORTED_D = -3, /* D not in {64, 128, 256} */
    ATTN_ERR_ALIGN = -4,         /* q, k, v or o not 16-byte aligned, or lse not 4-byte aligned */
    ATTN_ERR_SCALE = -5,         /* scale is NaN, infinite or negative */
    ATTN_ERR_LAUNCH = -6,        /* the HIP runtime refused the launch (see hipGetLastError) */
    ATTN_ERR_UNSUPPORTED = -7,   /* the entry point does not implement this combination of arguments */
    ATTN_ERR_WORKSPACE = -8      /* the workspace is too small */
} attn_status;

/*
 * attn_fwd -- enqueue one forward pass on `stream` and return (asynchronous).
 *
 *   q      device pointer, bf16, contiguous row-major [B][H][S_q][D]      (read only)
 *   k, v   device pointers, bf16, contiguous row-major [B][H][S_kv][D]    (read only)
 *   o      device pointer, bf16, [B][H][S_q][D]; every element is overwritten
 *   lse    device pointer, fp32, [B][H][S_q]; natural-log log-sum-exp of the
 *          scaled scores of each row; every element is overwritten
 *   B, H, S_q, S_kv   >= 1, any value (ragged tiles are masked inside the kernel)
 *   D      64, 128 or 256
 *   causal 0: every key is visible; non-zero: key j is visible to query i iff j <= i
 *   scale  multiplies QK^T before the softmax; finite and >= 0 (callers pass 1/sqrt(D))
 *   stream a hipStream_t passed as void* (NULL = the default stream)
 *
 * Ownership: the caller owns all five buffers and keeps them alive until the
 * work enqueued on `stream` has completed.  The library allocates nothing,
 * keeps no state between calls that changes a result (it remembers only, per
 * kernel and device, that a launch attribute has been set and how many workgroups
 * the chip holds at once) and never synchronises the device.  o/lse must
 * not overlap q/k/v.
 *
 * Errors: arguments are validated on the host before any HIP call; on a
 * validation error a negative attn_status is returned and nothing is
 * launched.  A launch the runtime rejects returns ATTN_ERR_LAUNCH.  The
 * function never aborts or throws.  NaN/Inf inside q, k, v are not checked
 * (the outputs are then unspecified).  Results are bitwise reproducible from
 * run to run (no atomics; workgroups take tiles in a fixed order).
 */
int attn_fwd(const void *q, const void *k, const void *v, void *o, float *lse,
             int B, int H, int S_q, int S_kv, int D, int causal, float scale,
             void *stream);

/*
 * attn_fwd_f16 -- the same operation on IEEE fp16 tensors, the element type of the
 * paper's Section 6 forward-attention evaluation (FP16, HEAD_DIM = 128).
 *
 * Arguments, layout, ownership and error behaviour are those of attn_fwd, except:
 *   q, k, v, o   hold IEEE binary16 instead of bf16; both contractions run on fp16
 *                MFMA with fp32 accumulation and P is rounded to fp16 (nearest even)
 *   scale        finite and > 0 (0 returns ATTN_ERR_SCALE)
 *   S_kv * D     below 2^30 (one head of K addressed with 32-bit byte offsets;
 *                larger returns ATTN_ERR_SHAPE)
 * Inputs whose scores or values overflow fp16 range are the caller's concern, as
 * NaN/Inf are for attn_fwd.
 */
int attn_fwd_f16(const void *q, const void *k, const void *v, void *o, float *lse,
                 int B, int H, int S_q, int S_kv, int D, int causal, float scale,
                 void *stream);

/*
 * attn_fwd_splitkv -- attn_fwd with the keys cut into n_split ranges that run as separate
 * workgroups, for shapes whose B * H * ceil(S_q / 256) query tiles cannot fill the 256 compute
 * units (long S_kv, few heads or queries).  Each range runs the loop of Fig. 1a on its keys and
 * leaves a normalised partial output and its log-sum-exp in the workspace; a second kernel merges
 * them:  lse = ln sum_s exp(lse_s),  o = sum_s exp(lse_s - lse) o_s  -- the accumulator
 * rescaling of Section 6.2 applied once more, across workgroups.
 *
 * Arguments, layout, ownership and error behaviour are those of attn_fwd, plus:
 *   workspace        device pointer, 16-byte aligned, owned by the caller, overwritten; must stay
 *                    valid until the work on `stream` has completed
 *   workspace_bytes  its size; at least attn_fwd_splitkv_workspace_bytes(B, H, S_q, D, n_split),
 *                    else ATTN_ERR_WORKSPACE
 *   n_split          1 .. 256 requested key ranges; ranges are rounded up to whole 64-key tiles,
 *                    so fewer may be used (one range = a plain attn_fwd launch)
 *   D                64 or 128 (256 returns ATTN_ERR_UNSUPPORTED_D)
 *   causal           must be 0 (ATTN_ERR_UNSUPPORTED otherwise)
 *   scale            finite and > 0
 * Results are bitwise reproducible for a given n_split; they differ from attn_fwd's in the last
 * bits (another summation order).
 */
int attn_fwd_splitkv(const void *q, const void *k, const void *v, void *o, float *lse,
                     void *workspace, long long workspace_bytes, int n_split,
                     int B, int H, int S_q, int S_kv, int D, int causal, float scale,
                     void *stream);

/* attn_fwd_splitkv on IEEE fp16 tensors (q, k, v, o); everything else as attn_fwd_splitkv; pairs with attn_fwd_f16. */
int attn_fwd_splitkv_f16(const void *q, const void *k, const void *v, void *o, float *lse,
                         void *workspace, long long workspace_bytes, int n_split,
                         int B, int H, int S_q, int S_kv, int D, int causal, float scale,
                         void *stream);

/* Bytes of workspace attn_fwd_splitkv (either element type) needs: n_split * B * H * S_q * (D + 1) * 4; -1 on invalid arguments. */
long long attn_fwd_splitkv_workspace_bytes(int B, int H, int S_q, int D, int n_split);

/*
 * Diagnostic, host only (no GPU call): which (head, tile) the workgroup with id `workgroup` of a launch of
 * n_heads * n_tiles workgroups works on -- the work decomposition of the kernels (XCD-aware; causal:
 * heaviest tiles first, in groups of heads that share an L2).  `head_bytes`: bytes of operands the
 * workgroups of one head stream (forward: K and V, 4 * S_kv * D; backward: 4 * (S_q + S_kv) * D); it sizes
 * the causal groups and is ignored otherwise.  `*head` = b*H + h, `*tile` = index of the tile of owner rows
 * (query tiles in the forward pass; the key-owner backward sweep counts its tiles from the other end).
 * Returns ATTN_OK, or ATTN_ERR_NULL / ATTN_ERR_SHAPE (n_heads, n_tiles < 1, head_bytes < 0, product above
 * 2^31 - 1, workgroup outside [0, n_heads * n_tiles)).
 */
int attn_workgroup_tile(int causal, int workgroup, int n_heads, int n_tiles, long long head_bytes,
                        int *head, int *tile);

/*
 * Diagnostic, host only (no GPU call): the forward kernels' workgroups are persistent -- a launch has at most
 * one workgroup per CU slot and each walks a queue of tiles.  `*entry` = the id (the `workgroup` argument of
 * attn_workgroup_tile) that workgroup `workgroup` of a launch of n_workgroups takes up in pass `pass` (0, 1, ...)
 * when n_entries tiles are queued, or -1 when that pass has none for it.  An XCD's workgroups share the XCD's
 * entries (id % 8); odd passes run through them in reverse, so that a slot pairs heavy with light tiles of a
 * causal launch.  n_workgroups >= n_entries: one entry each, in pass 0.
 * Returns ATTN_OK, or ATTN_ERR_NULL / ATTN_ERR_SHAPE (counts < 1, pass < 0, workgroup outside
 * [0, n_workgroups), n_workgroups < n_entries and not a multiple of 8).
 */
int attn_workgroup_queue_entry(int workgroup, int n_workgroups, int n_entries, int pass, int *entry);

/* Static, NUL-terminated description of an attn_status value; never freed. */
const char *attn_strerror(int status);

/* Library version: major * 10000 + minor * 100 + patch. */
int attn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MI355_ATTN_FWD_H */
