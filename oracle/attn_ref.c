/*
 * attn_ref.c -- fp64 CPU oracle for scaled-dot-product attention (forward).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU path is checked against.  It shares no code, header, table or helper
 * with the HIP library and must never be called from the product path: only
 * tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg use it.
 *
 * What it computes.  The paper's Section 3 running example (Fig. 1a) is a
 * simplified per-SM loop  O = 0; for i: S = gemm(Q, K[i]); P = exp(S);
 * O += gemm(P, V[i]).  The figure elides the softmax bookkeeping (max
 * subtraction, normalisation) that Section 6.2's discussion of "softmax
 * calculations" and "accumulator rescaling" refers to.  The tiled loop with a
 * running max is an exact algebraic re-association of ordinary softmax
 * attention, so the oracle is that plain definition written out, one row at a
 * time, with no tiles and no running rescale:
 *
 *   J(i)  = { j : 0 <= j < S_kv }                     if not causal
 *         = { j : 0 <= j < S_kv and j <= i }          if causal (top-left aligned)
 *   s_ij  = scale * sum_d q[b,h,i,d] * k[b,h,j,d]     j in J(i)
 *   m_i   = max_j s_ij
 *   l_i   = sum_j exp(s_ij - m_i)
 *   LSE_i = m_i + ln(l_i)                             (natural log)
 *   O_id  = (1/l_i) * sum_j exp(s_ij - m_i) * v[b,h,j,d]
 *
 * Everything is IEEE fp64.  Inputs are 16-bit patterns (uint16) widened
 * exactly: bf16 (attn_ref_f64), or IEEE binary16 (attn_ref_f64_f16), the
 * element type of the paper's Section 6 evaluation.  `scale` is the caller's
 * fp32 value widened exactly.  Outputs are fp64 and are not rounded.
 *
 * Layout: q [B][H][S_q][D], k and v [B][H][S_kv][D], contiguous, row-major.
 * Rows are addressed by a flat id  r = (b*H + h)*S_q + i.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double bf16_bits_to_f64(uint16_t bits)
{
    /* bf16 is the upper half of an IEEE binary32: widen by shifting. */
    uint32_t w = ((uint32_t)bits) << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

static double f16_bits_to_f64(uint16_t bits)
{
    /* IEEE 754 binary16: 1 sign bit, 5 exponent bits (bias 15), 10 fraction bits. */
    const int sign = bits >> 15;
    const int e = (bits >> 10) & 0x1f;
    const int f = bits & 0x3ff;
    double x;
    if (e == 0)
        x = ldexp((double)f, -24); /* zero and subnormals: f * 2^-10 * 2^-14 */
    else if (e == 31)
        x = f ? NAN : INFINITY;
    else
        x = ldexp(1.0 + (double)f / 1024.0, e - 15);
    return sign ? -x : x;
}

typedef double (*decode_fn)(uint16_t);

/* One output row.  `s` is scratch for S_kv doubles; `dec` widens one input element. */
static void attn_row(const uint16_t *q_row, const uint16_t *k_head, const uint16_t *v_head,
                     int64_t i, int S_kv, int D, int causal, double scale,
                     double *s, double *o_row, double *lse_out, decode_fn dec)
{
    int64_t n = S_kv;
    if (causal && i + 1 < n)
        n = i + 1; /* keys j <= i only */

    /* pass 1: scores and their maximum */
    double m = -INFINITY;
    for (int64_t j = 0; j < n; ++j) {
        const uint16_t *k_row = k_head + j * (int64_t)D;
        double dot = 0.0;
        for (int d = 0; d < D; ++d)
            dot += dec(q_row[d]) * dec(k_row[d]);
        s[j] = scale * dot;
        if (s[j] > m)
            m = s[j];
    }

    /* pass 2: normaliser and weighted sum of value rows */
    double l = 0.0;
    for (int d = 0; d < D; ++d)
        o_row[d] = 0.0;
    for (int64_t j = 0; j < n; ++j) {
        double p = exp(s[j] - m);
        const uint16_t *v_row = v_head + j * (int64_t)D;
        l += p;
        for (int d = 0; d < D; ++d)
            o_row[d] += p * dec(v_row[d]);
    }
    for (int d = 0; d < D; ++d)
        o_row[d] /= l;
    *lse_out = m + log(l);
}

/*
 * attn_ref_f64: compute n_rows output rows.
 *   rows == NULL : rows 0 .. n_rows-1 (pass n_rows = B*H*S_q for everything)
 *   rows != NULL : the listed flat row ids, in order
 *   o   : [n_rows][D] fp64,  lse : [n_rows] fp64
 *   n_threads <= 0 : OpenMP default
 * returns 0, or -1 on a bad argument / allocation failure.
 */
static int attn_ref_any(const uint16_t *q, const uint16_t *k, const uint16_t *v,
                        int B, int H, int S_q, int S_kv, int D, int causal, float scale,
                        int64_t n_rows, const int64_t *rows,
                        double *o, double *lse, int n_threads, decode_fn dec)
{
    if (!q || !k || !v || !o || !lse)
        return -1;
    if (B < 1 || H < 1 || S_q < 1 || S_kv < 1 || D < 1 || n_rows < 0)
        return -1;
    const int64_t total_rows = (int64_t)B * H * S_q;
    if (rows) {
        for (int64_t t = 0; t < n_rows; ++t)
            if (rows[t] < 0 || rows[t] >= total_rows)
                return -1;
    } else if (n_rows > total_rows) {
        return -1;
    }
    const double scale64 = (double)scale;
    int failed = 0;

#ifdef _OPENMP
#pragma omp parallel num_threads(n_threads > 0 ? n_threads : omp_get_max_threads())
#endif
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)S_kv);
        if (!s) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            failed = 1;
        }
#ifdef _OPENMP
#pragma omp for schedule(dynamic, 16)
#endif
        for (int64_t t = 0; t < n_rows; ++t) {
            if (!s)
                continue;
            const int64_t r = rows ? rows[t] : t;
            const int64_t bh = r / S_q;
            const int64_t i = r % S_q;
            attn_row(q + r * (int64_t)D,
                     k + bh * (int64_t)S_kv * D,
                     v + bh * (int64_t)S_kv * D,
                     i, S_kv, D, causal, scale64,
                     s, o + t * (int64_t)D, lse + t, dec);
        }
        free(s);
    }
    return failed ? -1 : 0;
}

int attn_ref_f64(const uint16_t *q, const uint16_t *k, const uint16_t *v,
                 int B, int H, int S_q, int S_kv, int D, int causal, float scale,
                 int64_t n_rows, const int64_t *rows,
                 double *o, double *lse, int n_threads)
{
    return attn_ref_any(q, k, v, B, H, S_q, S_kv, D, causal, scale, n_rows, rows, o, lse, n_threads,
                        bf16_bits_to_f64);
}

/* Same, with q, k, v holding IEEE binary16 bit patterns. */
int attn_ref_f64_f16(const uint16_t *q, const uint16_t *k, const uint16_t *v,
                     int B, int H, int S_q, int S_kv, int D, int causal, float scale,
                     int64_t n_rows, const int64_t *rows,
                     double *o, double *lse, int n_threads)
{
    return attn_ref_any(q, k, v, B, H, S_q, S_kv, D, causal, scale, n_rows, rows, o, lse, n_threads,
                        f16_bits_to_f64);
}

/* Number of threads an n_threads <= 0 call would use (for reporting). */
int attn_ref_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
