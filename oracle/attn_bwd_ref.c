/*
 * attn_bwd_ref.c -- fp64 CPU oracle for the backward pass of scaled-dot-product attention.
 *
 * TEST INFRASTRUCTURE ONLY.  Slow, plain definition that the GPU backward path is
 * checked against; shares no code, header, table or helper with the HIP library
 * and is never called from the product path.
 *
 * What it computes.  The paper's Section 6.3 evaluates the backward pass of the
 * attention of Section 6.2 ("five GEMMs and one exponential" per tile, then a
 * reduction of dQ).  Those five products are the chain rule applied to the
 * forward definition  O = softmax(scale * Q K^T) V; written out per query row i,
 * with dO the gradient of a scalar loss with respect to O:
 *
 *   J(i)   = visible keys (all j < S_kv; causal: also j <= i)
 *   s_ij   = scale * q_i . k_j                     j in J(i)
 *   p_ij   = exp(s_ij - m_i) / l_i                 (m_i = max_j s_ij, l_i = sum_j exp(s_ij - m_i))
 *   dp_ij  = dO_i . v_j                            (gradient w.r.t. p_ij)
 *   D_i    = sum_j p_ij * dp_ij                    (softmax Jacobian: every p_ij feels every s_ij')
 *   ds_ij  = p_ij * (dp_ij - D_i)                  (gradient w.r.t. s_ij)
 *   dQ_i   = scale * sum_j ds_ij * k_j
 *   dK_j   = scale * sum_i ds_ij * q_i             (sum over the rows i that see key j)
 *   dV_j   =         sum_i p_ij  * dO_i
 *
 * No tiles, no recomputation tricks, no use of a stored O or LSE: only q, k, v, dO.
 * Everything is IEEE fp64; inputs are 16-bit patterns (bf16, or IEEE binary16 when
 * is_f16 != 0) widened exactly; `scale` is the caller's fp32 value widened exactly.
 *
 * Layout: q, dO [B][H][S_q][D]; k, v [B][H][S_kv][D]; contiguous, row-major.
 * Heads are addressed by the flat id bh = b*H + h.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double bwd_bf16_to_f64(uint16_t bits)
{
    uint32_t w = ((uint32_t)bits) << 16; /* bf16 = upper half of a binary32 */
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

static double bwd_f16_to_f64(uint16_t bits)
{
    /* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits */
    const int sign = bits >> 15, e = (bits >> 10) & 0x1f, f = bits & 0x3ff;
    double x;
    if (e == 0)
        x = ldexp((double)f, -24);
    else if (e == 31)
        x = f ? NAN : INFINITY;
    else
        x = ldexp(1.0 + (double)f / 1024.0, e - 15);
    return sign ? -x : x;
}

/* widen one [n][D] block */
static void widen(const uint16_t *src, int64_t n, double *dst, int is_f16)
{
    for (int64_t t = 0; t < n; ++t)
        dst[t] = is_f16 ? bwd_f16_to_f64(src[t]) : bwd_bf16_to_f64(src[t]);
}

/*
 * One head.  qh, doh: [S_q][D]; kh, vh: [S_kv][D] (already fp64).
 * dq: [S_q][D]; dk, dv: [S_kv][D], all overwritten.
 */
static int bwd_head(const double *qh, const double *kh, const double *vh, const double *doh,
                    int S_q, int S_kv, int D, int causal, double scale,
                    double *dq, double *dk, double *dv, int n_threads)
{
    int failed = 0;
    const size_t kv_elems = (size_t)S_kv * D;
    memset(dk, 0, sizeof(double) * kv_elems);
    memset(dv, 0, sizeof(double) * kv_elems);

#ifdef _OPENMP
#pragma omp parallel num_threads(n_threads > 0 ? n_threads : omp_get_max_threads())
#endif
    {
        /* per-thread partial dK, dV (rows i are split over threads) and per-row scratch */
        double *pdk = (double *)calloc(kv_elems, sizeof(double));
        double *pdv = (double *)calloc(kv_elems, sizeof(double));
        double *p = (double *)malloc(sizeof(double) * (size_t)S_kv);
        double *ds = (double *)malloc(sizeof(double) * (size_t)S_kv);
        if (!pdk || !pdv || !p || !ds) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            failed = 1;
        }
#ifdef _OPENMP
#pragma omp for schedule(dynamic, 8)
#endif
        for (int i = 0; i < S_q; ++i) {
            if (!pdk || !pdv || !p || !ds)
                continue;
            const double *qi = qh + (size_t)i * D;
            const double *doi = doh + (size_t)i * D;
            int n = S_kv;
            if (causal && i + 1 < n)
                n = i + 1;
            /* scores, softmax */
            double m = -INFINITY;
            for (int j = 0; j < n; ++j) {
                const double *kj = kh + (size_t)j * D;
                double dot = 0.0;
                for (int d = 0; d < D; ++d)
                    dot += qi[d] * kj[d];
                p[j] = scale * dot;
                if (p[j] > m)
                    m = p[j];
            }
            double l = 0.0;
            for (int j = 0; j < n; ++j) {
                p[j] = exp(p[j] - m);
                l += p[j];
            }
            for (int j = 0; j < n; ++j)
                p[j] /= l;
            /* dp, D_i */
            double Di = 0.0;
            for (int j = 0; j < n; ++j) {
                const double *vj = vh + (size_t)j * D;
                double dp = 0.0;
                for (int d = 0; d < D; ++d)
                    dp += doi[d] * vj[d];
                ds[j] = dp;
                Di += p[j] * dp;
            }
            for (int j = 0; j < n; ++j)
                ds[j] = p[j] * (ds[j] - Di);
            /* dQ_i, and this row's terms of dK, dV */
            double *dqi = dq + (size_t)i * D;
            for (int d = 0; d < D; ++d)
                dqi[d] = 0.0;
            for (int j = 0; j < n; ++j) {
                const double *kj = kh + (size_t)j * D;
                double *dkj = pdk + (size_t)j * D;
                double *dvj = pdv + (size_t)j * D;
                for (int d = 0; d < D; ++d) {
                    dqi[d] += ds[j] * kj[d];
                    dkj[d] += ds[j] * qi[d];
                    dvj[d] += p[j] * doi[d];
                }
            }
            for (int d = 0; d < D; ++d)
                dqi[d] *= scale;
        }
        /* add the partials, one thread at a time (fp64: the order moves the last bits only) */
#ifdef _OPENMP
#pragma omp critical
#endif
        {
            if (pdk && pdv)
                for (size_t t = 0; t < kv_elems; ++t) {
                    dk[t] += pdk[t];
                    dv[t] += pdv[t];
                }
        }
        free(pdk);
        free(pdv);
        free(p);
        free(ds);
    }
    for (size_t t = 0; t < kv_elems; ++t)
        dk[t] *= scale;
    return failed ? -1 : 0;
}

/*
 * attn_bwd_ref_f64: gradients for n_heads heads.
 *   heads == NULL : heads 0 .. n_heads-1 (pass n_heads = B*H for everything)
 *   heads != NULL : the listed flat head ids b*H + h, in order
 *   dq : [n_heads][S_q][D], dk, dv : [n_heads][S_kv][D], fp64
 * returns 0, or -1 on a bad argument / allocation failure.
 */
int attn_bwd_ref_f64(const uint16_t *q, const uint16_t *k, const uint16_t *v, const uint16_t *d_o,
                     int B, int H, int S_q, int S_kv, int D, int causal, float scale, int is_f16,
                     int64_t n_heads, const int64_t *heads,
                     double *dq, double *dk, double *dv, int n_threads)
{
    if (!q || !k || !v || !d_o || !dq || !dk || !dv)
        return -1;
    if (B < 1 || H < 1 || S_q < 1 || S_kv < 1 || D < 1 || n_heads < 0)
        return -1;
    const int64_t BH = (int64_t)B * H;
    if (heads) {
        for (int64_t t = 0; t < n_heads; ++t)
            if (heads[t] < 0 || heads[t] >= BH)
                return -1;
    } else if (n_heads > BH) {
        return -1;
    }
    const size_t qe = (size_t)S_q * D, ke = (size_t)S_kv * D;
    double *qh = (double *)malloc(sizeof(double) * qe);
    double *doh = (double *)malloc(sizeof(double) * qe);
    double *kh = (double *)malloc(sizeof(double) * ke);
    double *vh = (double *)malloc(sizeof(double) * ke);
    int rc = (qh && doh && kh && vh) ? 0 : -1;
    for (int64_t t = 0; t < n_heads && rc == 0; ++t) {
        const int64_t bh = heads ? heads[t] : t;
        widen(q + bh * qe, (int64_t)qe, qh, is_f16);
        widen(d_o + bh * qe, (int64_t)qe, doh, is_f16);
        widen(k + bh * ke, (int64_t)ke, kh, is_f16);
        widen(v + bh * ke, (int64_t)ke, vh, is_f16);
        rc = bwd_head(qh, kh, vh, doh, S_q, S_kv, D, causal, (double)scale,
                      dq + t * qe, dk + t * ke, dv + t * ke, n_threads);
    }
    free(qh);
    free(doh);
    free(kh);
    free(vh);
    return rc;
}
