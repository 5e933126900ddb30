/*
 * CPU oracle for batched candidate-suffix attention over a shared prefix.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the HIP path is
 * checked against.  It shares no code with the HIP library and must never be called from
 * the product path (only from tests, the smoke check and the benchmark's cpu_baseline leg).
 *
 * What it computes (paper Eq. 2, scaled dot-product attention, and Eq. 3, the Standard KV
 * cache that repeats the prefix K/V once per candidate):
 *   for every candidate b and KV head k the prefix K/V is PHYSICALLY COPIED into a fresh
 *   per-candidate buffer, the candidate's own suffix K/V rows are appended after it
 *   (App. F.5: concatenate with the suffix K/V of the current layer), and every valid
 *   suffix query i attends to all P prefix rows plus suffix rows 0..i (causal), with a
 *   max-subtracted softmax.  PSKV is exact, not an approximation (Sec. 5.1 / App. D), so
 *   this plain definition is the expected result.
 *
 * Arithmetic: inputs are widened exactly to double; every sum is a sequential double sum.
 * Rows i >= suf_len[b] produce 0 (and lse = -inf, probs = 0).
 *
 * Layouts (contiguous, row-major): q [B,S,Hq,D]; k_suf,v_suf [B,S,Hkv,D];
 * k_pre,v_pre [P,Hkv,D]; out [B,S,Hq,D] double; lse [B,Hq,S] double (optional);
 * probs [B,Hq,S,P+S] double (optional, tests only).  Query head h uses KV head h / (Hq/Hkv).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { PSKV_ORACLE_F32 = 0, PSKV_ORACLE_BF16 = 1, PSKV_ORACLE_F64 = 2 };

static double widen(const void *base, int64_t idx, int dtype)
{
    if (dtype == PSKV_ORACLE_F32)
        return (double)((const float *)base)[idx];
    if (dtype == PSKV_ORACLE_F64)
        return ((const double *)base)[idx];
    /* bfloat16: the 16 stored bits are the high half of an IEEE binary32 */
    uint32_t bits = ((uint32_t)((const uint16_t *)base)[idx]) << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

int pskv_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* returns 0 on success, 1 on bad arguments, 2 on allocation failure */
int pskv_oracle_attn(int B, int S, int P, int Hq, int Hkv, int D, int dtype, double scale,
                     const void *q, const void *k_suf, const void *v_suf,
                     const void *k_pre, const void *v_pre, const int32_t *suf_len,
                     double *out, double *lse, double *probs, int nthreads)
{
    if (B < 0 || S < 1 || P < 0 || Hq < 1 || Hkv < 1 || D < 1 || Hq % Hkv != 0)
        return 1;
    if (dtype < 0 || dtype > 2 || !out || !q || !k_suf || !v_suf || (P > 0 && (!k_pre || !v_pre)))
        return 1;
    for (int b = 0; b < B; ++b)
        if (suf_len && (suf_len[b] < 0 || suf_len[b] > S))
            return 1;
    const int G = Hq / Hkv;
    const int64_t W = (int64_t)P + S; /* width of one probs row */
    int failed = 0;
#ifdef _OPENMP
    if (nthreads > 0)
        omp_set_num_threads(nthreads);
#else
    (void)nthreads;
#endif

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t bk = 0; bk < (int64_t)B * Hkv; ++bk) {
        const int b = (int)(bk / Hkv), k = (int)(bk % Hkv);
        const int len = suf_len ? suf_len[b] : S;
        const int64_t T = (int64_t)P + len; /* rows of this candidate's private cache */

        /* Eq. 3: this candidate's own copy of the prefix K/V, then its suffix K/V rows. */
        double *Kfull = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1) * D);
        double *Vfull = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1) * D);
        double *s = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1));
        if (!Kfull || !Vfull || !s) {
#pragma omp atomic write
            failed = 1;
            free(Kfull); free(Vfull); free(s);
            continue;
        }
        for (int64_t j = 0; j < P; ++j)
            for (int d = 0; d < D; ++d) {
                Kfull[j * D + d] = widen(k_pre, (j * Hkv + k) * D + d, dtype);
                Vfull[j * D + d] = widen(v_pre, (j * Hkv + k) * D + d, dtype);
            }
        for (int64_t t = 0; t < len; ++t)
            for (int d = 0; d < D; ++d) {
                const int64_t src = (((int64_t)b * S + t) * Hkv + k) * D + d;
                Kfull[(P + t) * D + d] = widen(k_suf, src, dtype);
                Vfull[(P + t) * D + d] = widen(v_suf, src, dtype);
            }

        for (int g = 0; g < G; ++g) {
            const int h = k * G + g;
            for (int i = 0; i < S; ++i) {
                double *o = out + (((int64_t)b * S + i) * Hq + h) * D;
                double *pr = probs ? probs + (((int64_t)b * Hq + h) * S + i) * W : NULL;
                for (int d = 0; d < D; ++d)
                    o[d] = 0.0;
                if (pr)
                    for (int64_t j = 0; j < W; ++j)
                        pr[j] = 0.0;
                if (i >= len) { /* padded query row */
                    if (lse)
                        lse[((int64_t)b * Hq + h) * S + i] = -INFINITY;
                    continue;
                }
                /* visible rows: all of the prefix, and suffix rows 0..i  ->  0 .. P+i */
                const int64_t nvis = (int64_t)P + i + 1;
                const int64_t qoff = (((int64_t)b * S + i) * Hq + h) * D;
                double m = -INFINITY;
                for (int64_t j = 0; j < nvis; ++j) {
                    double acc = 0.0;
                    for (int d = 0; d < D; ++d)
                        acc += widen(q, qoff + d, dtype) * Kfull[j * D + d];
                    s[j] = acc * scale;
                    if (s[j] > m)
                        m = s[j];
                }
                double denom = 0.0;
                for (int64_t j = 0; j < nvis; ++j) {
                    s[j] = exp(s[j] - m);
                    denom += s[j];
                }
                for (int64_t j = 0; j < nvis; ++j) {
                    const double p = s[j] / denom;
                    if (pr)
                        pr[j] = p; /* column j: prefix row j for j < P, suffix token t at column P+t */
                    for (int d = 0; d < D; ++d)
                        o[d] += p * Vfull[j * D + d];
                }
                if (lse)
                    lse[((int64_t)b * Hq + h) * S + i] = m + log(denom);
            }
        }
        free(Kfull); free(Vfull); free(s);
    }
    return failed ? 2 : 0;
}

/*
 * Batched multi-instruction form (paper Sec. 4.3, suffix-centric alignment; App. F.1, position
 * consistency under padding): Np instructions, each with its own prefix K/V, LEFT-padded to a
 * common Pp rows (the real rows of instruction n are the last pre_len[n] ones), and C
 * consecutive candidates per instruction (candidate b belongs to instruction b / C, B = Np*C).
 * A candidate attends to the real prefix rows of its own instruction and causally to its own
 * suffix rows; padding rows of the prefix are excluded from attention (they may hold anything).
 *
 * Same plain procedure as above: for every candidate and KV head the real prefix rows of the
 * candidate's instruction are physically copied into a private buffer (one prefix cache per
 * instruction, repeated over its candidates the Standard-KV way), the suffix rows are appended
 * and every valid query runs the max-subtracted softmax of Eq. 2 over the rows it may see.
 *
 * Layouts: k_pre,v_pre [Np,Pp,Hkv,D]; pre_len [Np] (NULL: every prefix has Pp real rows);
 * the rest as for pskv_oracle_attn.  probs (optional) is [B,Hq,S,Pp+S]: column j < Pp is the
 * padded prefix index j (0 on padding), column Pp+t is suffix token t.
 */
int pskv_oracle_attn_multi(int Np, int C, int S, int Pp, int Hq, int Hkv, int D, int dtype, double scale,
                           const void *q, const void *k_suf, const void *v_suf,
                           const void *k_pre, const void *v_pre, const int32_t *pre_len,
                           const int32_t *suf_len, double *out, double *lse, double *probs, int nthreads)
{
    if (Np < 0 || C < 0 || S < 1 || Pp < 0 || Hq < 1 || Hkv < 1 || D < 1 || Hq % Hkv != 0)
        return 1;
    if (dtype < 0 || dtype > 2 || !out || !q || !k_suf || !v_suf || (Pp > 0 && (!k_pre || !v_pre)))
        return 1;
    const int64_t B = (int64_t)Np * C;
    for (int n = 0; n < Np; ++n)
        if (pre_len && (pre_len[n] < 0 || pre_len[n] > Pp))
            return 1;
    for (int64_t b = 0; b < B; ++b)
        if (suf_len && (suf_len[b] < 0 || suf_len[b] > S))
            return 1;
    const int G = Hq / Hkv;
    const int64_t W = (int64_t)Pp + S;
    int failed = 0;
#ifdef _OPENMP
    if (nthreads > 0)
        omp_set_num_threads(nthreads);
#else
    (void)nthreads;
#endif

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t bk = 0; bk < B * Hkv; ++bk) {
        const int64_t b = bk / Hkv;
        const int k = (int)(bk % Hkv);
        const int n = (int)(b / C);                 /* the candidate's instruction */
        const int np = pre_len ? pre_len[n] : Pp;   /* its real prefix rows ...   */
        const int64_t first = (int64_t)Pp - np;     /* ... start here (left padding before) */
        const int len = suf_len ? suf_len[b] : S;
        const int64_t T = (int64_t)np + len;

        double *Kfull = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1) * D);
        double *Vfull = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1) * D);
        double *s = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1));
        if (!Kfull || !Vfull || !s) {
#pragma omp atomic write
            failed = 1;
            free(Kfull); free(Vfull); free(s);
            continue;
        }
        for (int64_t j = 0; j < np; ++j)
            for (int d = 0; d < D; ++d) {
                const int64_t src = ((((int64_t)n * Pp) + first + j) * Hkv + k) * D + d;
                Kfull[j * D + d] = widen(k_pre, src, dtype);
                Vfull[j * D + d] = widen(v_pre, src, dtype);
            }
        for (int64_t t = 0; t < len; ++t)
            for (int d = 0; d < D; ++d) {
                const int64_t src = ((b * S + t) * Hkv + k) * D + d;
                Kfull[(np + t) * D + d] = widen(k_suf, src, dtype);
                Vfull[(np + t) * D + d] = widen(v_suf, src, dtype);
            }

        for (int g = 0; g < G; ++g) {
            const int h = k * G + g;
            for (int i = 0; i < S; ++i) {
                double *o = out + ((b * S + i) * Hq + h) * D;
                double *pr = probs ? probs + ((b * Hq + h) * S + i) * W : NULL;
                for (int d = 0; d < D; ++d)
                    o[d] = 0.0;
                if (pr)
                    for (int64_t j = 0; j < W; ++j)
                        pr[j] = 0.0;
                if (i >= len) {
                    if (lse)
                        lse[(b * Hq + h) * S + i] = -INFINITY;
                    continue;
                }
                const int64_t nvis = (int64_t)np + i + 1; /* real prefix rows, suffix rows 0..i */
                const int64_t qoff = ((b * S + i) * Hq + h) * D;
                double m = -INFINITY;
                for (int64_t j = 0; j < nvis; ++j) {
                    double acc = 0.0;
                    for (int d = 0; d < D; ++d)
                        acc += widen(q, qoff + d, dtype) * Kfull[j * D + d];
                    s[j] = acc * scale;
                    if (s[j] > m)
                        m = s[j];
                }
                double denom = 0.0;
                for (int64_t j = 0; j < nvis; ++j) {
                    s[j] = exp(s[j] - m);
                    denom += s[j];
                }
                for (int64_t j = 0; j < nvis; ++j) {
                    const double p = s[j] / denom;
                    if (pr)
                        pr[j < np ? first + j : (int64_t)Pp + (j - np)] = p;
                    for (int d = 0; d < D; ++d)
                        o[d] += p * Vfull[j * D + d];
                }
                if (lse)
                    lse[(b * Hq + h) * S + i] = m + log(denom);
            }
        }
        free(Kfull); free(Vfull); free(s);
    }
    return failed ? 2 : 0;
}

/*
 * Backward pass of the single-prefix form with respect to the suffix side (the paper keeps the
 * computation graph of the suffix/target segment intact so that gradient-based synthesis can
 * differentiate through cached execution, Sec. 1 and Sec. 4.2; the prefix K/V is a constant).
 *
 * Definition: with out = f(q, k_suf, v_suf) the forward pass above and dout a given tensor of
 * the same shape, the result is the gradient of  L = sum(dout * out)  with respect to q, k_suf
 * and v_suf.  It is written here as the textbook derivative of Eq. 2, row by row: for a valid
 * query row with probabilities p_j over its visible rows (own copy of the prefix, then suffix
 * rows 0..i),
 *     dp_j = <dout_row, V_j>,   ds_j = p_j * (dp_j - sum_k p_k dp_k),
 *     dq_row += scale * sum_j ds_j K_j,   dK_j += scale * ds_j q_row,   dV_j += p_j dout_row,
 * where only the suffix rows j receive dK, dV (summed over the query heads that share the KV
 * head).  Padded query rows contribute nothing and get dq = 0; padded suffix rows get 0.
 * Not thread-parallel over candidates' shared outputs: one thread per candidate.
 */
int pskv_oracle_attn_bwd(int B, int S, int P, int Hq, int Hkv, int D, int dtype, double scale,
                         const void *q, const void *k_suf, const void *v_suf,
                         const void *k_pre, const void *v_pre, const int32_t *suf_len,
                         const double *dout, double *dq, double *dk_suf, double *dv_suf, int nthreads)
{
    if (B < 0 || S < 1 || P < 0 || Hq < 1 || Hkv < 1 || D < 1 || Hq % Hkv != 0)
        return 1;
    if (dtype < 0 || dtype > 2 || !dout || !dq || !dk_suf || !dv_suf || !q || !k_suf || !v_suf ||
        (P > 0 && (!k_pre || !v_pre)))
        return 1;
    for (int b = 0; b < B; ++b)
        if (suf_len && (suf_len[b] < 0 || suf_len[b] > S))
            return 1;
    const int G = Hq / Hkv;
    int failed = 0;
#ifdef _OPENMP
    if (nthreads > 0)
        omp_set_num_threads(nthreads);
#else
    (void)nthreads;
#endif

#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        const int len = suf_len ? suf_len[b] : S;
        const int64_t T = (int64_t)P + len;
        double *Kfull = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1) * D);
        double *Vfull = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1) * D);
        double *p = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1));
        double *dp = (double *)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1));
        if (!Kfull || !Vfull || !p || !dp) {
#pragma omp atomic write
            failed = 1;
            free(Kfull); free(Vfull); free(p); free(dp);
            continue;
        }
        for (int64_t x = 0; x < (int64_t)S * Hq * D; ++x)
            dq[(int64_t)b * S * Hq * D + x] = 0.0;
        for (int64_t x = 0; x < (int64_t)S * Hkv * D; ++x) {
            dk_suf[(int64_t)b * S * Hkv * D + x] = 0.0;
            dv_suf[(int64_t)b * S * Hkv * D + x] = 0.0;
        }
        for (int k = 0; k < Hkv; ++k) {
            /* this candidate's private cache: copy of the prefix, then its suffix rows (Eq. 3) */
            for (int64_t j = 0; j < P; ++j)
                for (int d = 0; d < D; ++d) {
                    Kfull[j * D + d] = widen(k_pre, (j * Hkv + k) * D + d, dtype);
                    Vfull[j * D + d] = widen(v_pre, (j * Hkv + k) * D + d, dtype);
                }
            for (int64_t t = 0; t < len; ++t)
                for (int d = 0; d < D; ++d) {
                    const int64_t src = (((int64_t)b * S + t) * Hkv + k) * D + d;
                    Kfull[(P + t) * D + d] = widen(k_suf, src, dtype);
                    Vfull[(P + t) * D + d] = widen(v_suf, src, dtype);
                }
            for (int g = 0; g < G; ++g) {
                const int h = k * G + g;
                for (int i = 0; i < len; ++i) {
                    const int64_t nvis = (int64_t)P + i + 1;
                    const int64_t roff = (((int64_t)b * S + i) * Hq + h) * D;
                    double m = -INFINITY;
                    for (int64_t j = 0; j < nvis; ++j) {
                        double acc = 0.0;
                        for (int d = 0; d < D; ++d)
                            acc += widen(q, roff + d, dtype) * Kfull[j * D + d];
                        p[j] = acc * scale;
                        if (p[j] > m)
                            m = p[j];
                    }
                    double denom = 0.0;
                    for (int64_t j = 0; j < nvis; ++j) {
                        p[j] = exp(p[j] - m);
                        denom += p[j];
                    }
                    double mean_dp = 0.0; /* sum_k p_k dp_k */
                    for (int64_t j = 0; j < nvis; ++j) {
                        p[j] /= denom;
                        double acc = 0.0;
                        for (int d = 0; d < D; ++d)
                            acc += dout[roff + d] * Vfull[j * D + d];
                        dp[j] = acc;
                        mean_dp += p[j] * acc;
                    }
                    for (int64_t j = 0; j < nvis; ++j) {
                        const double ds = p[j] * (dp[j] - mean_dp);
                        for (int d = 0; d < D; ++d)
                            dq[roff + d] += scale * ds * Kfull[j * D + d];
                        if (j >= P) { /* a suffix row of this candidate */
                            const int64_t koff = (((int64_t)b * S + (j - P)) * Hkv + k) * D;
                            for (int d = 0; d < D; ++d) {
                                dk_suf[koff + d] += scale * ds * widen(q, roff + d, dtype);
                                dv_suf[koff + d] += p[j] * dout[roff + d];
                            }
                        }
                    }
                }
            }
        }
        free(Kfull); free(Vfull); free(p); free(dp);
    }
    return failed ? 2 : 0;
}
