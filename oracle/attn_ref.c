/*
 * fp64 CPU oracle for single-token grouped-query decode attention over a KV
 * cache compressed per head.  TEST INFRASTRUCTURE ONLY: nothing on the product
 * path may call this; it exists so that the GPU kernels can be checked against
 * a definition that is obviously right, and it shares no code with them.
 *
 * What is computed.  The paper's setting (Introduction; Related Work,
 * "Imbalanced Per-Head Compression"; Section 3.2, latency of decoding one
 * token) is ordinary scaled-dot-product attention of one new query token per
 * sequence, where every attention head keeps its own number of cached tokens.
 * The paper does not print the formula; it is the standard one:
 *
 *     s_t  = scale * <q, K_t>            t = 0 .. len-1
 *     w_t  = exp(s_t - max_t s_t)
 *     out  = sum_t w_t V_t / sum_t w_t
 *     lse  = max_t s_t + log(sum_t w_t)
 *
 * Readings taken where the paper is silent: the budget is per KV head and the
 * G = Hq/Hkv query heads [h*G, (h+1)*G) share KV head h; the cache already
 * holds every token to attend to (no mask, no positions); an empty head gives
 * out = 0 and lse = -inf.
 *
 * Everything is plain loops in double precision with left-to-right sums: no
 * tiling, no running maximum, no chunking.  The only parallelism is an OpenMP
 * loop over independent (sequence, query head) outputs.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_BF16 = 0, ORACLE_F32 = 1, ORACLE_F64 = 2 };

static double load_elem(const void *base, int64_t idx, int dtype)
{
    if (dtype == ORACLE_BF16) {
        /* bf16 is the upper half of an IEEE binary32: widening is exact. */
        uint32_t bits = (uint32_t)((const uint16_t *)base)[idx] << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    }
    if (dtype == ORACLE_F32)
        return (double)((const float *)base)[idx];
    return ((const double *)base)[idx];
}

/*
 * Softmax statistics and unnormalised weighted sum over rows
 * [row0, row0 + n) of K and V for one query vector:
 *   m = max s_t, l = sum exp(s_t - m), acc[d] = sum exp(s_t - m) V[t][d].
 * n == 0 gives m = -inf, l = 0, acc = 0.  `s` is scratch of n doubles.
 */
static void scores_and_sums(const void *q, int64_t q_idx0, const void *k, const void *v,
                            int64_t row0, int64_t n, int D, int dtype, double scale,
                            double *s, double *m_out, double *l_out, double *acc)
{
    for (int d = 0; d < D; ++d)
        acc[d] = 0.0;
    if (n <= 0) {
        *m_out = -INFINITY;
        *l_out = 0.0;
        return;
    }
    for (int64_t t = 0; t < n; ++t) {
        double dot = 0.0;
        for (int d = 0; d < D; ++d)
            dot += load_elem(q, q_idx0 + d, dtype) * load_elem(k, (row0 + t) * D + d, dtype);
        s[t] = scale * dot;
    }
    double m = s[0];
    for (int64_t t = 1; t < n; ++t)
        if (s[t] > m)
            m = s[t];
    double l = 0.0;
    for (int64_t t = 0; t < n; ++t) {
        double w = exp(s[t] - m);
        l += w;
        for (int d = 0; d < D; ++d)
            acc[d] += w * load_elem(v, (row0 + t) * D + d, dtype);
    }
    *m_out = m;
    *l_out = l;
}

/*
 * Full attention.  q [B][Hq][D], k/v [rows][D] (dtype as given), off/len [B][Hkv].
 * sel: optional list of n_sel flat output indices b*Hq+hq to compute (others are
 * left untouched); NULL computes all.  out [B][Hq][D] and lse [B][Hq] are double.
 * Returns 0, or -1 on bad arguments.
 */
int fairkv_oracle_attn(const void *q, const void *k, const void *v,
                       const int64_t *off, const int32_t *len,
                       int B, int Hq, int Hkv, int D, int dtype, double scale,
                       const int32_t *sel, int n_sel,
                       double *out, double *lse, int n_threads)
{
    if (!q || !k || !v || !off || !len || !out || !lse)
        return -1;
    if (B <= 0 || Hq <= 0 || Hkv <= 0 || D <= 0 || Hq % Hkv != 0)
        return -1;
    if (dtype != ORACLE_BF16 && dtype != ORACLE_F32 && dtype != ORACLE_F64)
        return -1;
    const int G = Hq / Hkv;
    const int total = sel ? n_sel : B * Hq;
#ifdef _OPENMP
    if (n_threads > 0)
        omp_set_num_threads(n_threads);
#else
    (void)n_threads;
#endif
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(| : bad)
    for (int i = 0; i < total; ++i) {
        const int flat = sel ? sel[i] : i;
        if (flat < 0 || flat >= B * Hq) {
            bad = 1;
            continue;
        }
        const int b = flat / Hq, hq = flat % Hq, h = hq / G;
        const int64_t n = len[b * Hkv + h];
        const int64_t row0 = off[b * Hkv + h];
        double *o = out + (int64_t)flat * D;
        if (n < 0) {
            bad = 1;
            continue;
        }
        double *s = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
        double m, l;
        scores_and_sums(q, (int64_t)flat * D, k, v, row0, n, D, dtype, scale, s, &m, &l, o);
        if (n == 0) {
            lse[flat] = -INFINITY;
        } else {
            for (int d = 0; d < D; ++d)
                o[d] /= l;
            lse[flat] = m + log(l);
        }
        free(s);
    }
    return bad ? -1 : 0;
}

/*
 * Several new tokens per sequence at once (a draft of q_len tokens being verified): the cache
 * already holds their K/V as the last q_len rows of every head, and new token i (0-based) sees
 * the rows before the new tokens that follow it: rows [0, len - (q_len - 1 - i)), none if that
 * is not positive.  This is ordinary causal attention restricted to the kept tokens; with
 * q_len = 1 it is fairkv_oracle_attn.  q [B][q_len][Hq][D]; out [B][q_len][Hq][D] and
 * lse [B][q_len][Hq] are double.  Returns 0, or -1 on bad arguments.
 */
int fairkv_oracle_attn_multi(const void *q, const void *k, const void *v,
                             const int64_t *off, const int32_t *len,
                             int B, int q_len, int Hq, int Hkv, int D, int dtype, double scale,
                             double *out, double *lse, int n_threads)
{
    if (!q || !k || !v || !off || !len || !out || !lse)
        return -1;
    if (B <= 0 || q_len <= 0 || Hq <= 0 || Hkv <= 0 || D <= 0 || Hq % Hkv != 0)
        return -1;
    if (dtype != ORACLE_BF16 && dtype != ORACLE_F32 && dtype != ORACLE_F64)
        return -1;
    const int G = Hq / Hkv;
    const int total = B * q_len * Hq;
#ifdef _OPENMP
    if (n_threads > 0)
        omp_set_num_threads(n_threads);
#else
    (void)n_threads;
#endif
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(| : bad)
    for (int flat = 0; flat < total; ++flat) {
        const int hq = flat % Hq, i = (flat / Hq) % q_len, b = flat / (Hq * q_len), h = hq / G;
        const int64_t len_bh = len[b * Hkv + h];
        const int64_t row0 = off[b * Hkv + h];
        if (len_bh < 0) {
            bad = 1;
            continue;
        }
        int64_t n = len_bh - (q_len - 1 - i);
        if (n < 0)
            n = 0;
        double *o = out + (int64_t)flat * D;
        double *s = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
        double m, l;
        scores_and_sums(q, (int64_t)flat * D, k, v, row0, n, D, dtype, scale, s, &m, &l, o);
        if (n == 0) {
            lse[flat] = -INFINITY;
        } else {
            for (int d = 0; d < D; ++d)
                o[d] /= l;
            lse[flat] = m + log(l);
        }
        free(s);
    }
    return bad ? -1 : 0;
}

/*
 * One token chunk of one (sequence, query head): rows [off + t0, off + t0 + n)
 * of that head's cache.  Gives the chunk's (m, l, unnormalised acc[D]).  Used
 * only to pin the chunk-merge identity (chunked-and-merged == unchunked).
 */
int fairkv_oracle_attn_chunk(const void *q, const void *k, const void *v,
                             int64_t q_idx0, int64_t row0, int64_t n, int D, int dtype,
                             double scale, double *m, double *l, double *acc)
{
    if (!q || !k || !v || !m || !l || !acc || D <= 0 || n < 0)
        return -1;
    double *s = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
    scores_and_sums(q, q_idx0, k, v, row0, n, D, dtype, scale, s, m, l, acc);
    free(s);
    return 0;
}

int fairkv_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
