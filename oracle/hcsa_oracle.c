/*
 * CPU oracle for Head-Centric Sparse Attention (dLLM-Serve, Section 4.5).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * GPU library must compute.  It shares no code, header, table or helper with
 * the HIP path and is never called by it; only the tests, the smoke check and
 * the benchmark's cpu_baseline leg load it.  All pointers are HOST pointers.
 *
 * Layout (packed variable length, contiguous):
 *   q   [total_q , Hq , D]     cu_q  [B+1] prefix sums of per-sequence query rows
 *   k,v [total_kv, Hkv, D]     cu_kv [B+1] prefix sums of per-sequence KV lengths
 *   idx [Hq, total_k] int32    cu_k  [B+1] prefix sums of per-sequence kept rows;
 *                              entries are positions LOCAL to their sequence
 *   dtype 0: float32 elements; dtype 1: bfloat16 elements given as uint16 bits.
 *   Query head h reads KV head h / (Hq / Hkv).
 *
 * What follows which passage:
 *   oracle_score   per-head importance score, Section 4.5 Eq. (6): block queries
 *                  against every key of the sequence, then a local max-pool of
 *                  odd width w.  The reduction of the block's per-query scores
 *                  to one number is not stated in the paper; here it is the sum
 *                  over the block's queries (same order as their mean).
 *   oracle_topk    I^h = TopK(S_{h,:}, k), Section 4.5 (text under Eq. (6)),
 *                  under the total order "larger score first, equal scores:
 *                  lower position first", written out ascending by position.
 *   oracle_attend  Softmax(Q K^T / sqrt(d)) V restricted to the kept rows of
 *                  each head: Section 2.3 Eq. (4) (Reuse) and, with every
 *                  position kept, Eq. (3) (Refresh).  Bidirectional, no mask,
 *                  no position term (keys already carry positions, Section 4.5).
 *
 * Precision.  Attention is evaluated in fp64.  The score decides an integer
 * result (which rows are kept), so its arithmetic is part of the definition and
 * is taken in the kernel's precision, fp32, in one fixed order:
 *   qsum[d] = (((0 + Q[0,h,d]) + Q[1,h,d]) + ... )          fp32 adds, rows ascending
 *   acc = 0;  acc = fmaf(qsum[d], K[j,g,d], acc)  d = 0..D-1  one rounding per step
 *   s = acc + 0.0f                                          (-0 becomes +0)
 * A second, fp64 score (sum over the block of the individual dot products) is
 * returned beside it so a disagreement can be classified.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_BAD_ARG 1
#define ORACLE_NO_MEM 2

static inline float widen(const void *base, int dtype, int64_t i)
{
    if (dtype == 0)
        return ((const float *)base)[i];
    uint32_t u = ((uint32_t)((const uint16_t *)base)[i]) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static int check_common(int dtype, int B, int Hq, int Hkv, int D,
                        const int32_t *cu_q, const int32_t *cu_kv)
{
    if (dtype != 0 && dtype != 1) return ORACLE_BAD_ARG;
    if (B < 0 || Hq < 1 || Hkv < 1 || D < 1 || Hq % Hkv != 0) return ORACLE_BAD_ARG;
    if (!cu_q || !cu_kv) return ORACLE_BAD_ARG;
    if (cu_q[0] != 0 || cu_kv[0] != 0) return ORACLE_BAD_ARG;
    for (int b = 0; b < B; ++b)
        if (cu_q[b + 1] < cu_q[b] || cu_kv[b + 1] < cu_kv[b]) return ORACLE_BAD_ARG;
    return ORACLE_OK;
}

/* Eq. (6): s32 [Hq, total_kv] (fp32, canonical order, after pooling),
 * s64 [Hq, total_kv] (fp64 sum of the block's dot products, after pooling), either may be NULL. */
int oracle_score(int dtype, int B, int Hq, int Hkv, int D,
                 const void *q, const void *k,
                 const int32_t *cu_q, const int32_t *cu_kv,
                 int pool_w, float *s32, double *s64)
{
    int rc = check_common(dtype, B, Hq, Hkv, D, cu_q, cu_kv);
    if (rc) return rc;
    if (pool_w < 1 || pool_w % 2 == 0) return ORACLE_BAD_ARG;
    const int G = Hq / Hkv;
    const int64_t total_kv = cu_kv[B];
    const int half = pool_w / 2;
    int failed = 0;

#pragma omp parallel for schedule(dynamic)
    for (int bh = 0; bh < B * Hq; ++bh) {
        const int b = bh / Hq, h = bh % Hq, g = h / G;
        const int64_t q0 = cu_q[b], nq = cu_q[b + 1] - cu_q[b];
        const int64_t k0 = cu_kv[b], L = cu_kv[b + 1] - cu_kv[b];
        float *qsum = (float *)malloc(sizeof(float) * (size_t)D);
        float *raw32 = (float *)malloc(sizeof(float) * (size_t)(L > 0 ? L : 1));
        double *raw64 = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1));
        if (!qsum || !raw32 || !raw64) {
            failed = 1;
            free(qsum); free(raw32); free(raw64);
            continue;
        }
        for (int d = 0; d < D; ++d) {
            float a = 0.0f;
            for (int64_t i = 0; i < nq; ++i)
                a = a + widen(q, dtype, ((q0 + i) * Hq + h) * D + d);
            qsum[d] = a;
        }
        for (int64_t j = 0; j < L; ++j) {
            const int64_t krow = ((k0 + j) * Hkv + g) * D;
            float acc = 0.0f;
            for (int d = 0; d < D; ++d)
                acc = fmaf(qsum[d], widen(k, dtype, krow + d), acc);
            raw32[j] = acc + 0.0f;
            if (s64) {
                double tot = 0.0;
                for (int64_t i = 0; i < nq; ++i) {
                    const int64_t qrow = ((q0 + i) * Hq + h) * D;
                    double dot = 0.0;
                    for (int d = 0; d < D; ++d)
                        dot += (double)widen(q, dtype, qrow + d) * (double)widen(k, dtype, krow + d);
                    tot += dot;
                }
                raw64[j] = tot;
            }
        }
        /* local max-pool over positions j-half .. j+half, clipped to the sequence */
        for (int64_t j = 0; j < L; ++j) {
            int64_t lo = j - half < 0 ? 0 : j - half;
            int64_t hi = j + half > L - 1 ? L - 1 : j + half;
            float m32 = raw32[lo];
            double m64 = s64 ? raw64[lo] : 0.0;
            for (int64_t m = lo + 1; m <= hi; ++m) {
                if (raw32[m] > m32) m32 = raw32[m];
                if (s64 && raw64[m] > m64) m64 = raw64[m];
            }
            if (s32) s32[(int64_t)h * total_kv + k0 + j] = m32;
            if (s64) s64[(int64_t)h * total_kv + k0 + j] = m64;
        }
        free(qsum); free(raw32); free(raw64);
    }
    return failed ? ORACLE_NO_MEM : ORACLE_OK;
}

typedef struct {
    float s;
    int32_t j;
} scored_pos;

/* larger score first; equal scores (IEEE ==): lower position first */
static int by_score_then_pos(const void *a, const void *b)
{
    const scored_pos *x = (const scored_pos *)a, *y = (const scored_pos *)b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    return (x->j > y->j) - (x->j < y->j);
}

static int by_pos(const void *a, const void *b)
{
    const scored_pos *x = (const scored_pos *)a, *y = (const scored_pos *)b;
    return (x->j > y->j) - (x->j < y->j);
}

/* TopK(S_{h,:}, k_b) for every (sequence, head); s [Hq, total_kv]; idx_out [Hq, total_k]. */
int oracle_topk(int B, int Hq, const float *s,
                const int32_t *cu_kv, const int32_t *cu_k, int32_t *idx_out)
{
    if (B < 0 || Hq < 1 || !s || !cu_kv || !cu_k || !idx_out) return ORACLE_BAD_ARG;
    if (cu_kv[0] != 0 || cu_k[0] != 0) return ORACLE_BAD_ARG;
    for (int b = 0; b < B; ++b) {
        const int64_t L = cu_kv[b + 1] - cu_kv[b], kb = cu_k[b + 1] - cu_k[b];
        if (L < 0 || kb < 0 || kb > L) return ORACLE_BAD_ARG;
    }
    const int64_t total_kv = cu_kv[B], total_k = cu_k[B];
    int failed = 0;

#pragma omp parallel for schedule(dynamic)
    for (int bh = 0; bh < B * Hq; ++bh) {
        const int b = bh / Hq, h = bh % Hq;
        const int64_t k0 = cu_kv[b], L = cu_kv[b + 1] - cu_kv[b];
        const int64_t o0 = cu_k[b], kb = cu_k[b + 1] - cu_k[b];
        if (kb == 0) continue;
        scored_pos *p = (scored_pos *)malloc(sizeof(scored_pos) * (size_t)L);
        if (!p) { failed = 1; continue; }
        for (int64_t j = 0; j < L; ++j) {
            p[j].s = s[(int64_t)h * total_kv + k0 + j];
            p[j].j = (int32_t)j;
        }
        qsort(p, (size_t)L, sizeof(scored_pos), by_score_then_pos);
        qsort(p, (size_t)kb, sizeof(scored_pos), by_pos);
        for (int64_t t = 0; t < kb; ++t)
            idx_out[(int64_t)h * total_k + o0 + t] = p[t].j;
        free(p);
    }
    return failed ? ORACLE_NO_MEM : ORACLE_OK;
}

/* score + top-k in one call (what the library's selection entry point computes) */
int oracle_select(int dtype, int B, int Hq, int Hkv, int D,
                  const void *q, const void *k,
                  const int32_t *cu_q, const int32_t *cu_kv, const int32_t *cu_k,
                  int pool_w, int32_t *idx_out)
{
    int rc = check_common(dtype, B, Hq, Hkv, D, cu_q, cu_kv);
    if (rc) return rc;
    const int64_t total_kv = cu_kv[B];
    float *s = (float *)malloc(sizeof(float) * (size_t)(total_kv > 0 ? total_kv : 1) * (size_t)Hq);
    if (!s) return ORACLE_NO_MEM;
    rc = oracle_score(dtype, B, Hq, Hkv, D, q, k, cu_q, cu_kv, pool_w, s, NULL);
    if (!rc) rc = oracle_topk(B, Hq, s, cu_kv, cu_k, idx_out);
    free(s);
    return rc;
}

/* Selection variants.
 *
 * forced_tail = n > 0: Section 2.3 Eq. (4) attends over [K_b; K_cache], the active block's own keys
 * and values beside the cache.  With the block stored as the last n positions of the sequence, those
 * n positions are always kept and never ranked; the k_b - n best of the candidates 0 .. L_b-n-1 are
 * chosen as usual (the pooling window is clipped to the candidates) and the n block positions are
 * appended, so the list stays ascending.
 *
 * head_sum != 0: the shared selection of Section 2.4 Eq. (5): the pooled per-head scores are summed
 * over the query heads (fp32, ascending head, starting from +0), one TopK per sequence is taken, and
 * every head gets the same list.
 */
int oracle_select_ex(int dtype, int B, int Hq, int Hkv, int D,
                     const void *q, const void *k,
                     const int32_t *cu_q, const int32_t *cu_kv, const int32_t *cu_k,
                     int pool_w, int forced_tail, int head_sum, int32_t *idx_out)
{
    int rc = check_common(dtype, B, Hq, Hkv, D, cu_q, cu_kv);
    if (rc) return rc;
    if (pool_w < 1 || pool_w % 2 == 0 || forced_tail < 0 || !cu_k || !idx_out) return ORACLE_BAD_ARG;
    if (cu_k[0] != 0) return ORACLE_BAD_ARG;
    for (int b = 0; b < B; ++b) {
        const int64_t L = cu_kv[b + 1] - cu_kv[b], kb = cu_k[b + 1] - cu_k[b];
        if (kb < 0 || kb > L) return ORACLE_BAD_ARG;
        if (kb > 0 && (kb < forced_tail || L < forced_tail)) return ORACLE_BAD_ARG;
    }
    const int64_t total_kv = cu_kv[B], total_k = cu_k[B];
    const int half = pool_w / 2;
    float *raw = (float *)malloc(sizeof(float) * (size_t)(total_kv > 0 ? total_kv : 1) * (size_t)Hq);
    if (!raw) return ORACLE_NO_MEM;
    rc = oracle_score(dtype, B, Hq, Hkv, D, q, k, cu_q, cu_kv, 1, raw, NULL);   /* unpooled Eq. (6) scores */
    if (rc) { free(raw); return rc; }

    for (int b = 0; b < B; ++b) {
        const int64_t k0 = cu_kv[b], L = cu_kv[b + 1] - cu_kv[b];
        const int64_t o0 = cu_k[b], kb = cu_k[b + 1] - cu_k[b];
        if (kb == 0) continue;
        const int64_t Lc = L - forced_tail, kc = kb - forced_tail;   /* candidates, and how many of them are kept */
        float *pooled = (float *)malloc(sizeof(float) * (size_t)(Lc > 0 ? Lc : 1) * (size_t)Hq);
        scored_pos *p = (scored_pos *)malloc(sizeof(scored_pos) * (size_t)(Lc > 0 ? Lc : 1));
        if (!pooled || !p) { free(pooled); free(p); free(raw); return ORACLE_NO_MEM; }
        for (int h = 0; h < Hq; ++h)
            for (int64_t j = 0; j < Lc; ++j) {
                int64_t lo = j - half < 0 ? 0 : j - half;
                int64_t hi = j + half > Lc - 1 ? Lc - 1 : j + half;
                float m = raw[(int64_t)h * total_kv + k0 + lo];
                for (int64_t t = lo + 1; t <= hi; ++t)
                    if (raw[(int64_t)h * total_kv + k0 + t] > m) m = raw[(int64_t)h * total_kv + k0 + t];
                pooled[(int64_t)h * Lc + j] = m;
            }
        const int lists = head_sum ? 1 : Hq;
        for (int li = 0; li < lists; ++li) {
            for (int64_t j = 0; j < Lc; ++j) {
                float sc;
                if (head_sum) {
                    sc = 0.0f;
                    for (int h = 0; h < Hq; ++h) sc = sc + pooled[(int64_t)h * Lc + j];
                } else {
                    sc = pooled[(int64_t)li * Lc + j];
                }
                p[j].s = sc;
                p[j].j = (int32_t)j;
            }
            qsort(p, (size_t)Lc, sizeof(scored_pos), by_score_then_pos);
            qsort(p, (size_t)kc, sizeof(scored_pos), by_pos);
            for (int h = head_sum ? 0 : li; h < (head_sum ? Hq : li + 1); ++h) {
                for (int64_t t = 0; t < kc; ++t) idx_out[(int64_t)h * total_k + o0 + t] = p[t].j;
                for (int64_t t = 0; t < forced_tail; ++t)
                    idx_out[(int64_t)h * total_k + o0 + kc + t] = (int32_t)(Lc + t);
            }
        }
        free(pooled); free(p);
    }
    free(raw);
    return ORACLE_OK;
}


/* Eq. (4) over each head's kept rows (seq_mode[b] == 0, rows idx[h, cu_k[b] .. cu_k[b+1]))
 * and Eq. (3) over all rows (seq_mode[b] == 1); seq_mode NULL means all sparse.
 * o_out [total_q, Hq, D] in fp64. */
int oracle_attend(int dtype, int B, int Hq, int Hkv, int D,
                  const void *q, const void *k, const void *v,
                  const int32_t *cu_q, const int32_t *cu_kv,
                  const int32_t *idx, const int32_t *cu_k, const uint8_t *seq_mode,
                  double softmax_scale, double *o_out)
{
    int rc = check_common(dtype, B, Hq, Hkv, D, cu_q, cu_kv);
    if (rc) return rc;
    if (!o_out) return ORACLE_BAD_ARG;
    int any_sparse = 0;
    for (int b = 0; b < B; ++b)
        if (!seq_mode || seq_mode[b] == 0) any_sparse = 1;
    if (any_sparse && (!idx || !cu_k)) return ORACLE_BAD_ARG;
    const int G = Hq / Hkv;
    const int64_t total_q = cu_q[B];
    const int64_t total_k = cu_k ? cu_k[B] : 0;
    int failed = 0;

    /* validate indices before computing anything */
    for (int b = 0; b < B; ++b) {
        if (seq_mode && seq_mode[b] != 0) {
            if (seq_mode[b] != 1) return ORACLE_BAD_ARG;
            continue;
        }
        const int64_t L = cu_kv[b + 1] - cu_kv[b];
        for (int h = 0; h < Hq; ++h)
            for (int64_t t = cu_k[b]; t < cu_k[b + 1]; ++t) {
                int32_t j = idx[(int64_t)h * total_k + t];
                if (j < 0 || j >= L) return ORACLE_BAD_ARG;
            }
    }

#pragma omp parallel for schedule(dynamic)
    for (int64_t rh = 0; rh < total_q * Hq; ++rh) {
        const int64_t row = rh / Hq;
        const int h = (int)(rh % Hq), g = h / G;
        int b = 0;
        while (cu_q[b + 1] <= row) ++b;
        const int dense = seq_mode && seq_mode[b] == 1;
        const int64_t k0 = cu_kv[b], L = cu_kv[b + 1] - cu_kv[b];
        const int64_t n = dense ? L : (int64_t)(cu_k[b + 1] - cu_k[b]);
        double *out = o_out + (row * Hq + h) * D;
        if (n == 0) {                      /* nothing to attend to: defined as zero */
            for (int d = 0; d < D; ++d) out[d] = 0.0;
            continue;
        }
        double *z = (double *)malloc(sizeof(double) * (size_t)n);
        if (!z) { failed = 1; continue; }
        const int64_t qrow = (row * Hq + h) * D;
        double zmax = -INFINITY;
        for (int64_t t = 0; t < n; ++t) {
            const int64_t j = dense ? t : (int64_t)idx[(int64_t)h * total_k + cu_k[b] + t];
            const int64_t krow = ((k0 + j) * Hkv + g) * D;
            double dot = 0.0;
            for (int d = 0; d < D; ++d)
                dot += (double)widen(q, dtype, qrow + d) * (double)widen(k, dtype, krow + d);
            z[t] = softmax_scale * dot;
            if (z[t] > zmax) zmax = z[t];
        }
        double denom = 0.0;
        for (int d = 0; d < D; ++d) out[d] = 0.0;
        for (int64_t t = 0; t < n; ++t) {
            const int64_t j = dense ? t : (int64_t)idx[(int64_t)h * total_k + cu_k[b] + t];
            const int64_t vrow = ((k0 + j) * Hkv + g) * D;
            const double p = exp(z[t] - zmax);
            denom += p;
            for (int d = 0; d < D; ++d)
                out[d] += p * (double)widen(v, dtype, vrow + d);
        }
        for (int d = 0; d < D; ++d) out[d] /= denom;
        free(z);
    }
    return failed ? ORACLE_NO_MEM : ORACLE_OK;
}
