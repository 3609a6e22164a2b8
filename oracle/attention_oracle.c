/*
 * fp64 CPU oracle for attention of a short token segment over a long cached
 * context.  TEST INFRASTRUCTURE ONLY: nothing on the product path may call it.
 *
 * What it computes is the plain definition, one output row at a time:
 *
 *     out = softmax(q K^T / sqrt(d_k)) V                 (paper Sec. 3.2, Eq. 1)
 *
 * with K, V = the cached context (Sec. 3.2, Eq. 2: K_ctx, V_ctx), optionally
 * followed by a few "extra" keys that are not in the cache: the new chunk of a
 * data-plane append (Alg. 1: K.append(Forward(tokens, K))) or the ephemeral
 * Region-2 tokens of a query (Sec. 3.3; Sec. 3.9.3 "Extend" then "Clear").
 *
 * Deliberately naive: three passes per row (scores, exponentials, weighted sum),
 * everything in double, keys visited in ascending position, no tiling, no
 * running maximum, no splitting.  Inputs are either IEEE fp32 or bf16 (upper 16
 * bits of an fp32) and are widened to double exactly.
 *
 * Readings of the paper taken here (the paper does not fix them):
 *   - grouped-query attention: query head h reads KV head h / (Hq / Hkv);
 *   - which extra keys a row may see is given by the caller as a count of
 *     leading extra keys (vis[i]); causal masking is expressed through it;
 *   - natural exponential, log-sum-exp returned in natural-log units.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

static double widen(const void *base, int dtype, int64_t idx)
{
    if (dtype == ORACLE_F32) {
        return (double)((const float *)base)[idx];
    } else {
        uint32_t bits = ((uint32_t)((const uint16_t *)base)[idx]) << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    }
}

/*
 * One output row: query token i, query head h.
 *   q      [m][Hq][d]       query rows
 *   kc, vc [n][Hkv][d]      cached keys / values (may be NULL when n == 0)
 *   ke, ve [n_extra][Hkv][d] extra keys / values (may be NULL when n_vis == 0)
 *   n_vis  number of leading extra keys this row may see
 *   out    [d] doubles, *lse natural-log log-sum-exp of the scaled scores
 *   work   scratch of n + n_vis doubles
 * Returns 0, or -1 when the row has no visible key at all.
 */
static int one_row(int dtype, const void *q, int64_t i, int h,
                   const void *kc, const void *vc, int64_t n,
                   const void *ke, const void *ve, int64_t n_vis,
                   int Hq, int Hkv, int d, double scale,
                   double *out, double *lse, double *work)
{
    const int G = Hq / Hkv;
    const int g = h / G;
    const int64_t total = n + n_vis;
    if (total <= 0) return -1;

    const int64_t qoff = (i * Hq + h) * (int64_t)d;

    /* pass 1: scaled scores, ascending key position; running max */
    double mx = -INFINITY;
    for (int64_t j = 0; j < total; ++j) {
        const void *kb = (j < n) ? kc : ke;
        const int64_t jj = (j < n) ? j : j - n;
        const int64_t koff = (jj * Hkv + g) * (int64_t)d;
        double acc = 0.0;
        for (int t = 0; t < d; ++t)
            acc += widen(q, dtype, qoff + t) * widen(kb, dtype, koff + t);
        acc *= scale;
        work[j] = acc;
        if (acc > mx) mx = acc;
    }
    /* pass 2: exponentials and their sum */
    double l = 0.0;
    for (int64_t j = 0; j < total; ++j) {
        work[j] = exp(work[j] - mx);
        l += work[j];
    }
    /* pass 3: weighted sum of values, then normalise */
    for (int t = 0; t < d; ++t) out[t] = 0.0;
    for (int64_t j = 0; j < total; ++j) {
        const void *vb = (j < n) ? vc : ve;
        const int64_t jj = (j < n) ? j : j - n;
        const int64_t voff = (jj * Hkv + g) * (int64_t)d;
        const double p = work[j];
        for (int t = 0; t < d; ++t)
            out[t] += p * widen(vb, dtype, voff + t);
    }
    for (int t = 0; t < d; ++t) out[t] /= l;
    *lse = mx + log(l);
    return 0;
}

/*
 * All rows of a segment of m query tokens.
 *   vis [m]  number of leading extra keys visible to token i (NULL => 0 for all)
 *   out [m][Hq][d] doubles, lse [m][Hq] doubles
 * Returns 0, -1 if some row has no visible key (that row is left untouched),
 * -2 on bad arguments, -3 on allocation failure.
 */
int oracle_attention(int dtype, const void *q, int64_t m,
                     const void *kc, const void *vc, int64_t n,
                     const void *ke, const void *ve, int64_t n_extra,
                     const int64_t *vis,
                     int Hq, int Hkv, int d, double scale,
                     double *out, double *lse)
{
    if (Hq <= 0 || Hkv <= 0 || d <= 0 || Hq % Hkv != 0 || m < 0 || n < 0 || n_extra < 0)
        return -2;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return -2;
    int status = 0;
#pragma omp parallel
    {
        double *work = (double *)malloc(sizeof(double) * (size_t)(n + n_extra + 1));
        if (!work) {
#pragma omp critical
            status = -3;
        } else {
#pragma omp for collapse(2) schedule(dynamic, 1)
            for (int64_t i = 0; i < m; ++i) {
                for (int h = 0; h < Hq; ++h) {
                    int64_t nv = vis ? vis[i] : 0;
                    if (nv < 0 || nv > n_extra) {
#pragma omp critical
                        status = -2;
                        continue;
                    }
                    int rc = one_row(dtype, q, i, h, kc, vc, n, ke, ve, nv,
                                     Hq, Hkv, d, scale,
                                     out + (i * Hq + h) * (int64_t)d,
                                     lse + (i * Hq + h), work);
                    if (rc != 0) {
#pragma omp critical
                        if (status == 0) status = -1;
                    }
                }
            }
            free(work);
        }
    }
    return status;
}

/*
 * A chosen subset of rows: rows[r] = {token i, head h} pairs.
 *   out [n_rows][d] doubles, lse [n_rows] doubles
 * Used on full-size workloads where computing every row would take too long.
 */
int oracle_attention_rows(int dtype, const void *q, int64_t m,
                          const void *kc, const void *vc, int64_t n,
                          const void *ke, const void *ve, int64_t n_extra,
                          const int64_t *vis,
                          int Hq, int Hkv, int d, double scale,
                          const int64_t *rows, int64_t n_rows,
                          double *out, double *lse)
{
    if (Hq <= 0 || Hkv <= 0 || d <= 0 || Hq % Hkv != 0 || m < 0 || n < 0 || n_extra < 0)
        return -2;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return -2;
    for (int64_t r = 0; r < n_rows; ++r) {
        if (rows[2 * r] < 0 || rows[2 * r] >= m || rows[2 * r + 1] < 0 || rows[2 * r + 1] >= Hq)
            return -2;
    }
    int status = 0;
#pragma omp parallel
    {
        double *work = (double *)malloc(sizeof(double) * (size_t)(n + n_extra + 1));
        if (!work) {
#pragma omp critical
            status = -3;
        } else {
#pragma omp for schedule(dynamic, 1)
            for (int64_t r = 0; r < n_rows; ++r) {
                const int64_t i = rows[2 * r];
                const int h = (int)rows[2 * r + 1];
                int64_t nv = vis ? vis[i] : 0;
                if (nv < 0 || nv > n_extra) {
#pragma omp critical
                    status = -2;
                    continue;
                }
                int rc = one_row(dtype, q, i, h, kc, vc, n, ke, ve, nv,
                                 Hq, Hkv, d, scale, out + r * (int64_t)d, lse + r, work);
                if (rc != 0) {
#pragma omp critical
                    if (status == 0) status = -1;
                }
            }
            free(work);
        }
    }
    return status;
}

/* Threads the parallel regions above will use (reported by the benchmark). */
#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
#else
int oracle_num_threads(void) { return 1; }
#endif
