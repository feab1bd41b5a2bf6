/*
 * CPU oracle for batched IVF-Flat top-k search.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, query-major implementation of what the retrieval stage of the
 * paper computes (Section 2.2: similarity between a query and the stored
 * vectors, top-k nearest returned; the IVF index restricts the search to the
 * nprobe clusters whose centroids are closest to the query; Section 4.4: the
 * partial results of a request are merged into one top-k).  The paper gives the
 * method only in prose; the cluster-major schedule of the GPU path changes the
 * order of the work, not the answer, so the oracle is the textbook definition
 * written out.  Every score is accumulated in double, index ascending.
 *
 * Only tests, the smoke check and the cpu_baseline leg of the benchmark may use
 * this file.  It shares no code with the HIP path.
 *
 * Conventions (all are readings of points the paper leaves open):
 *   metric 0 = inner product, larger is better (the paper's "cosine similarity"
 *              on vectors the caller has normalised);
 *   metric 1 = squared L2 distance (no square root), smaller is better,
 *              computed in the direct form sum (q_i - x_i)^2;
 *   the coarse step uses the same metric as the fine step;
 *   ties: lower centroid index first (coarse), lower id first (fine);
 *   fewer than k candidates: ids padded with -1, scores with -inf (IP) or
 *   +inf (L2);
 *   dtype 0 = float32, 1 = IEEE binary16, 2 = bfloat16 storage of the database
 *   rows; a stored value is converted exactly to double.  Queries and
 *   centroids are float32.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_IP = 0, ORACLE_L2 = 1 };
enum { ORACLE_F32 = 0, ORACLE_F16 = 1, ORACLE_BF16 = 2 };

/* exact binary16 -> double */
static double half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int exp = (h >> 10) & 0x1f;
    int man = h & 0x3ff;
    double v;
    if (exp == 0)
        v = ldexp((double)man, -24);               /* subnormal: man * 2^-24 */
    else if (exp == 31)
        v = man ? NAN : INFINITY;
    else
        v = ldexp((double)(man | 0x400), exp - 25); /* (1024+man) * 2^(exp-25) */
    return sign ? -v : v;
}

/* exact bfloat16 -> double: a bfloat16 is the upper half of a float32 */
static double bf16_to_double(uint16_t b)
{
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static inline double stored_value(const void *base, int dtype, int64_t idx)
{
    switch (dtype) {
    case ORACLE_F32: return (double)((const float *)base)[idx];
    case ORACLE_F16: return half_to_double(((const uint16_t *)base)[idx]);
    default:         return bf16_to_double(((const uint16_t *)base)[idx]);
    }
}

/* score of one (query, stored row) pair */
static double pair_score(const float *q, const void *rows, int dtype, int64_t row,
                         int d, int metric)
{
    double acc = 0.0;
    int64_t base = row * (int64_t)d;
    if (metric == ORACLE_IP) {
        for (int i = 0; i < d; i++)
            acc += (double)q[i] * stored_value(rows, dtype, base + i);
    } else {
        for (int i = 0; i < d; i++) {
            double t = (double)q[i] - stored_value(rows, dtype, base + i);
            acc += t * t;
        }
    }
    return acc;
}

/* is candidate (s1,id1) strictly better than (s2,id2)? */
static inline int better(double s1, int64_t id1, double s2, int64_t id2, int metric)
{
    if (s1 != s2)
        return metric == ORACLE_IP ? (s1 > s2) : (s1 < s2);
    return id1 < id2;
}

/* sorted best-first list of at most k entries; insert by shifting */
typedef struct {
    int k, n, metric;
    double *s;
    int64_t *id;
} topk_t;

static void topk_push(topk_t *t, double s, int64_t id)
{
    if (t->n == t->k && !better(s, id, t->s[t->k - 1], t->id[t->k - 1], t->metric))
        return;
    int pos = (t->n < t->k) ? t->n : t->k - 1;
    while (pos > 0 && better(s, id, t->s[pos - 1], t->id[pos - 1], t->metric)) {
        t->s[pos] = t->s[pos - 1];
        t->id[pos] = t->id[pos - 1];
        pos--;
    }
    t->s[pos] = s;
    t->id[pos] = id;
    if (t->n < t->k)
        t->n++;
}

static void topk_emit(const topk_t *t, int64_t *out_ids, double *out_scores)
{
    double pad = (t->metric == ORACLE_IP) ? -INFINITY : INFINITY;
    for (int j = 0; j < t->k; j++) {
        out_ids[j] = (j < t->n) ? t->id[j] : -1;
        out_scores[j] = (j < t->n) ? t->s[j] : pad;
    }
}

/* number of threads the query loops use from now on (for timing the oracle on one core); no arithmetic changes */
void oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Coarse step (Section 2.2: the choice of the clusters whose centroids are closest to the query).
 * out_probe[q*nprobe + r] = index of the r-th best centroid for query q,
 * out_scores likewise (double).  Returns 0, or -1 on bad arguments.
 */
int oracle_coarse(const float *queries, int64_t nq, const float *centroids, int64_t nlist,
                  int d, int metric, int nprobe, int32_t *out_probe, double *out_scores)
{
    if (!queries || !centroids || !out_probe || nq < 0 || nlist < 1 || d < 1 ||
        nprobe < 1 || nprobe > nlist || (metric != ORACLE_IP && metric != ORACLE_L2))
        return -1;
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t q = 0; q < nq; q++) {
        topk_t t = { nprobe, 0, metric, malloc(sizeof(double) * nprobe),
                     malloc(sizeof(int64_t) * nprobe) };
        int64_t *ids = malloc(sizeof(int64_t) * nprobe);
        double *sc = malloc(sizeof(double) * nprobe);
        if (!t.s || !t.id || !ids || !sc) {
            fail = 1;
        } else {
            const float *qv = queries + q * (int64_t)d;
            for (int64_t j = 0; j < nlist; j++)
                topk_push(&t, pair_score(qv, centroids, ORACLE_F32, j, d, metric), j);
            topk_emit(&t, ids, sc);
            for (int r = 0; r < nprobe; r++) {
                out_probe[q * nprobe + r] = (int32_t)ids[r];
                if (out_scores)
                    out_scores[q * nprobe + r] = sc[r];
            }
        }
        free(t.s); free(t.id); free(ids); free(sc);
    }
    return fail ? -2 : 0;
}

/*
 * Fine step with the probe lists given: for each query scan every row of every
 * probed list (Section 2.2: the search is restricted to the selected clusters),
 * keep the k best (Section 4.4: per-request merge).  probe[q*nprobe + r] < 0
 * means "no list in this position" and is skipped.
 * list l holds rows offsets[l] .. offsets[l+1]-1 of `vectors`; ids[row] is the
 * label reported for that row.
 */
int oracle_scan(const float *queries, int64_t nq, int d, const int64_t *offsets, int64_t nlist,
                const void *vectors, int dtype, const int64_t *ids, const int32_t *probe,
                int nprobe, int k, int metric, int64_t *out_ids, double *out_scores)
{
    if (!queries || !offsets || !vectors || !ids || !probe || !out_ids || !out_scores ||
        nq < 0 || d < 1 || nprobe < 1 || k < 1 || dtype < 0 || dtype > 2 ||
        (metric != ORACLE_IP && metric != ORACLE_L2))
        return -1;
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t q = 0; q < nq; q++) {
        topk_t t = { k, 0, metric, malloc(sizeof(double) * k), malloc(sizeof(int64_t) * k) };
        if (!t.s || !t.id) {
            fail = 1;
        } else {
            const float *qv = queries + q * (int64_t)d;
            for (int r = 0; r < nprobe; r++) {
                int32_t l = probe[q * nprobe + r];
                if (l < 0 || l >= nlist)
                    continue;
                for (int64_t row = offsets[l]; row < offsets[l + 1]; row++)
                    topk_push(&t, pair_score(qv, vectors, dtype, row, d, metric), ids[row]);
            }
            topk_emit(&t, out_ids + q * k, out_scores + q * k);
        }
        free(t.s); free(t.id);
    }
    return fail ? -2 : 0;
}

/* Whole search = coarse step, then fine step on the lists it selected. */
int oracle_ivf_search(const float *queries, int64_t nq, int d, const float *centroids,
                      const int64_t *offsets, int64_t nlist, const void *vectors, int dtype,
                      const int64_t *ids, int nprobe, int k, int metric,
                      int32_t *out_probe, int64_t *out_ids, double *out_scores)
{
    int rc = oracle_coarse(queries, nq, centroids, nlist, d, metric, nprobe, out_probe, NULL);
    if (rc)
        return rc;
    return oracle_scan(queries, nq, d, offsets, nlist, vectors, dtype, ids, out_probe, nprobe, k,
                       metric, out_ids, out_scores);
}

/* Exact search: every one of the n stored rows is a candidate (no index). */
int oracle_bruteforce(const float *queries, int64_t nq, int d, const void *vectors, int dtype,
                      const int64_t *ids, int64_t n, int k, int metric, int64_t *out_ids,
                      double *out_scores)
{
    if (!queries || !vectors || !ids || !out_ids || !out_scores || nq < 0 || d < 1 || n < 0 ||
        k < 1 || dtype < 0 || dtype > 2 || (metric != ORACLE_IP && metric != ORACLE_L2))
        return -1;
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t q = 0; q < nq; q++) {
        topk_t t = { k, 0, metric, malloc(sizeof(double) * k), malloc(sizeof(int64_t) * k) };
        if (!t.s || !t.id) {
            fail = 1;
        } else {
            const float *qv = queries + q * (int64_t)d;
            for (int64_t row = 0; row < n; row++)
                topk_push(&t, pair_score(qv, vectors, dtype, row, d, metric), ids[row]);
            topk_emit(&t, out_ids + q * k, out_scores + q * k);
        }
        free(t.s); free(t.id);
    }
    return fail ? -2 : 0;
}

/* Scores of n chosen (query, row) pairs: out[i] = score(queries[qidx[i]], row ridx[i]). */
int oracle_pair_scores(const float *queries, int d, const void *vectors, int dtype, int metric,
                       const int64_t *qidx, const int64_t *ridx, int64_t n, double *out)
{
    if (!queries || !vectors || !qidx || !ridx || !out || d < 1 || dtype < 0 || dtype > 2)
        return -1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; i++)
        out[i] = pair_score(queries + qidx[i] * (int64_t)d, vectors, dtype, ridx[i], d, metric);
    return 0;
}
