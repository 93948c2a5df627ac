/*
 * CPU oracle for batched IVF-Flat search.  TEST INFRASTRUCTURE ONLY: nothing on the
 * product path may call, link or load this file.  It shares no code with the HIP library.
 *
 * What it computes (the plain definition of exact IVF-Flat probing with a full list scan;
 * the paper, Sec. 3.2, fixes only the frame -- vectors resident, a per-request candidate
 * list merged unit by unit, a request finished when all its units are done, top-k returned,
 * Sec. 3.1 last paragraph -- and requires that batching leaves results unchanged):
 *
 *   1. coarse score of the query against every centroid j, in fp64 on the stored values:
 *        L2: a_j = sum_i (q_i - C_ji)^2        IP: a_j = sum_i q_i * C_ji
 *   2. probe set = the nprobe best centroids (L2 smallest, IP largest), ties -> smaller j
 *   3. candidates = union of the probed lists, every vector of every probed list
 *   4. score of each candidate x:  L2: sum_i (q_i - x_i)^2 (squared, difference form)
 *                                  IP: sum_i q_i * x_i
 *   5. order by (score best first, id ascending); return the first min(k, #candidates)
 *
 * All sums run i = 0..d-1 in order, in double.  fp16 inputs are widened bit by bit here.
 * No blocking, no pruning, no sharing of list reads between queries.
 *
 * Pins (tests marked "not gpu"): brute-force kNN when nprobe == nlist; a hand-computed 1-D
 * example with ties and short lists; integer-exact data against int64 arithmetic; the
 * unit-norm identity between L2 and IP; output invariants.  The k-means used to build an
 * index is not part of this file and is "parity unpinned" beyond the index checker.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORA_L2 = 0, ORA_IP = 1 };
enum { ORA_F32 = 0, ORA_F16 = 1 };

/* IEEE binary16 -> double, bit by bit (sign, 5-bit exponent, 10-bit fraction). */
static double half_bits_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int f = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)f, -24);                 /* subnormal: f * 2^-10 * 2^-14 */
    else if (e == 31)
        v = f ? NAN : INFINITY;
    else
        v = ldexp((double)(f + 1024), e - 25);     /* (1 + f/1024) * 2^(e-15) */
    return sign ? -v : v;
}

static inline double elem(const void *p, int dtype, size_t i)
{
    if (dtype == ORA_F32)
        return (double)((const float *)p)[i];
    return half_bits_to_double(((const uint16_t *)p)[i]);
}

/* widen one stored row (query or base vector) to double */
static void widen_row(const void *row, int dtype, uint32_t d, double *out)
{
    for (uint32_t i = 0; i < d; ++i)
        out[i] = elem(row, dtype, i);
}

static double score_dd(const double *q, const double *x, uint32_t d, int metric)
{
    double s = 0.0;
    if (metric == ORA_L2) {
        for (uint32_t i = 0; i < d; ++i) {
            double t = q[i] - x[i];
            s += t * t;
        }
    } else {
        for (uint32_t i = 0; i < d; ++i)
            s += q[i] * x[i];
    }
    return s;
}

/* "a is better than b" under the metric, id/index as the tie-break */
typedef struct {
    double score;
    int64_t id;
} cand_t;

static int cmp_l2(const void *pa, const void *pb)
{
    const cand_t *a = (const cand_t *)pa, *b = (const cand_t *)pb;
    if (a->score < b->score) return -1;
    if (a->score > b->score) return 1;
    return (a->id > b->id) - (a->id < b->id);
}

static int cmp_ip(const void *pa, const void *pb)
{
    const cand_t *a = (const cand_t *)pa, *b = (const cand_t *)pb;
    if (a->score > b->score) return -1;
    if (a->score < b->score) return 1;
    return (a->id > b->id) - (a->id < b->id);
}

/* Step 1: coarse scores of one query against all centroids (centroids are fp32 values). */
int ivf_oracle_coarse(const float *centroids, uint32_t nlist, uint32_t d,
                      const void *q, int dtype, int metric, double *scores_out)
{
    if (!centroids || !q || !scores_out || d == 0) return -1;
    double *qd = (double *)malloc(sizeof(double) * d);
    double *cd = (double *)malloc(sizeof(double) * d);
    if (!qd || !cd) { free(qd); free(cd); return -2; }
    widen_row(q, dtype, d, qd);
    for (uint32_t j = 0; j < nlist; ++j) {
        for (uint32_t i = 0; i < d; ++i) cd[i] = (double)centroids[(size_t)j * d + i];
        scores_out[j] = score_dd(qd, cd, d, metric);
    }
    free(qd); free(cd);
    return 0;
}

/* Step 2: the nprobe best centroids in rank order, ties -> smaller centroid number. */
int ivf_oracle_probe(const double *scores, uint32_t nlist, uint32_t nprobe, int metric,
                     uint32_t *probe_out)
{
    if (!scores || !probe_out || nprobe == 0 || nprobe > nlist) return -1;
    cand_t *c = (cand_t *)malloc(sizeof(cand_t) * nlist);
    if (!c) return -2;
    for (uint32_t j = 0; j < nlist; ++j) { c[j].score = scores[j]; c[j].id = j; }
    qsort(c, nlist, sizeof(cand_t), metric == ORA_L2 ? cmp_l2 : cmp_ip);
    for (uint32_t r = 0; r < nprobe; ++r) probe_out[r] = (uint32_t)c[r].id;
    free(c);
    return 0;
}

/* Steps 3-5 for a given probe set.  cand_ids/cand_scores (capacity cand_cap) receive ALL
 * candidates in final order when non-NULL; ids_out/dist_out receive the first k.
 * X is the base in its original row order; list_off/list_ids describe the partition. */
int ivf_oracle_scan(const void *X, int dtype, uint64_t n, uint32_t d,
                    const uint64_t *list_off, const int64_t *list_ids, uint32_t nlist,
                    const uint32_t *probe, uint32_t nprobe,
                    const void *q, int metric, uint32_t k,
                    int64_t *ids_out, double *dist_out, uint32_t *n_out,
                    int64_t *cand_ids, double *cand_scores, uint64_t cand_cap, uint64_t *n_cand_out)
{
    if (!X || !list_off || !list_ids || !probe || !q || d == 0) return -1;
    size_t esz = dtype == ORA_F32 ? 4 : 2;
    uint64_t total = 0;
    for (uint32_t r = 0; r < nprobe; ++r) {
        if (probe[r] >= nlist) return -1;
        total += list_off[probe[r] + 1] - list_off[probe[r]];
    }
    cand_t *c = (cand_t *)malloc(sizeof(cand_t) * (total ? total : 1));
    double *qd = (double *)malloc(sizeof(double) * d);
    double *xd = (double *)malloc(sizeof(double) * d);
    if (!c || !qd || !xd) { free(c); free(qd); free(xd); return -2; }
    widen_row(q, dtype, d, qd);
    uint64_t m = 0;
    for (uint32_t r = 0; r < nprobe; ++r) {
        uint32_t l = probe[r];
        for (uint64_t p = list_off[l]; p < list_off[l + 1]; ++p) {
            int64_t id = list_ids[p];
            if (id < 0 || (uint64_t)id >= n) { free(c); free(qd); free(xd); return -3; }
            widen_row((const char *)X + (size_t)id * d * esz, dtype, d, xd);
            c[m].score = score_dd(qd, xd, d, metric);
            c[m].id = id;
            ++m;
        }
    }
    qsort(c, m, sizeof(cand_t), metric == ORA_L2 ? cmp_l2 : cmp_ip);
    uint32_t kk = (uint32_t)(m < k ? m : k);
    if (n_out) *n_out = kk;
    if (ids_out && dist_out) {
        for (uint32_t r = 0; r < kk; ++r) { ids_out[r] = c[r].id; dist_out[r] = c[r].score; }
        for (uint32_t r = kk; r < k; ++r) {
            ids_out[r] = -1;
            dist_out[r] = metric == ORA_L2 ? INFINITY : -INFINITY;
        }
    }
    if (n_cand_out) *n_cand_out = m;
    if (cand_ids && cand_scores) {
        uint64_t w = m < cand_cap ? m : cand_cap;
        for (uint64_t r = 0; r < w; ++r) { cand_ids[r] = c[r].id; cand_scores[r] = c[r].score; }
    }
    free(c); free(qd); free(xd);
    return 0;
}

/* Steps 1-5 for one query.  probe_out (nprobe entries) may be NULL. */
int ivf_oracle_search(const void *X, int dtype, uint64_t n, uint32_t d,
                      const float *centroids, uint32_t nlist,
                      const uint64_t *list_off, const int64_t *list_ids,
                      const void *q, uint32_t k, uint32_t nprobe, int metric,
                      uint32_t *probe_out, int64_t *ids_out, double *dist_out, uint32_t *n_out)
{
    if (nprobe == 0 || nprobe > nlist || k == 0) return -1;
    double *a = (double *)malloc(sizeof(double) * nlist);
    uint32_t *probe = (uint32_t *)malloc(sizeof(uint32_t) * nprobe);
    if (!a || !probe) { free(a); free(probe); return -2; }
    int rc = ivf_oracle_coarse(centroids, nlist, d, q, dtype, metric, a);
    if (!rc) rc = ivf_oracle_probe(a, nlist, nprobe, metric, probe);
    if (!rc) rc = ivf_oracle_scan(X, dtype, n, d, list_off, list_ids, nlist, probe, nprobe, q, metric, k,
                                  ids_out, dist_out, n_out, NULL, NULL, 0, NULL);
    if (!rc && probe_out) memcpy(probe_out, probe, sizeof(uint32_t) * nprobe);
    free(a); free(probe);
    return rc;
}

/* A batch of queries, each with its own k / nprobe / metric against ONE index; queries are
 * independent, so they are simply run one after another (OpenMP spreads them over cores).
 * Outputs are kmax / nprobe_max wide per query.  Returns the first non-zero status. */
int ivf_oracle_search_batch(const void *X, int dtype, uint64_t n, uint32_t d,
                            const float *centroids, uint32_t nlist,
                            const uint64_t *list_off, const int64_t *list_ids,
                            const void *queries, uint32_t nq,
                            const uint32_t *k, const uint32_t *nprobe, const uint32_t *metric,
                            uint32_t kmax, uint32_t nprobe_max,
                            uint32_t *probe_out, int64_t *ids_out, double *dist_out, uint32_t *n_out,
                            int *threads_used)
{
    size_t esz = dtype == ORA_F32 ? 4 : 2;
    int status = 0;
    int nthreads = 1;
#pragma omp parallel
    {
#pragma omp single
        {
#ifdef _OPENMP
            nthreads = omp_get_num_threads();
#endif
        }
#pragma omp for schedule(dynamic, 1)
        for (int64_t i = 0; i < (int64_t)nq; ++i) {
            if (k[i] > kmax || nprobe[i] > nprobe_max) {
#pragma omp critical
                status = status ? status : -1;
                continue;
            }
            /* per-query outputs are padded to kmax; the callee pads only up to k[i] */
            for (uint32_t r = 0; r < kmax; ++r) {
                ids_out[(size_t)i * kmax + r] = -1;
                dist_out[(size_t)i * kmax + r] = metric[i] == ORA_L2 ? INFINITY : -INFINITY;
            }
            int rc = ivf_oracle_search(X, dtype, n, d, centroids, nlist, list_off, list_ids,
                                       (const char *)queries + (size_t)i * d * esz,
                                       k[i], nprobe[i], (int)metric[i],
                                       probe_out ? probe_out + (size_t)i * nprobe_max : NULL,
                                       ids_out + (size_t)i * kmax, dist_out + (size_t)i * kmax,
                                       n_out + i);
            if (rc) {
#pragma omp critical
                status = status ? status : rc;
            }
        }
    }
    if (threads_used) *threads_used = nthreads;
    return status;
}

/* exposed so a test can pin the half conversion against numpy's own */
double ivf_oracle_half_to_double(uint16_t h) { return half_bits_to_double(h); }
