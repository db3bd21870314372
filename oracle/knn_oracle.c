/*
 * knn_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, obviously-correct CPU statement of what exact brute-force
 * k-nearest-neighbour search computes.  It exists only so that tests, the
 * smoke check and the benchmark's CPU-baseline leg have something independent
 * to compare the GPU library against.  It shares no code, header, table or
 * helper with the GPU path and nothing in the product may call it.
 *
 * What it computes (paper, Sect. 3 "Description of the problem"):
 *   for every query vector q_i, the k reference indices j_1..j_k whose
 *   distances delta(q_i, r_j) are the k smallest, listed in non-decreasing
 *   order of distance, such that every reference left out is at least as far
 *   as the k-th one listed.
 * The method of the paper is brute force and reaches exactly this result, so
 * the oracle is the definition written out: all nr distances of a row, a full
 * sort of the row, the first k entries.
 *
 * Readings of the paper that this file fixes:
 *   - delta is evaluated as the coordinate-by-coordinate fold of Sect. 3
 *     ("cumulatively computable"): a_1 = initial value,
 *     a_{c+1} = dbar(u_c, v_c, a_c), delta = a_{d+1}.  The paper's recurrence
 *     writes n where the coordinate count d is meant.
 *   - a vector is never its own neighbour: the algorithm of Sect. 4 only ever
 *     evaluates delta(v_x, v_y) for x > y, so the pair (i, i) is never pushed
 *     to a heap.  Exclusion is by index; a different row with identical
 *     coordinates is a legitimate neighbour at distance 0.
 *   - the paper accepts any resolution of ties (its conditions use <=); this
 *     oracle resolves them by the lower reference index so that the answer is
 *     unique.
 *   - indices are 0-based (the paper counts from 1).
 *   - all arithmetic is IEEE double on the exact fp32 input values.
 *
 * Distances (metric argument):
 *   0  squared Euclidean   sum_c (u_c - v_c)^2           (direct differences)
 *   1  cosine distance     1 - (u.v) / (|u| |v|);  1 if either vector is zero
 *   2  squared Hellinger   sum_c (sqrt(u_c) - sqrt(v_c))^2   (Sect. 7, Eq. 1;
 *      the printed formula lacks the square, without which it would not be
 *      symmetric as Sect. 3 requires).  Inputs must be >= 0.
 * Further cumulatively computable distances in the sense of Sect. 3 (the paper
 * asks only that delta be such a fold; it names Kullback-Leibler as the distance
 * of the work it compares with, Sect. 2, and notes in Sect. 3 that a distance
 * that is not symmetric needs both orders of every pair):
 *   3  Manhattan (L1)      dbar(u, v, a) = a + |u - v|
 *   4  Chebyshev (L-inf)   dbar(u, v, a) = max(a, |u - v|)
 *   5  Kullback-Leibler    dbar(u, v, a) = a + u ln(u / v), a term with u = 0
 *      counting 0; delta(q, r) takes the QUERY as the first argument, so it is
 *      not symmetric.  Inputs must be >= 0 and references > 0 wherever the
 *      query is > 0 (no normalisation is applied or required).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    double dist;
    int32_t idx;
} pair_t;

/* Order of Sect. 3's output list, made total: distance first, index second. */
static int pair_less(const void *pa, const void *pb)
{
    const pair_t *a = (const pair_t *)pa;
    const pair_t *b = (const pair_t *)pb;
    if (a->dist < b->dist) return -1;
    if (a->dist > b->dist) return 1;
    if (a->idx < b->idx) return -1;
    if (a->idx > b->idx) return 1;
    return 0;
}

/* delta(u, v) as the fold a_{c+1} = dbar(u_c, v_c, a_c) of Sect. 3. */
static double delta(const float *u, const float *v, int32_t d, int metric)
{
    if (metric == 0) {
        double a = 0.0;
        for (int32_t c = 0; c < d; ++c) {
            double t = (double)u[c] - (double)v[c];
            a = a + t * t;
        }
        return a;
    }
    if (metric == 1) {
        double uv = 0.0, uu = 0.0, vv = 0.0;
        for (int32_t c = 0; c < d; ++c) {
            double x = (double)u[c], y = (double)v[c];
            uv = uv + x * y;
            uu = uu + x * x;
            vv = vv + y * y;
        }
        if (uu == 0.0 || vv == 0.0) return 1.0;
        return 1.0 - uv / (sqrt(uu) * sqrt(vv));
    }
    if (metric == 2) {
        double a = 0.0;
        for (int32_t c = 0; c < d; ++c) {
            double t = sqrt((double)u[c]) - sqrt((double)v[c]);
            a = a + t * t;
        }
        return a;
    }
    if (metric == 3) {
        double a = 0.0;
        for (int32_t c = 0; c < d; ++c) a = a + fabs((double)u[c] - (double)v[c]);
        return a;
    }
    if (metric == 4) {
        double a = 0.0;
        for (int32_t c = 0; c < d; ++c) {
            double t = fabs((double)u[c] - (double)v[c]);
            if (t > a) a = t;
        }
        return a;
    }
    /* metric == 5 */
    {
        double a = 0.0;
        for (int32_t c = 0; c < d; ++c) {
            double x = (double)u[c], y = (double)v[c];
            if (x > 0.0) a = a + x * log(x / y);
        }
        return a;
    }
}

/* One distance, exported so the comparator can price any (query, reference). */
double knn_oracle_delta(const float *u, const float *v, int32_t d, int32_t metric)
{
    return delta(u, v, d, metric);
}

/*
 * Distances of given (query, reference) pairs: out[i, r] = delta(Q[i], R[idx[i, r]]).
 * Used by the comparator to price whatever neighbour list it is handed.
 * An index outside [0, nr) yields NaN.
 */
int32_t knn_oracle_pair_dists(const float *Q, int64_t nq, const float *R, int64_t nr,
                              int32_t d, int32_t k, int32_t metric,
                              const int32_t *idx, double *out)
{
    if (!Q || !R || !idx || !out) return 1;
    if (nq < 1 || nr < 1 || d < 1 || k < 1) return 1;
    if (metric < 0 || metric > 5) return 1;
    for (int64_t i = 0; i < nq; ++i) {
        for (int32_t r = 0; r < k; ++r) {
            int64_t j = idx[(size_t)i * (size_t)k + (size_t)r];
            out[(size_t)i * (size_t)k + (size_t)r] =
                (j < 0 || j >= nr) ? NAN
                                   : delta(Q + (size_t)i * (size_t)d, R + (size_t)j * (size_t)d, d, metric);
        }
    }
    return 0;
}

/*
 * Batched partial sort (paper, Sect. 6 "Phase 2: taking k smallest elements", and its
 * closing remark in Sect. 8 that the simultaneous partial sort of many arrays matters on
 * its own): for every row of A[m, n] (row stride lda), the k smallest entries in
 * non-decreasing order with their column numbers, ties to the lower column.
 * Written as the definition: full sort of the row by (value, column), first k.
 */
int32_t knn_oracle_select(const float *A, int64_t m, int64_t n, int64_t lda, int32_t k,
                          int32_t *idx, float *val)
{
    if (!A || !idx || !val) return 1;
    if (m < 1 || n < 1 || lda < n || k < 1 || k > n) return 1;
    if (n > (int64_t)INT32_MAX) return 1;
    int32_t failed = 0;
#pragma omp parallel
    {
        pair_t *row = (pair_t *)malloc((size_t)n * sizeof(pair_t));
        if (!row) {
#pragma omp atomic write
            failed = 2;
        }
#pragma omp for schedule(dynamic, 1)
        for (int64_t i = 0; i < m; ++i) {
            if (!row) continue;
            for (int64_t j = 0; j < n; ++j) {
                row[j].dist = (double)A[(size_t)i * (size_t)lda + (size_t)j];
                row[j].idx = (int32_t)j;
            }
            qsort(row, (size_t)n, sizeof(pair_t), pair_less);
            for (int32_t r = 0; r < k; ++r) {
                idx[(size_t)i * (size_t)k + (size_t)r] = row[r].idx;
                val[(size_t)i * (size_t)k + (size_t)r] = (float)row[r].dist;
            }
        }
        free(row);
    }
    return failed;
}

int32_t knn_oracle_threads(void)
{
#ifdef _OPENMP
    return (int32_t)omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Q[nq, d], R[nr, d]: row-major fp32 on the host.
 * self_idx[nq]: reference index that IS query i and must be skipped, or -1.
 *               May be NULL (nothing skipped).
 * idx[nq, k], dist[nq, k]: outputs, ascending by (dist, idx).
 * next_dist[nq]: distance of the (k+1)-th entry of the sorted row, +inf if the
 *               row has only k candidates.  May be NULL.
 * Returns 0 on success, 1 on bad arguments, 2 if memory ran out.
 */
int32_t knn_oracle_search(const float *Q, int64_t nq, const float *R, int64_t nr,
                          int32_t d, int32_t k, int32_t metric,
                          const int64_t *self_idx,
                          int32_t *idx, double *dist, double *next_dist)
{
    if (!Q || !R || !idx || !dist) return 1;
    if (nq < 1 || nr < 1 || d < 1 || k < 1) return 1;
    if (metric < 0 || metric > 5) return 1;
    if (nr > (int64_t)INT32_MAX) return 1;
    int32_t failed = 0;

#pragma omp parallel
    {
        pair_t *row = (pair_t *)malloc((size_t)nr * sizeof(pair_t));
        if (!row) {
#pragma omp atomic write
            failed = 2;
        }
#pragma omp for schedule(dynamic, 1)
        for (int64_t i = 0; i < nq; ++i) {
            if (!row) continue;
            const float *q = Q + (size_t)i * (size_t)d;
            int64_t self = self_idx ? self_idx[i] : -1;
            int64_t m = 0;
            for (int64_t j = 0; j < nr; ++j) {
                if (j == self) continue;
                row[m].dist = delta(q, R + (size_t)j * (size_t)d, d, metric);
                row[m].idx = (int32_t)j;
                ++m;
            }
            if (m < (int64_t)k) {
#pragma omp atomic write
                failed = 1;
                continue;
            }
            qsort(row, (size_t)m, sizeof(pair_t), pair_less);
            for (int32_t r = 0; r < k; ++r) {
                idx[(size_t)i * (size_t)k + (size_t)r] = row[r].idx;
                dist[(size_t)i * (size_t)k + (size_t)r] = row[r].dist;
            }
            if (next_dist) next_dist[i] = (m > (int64_t)k) ? row[k].dist : INFINITY;
        }
        free(row);
    }
    return failed;
}
