/*
 * CPU oracle for Lloyd's K-means -- TEST INFRASTRUCTURE, not product code.
 *
 * Only the test-suite, the smoke check and the benchmark's cpu_baseline leg may
 * call this file.  It shares no code with the HIP path and is deliberately
 * plain: every function is the textbook definition written out in float64,
 * with no blocking, fusion or algebraic rewriting.
 *
 *   assignment  : Section 2, Eq. (1)  -- nearest centroid in Euclidean norm;
 *                 the square root is dropped as Section 3.1.2 allows, and the
 *                 distance is evaluated in the direct-difference form of the
 *                 basic kernel of Section 3.1.1 (NOT the norm expansion of
 *                 Section 3.1.2, which is what the GPU path is checked for).
 *   update      : Section 2, Eq. (2)  -- mean of the points of each cluster.
 *   fit         : Section 2           -- alternate the two steps from Y^(0).
 *
 * Readings where the paper is silent: exact ties go to the lowest centroid
 * index; an empty cluster keeps its previous centroid; the loop runs a fixed
 * number of iterations; the initial centroids are K distinct data points.
 *
 * dtype: 0 = float32 storage, 1 = float64 storage.  Stored values are promoted
 * exactly to double; all arithmetic is double.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static inline double ld(int dtype, const void *p, int64_t i)
{
    return dtype == 0 ? (double)((const float *)p)[i] : ((const double *)p)[i];
}

/* Squared Euclidean distance between row i of X and row j of C, summed in
 * increasing feature index. */
static double sqdist(int dtype, const void *X, int64_t i, const void *C, int64_t j, int D)
{
    double s = 0.0;
    for (int d = 0; d < D; ++d) {
        double diff = ld(dtype, X, i * (int64_t)D + d) - ld(dtype, C, j * (int64_t)D + d);
        s += diff * diff;
    }
    return s;
}

/* Eq. (1) for the listed rows (rows == NULL: all rows 0..nrows-1).
 * labels[r]  = smallest j attaining the minimum distance,
 * best[r]    = that (squared) distance,
 * second[r]  = the smallest distance over the other centroids (+inf if K==1).
 */
int oracle_assign_rows(int dtype, const void *X, const void *C, const int64_t *rows,
                       int64_t nrows, int D, int K, int32_t *labels, double *best, double *second)
{
    if (nrows < 0 || D < 1 || K < 1) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < nrows; ++r) {
        int64_t i = rows ? rows[r] : r;
        double b = INFINITY, s = INFINITY;
        int32_t bj = 0;
        for (int j = 0; j < K; ++j) {
            double d = sqdist(dtype, X, i, C, j, D);
            if (d < b) {
                s = b;
                b = d;
                bj = j;
            } else if (d < s) {
                s = d;
            }
        }
        labels[r] = bj;
        if (best) best[r] = b;
        if (second) second[r] = s;
    }
    return 0;
}

int oracle_assign(int dtype, const void *X, const void *C, int64_t N, int D, int K,
                  int32_t *labels, double *best, double *second)
{
    return oracle_assign_rows(dtype, X, C, NULL, N, D, K, labels, best, second);
}

/* Eq. (2).  Sums run over points in increasing index; one rounding to the
 * storage dtype at the end.  C holds the previous centroids on entry (kept for
 * empty clusters) and the new ones on return.  The feature columns are
 * independent, so they are shared among threads; each column still adds its
 * points in increasing i. */
int oracle_update(int dtype, const void *X, const int32_t *labels, int64_t N, int D, int K,
                  void *C, int64_t *counts)
{
    if (N < 0 || D < 1 || K < 1) return 1;
    for (int64_t i = 0; i < N; ++i)
        if (labels[i] < 0 || labels[i] >= K) return 2;
    double *sum = (double *)calloc((size_t)K * D, sizeof(double));
    if (!sum) return 3;
    for (int j = 0; j < K; ++j) counts[j] = 0;
    for (int64_t i = 0; i < N; ++i) counts[labels[i]] += 1;
#pragma omp parallel for schedule(static)
    for (int d = 0; d < D; ++d)
        for (int64_t i = 0; i < N; ++i)
            sum[(int64_t)labels[i] * D + d] += ld(dtype, X, i * (int64_t)D + d);
    for (int j = 0; j < K; ++j) {
        if (counts[j] == 0) continue;
        for (int d = 0; d < D; ++d) {
            double m = sum[(int64_t)j * D + d] / (double)counts[j];
            if (dtype == 0)
                ((float *)C)[(int64_t)j * D + d] = (float)m;
            else
                ((double *)C)[(int64_t)j * D + d] = m;
        }
    }
    free(sum);
    return 0;
}

/* Lloyd iterations from the initial centroids already stored in C.
 * For t = 1..iters: labels_t = assign(X, C_{t-1}); J_t = sum of best distances;
 * C_t = update(X, labels_t).  On return C = C_iters, labels = labels_iters (taken
 * with respect to C_{iters-1}), counts likewise, inertia[t-1] = J_t.
 * C_hist (optional, iters*K*D entries of the storage dtype) receives C_1..C_iters
 * and labels_hist (optional, iters*N) receives labels_1..labels_iters. */
int oracle_fit(int dtype, const void *X, int64_t N, int D, int K, int iters, void *C,
               int32_t *labels, int64_t *counts, double *inertia, void *C_hist,
               int32_t *labels_hist)
{
    if (N < 1 || D < 1 || K < 1 || iters < 0) return 1;
    size_t esz = dtype == 0 ? sizeof(float) : sizeof(double);
    double *best = (double *)malloc((size_t)N * sizeof(double));
    if (!best) return 3;
    for (int t = 0; t < iters; ++t) {
        int rc = oracle_assign(dtype, X, C, N, D, K, labels, best, NULL);
        if (rc) { free(best); return rc; }
        double J = 0.0;
        for (int64_t i = 0; i < N; ++i) J += best[i];
        if (inertia) inertia[t] = J;
        rc = oracle_update(dtype, X, labels, N, D, K, C, counts);
        if (rc) { free(best); return rc; }
        if (C_hist) memcpy((char *)C_hist + (size_t)t * K * D * esz, C, (size_t)K * D * esz);
        if (labels_hist) memcpy(labels_hist + (size_t)t * N, labels, (size_t)N * sizeof(int32_t));
    }
    free(best);
    return 0;
}

/* ---- seeded choice of K distinct point indices ---------------------------
 * The paper does not say how Y^(0) is chosen; the workloads use K distinct data
 * points.  When the caller gives no explicit initial centroids, the index set is
 * drawn by Floyd's sampling algorithm driven by the SplitMix64 generator
 * (Steele, Lea, Flood 2014): for j = N-K .. N-1, t = next() mod (j+1); take t
 * unless already taken, else take j.  Indices are returned in order of
 * selection.  The HIP library implements the same published procedure on its
 * own. */
static uint64_t splitmix64_next(uint64_t *state)
{
    uint64_t z = (*state += 0x9E3779B97F4A7C15ULL);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

void oracle_splitmix64(uint64_t seed, int n, uint64_t *out)
{
    uint64_t s = seed;
    for (int i = 0; i < n; ++i) out[i] = splitmix64_next(&s);
}

int oracle_seeded_indices(uint64_t seed, int64_t N, int K, int64_t *idx)
{
    if (K < 1 || N < K) return 1;
    uint64_t s = seed;
    int n = 0;
    for (int64_t j = N - K; j < N; ++j) {
        int64_t t = (int64_t)(splitmix64_next(&s) % (uint64_t)(j + 1));
        int taken = 0;
        for (int q = 0; q < n; ++q)
            if (idx[q] == t) { taken = 1; break; }
        idx[n++] = taken ? j : t;
    }
    return 0;
}
