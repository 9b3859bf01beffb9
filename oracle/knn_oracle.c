/*
 * CPU oracle for exact brute-force k-nearest-neighbour search.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * GPU library is checked against.  Only tests, the smoke check and the
 * cpu_baseline leg of the benchmark may call it; the product path never does.
 * It shares no code, header, table or helper with the HIP library.
 *
 * What it computes (paper section 5.2, "K-Nearest Neighbours": a kNN query
 * selects the k closest data points to each query point; brute force forms the
 * pairwise distances between m queries and n points and takes the top k):
 *
 *     D[i][j] = sum_{t<d} (Q[i][t] - X[j][t])^2          (fp64, t ascending)
 *
 * evaluated in the naive "difference" form of section 4.1 (the left-hand side
 * of the identity sum (x-y)^2 = sum x^2 + y^2 - 2xy that the paper's
 * match-and-replace pass rewrites).  Row i of the result holds the k pairs
 * (D[i][j], j) that are smallest under the lexicographic order
 * (distance, index), listed ascending.  The paper does not say how equal
 * distances are ordered; the lower index wins here.
 *
 * Two selection routines are given and both are pinned by the CPU tests:
 *   oracle_knn_fullsort : the definition written out - all n distances, one
 *                         full sort by (distance, index), first k taken.
 *   oracle_knn          : same result by a bounded max-heap per row; this is
 *                         the one used at sizes where n full sorts are too slow.
 *
 * Pins (tests/test_oracle_pins.py): numpy brute force with a stable argsort on
 * tiny inputs for every k, closed forms (integer line, scaled orthogonal
 * basis), duplicated points, k=1 == argmin, k=n == stable argsort,
 * torch.cdist cross-check, the norm-expansion identity of section 4.1,
 * permutation and translation invariance, zero self-distance.
 *
 * Second metric (the cosine rows of the paper's kNN table, section 5.2 / appendix):
 *     C[i][j] = max(0, 1 - <q_i, x_j> / (|q_i| |x_j|)),   1 if either vector is zero,
 * with the three sums accumulated in fp64 in ascending t.  Same selection, same order.
 * Pins: numpy brute force, orthogonal and antipodal closed forms, exact invariance under
 * power-of-two scaling, agreement with the Euclidean oracle on unit-normalised data.
 *
 * Third metric (the L1 rows of the same table):
 *     M[i][j] = sum_t |q_it - x_jt|, fp64, ascending t.
 * Pins: numpy brute force (exact on integer grids), the integer line (distance |i - j|),
 * scipy's cityblock cdist, the norm inequalities L2 <= L1 <= sqrt(d) L2.
 *
 * Kernel matrix-vector product (paper section 5.1 and the appendix):
 *     y_i = sum_j k(x_i, z_j) v_j,   k(x, z) = variance * exp(-0.5 |x - z|^2 / lengthscale^2),
 * the squared-exponential kernel, distances in the difference form above, everything in
 * fp64, j ascending.  Pins: dense numpy K @ v, closed forms (one point, two points at a
 * known distance, huge lengthscale), symmetry v'(Kw) = w'(Kv), linearity in v.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC (no -ffast-math, no FMA contraction).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    double dist;
    int64_t idx;
} pair_t;

/* (distance, index) lexicographic "a comes before b". */
static int pair_before(const pair_t *a, const pair_t *b)
{
    if (a->dist < b->dist) return 1;
    if (a->dist > b->dist) return 0;
    return a->idx < b->idx;
}

static int pair_qsort_cmp(const void *pa, const void *pb)
{
    const pair_t *a = (const pair_t *)pa, *b = (const pair_t *)pb;
    if (pair_before(a, b)) return -1;
    if (pair_before(b, a)) return 1;
    return 0;
}

/* Squared Euclidean distance of one pair, naive difference form, fp64.
 * Section 4.1 (entries (x - y)^2 summed over the dimension). */
double oracle_sqdist(const float *q, const float *x, int32_t d)
{
    double acc = 0.0;
    for (int32_t t = 0; t < d; ++t) {
        double diff = (double)q[t] - (double)x[t];
        acc += diff * diff;
    }
    return acc;
}

/* Same distance through the expanded form of section 4.1,
 * sum x^2 + sum y^2 - 2 sum xy, in fp64.  Only used by the tests that check
 * the two forms against each other. */
double oracle_sqdist_expanded(const float *q, const float *x, int32_t d)
{
    double qq = 0.0, xx = 0.0, qx = 0.0;
    for (int32_t t = 0; t < d; ++t) {
        qq += (double)q[t] * (double)q[t];
        xx += (double)x[t] * (double)x[t];
        qx += (double)q[t] * (double)x[t];
    }
    return qq + xx - 2.0 * qx;
}

/* Cosine distance of one pair, fp64: 1 - <q,x> / (|q| |x|), clamped at 0; 1 for a zero vector. */
double oracle_cosdist(const float *q, const float *x, int32_t d)
{
    double qq = 0.0, xx = 0.0, qx = 0.0;
    for (int32_t t = 0; t < d; ++t) {
        qq += (double)q[t] * (double)q[t];
        xx += (double)x[t] * (double)x[t];
        qx += (double)q[t] * (double)x[t];
    }
    if (qq == 0.0 || xx == 0.0) return 1.0;
    double c = 1.0 - qx / (sqrt(qq) * sqrt(xx));
    return c < 0.0 ? 0.0 : c;
}

/* L1 (Manhattan) distance of one pair, fp64, ascending t. */
double oracle_l1dist(const float *q, const float *x, int32_t d)
{
    double acc = 0.0;
    for (int32_t t = 0; t < d; ++t) acc += fabs((double)q[t] - (double)x[t]);
    return acc;
}

#define ORACLE_METRIC_L2SQ 0
#define ORACLE_METRIC_COSINE 1
#define ORACLE_METRIC_L1 2

static double pair_distance(const float *q, const float *x, int32_t d, int32_t metric)
{
    if (metric == ORACLE_METRIC_COSINE) return oracle_cosdist(q, x, d);
    if (metric == ORACLE_METRIC_L1) return oracle_l1dist(q, x, d);
    return oracle_sqdist(q, x, d);
}

/* Max-heap on (distance, index): the root is the entry that comes LAST. */
static void heap_sift_down(pair_t *h, int64_t size, int64_t pos)
{
    for (;;) {
        int64_t l = 2 * pos + 1, r = l + 1, top = pos;
        if (l < size && pair_before(&h[top], &h[l])) top = l;
        if (r < size && pair_before(&h[top], &h[r])) top = r;
        if (top == pos) return;
        pair_t tmp = h[pos];
        h[pos] = h[top];
        h[top] = tmp;
        pos = top;
    }
}

static void heap_sift_up(pair_t *h, int64_t pos)
{
    while (pos > 0) {
        int64_t parent = (pos - 1) / 2;
        if (!pair_before(&h[parent], &h[pos])) return;
        pair_t tmp = h[pos];
        h[pos] = h[parent];
        h[parent] = tmp;
        pos = parent;
    }
}

/* One row, heap selection of the kk = min(k+1, n) first pairs. */
static void row_select_heap(const float *q, const float *X, int64_t ldx, int64_t n,
                            int32_t d, int64_t kk, pair_t *heap, int32_t metric)
{
    int64_t size = 0;
    for (int64_t j = 0; j < n; ++j) {
        pair_t cur;
        cur.dist = pair_distance(q, X + j * ldx, d, metric);
        cur.idx = j;
        if (size < kk) {
            heap[size] = cur;
            heap_sift_up(heap, size);
            ++size;
        } else if (pair_before(&cur, &heap[0])) {
            heap[0] = cur;
            heap_sift_down(heap, size, 0);
        }
    }
    qsort(heap, (size_t)size, sizeof(pair_t), pair_qsort_cmp);
}

/*
 * oracle_knn: rows[r] (r < nrows) names the query rows to evaluate; rows ==
 * NULL means rows 0..nrows-1.  Outputs are [nrows, k]: idx (int64), dist
 * (fp64).  next_dist[r] receives the (k+1)-th smallest distance of that row
 * (+inf when k == n) so that a caller can measure the gap behind the k-th
 * neighbour.  Returns 0, or -1 on bad arguments / allocation failure.
 */
int oracle_knn_metric(const float *Q, int64_t ldq, const float *X, int64_t ldx,
                      int64_t n, int32_t d, int32_t k,
                      const int64_t *rows, int64_t nrows,
                      int64_t *idx, double *dist, double *next_dist, int32_t nthreads,
                      int32_t metric)
{
    if (!Q || !X || !idx || !dist || n < 1 || d < 1 || k < 1 || k > n || nrows < 0 ||
        ldq < d || ldx < d)
        return -1;
    int64_t kk = (int64_t)k + 1 <= n ? (int64_t)k + 1 : n;
    int failed = 0;
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel num_threads(nthreads)
    {
        pair_t *heap = (pair_t *)malloc((size_t)kk * sizeof(pair_t));
        if (!heap) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (int64_t r = 0; r < nrows; ++r) {
            if (!heap) continue;
            int64_t i = rows ? rows[r] : r;
            row_select_heap(Q + i * ldq, X, ldx, n, d, kk, heap, metric);
            for (int32_t p = 0; p < k; ++p) {
                idx[r * k + p] = heap[p].idx;
                dist[r * k + p] = heap[p].dist;
            }
            if (next_dist) next_dist[r] = (kk > k) ? heap[k].dist : INFINITY;
        }
        free(heap);
    }
    return failed ? -1 : 0;
}

int oracle_knn(const float *Q, int64_t ldq, const float *X, int64_t ldx,
               int64_t n, int32_t d, int32_t k,
               const int64_t *rows, int64_t nrows,
               int64_t *idx, double *dist, double *next_dist, int32_t nthreads)
{
    return oracle_knn_metric(Q, ldq, X, ldx, n, d, k, rows, nrows, idx, dist, next_dist, nthreads,
                             ORACLE_METRIC_L2SQ);
}

/*
 * oracle_knn_fullsort: the definition written out.  For every requested row
 * all n (distance, index) pairs are formed, sorted once by (distance, index)
 * and the first k are reported.  Single-threaded, O(n log n) per row.
 */
int oracle_knn_fullsort_metric(const float *Q, int64_t ldq, const float *X, int64_t ldx,
                               int64_t n, int32_t d, int32_t k,
                               const int64_t *rows, int64_t nrows,
                               int64_t *idx, double *dist, double *next_dist, int32_t metric)
{
    if (!Q || !X || !idx || !dist || n < 1 || d < 1 || k < 1 || k > n || nrows < 0 ||
        ldq < d || ldx < d)
        return -1;
    pair_t *all = (pair_t *)malloc((size_t)n * sizeof(pair_t));
    if (!all) return -1;
    for (int64_t r = 0; r < nrows; ++r) {
        int64_t i = rows ? rows[r] : r;
        for (int64_t j = 0; j < n; ++j) {
            all[j].dist = pair_distance(Q + i * ldq, X + j * ldx, d, metric);
            all[j].idx = j;
        }
        qsort(all, (size_t)n, sizeof(pair_t), pair_qsort_cmp);
        for (int32_t p = 0; p < k; ++p) {
            idx[r * k + p] = all[p].idx;
            dist[r * k + p] = all[p].dist;
        }
        if (next_dist) next_dist[r] = (k < n) ? all[k].dist : INFINITY;
    }
    free(all);
    return 0;
}

int oracle_knn_fullsort(const float *Q, int64_t ldq, const float *X, int64_t ldx,
                        int64_t n, int32_t d, int32_t k,
                        const int64_t *rows, int64_t nrows,
                        int64_t *idx, double *dist, double *next_dist)
{
    return oracle_knn_fullsort_metric(Q, ldq, X, ldx, n, d, k, rows, nrows, idx, dist, next_dist,
                                      ORACLE_METRIC_L2SQ);
}

/*
 * oracle_kmv: y[i] = sum_j variance * exp(-0.5 * |X[i] - Z[j]|^2 / lengthscale^2) * v[j].
 * X [n, d], Z [m, d] fp32 row-major (leading dimensions in elements), v [m] fp32, y [n] fp64.
 * rows == NULL: all n rows; else y has nrows entries for the listed rows.
 */
int oracle_kmv(const float *X, int64_t ldx, const float *Z, int64_t ldz, const float *v,
               int64_t n, int64_t m, int32_t d, double variance, double lengthscale,
               const int64_t *rows, int64_t nrows, double *y, int32_t nthreads)
{
    if (!X || !Z || !v || !y || n < 0 || m < 0 || d < 1 || ldx < d || ldz < d || !(lengthscale > 0.0))
        return -1;
    if (nthreads < 1) nthreads = 1;
    const double inv = -0.5 / (lengthscale * lengthscale);
#pragma omp parallel for num_threads(nthreads) schedule(dynamic, 4)
    for (int64_t r = 0; r < nrows; ++r) {
        int64_t i = rows ? rows[r] : r;
        double acc = 0.0;
        for (int64_t j = 0; j < m; ++j)
            acc += variance * exp(inv * oracle_sqdist(X + i * ldx, Z + j * ldz, d)) * (double)v[j];
        y[r] = acc;
    }
    return 0;
}

/*
 * oracle_kmv_f64: the same product with fp64 inputs, the precision in which paper section
 * 5.1 evaluates it.  X [n, d], Z [m, d], v [m] fp64 row-major; everything in fp64, the
 * squared distance in difference form with t ascending, the sum with j ascending.
 */
int oracle_kmv_f64(const double *X, int64_t ldx, const double *Z, int64_t ldz, const double *v,
                   int64_t n, int64_t m, int32_t d, double variance, double lengthscale,
                   const int64_t *rows, int64_t nrows, double *y, int32_t nthreads)
{
    if (!X || !Z || !v || !y || n < 0 || m < 0 || d < 1 || ldx < d || ldz < d || !(lengthscale > 0.0))
        return -1;
    if (nthreads < 1) nthreads = 1;
    const double inv = -0.5 / (lengthscale * lengthscale);
#pragma omp parallel for num_threads(nthreads) schedule(dynamic, 4)
    for (int64_t r = 0; r < nrows; ++r) {
        int64_t i = rows ? rows[r] : r;
        const double *x = X + i * ldx;
        double acc = 0.0;
        for (int64_t j = 0; j < m; ++j) {
            const double *z = Z + j * ldz;
            double sq = 0.0;
            for (int32_t t = 0; t < d; ++t) {
                double df = x[t] - z[t];
                sq += df * df;
            }
            acc += variance * exp(inv * sq) * v[j];
        }
        y[r] = acc;
    }
    return 0;
}

/*
 * oracle_sgpr_accumulate: the two data-sized sums of sparse Gaussian process regression
 * (paper section 5.3) that a memory-efficient implementation accumulates over the data
 * instead of storing the m x n matrix K_uf:
 *     A[i][j] = sum_t K_uf[i][t] * K_uf[j][t]        (A = K_uf K_fu, m x m)
 *     b[i]    = sum_t K_uf[i][t] * y[t]              (b = K_uf y,    m)
 * with K_uf[i][t] = variance * exp(-0.5 * |U[i] - X[t]|^2 / lengthscale^2), the squared-
 * exponential kernel of section 5.1 between the m inducing points U and the n data points X.
 * Here the definition is written out: K_uf is stored whole (fp64, m * n values - small cases
 * only) and the sums run over t ascending.  A is m x m row-major.
 */
int oracle_sgpr_accumulate(const float *U, int64_t ldu, const float *X, int64_t ldx, const float *y,
                           int64_t m, int64_t n, int32_t d, double variance, double lengthscale,
                           double *A, double *b, int32_t nthreads)
{
    if (!U || !X || !y || !A || !b || m < 1 || n < 0 || d < 1 || ldu < d || ldx < d ||
        !(lengthscale > 0.0))
        return -1;
    if (nthreads < 1) nthreads = 1;
    const double inv = -0.5 / (lengthscale * lengthscale);
    double *K = (double *)malloc(sizeof(double) * (size_t)m * (size_t)(n > 0 ? n : 1));
    if (!K) return -2;
#pragma omp parallel for num_threads(nthreads) schedule(static)
    for (int64_t i = 0; i < m; ++i)
        for (int64_t t = 0; t < n; ++t)
            K[i * n + t] = variance * exp(inv * oracle_sqdist(U + i * ldu, X + t * ldx, d));
#pragma omp parallel for num_threads(nthreads) schedule(dynamic, 1)
    for (int64_t i = 0; i < m; ++i) {
        for (int64_t j = 0; j < m; ++j) {
            double acc = 0.0;
            for (int64_t t = 0; t < n; ++t) acc += K[i * n + t] * K[j * n + t];
            A[i * m + j] = acc;
        }
        double acc = 0.0;
        for (int64_t t = 0; t < n; ++t) acc += K[i * n + t] * (double)y[t];
        b[i] = acc;
    }
    free(K);
    return 0;
}

/*
 * oracle_sgpr_entries: the listed entries A[ii[p]][jj[p]] of the same matrix, each summed
 * directly over the data (no stored K_uf), for spot checks at sizes where the full routine
 * does not fit.
 */
int oracle_sgpr_entries(const float *U, int64_t ldu, const float *X, int64_t ldx, int64_t m,
                        int64_t n, int32_t d, double variance, double lengthscale,
                        const int64_t *ii, const int64_t *jj, int64_t count, double *out,
                        int32_t nthreads)
{
    if (!U || !X || !ii || !jj || !out || m < 1 || n < 0 || d < 1 || ldu < d || ldx < d ||
        !(lengthscale > 0.0))
        return -1;
    if (nthreads < 1) nthreads = 1;
    const double inv = -0.5 / (lengthscale * lengthscale);
#pragma omp parallel for num_threads(nthreads) schedule(dynamic, 1)
    for (int64_t p = 0; p < count; ++p) {
        const float *ui = U + ii[p] * ldu, *uj = U + jj[p] * ldu;
        double acc = 0.0;
        for (int64_t t = 0; t < n; ++t) {
            const float *x = X + t * ldx;
            acc += (variance * exp(inv * oracle_sqdist(ui, x, d))) *
                   (variance * exp(inv * oracle_sqdist(uj, x, d)));
        }
        out[p] = acc;
    }
    return 0;
}

/* Number of threads an OpenMP region of the requested width really gets. */
int32_t oracle_threads_used(int32_t nthreads)
{
    int32_t got = 1;
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel num_threads(nthreads)
    {
#pragma omp single
        {
#ifdef _OPENMP
            got = (int32_t)omp_get_num_threads();
#endif
        }
    }
    return got;
}
