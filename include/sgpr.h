/*
 * sgpr.h - C ABI of the MI355X (gfx950) accumulations of sparse Gaussian process regression
 * with a caller-given device-memory limit.  Part of the same shared library as knn.h and
 * kmv.h and sharing their conventions (row-major fp32 matrices with leading dimensions in
 * elements, DEVICE / HOST pointers, decimal size units, no ownership taken, knn_status return
 * codes, knn_last_hip_error()).
 *
 * Operation (paper section 5.3): sparse variational GP regression with m inducing points
 * needs, from the n data points, only
 *     A = K_uf K_fu   (m x m)        and        b = K_uf y   (m),
 * where K_uf[i][t] = variance * exp(-1/2 * ||u_i - x_t||^2 / lengthscale^2) is the m x n
 * squared-exponential kernel matrix of section 5.1 between inducing points and data.  A
 * straightforward implementation stores K_uf (O(n m) memory); the memory-efficient
 * procedure the section refers to sums over the data in chunks and needs O(m^2).  Here the
 * data axis is cut into chunks of chunk_cols points (section 4.3: the largest splittable
 * axis); one chunk of K_uf lives in the workspace, is multiplied by its own transpose on the
 * fp32 matrix cores and added to A in fp64, and is dropped.  When m is small (few 128 x 128
 * tiles of A for 256 compute units) and the limit has room, the columns of a chunk are cut
 * into col_groups groups whose products run concurrently into partial copies of A kept in
 * the workspace; the copies are added in a fixed order at the end.
 */
#ifndef SGPR_MI355X_H
#define SGPR_MI355X_H

#include <stdint.h>

#include "knn.h"

#ifdef __cplusplus
extern "C" {
#endif

#define SGPR_MAX_CHUNK_COLS 4096 /* longest run of products summed in fp32 before fp64 takes over */

typedef struct {
    int64_t m, n;
    int32_t d;
    int32_t col_groups;       /* column groups of a chunk multiplied concurrently (1, 2, 4, 8) */
    int64_t chunk_cols;       /* data points per chunk (multiple of 16, or n)            */
    int64_t n_chunks;         /* ceil(n / chunk_cols); 0 when n == 0                     */
    int64_t chunk_ld;         /* leading dimension of the K_uf chunk in the workspace    */
    uint64_t workspace_bytes; /* chunk (m * chunk_ld * 4) + (col_groups - 1) partial
                                 copies of A (m * m * 8 each), aligned  <= limit         */
    uint64_t min_limit_bytes; /* a chunk of 16 points                                    */
} sgpr_plan_t;

/*
 * HOST.  m >= 1 inducing points, n >= 0 data points, d >= 1.  Returns KNN_OK,
 * KNN_ERR_INVALID_ARG, KNN_ERR_UNSUPPORTED (m > 2^17 or n > 2^31 - 65536) or
 * KNN_ERR_MEM_LIMIT_TOO_SMALL (then *out still carries min_limit_bytes).
 */
knn_status sgpr_plan(int64_t m, int64_t n, int32_t d, uint64_t mem_limit_bytes,
                     sgpr_plan_t *out /* HOST */);

/*
 * sgpr_accumulate - A = K_uf K_fu and b = K_uf y (section 5.3).
 *   U [m, d], ldu     DEVICE in, fp32 inducing points
 *   X [n, d], ldx     DEVICE in, fp32 data points
 *   y [n]             DEVICE in, fp32 targets
 *   variance >= 0, lengthscale > 0 (finite)
 *   workspace         DEVICE, 256-byte aligned, workspace_bytes >= plan.workspace_bytes
 *   A [m, m], lda     DEVICE out, fp64, row-major, lda >= m; fully overwritten, exactly symmetric
 *   b [m]             DEVICE out, fp64; fully overwritten
 *   hip_stream        hipStream_t (NULL: default stream); the call only enqueues work and
 *                     allocates nothing.
 * Arithmetic: K_uf entries in fp32 (difference-form distance, hardware exp2); products and
 * their sums over one chunk in fp32 on the matrix cores; sums over chunks in fp64.  Every
 * entry is summed in a fixed order; the result depends on the limit only through the chunk
 * length (last bits).
 */
knn_status sgpr_accumulate(const float *U, int64_t ldu, const float *X, int64_t ldx,
                           const float *y, int64_t m, int64_t n, int32_t d, double variance,
                           double lengthscale, uint64_t mem_limit_bytes, void *workspace,
                           uint64_t workspace_bytes, double *A, int64_t lda, double *b,
                           void *hip_stream);

#ifdef __cplusplus
}
#endif

#endif /* SGPR_MI355X_H */
