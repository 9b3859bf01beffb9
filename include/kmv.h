/*
 * kmv.h - C ABI of the MI355X (gfx950) kernel matrix-vector product with a
 * caller-given device-memory limit.  Part of the same shared library as knn.h
 * and sharing its conventions (row-major fp32 matrices with leading
 * dimensions in elements, DEVICE / HOST pointers, decimal size units, no
 * ownership taken, knn_status return codes, knn_last_hip_error()).
 *
 * Operation (paper section 5.1 and the appendix that shows its graph before
 * and after splitting):  y = K v  with
 *     K[i][j] = variance * exp(-1/2 * ||x_i - z_j||^2 / lengthscale^2),
 * the squared-exponential kernel between the n rows of X and the m rows of Z.
 * The n x m matrix K is the big intermediate of section 4.3: it is produced
 * tile by tile in registers, multiplied by the matching piece of v and summed
 * at once, so it never exists in memory.  The paper evaluates the expression
 * in double precision.  Two families of entry points: kmv_plan / kmv_apply
 * take fp32 points, evaluate each K entry in fp32 (one hardware exp2 per pair)
 * and carry every sum longer than 64 terms in fp64; kmv_plan_f64 /
 * kmv_apply_f64 take fp64 points and compute in fp64 throughout.  y is fp64
 * in both.
 */
#ifndef KMV_MI355X_H
#define KMV_MI355X_H

#include <stdint.h>

#include "knn.h"

#ifdef __cplusplus
extern "C" {
#endif

/* kernel families (kmv_plan_t.path) */
#define KMV_PATH_LOWD 0 /* d <= 8: difference-form squared distance on the vector ALU   */
#define KMV_PATH_MFMA 1 /* d  > 8: section 4.1 expansion, matrix-core tile of X Z^T (bf16
                           instructions on three-piece splits: fp32-accurate products) */
#define KMV_PATH_VALU 2 /* fp64 entry points, d > 8: difference form, row re-read in chunks */

/*
 * The plan.  One workgroup owns tile_rows rows of X (one row of K per lane)
 * and walks a range of the m points; the point axis is cut into n_splits
 * ranges as far as that fills the GPU (small n) or evens out its last round
 * of workgroups (path 1) and the limit has room, each range giving a partial
 * sum per row in the workspace (fp64, [n_splits][n]) that a last kernel adds
 * in ascending range order.  With n_splits == 1 the sums go straight to y.
 * n_splits depends on the limit, so y can differ between limits by the fp64
 * rounding of the range sums.  Path 1 also keeps c * ||z_j||^2 (fp32, m values) in the
 * workspace, c = log2(e) / (2 lengthscale^2).
 */
typedef struct {
    int64_t n, m;
    int32_t d;
    int32_t path;      /* KMV_PATH_*                                      */
    int32_t tile_rows; /* rows of X per workgroup                         */
    int32_t n_splits;  /* ranges the point axis is cut into               */
    int64_t norms_bytes;     /* path 1: the scaled norms of Z, else 0     */
    int64_t partials_bytes;  /* n_splits > 1: the partial sums, else 0    */
    int64_t workspace_bytes; /* norms_bytes + partials_bytes  <= limit    */
    int64_t min_limit_bytes; /* smallest limit that can run this shape    */
} kmv_plan_t;

/*
 * HOST.  Fills *out for the shape and limit given (section 4.3: the split is
 * chosen so that everything the library keeps stays under the limit).
 * n >= 0 rows of X, m >= 0 rows of Z, d >= 1, mem_limit_bytes >= 0.
 * Returns KNN_OK, KNN_ERR_INVALID_ARG, KNN_ERR_UNSUPPORTED (n or m above
 * 2^31 - 65536) or KNN_ERR_MEM_LIMIT_TOO_SMALL (then *out still carries
 * min_limit_bytes).
 */
int kmv_plan(int64_t n, int64_t m, int32_t d, int64_t mem_limit_bytes, kmv_plan_t* out);

/*
 * y = K(X, Z) v  (section 5.1; kernel as defined in the appendix).
 *   X          DEVICE  fp32 [n][ldx], ldx >= d      rows x_i
 *   Z          DEVICE  fp32 [m][ldz], ldz >= d      rows z_j (may alias X)
 *   v          DEVICE  fp32 [m]
 *   variance   sigma^2 >= 0, lengthscale l > 0 (both finite)
 *   workspace  DEVICE  256-byte aligned, workspace_bytes >= plan.workspace_bytes
 *              (may be NULL when the plan needs 0 bytes); contents are scratch
 *   y          DEVICE  fp64 [n], fully overwritten (all zeros when m == 0)
 *   stream     hipStream_t (NULL: the default stream).  The call only
 *              enqueues work; it allocates nothing and does not synchronise.
 * Each y_i is a sum in a fixed order (64-point groups in fp32, groups and
 * ranges in fp64), so results do not depend on timing; they may differ in the
 * last bits between two limits that give different n_splits.
 * Errors as kmv_plan, plus KNN_ERR_WORKSPACE_TOO_SMALL and KNN_ERR_HIP.
 */
int kmv_apply(const float* X, int64_t ldx, const float* Z, int64_t ldz, const float* v, int64_t n,
              int64_t m, int32_t d, double variance, double lengthscale, int64_t mem_limit_bytes,
              void* workspace, int64_t workspace_bytes, double* y, void* stream);

/*
 * The same product in the precision section 5.1 evaluates it in: X, Z, v are
 * fp64 (DEVICE, row-major, leading dimensions in elements) and every
 * operation is fp64 - difference-form squared distance with the columns in
 * ascending order, the math library's exp, one fused multiply-add per point
 * into a single accumulator with the points in ascending order (per range).
 * Vector-ALU kernels for every d (path 0 or 2); the workspace holds only the
 * partial sums of the ranges (norms_bytes == 0).  Otherwise as kmv_plan /
 * kmv_apply.
 */
int kmv_plan_f64(int64_t n, int64_t m, int32_t d, int64_t mem_limit_bytes, kmv_plan_t* out);

int kmv_apply_f64(const double* X, int64_t ldx, const double* Z, int64_t ldz, const double* v,
                  int64_t n, int64_t m, int32_t d, double variance, double lengthscale,
                  int64_t mem_limit_bytes, void* workspace, int64_t workspace_bytes, double* y,
                  void* stream);

#ifdef __cplusplus
}
#endif

#endif /* KMV_MI355X_H */
