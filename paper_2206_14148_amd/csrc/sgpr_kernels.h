// Internal launcher interface between the SGPR C ABI (sgpr_api.hip) and its gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace sgpr {

// A[0..m)[0..m) = 0 and (b != nullptr) b[0..m) = 0.
hipError_t launch_zero(double* A, int64_t lda, double* b, int64_t m, hipStream_t stream);

// Kc[i][c] = variance * exp2(-c2 * |U[i] - X[c0 + c]|^2) for i < m, c < cols (fp32, ld = ldk).
hipError_t launch_kuf(const float* U, int64_t ldu, const float* X, int64_t ldx, int64_t m,
                      int64_t c0, int64_t cols, int d, float c2, float variance, float* Kc,
                      int64_t ldk, hipStream_t stream);

// Lower triangle (whole diagonal tiles): A[j][i] += sum_c Kc[j][c] * Kc[i][c].  The columns are
// cut into `groups` runs (multiples of 16); run 0 adds into A, run g > 0 into the m x m copy
// copies + (g - 1) * copy_stride (leading dimension m).
hipError_t launch_syrk(const float* Kc, int64_t ldk, int64_t m, int64_t cols, int groups, double* A,
                       int64_t lda, double* copies, int64_t copy_stride, hipStream_t stream);

// Lower triangle: A[j][i] += copy_0[j][i] + copy_1[j][i] + ... in that order.
hipError_t launch_add_copies(double* A, int64_t lda, const double* copies, int64_t copy_stride,
                             int ncopies, int64_t m, hipStream_t stream);

// b[i] += sum_c Kc[i][c] * y[c0 + c].
hipError_t launch_kufy(const float* Kc, int64_t ldk, int64_t m, int64_t cols, const float* y,
                       double* b, hipStream_t stream);

// A[i][j] = A[j][i] for j > i.
hipError_t launch_symmetrize(double* A, int64_t lda, int64_t m, hipStream_t stream);

}  // namespace sgpr
