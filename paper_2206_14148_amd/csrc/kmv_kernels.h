// Internal launcher interface between the kernel matrix-vector C ABI (kmv_api.hip) and its
// gfx950 kernels.  c2 = log2(e) / (2 lengthscale^2), so K = variance * exp2(-c2 * sqdist).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace kmv {

constexpr int kLowdMaxD = 8;      // difference form on the vector ALU up to here
constexpr int kLowdTileRows = 256;
constexpr int kMfmaTileRows = 128;
constexpr int kMfmaKC = 16;      // coordinates per pipeline step
constexpr int kMfmaResidentChunks = 4;  // d <= 64: the bf16 pieces of a row of X stay in registers
constexpr int kGroup = 64;        // points per fp32 partial sum
constexpr int kMaxSplits = 64;

// zn[j] = -c2 * sum_t Z[j][t]^2 (fp32): the start value of the MFMA accumulators.
hipError_t launch_scaled_norms(const float* Z, int64_t ldz, int64_t m, int d, float c2, float* zn,
                               hipStream_t stream);

// d <= kLowdMaxD.  out[s * n + i] = variance * sum over range s of K-without-variance * v.
hipError_t launch_lowd(const float* X, int64_t ldx, const float* Z, int64_t ldz, const float* v,
                       int64_t n, int64_t m, int d, float c2, double variance, int S, double* out,
                       hipStream_t stream);

// d > kLowdMaxD: squared distance through the expansion, X Z^T on bf16 MFMA over three-piece
// splits of the fp32 values (products as accurate as fp32's).
hipError_t launch_mfma(const float* X, int64_t ldx, const float* Z, int64_t ldz, const float* v,
                       const float* zn, int64_t n, int64_t m, int d, float c2, double variance, int S,
                       double* out, hipStream_t stream);

// fp64 inputs and arithmetic (the precision of paper section 5.1), any d: d <= kLowdMaxD keeps
// the row in registers, larger d re-reads it in chunks.  negc = -1 / (2 lengthscale^2).
hipError_t launch_f64(const double* X, int64_t ldx, const double* Z, int64_t ldz, const double* v,
                      int64_t n, int64_t m, int d, double negc, double variance, int S, double* out,
                      hipStream_t stream);

// y[i] = sum_s partials[s * n + i], s ascending.
hipError_t launch_reduce(const double* partials, int S, int64_t n, double* y, hipStream_t stream);

// y[i] = 0.
hipError_t launch_zero(double* y, int64_t n, hipStream_t stream);

}  // namespace kmv
