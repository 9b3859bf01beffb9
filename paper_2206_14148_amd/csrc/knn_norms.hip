// gfx950 (CDNA4, MI355X): squared row norms, the  sum x^2  term of the expansion in paper
// section 4.1, and their reciprocal square roots (the row scale of the cosine metric).
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>

#include "knn_config.h"
#include "knn_device.h"
#include "knn_kernels.h"

namespace knn {

namespace {

// ---------------------------------------------------------------------------------------
// Row norms (section 4.1, the sum x^2 term): one wave per row, fixed summation order.
// ---------------------------------------------------------------------------------------
// inverse != 0 writes 1 / sqrt(sum) instead (0 for a zero row): the cosine metric's row scale.
__global__ __launch_bounds__(256) void knn_row_norms_kernel(const float* __restrict__ X,
                                                            int64_t ldx, int64_t n, int d,
                                                            int inverse, float* __restrict__ xn) {
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    for (int64_t j = wave; j < n; j += nwaves) {
        const float* row = X + j * ldx;
        float acc = 0.f;
        for (int t = lane; t < d; t += kWave) acc = fmaf(row[t], row[t], acc);
#pragma unroll
        for (int s = 32; s > 0; s >>= 1) acc += __shfl_xor(acc, s);
        if (inverse) acc = acc > 0.f ? 1.f / sqrtf(acc) : 0.f;
        if (lane == 0) xn[j] = acc;
    }
}

}  // namespace

hipError_t launch_row_norms(const float* X, int64_t ldx, int64_t n, int d, bool inverse, float* xn,
                            hipStream_t stream) {
    int64_t blocks = (n + 3) / 4;
    if (blocks > 16384) blocks = 16384;
    knn_row_norms_kernel<<<dim3((unsigned)blocks), dim3(256), 0, stream>>>(X, ldx, n, d,
                                                                           inverse ? 1 : 0, xn);
    return hipGetLastError();
}
}  // namespace knn
