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
// resid != null: resid[0] also gets max_j |x_j - bf16(x_j)|^2 (bits of a non-negative float, an
// integer maximum orders them; zeroed beforehand), the largest rounding residual that the bf16
// filters of the d > 8 kernels have to allow for - from the same pass over X.
__global__ __launch_bounds__(256) void knn_row_norms_kernel(const float* __restrict__ X,
                                                            int64_t ldx, int64_t n, int d,
                                                            int inverse, float* __restrict__ xn,
                                                            unsigned* __restrict__ resid) {
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    float worst = 0.f;
    for (int64_t j = wave; j < n; j += nwaves) {
        const float* row = X + j * ldx;
        float acc = 0.f, res = 0.f;
        for (int t = lane; t < d; t += kWave) {
            const float v = row[t];
            acc = fmaf(v, v, acc);
            // v minus its bf16 rounding (round to nearest even), exact in fp32
            const unsigned u = __float_as_uint(v);
            const float r = v - __uint_as_float((u + 0x7fffu + ((u >> 16) & 1u)) & 0xffff0000u);
            res = fmaf(r, r, res);
        }
#pragma unroll
        for (int s = 32; s > 0; s >>= 1) {
            acc += __shfl_xor(acc, s);
            res += __shfl_xor(res, s);
        }
        if (inverse) acc = acc > 0.f ? 1.f / sqrtf(acc) : 0.f;
        if (lane == 0) xn[j] = acc;
        worst = fmaxf(worst, res);
    }
    if (resid) {  // one atomic per workgroup (they all go to the same word)
        __shared__ float wmax[4];
        if (lane == 0) wmax[threadIdx.x >> 6] = worst;
        __syncthreads();
        if (threadIdx.x == 0)
            atomicMax(resid, __float_as_uint(fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]))));
    }
}

}  // namespace

hipError_t launch_row_norms(const float* X, int64_t ldx, int64_t n, int d, bool inverse, float* xn,
                            hipStream_t stream, void* resid) {
    int64_t blocks = (n + 3) / 4;
    if (blocks > 4096) blocks = 4096;
    knn_row_norms_kernel<<<dim3((unsigned)blocks), dim3(256), 0, stream>>>(
        X, ldx, n, d, inverse ? 1 : 0, xn, static_cast<unsigned*>(resid));
    return hipGetLastError();
}
}  // namespace knn
