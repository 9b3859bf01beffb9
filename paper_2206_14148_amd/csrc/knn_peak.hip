// Measured matrix-core peak of the GPU this process runs on: a loop of nothing but MFMAs, so that
// roofline fractions can be quoted against what the chip sustains as well as against the
// published figure (under matrix-core load the engine clock settles below its 2.4 GHz maximum).
#include <hip/hip_runtime.h>

#include <cstdint>

#include "../../include/knn.h"
#include "knn_config.h"

namespace knn {
void set_last_hip_error(hipError_t e, const char* what);
}

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kPeakUnroll = 16;  // MFMAs per accumulator and loop iteration

// 8 waves per workgroup, one workgroup per compute unit: two waves per SIMD, four independent
// accumulators each, operands that never change.  out gets one word per thread (the sums: they
// keep the loop alive).
template <bool BF16>
__global__ __launch_bounds__(512, 2) void knn_mfma_peak_kernel(int iters, float seed, float* __restrict__ out) {
    f32x16 acc[4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[u][e] = 0.f;
    // Eight different A and B operands of pseudo-random bits, taken in turn: operands that never
    // change (or all zeros) toggle hardly a wire, draw far less power than real data and flatter
    // the result.  Magnitudes stay below 2^-4 and signs are mixed, so the sums stay far from
    // overflow.
    bf16x8 a8[8], b8[8];
    unsigned h = (threadIdx.x * 2654435761u) ^ (blockIdx.x * 40503u) ^ (unsigned)__float_as_uint(seed);
#pragma unroll
    for (int r = 0; r < 8; ++r) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            h = h * 1664525u + 1013904223u;
            // sign and 7 mantissa bits random, exponent 2^-8 .. 2^-5
            const unsigned short ua = (unsigned short)(((h >> 16) & 0x807f) | ((119 + ((h >> 8) & 3)) << 7));
            h = h * 1664525u + 1013904223u;
            const unsigned short ub = (unsigned short)(((h >> 16) & 0x807f) | ((119 + ((h >> 8) & 3)) << 7));
            a8[r][e] = __builtin_bit_cast(__bf16, ua);
            b8[r][e] = __builtin_bit_cast(__bf16, ub);
        }
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < kPeakUnroll; ++r) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (BF16)
                    acc[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a8[(r + u) & 7], b8[(r + 3 * u) & 7], acc[u], 0, 0, 0);
                else
                    acc[u] = __builtin_amdgcn_mfma_f32_32x32x2f32((float)a8[(r + u) & 7][u], (float)b8[r & 7][u],
                                                               acc[u], 0, 0, 0);
            }
        }
    }
    float s = 0.f;
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[u][e];
    out[blockIdx.x * 512 + threadIdx.x] = s;
}

}  // namespace

extern "C" knn_status knn_measure_mfma_peak(int32_t dtype, void* scratch, uint64_t scratch_bytes,
                                            void* hip_stream, float* tflops_out) {
    if (!tflops_out || !scratch || (dtype != 0 && dtype != 1)) return KNN_ERR_INVALID_ARG;
    const int blocks = knn::kNumCU;
    if (scratch_bytes < (uint64_t)blocks * 512 * 4) return KNN_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipError_t e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&e1);
    // about 15 ms of MFMAs at the published rate
    const int iters = dtype == 0 ? 9000 : 600;
    float* out = static_cast<float*>(scratch);
    float best = 0.f;
    for (int rep = 0; rep < 3 && e == hipSuccess; ++rep) {
        if (rep == 1) e = hipEventRecord(e0, stream);
        if (e != hipSuccess) break;
        if (dtype == 0) knn_mfma_peak_kernel<true><<<dim3(blocks), dim3(512), 0, stream>>>(iters, 0.0078125f, out);
        else knn_mfma_peak_kernel<false><<<dim3(blocks), dim3(512), 0, stream>>>(iters, 0.0078125f, out);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipEventRecord(e1, stream);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (e != hipSuccess) {
        knn::set_last_hip_error(e, "MFMA peak measurement");
        return KNN_ERR_HIP;
    }
    // two timed launches; flops per MFMA: 32 x 32 x K x 2
    const double flops_per_mfma = dtype == 0 ? 32768.0 : 4096.0;
    const double flops = 2.0 * (double)blocks * 8.0 * (double)iters * kPeakUnroll * 4.0 * flops_per_mfma;
    best = (float)(flops / ((double)ms * 1e-3) / 1e12);
    *tflops_out = best;
    return KNN_OK;
}
