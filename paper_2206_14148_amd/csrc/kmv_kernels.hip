// gfx950 (CDNA4, MI355X) kernels for the kernel matrix-vector product  y = K v  with the
// squared-exponential kernel (paper section 5.1; kernel formula in the appendix).  The
// n x m matrix K is the intermediate that section 4.3 keeps from being materialised: here
// a lane owns one row of K, produces its entries a few at a time in registers, multiplies
// them by v and adds them up, so K costs no memory at all.
//
// Summation order of one y_i, whatever the launch shape: points in ascending j inside
// groups of 64 (fp32, one fused multiply-add per point), groups in ascending order (fp64),
// point ranges in ascending order (fp64).
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>

#include "kmv_kernels.h"
#include "knn_config.h"
#include "knn_device.h"

namespace kmv {

namespace {

using knn::f32x16;
using knn::f32x4;
using knn::kInf;
using knn::load_row4;
using knn::mask_row4;

__global__ __launch_bounds__(256) void kmv_scaled_norms_kernel(const float* __restrict__ Z,
                                                               int64_t ldz, int64_t m, int d,
                                                               float c2, float* __restrict__ zn) {
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    for (int64_t j = wave; j < m; j += nwaves) {
        const float* p = Z + j * ldz;
        float acc = 0.f;
        for (int t = lane; t < d; t += 64) acc = fmaf(p[t], p[t], acc);
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) acc += __shfl_xor(acc, o);
        if (lane == 0) zn[j] = -c2 * acc;
    }
}

__global__ __launch_bounds__(256) void kmv_zero_kernel(double* __restrict__ y, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) y[i] = 0.0;
}

__global__ __launch_bounds__(256) void kmv_reduce_kernel(const double* __restrict__ partials, int S,
                                                         int64_t n, double* __restrict__ y) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    double acc = partials[i];
    for (int s = 1; s < S; ++s) acc += partials[(int64_t)s * n + i];
    y[i] = acc;
}

// ---------------------------------------------------------------------------------------
// d <= 8: one row x_i per lane in registers; the points z_j and the values v_j are the same
// for the whole wave, so they arrive through scalar loads and cost no vector work.  Per pair:
// d subtractions, d multiply-adds, one multiply by -c2, one hardware exp2, one multiply-add.
// ---------------------------------------------------------------------------------------
template <int D, bool CONTIG>
__global__ __launch_bounds__(kLowdTileRows) void kmv_lowd_kernel(
    const float* __restrict__ X, int64_t ldx, const float* __restrict__ Z, int64_t ldz_arg,
    const float* __restrict__ v, int n, int m, int split_len, float negc2, double variance,
    double* __restrict__ out) {
    constexpr int U = 8;
    const int64_t ldz = CONTIG ? (int64_t)D : ldz_arg;
    const int s = blockIdx.y;
    const int i = blockIdx.x * kLowdTileRows + threadIdx.x;
    const bool active = i < n;
    float x[D];
#pragma unroll
    for (int t = 0; t < D; ++t) x[t] = active ? X[(int64_t)i * ldx + t] : 0.f;

    auto term = [&](const float* __restrict__ zp, float vj, float part) {
        float df = x[0] - zp[0];
        float sq = df * df;
#pragma unroll
        for (int t = 1; t < D; ++t) {
            df = x[t] - zp[t];
            sq = fmaf(df, df, sq);
        }
        return fmaf(__builtin_amdgcn_exp2f(sq * negc2), vj, part);
    };

    const int j0 = s * split_len;  // split_len is a multiple of kGroup
    const int j1 = min(m, j0 + split_len);
    const float* zp = Z + (int64_t)j0 * ldz;  // uniform: read with scalar loads
    const float* vp = v + j0;
    double total = 0.0;
    int j = j0;
    for (; j + kGroup <= j1; j += kGroup) {
        float part = 0.f;
        for (int g = 0; g < kGroup; g += U, zp += U * ldz, vp += U) {
#pragma unroll
            for (int u = 0; u < U; ++u) part = term(zp + u * ldz, vp[u], part);
        }
        total += (double)part;
    }
    if (j < j1) {
        float part = 0.f;
        for (; j < j1; ++j, zp += ldz, ++vp) part = term(zp, vp[0], part);
        total += (double)part;
    }
    if (active) out[(int64_t)s * n + i] = variance * total;
}

// ---------------------------------------------------------------------------------------
// d > 8: a workgroup of 4 waves owns 128 rows of X and walks its point range in tiles of 128
// points.  Points are the M side and rows of X the N side of v_mfma_f32_32x32x2_f32, so the
// 16 accumulator values a lane holds per 32x32 block belong to ONE row x_i (column = lane %
// 32) and 16 different points.  The accumulators start at -c2 |z_j|^2 and receive
// (2 c2 x_i) . z_j; adding -c2 |x_i|^2 gives the exponent -c2 |x_i - z_j|^2 of the expansion
// in section 4.1.  Both operands stream through LDS in chunks of 16 columns, double buffered,
// with the global loads of step s+2 in flight during step s.
// ---------------------------------------------------------------------------------------
template <bool ALIGNED>
__global__ __launch_bounds__(256, 2) void kmv_mfma_kernel(
    const float* __restrict__ X, int64_t ldx, const float* __restrict__ Z, int64_t ldz,
    const float* __restrict__ v, const float* __restrict__ zn, int n, int m, int d, int split_len,
    float c2, double variance, double* __restrict__ out) {
    constexpr int TR = kMfmaTileRows, TZ = 128, KC = knn::kMfmaKC, RS = knn::kMfmaRowStride;
    extern __shared__ __align__(16) unsigned char smem[];
    float* zs = reinterpret_cast<float*>(smem);  // [2][TZ][RS]
    float* xs = zs + 2 * TZ * RS;                // [2][TR][RS]
    float* zns = xs + 2 * TR * RS;               // [2][TZ] accumulator start values
    float* vs = zns + 2 * TZ;                    // [2][TZ] pieces of v
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int i32 = lane & 31;
    const int h = lane >> 5;
    const int s = blockIdx.y;
    const int wg_row0 = blockIdx.x * TR;
    const int my_row = wave * 32 + i32;
    const int r = wg_row0 + my_row;
    const bool active = r < n;

    // -c2 |x_i|^2 of this lane's row, summed in ascending t
    float nxn = 0.f;
    if (active) {
        const float* p = X + (int64_t)r * ldx;
        float acc = 0.f;
        for (int t = 0; t < d; ++t) acc = fmaf(p[t], p[t], acc);
        nxn = -c2 * acc;
    }

    const int j0 = s * split_len;  // split_len is a multiple of TZ
    const int j1 = min(m, j0 + split_len);
    const int ntiles = (j1 > j0) ? (j1 - j0 + TZ - 1) / TZ : 0;
    const int nch = (d + KC - 1) / KC;
    const int total = ntiles * nch;
    const float bscale = 2.f * c2;

    const int srow = tid >> 2;
    const int scol = (tid & 3) * 4;

    struct Staged {
        f32x4 z0, z1, x0, x1;
        float znv, vv;
    };
    // Branch-free on purpose: every call issues the same loads from clamped addresses, so the
    // compiler can count the newer loads still in flight when an older set is consumed.
    auto fetch = [&](int step, Staged& g) {
        const int tile = step / nch;
        const int c = step - tile * nch;
        const int col = c * KC + scol;
        const int64_t jr = (int64_t)j0 + (int64_t)tile * TZ + srow;
        g.z0 = load_row4<ALIGNED>(Z, ldz, jr, j1, col, d);
        g.z1 = load_row4<ALIGNED>(Z, ldz, jr + 64, j1, col, d);
        g.x0 = load_row4<ALIGNED>(X, ldx, (int64_t)wg_row0 + srow, n, col, d);
        g.x1 = load_row4<ALIGNED>(X, ldx, (int64_t)wg_row0 + srow + 64, n, col, d);
        const int64_t jj = (int64_t)j0 + (int64_t)tile * TZ + (tid & (TZ - 1));
        const int64_t jc = jj < j1 ? jj : j1 - 1;
        g.znv = zn[jc];
        g.vv = v[jc];
    };
    auto stash = [&](int step, const Staged& g) {
        const int tile = step / nch;
        const int c = step - tile * nch;
        const int buf = step & 1;
        const int col = c * KC + scol;
        const int64_t jr = (int64_t)j0 + (int64_t)tile * TZ + srow;
        float* zb = zs + buf * TZ * RS;
        float* xb = xs + buf * TR * RS;
        *reinterpret_cast<f32x4*>(zb + srow * RS + scol) = mask_row4(g.z0, jr < j1, col, d, 1.f);
        *reinterpret_cast<f32x4*>(zb + (srow + 64) * RS + scol) =
            mask_row4(g.z1, jr + 64 < j1, col, d, 1.f);
        *reinterpret_cast<f32x4*>(xb + srow * RS + scol) =
            mask_row4(g.x0, wg_row0 + srow < n, col, d, bscale);
        *reinterpret_cast<f32x4*>(xb + (srow + 64) * RS + scol) =
            mask_row4(g.x1, wg_row0 + srow + 64 < n, col, d, bscale);
        if (c == 0 && tid < TZ) {
            const int64_t jj = (int64_t)j0 + (int64_t)tile * TZ + tid;
            // points past the range: exponent -inf and weight 0, so they add exactly 0
            zns[(tile & 1) * TZ + tid] = jj < j1 ? g.znv : -kInf;
            vs[(tile & 1) * TZ + tid] = jj < j1 ? g.vv : 0.f;
        }
    };

    f32x16 acc[4];
    double sum = 0.0;

    Staged set_even, set_odd;
    if (total > 0) {
        fetch(0, set_even);
        stash(0, set_even);
    }
    if (total > 1) fetch(1, set_odd);
    __syncthreads();

    auto run_step = [&](int step, Staged& mine, const Staged& next) {
        const int tile = step / nch;
        const int c = step - tile * nch;
        const int buf = step & 1;
        fetch(step + 2 < total ? step + 2 : total - 1, mine);  // past the end: a harmless re-load

        if (c == 0) {
            const float* zt = zns + (tile & 1) * TZ;
#pragma unroll
            for (int pb = 0; pb < 4; ++pb) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const f32x4 w = *reinterpret_cast<const f32x4*>(zt + pb * 32 + g * 8 + h * 4);
                    acc[pb][g * 4 + 0] = w[0];
                    acc[pb][g * 4 + 1] = w[1];
                    acc[pb][g * 4 + 2] = w[2];
                    acc[pb][g * 4 + 3] = w[3];
                }
            }
        }
        {
            const float* zb = zs + buf * TZ * RS;
            const float* xb = xs + buf * TR * RS;
            f32x4 b[KC / 8], a[KC / 8][4];
#pragma unroll
            for (int g = 0; g < KC / 8; ++g) {
                const int col = g * 8 + h * 4;
                b[g] = *reinterpret_cast<const f32x4*>(xb + my_row * RS + col);
#pragma unroll
                for (int pb = 0; pb < 4; ++pb)
                    a[g][pb] = *reinterpret_cast<const f32x4*>(zb + (pb * 32 + i32) * RS + col);
            }
#pragma unroll
            for (int g = 0; g < KC / 8; ++g) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
#pragma unroll
                    for (int pb = 0; pb < 4; ++pb)
                        acc[pb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[g][pb][e], b[g][e], acc[pb], 0, 0, 0);
                }
                if (g == 0 && step + 1 < total) stash(step + 1, next);
            }
        }

        if (c == nch - 1) {
            // This lane's 64 points of the tile, in ascending j: block pb, register group g,
            // element e is point pb*32 + g*8 + h*4 + e.  The two halves of the wave hold
            // interleaved runs of 4 points; they are added at the very end.
            const float* vt = vs + (tile & 1) * TZ;
            float part = 0.f;
#pragma unroll
            for (int pb = 0; pb < 4; ++pb) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const f32x4 w = *reinterpret_cast<const f32x4*>(vt + pb * 32 + g * 8 + h * 4);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float arg = fminf(acc[pb][g * 4 + e] + nxn, 0.f);
                        part = fmaf(__builtin_amdgcn_exp2f(arg), w[e], part);
                    }
                }
            }
            sum += (double)part;
        }
        __syncthreads();
    };
    for (int step = 0; step < total; step += 2) {
        run_step(step, set_even, set_odd);
        if (step + 1 < total) run_step(step + 1, set_odd, set_even);
    }
    const double other = __shfl_xor(sum, 32);
    if (active && h == 0) out[(int64_t)s * n + r] = variance * (sum + other);
}

// ---------------------------------------------------------------------------------------
// fp64 variant, d <= 8: the low-d kernel with every operation in fp64 and the library's exp.
// The sum runs over j ascending in one fp64 accumulator.
// ---------------------------------------------------------------------------------------
template <int D, bool CONTIG>
__global__ __launch_bounds__(kLowdTileRows) void kmv_lowd_f64_kernel(
    const double* __restrict__ X, int64_t ldx, const double* __restrict__ Z, int64_t ldz_arg,
    const double* __restrict__ v, int n, int m, int split_len, double negc, double variance,
    double* __restrict__ out) {
    constexpr int U = 4;
    const int64_t ldz = CONTIG ? (int64_t)D : ldz_arg;
    const int s = blockIdx.y;
    const int i = blockIdx.x * kLowdTileRows + threadIdx.x;
    const bool active = i < n;
    double x[D];
#pragma unroll
    for (int t = 0; t < D; ++t) x[t] = active ? X[(int64_t)i * ldx + t] : 0.0;

    auto term = [&](const double* __restrict__ zp, double vj, double total) {
        double df = x[0] - zp[0];
        double sq = df * df;
#pragma unroll
        for (int t = 1; t < D; ++t) {
            df = x[t] - zp[t];
            sq = fma(df, df, sq);
        }
        return fma(exp(sq * negc), vj, total);
    };

    const int j0 = s * split_len;
    const int j1 = min(m, j0 + split_len);
    const double* zp = Z + (int64_t)j0 * ldz;  // uniform: read with scalar loads
    const double* vp = v + j0;
    double total = 0.0;
    int j = j0;
    for (; j + U <= j1; j += U, zp += U * ldz, vp += U) {
#pragma unroll
        for (int u = 0; u < U; ++u) total = term(zp + u * ldz, vp[u], total);
    }
    for (; j < j1; ++j, zp += ldz, ++vp) total = term(zp, vp[0], total);
    if (active) out[(int64_t)s * n + i] = variance * total;
}

// ---------------------------------------------------------------------------------------
// fp64 variant, any d: one row per lane; a group of 8 wave-uniform points (scalar loads)
// keeps one running squared distance each while the row is walked in chunks of 4 columns,
// so a row value is loaded once per 8 points.  Columns in ascending order, points in
// ascending order, one fp64 accumulator.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(kLowdTileRows) void kmv_anyd_f64_kernel(
    const double* __restrict__ X, int64_t ldx, const double* __restrict__ Z, int64_t ldz,
    const double* __restrict__ v, int n, int m, int d, int split_len, double negc, double variance,
    double* __restrict__ out) {
    constexpr int P = 8, TC = 4;
    const int s = blockIdx.y;
    const int i = blockIdx.x * kLowdTileRows + threadIdx.x;
    const bool active = i < n;
    const double* __restrict__ xrow = X + (int64_t)(active ? i : n - 1) * ldx;  // in bounds for idle lanes
    const int j0 = s * split_len;
    const int j1 = min(m, j0 + split_len);
    const double* zp = Z + (int64_t)j0 * ldz;  // uniform
    const double* vp = v + j0;
    double total = 0.0;
    int j = j0;
    for (; j + P <= j1; j += P, zp += P * ldz, vp += P) {
        double sq[P];
#pragma unroll
        for (int p = 0; p < P; ++p) sq[p] = 0.0;
        int c = 0;
        for (; c + TC <= d; c += TC) {
            double xr[TC];
#pragma unroll
            for (int t = 0; t < TC; ++t) xr[t] = xrow[c + t];
#pragma unroll
            for (int p = 0; p < P; ++p) {
#pragma unroll
                for (int t = 0; t < TC; ++t) {
                    const double df = xr[t] - zp[p * ldz + c + t];
                    sq[p] = fma(df, df, sq[p]);
                }
            }
        }
        for (; c < d; ++c) {
            const double xr = xrow[c];
#pragma unroll
            for (int p = 0; p < P; ++p) {
                const double df = xr - zp[p * ldz + c];
                sq[p] = fma(df, df, sq[p]);
            }
        }
#pragma unroll
        for (int p = 0; p < P; ++p) total = fma(exp(sq[p] * negc), vp[p], total);
    }
    for (; j < j1; ++j, zp += ldz, ++vp) {
        double sq = 0.0;
        for (int c = 0; c < d; ++c) {
            const double df = xrow[c] - zp[c];
            sq = fma(df, df, sq);
        }
        total = fma(exp(sq * negc), vp[0], total);
    }
    if (active) out[(int64_t)s * n + i] = variance * total;
}

int64_t split_length(int64_t m, int S, int tile) {
    int64_t len = (m + S - 1) / S;
    return (len + tile - 1) / tile * tile;
}

}  // namespace

hipError_t launch_scaled_norms(const float* Z, int64_t ldz, int64_t m, int d, float c2, float* zn,
                               hipStream_t stream) {
    if (m == 0) return hipSuccess;
    int64_t blocks = (m + 3) / 4;
    if (blocks > 16384) blocks = 16384;
    kmv_scaled_norms_kernel<<<dim3((unsigned)blocks), dim3(256), 0, stream>>>(Z, ldz, m, d, c2, zn);
    return hipGetLastError();
}

hipError_t launch_zero(double* y, int64_t n, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    kmv_zero_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream>>>(y, n);
    return hipGetLastError();
}

hipError_t launch_reduce(const double* partials, int S, int64_t n, double* y, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    kmv_reduce_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream>>>(partials, S, n, y);
    return hipGetLastError();
}

template <int D>
static hipError_t launch_lowd_d(const float* X, int64_t ldx, const float* Z, int64_t ldz,
                                const float* v, int64_t n, int64_t m, float c2, double variance,
                                int S, double* out, hipStream_t stream) {
    const dim3 grid((unsigned)((n + kLowdTileRows - 1) / kLowdTileRows), (unsigned)S);
    const int split_len = (int)split_length(m, S, kGroup);
    if (ldz == D) {
        kmv_lowd_kernel<D, true><<<grid, dim3(kLowdTileRows), 0, stream>>>(
            X, ldx, Z, ldz, v, (int)n, (int)m, split_len, -c2, variance, out);
    } else {
        kmv_lowd_kernel<D, false><<<grid, dim3(kLowdTileRows), 0, stream>>>(
            X, ldx, Z, ldz, v, (int)n, (int)m, split_len, -c2, variance, out);
    }
    return hipGetLastError();
}

hipError_t launch_lowd(const float* X, int64_t ldx, const float* Z, int64_t ldz, const float* v,
                       int64_t n, int64_t m, int d, float c2, double variance, int S, double* out,
                       hipStream_t stream) {
    if (n == 0) return hipSuccess;
    switch (d) {
        case 1: return launch_lowd_d<1>(X, ldx, Z, ldz, v, n, m, c2, variance, S, out, stream);
        case 2: return launch_lowd_d<2>(X, ldx, Z, ldz, v, n, m, c2, variance, S, out, stream);
        case 3: return launch_lowd_d<3>(X, ldx, Z, ldz, v, n, m, c2, variance, S, out, stream);
        case 4: return launch_lowd_d<4>(X, ldx, Z, ldz, v, n, m, c2, variance, S, out, stream);
        case 5: return launch_lowd_d<5>(X, ldx, Z, ldz, v, n, m, c2, variance, S, out, stream);
        case 6: return launch_lowd_d<6>(X, ldx, Z, ldz, v, n, m, c2, variance, S, out, stream);
        case 7: return launch_lowd_d<7>(X, ldx, Z, ldz, v, n, m, c2, variance, S, out, stream);
        case 8: return launch_lowd_d<8>(X, ldx, Z, ldz, v, n, m, c2, variance, S, out, stream);
        default: return hipErrorInvalidValue;
    }
}

template <int D>
static hipError_t launch_f64_d(const double* X, int64_t ldx, const double* Z, int64_t ldz,
                               const double* v, int64_t n, int64_t m, double negc, double variance,
                               int S, double* out, hipStream_t stream) {
    const dim3 grid((unsigned)((n + kLowdTileRows - 1) / kLowdTileRows), (unsigned)S);
    const int split_len = (int)split_length(m, S, kGroup);
    if (ldz == D) {
        kmv_lowd_f64_kernel<D, true><<<grid, dim3(kLowdTileRows), 0, stream>>>(
            X, ldx, Z, ldz, v, (int)n, (int)m, split_len, negc, variance, out);
    } else {
        kmv_lowd_f64_kernel<D, false><<<grid, dim3(kLowdTileRows), 0, stream>>>(
            X, ldx, Z, ldz, v, (int)n, (int)m, split_len, negc, variance, out);
    }
    return hipGetLastError();
}

hipError_t launch_f64(const double* X, int64_t ldx, const double* Z, int64_t ldz, const double* v,
                      int64_t n, int64_t m, int d, double negc, double variance, int S, double* out,
                      hipStream_t stream) {
    if (n == 0) return hipSuccess;
    switch (d) {
        case 1: return launch_f64_d<1>(X, ldx, Z, ldz, v, n, m, negc, variance, S, out, stream);
        case 2: return launch_f64_d<2>(X, ldx, Z, ldz, v, n, m, negc, variance, S, out, stream);
        case 3: return launch_f64_d<3>(X, ldx, Z, ldz, v, n, m, negc, variance, S, out, stream);
        case 4: return launch_f64_d<4>(X, ldx, Z, ldz, v, n, m, negc, variance, S, out, stream);
        case 5: return launch_f64_d<5>(X, ldx, Z, ldz, v, n, m, negc, variance, S, out, stream);
        case 6: return launch_f64_d<6>(X, ldx, Z, ldz, v, n, m, negc, variance, S, out, stream);
        case 7: return launch_f64_d<7>(X, ldx, Z, ldz, v, n, m, negc, variance, S, out, stream);
        case 8: return launch_f64_d<8>(X, ldx, Z, ldz, v, n, m, negc, variance, S, out, stream);
        default: break;
    }
    const dim3 grid((unsigned)((n + kLowdTileRows - 1) / kLowdTileRows), (unsigned)S);
    const int split_len = (int)split_length(m, S, kGroup);
    kmv_anyd_f64_kernel<<<grid, dim3(kLowdTileRows), 0, stream>>>(
        X, ldx, Z, ldz, v, (int)n, (int)m, d, split_len, negc, variance, out);
    return hipGetLastError();
}

hipError_t launch_mfma(const float* X, int64_t ldx, const float* Z, int64_t ldz, const float* v,
                       const float* zn, int64_t n, int64_t m, int d, float c2, double variance, int S,
                       double* out, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    const size_t lds = (size_t)(4 * 128 * knn::kMfmaRowStride + 4 * 128) * 4;
    const dim3 grid((unsigned)((n + kMfmaTileRows - 1) / kMfmaTileRows), (unsigned)S);
    const int split_len = (int)split_length(m, S, 128);
    const bool aligned = (reinterpret_cast<uintptr_t>(X) % 16 == 0) &&
                         (reinterpret_cast<uintptr_t>(Z) % 16 == 0) && (ldx % 4 == 0) &&
                         (ldz % 4 == 0) && (d % 4 == 0);
    if (aligned) {
        kmv_mfma_kernel<true><<<grid, dim3(256), lds, stream>>>(
            X, ldx, Z, ldz, v, zn, (int)n, (int)m, d, split_len, c2, variance, out);
    } else {
        kmv_mfma_kernel<false><<<grid, dim3(256), lds, stream>>>(
            X, ldx, Z, ldz, v, zn, (int)n, (int)m, d, split_len, c2, variance, out);
    }
    return hipGetLastError();
}

}  // namespace kmv
