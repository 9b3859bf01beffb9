// gfx950 (CDNA4, MI355X) kernels for the data-sized sums of sparse GP regression (paper
// section 5.3): A = K_uf K_fu and b = K_uf y, accumulated over chunks of the data so that only
// one m x chunk piece of the kernel matrix K_uf ever exists (section 4.3: split the largest
// axis, keep the big intermediate inside one iteration).
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>

#include "knn_config.h"
#include "knn_device.h"
#include "sgpr_kernels.h"

namespace sgpr {

namespace {

using knn::f32x16;
using knn::f32x4;
using knn::load_row4;
using knn::mask_row4;

constexpr int kRowsPerThread = 8;  // inducing points per thread of the K_uf kernel

__global__ __launch_bounds__(256) void sgpr_zero_kernel(double* __restrict__ A, int64_t lda,
                                                        double* __restrict__ b, int m) {
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= m) return;
    for (int i = blockIdx.y; i < m; i += gridDim.y) A[(int64_t)i * lda + j] = 0.0;
    if (blockIdx.y == 0 && b) b[j] = 0.0;
}

// One data point per thread (consecutive threads: consecutive columns of the chunk, so the
// stores are coalesced), 8 inducing points per thread: their coordinates are the same for the
// whole workgroup and come through scalar loads, the data point's coordinate is loaded once
// per dimension and used 8 times.  Difference form, columns in ascending order.
__global__ __launch_bounds__(256) void sgpr_kuf_kernel(const float* __restrict__ U, int64_t ldu,
                                                       const float* __restrict__ X, int64_t ldx,
                                                       int m, int64_t c0, int cols, int d,
                                                       float negc2, float variance,
                                                       float* __restrict__ Kc, int64_t ldk) {
    constexpr int R = kRowsPerThread;
    const int c = blockIdx.x * 256 + threadIdx.x;
    const int i0 = blockIdx.y * R;
    const float* __restrict__ xp = X + (c0 + (c < cols ? c : cols - 1)) * ldx;  // clamped: in bounds
    float sq[R];
#pragma unroll
    for (int r = 0; r < R; ++r) sq[r] = 0.f;
    for (int t = 0; t < d; ++t) {
        const float xv = xp[t];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int i = min(i0 + r, m - 1);  // uniform; rows past m repeat the last one
            const float df = xv - U[(int64_t)i * ldu + t];
            sq[r] = fmaf(df, df, sq[r]);
        }
    }
    if (c >= cols) return;
#pragma unroll
    for (int r = 0; r < R; ++r)
        if (i0 + r < m)
            Kc[(int64_t)(i0 + r) * ldk + c] = variance * __builtin_amdgcn_exp2f(sq[r] * negc2);
}

// One wave per inducing point: fp32 products, one fp64 sum per lane over its columns
// (ascending), lanes added in a fixed butterfly.
__global__ __launch_bounds__(256) void sgpr_kufy_kernel(const float* __restrict__ Kc, int64_t ldk,
                                                        int m, int cols,
                                                        const float* __restrict__ y,
                                                        double* __restrict__ b) {
    const int lane = threadIdx.x & 63;
    const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= m) return;
    const float* __restrict__ row = Kc + (int64_t)i * ldk;
    double acc = 0.0;
    for (int c = lane; c < cols; c += 64) acc += (double)(row[c] * y[c]);
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) acc += __shfl_xor(acc, o);
    if (lane == 0) b[i] += acc;
}

__global__ __launch_bounds__(256) void sgpr_add_copies_kernel(double* __restrict__ A, int64_t lda,
                                                              const double* __restrict__ copies,
                                                              int64_t copy_stride, int ncopies,
                                                              int m) {
    const int i = blockIdx.x * 256 + threadIdx.x;  // column
    if (i >= m) return;
    for (int j = blockIdx.y; j < m; j += gridDim.y) {
        if (i > (j | 127)) continue;  // above the diagonal tile of row j: nothing was summed there
        double acc = A[(int64_t)j * lda + i];
        for (int g = 0; g < ncopies; ++g) acc += copies[(int64_t)g * copy_stride + (int64_t)j * m + i];
        A[(int64_t)j * lda + i] = acc;
    }
}

__global__ __launch_bounds__(256) void sgpr_symmetrize_kernel(double* __restrict__ A, int64_t lda,
                                                              int m) {
    // 16 x 16 tile of the strict upper triangle, read from its mirror image through LDS so
    // that both the loads and the stores run along rows
    __shared__ double tile[16][17];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int bi = blockIdx.y, bj = blockIdx.x;  // target tile: rows bi, columns bj
    if (bj < bi) return;
    const int sr = bj * 16 + ty, sc = bi * 16 + tx;  // source element A[sr][sc] (lower triangle)
    tile[ty][tx] = (sr < m && sc < m) ? A[(int64_t)sr * lda + sc] : 0.0;
    __syncthreads();
    const int r = bi * 16 + ty, c = bj * 16 + tx;
    if (r < m && c < m && c > r) A[(int64_t)r * lda + c] = tile[tx][ty];
}

// ---------------------------------------------------------------------------------------
// Chunk product on the matrix cores.  A workgroup of 4 waves owns one 128 x 128 tile of the
// lower triangle (tile row tj >= tile column ti) and walks the chunk's columns in steps of 16:
// rows of tile tj are the M side and rows of tile ti the N side of v_mfma_f32_32x32x2_f32,
// both staged through LDS, double buffered, with the global loads of step s+2 in flight
// during step s.  At the end every lane holds, per 32 x 32 block, 16 values of one column
// i = lane % 32, so for a fixed register the 32 lanes of a half wave write 32 consecutive
// fp64 entries of one row of A.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256, 2) void sgpr_syrk_kernel(const float* __restrict__ Kc_all,
                                                           int64_t ldk, int m, int cols_all,
                                                           int group_cols,
                                                           double* __restrict__ A0, int64_t lda0,
                                                           double* __restrict__ copies,
                                                           int64_t copy_stride) {
    // column group blockIdx.y: its run of columns and the matrix its sums go to
    const int grp = blockIdx.y;
    const float* __restrict__ Kc = Kc_all + (int64_t)grp * group_cols;
    const int cols = min(group_cols, cols_all - grp * group_cols);
    if (cols <= 0) return;  // whole workgroup, before any barrier
    double* __restrict__ A = grp == 0 ? A0 : copies + (int64_t)(grp - 1) * copy_stride;
    const int64_t lda = grp == 0 ? lda0 : (int64_t)m;
    constexpr int T = 128, KC = knn::kMfmaKC, RS = knn::kMfmaRowStride;
    extern __shared__ __align__(16) unsigned char smem[];
    float* js = reinterpret_cast<float*>(smem);  // [2][T][RS] rows of tile tj
    float* is = js + 2 * T * RS;                 // [2][T][RS] rows of tile ti
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int i32 = lane & 31;
    const int h = lane >> 5;

    // blockIdx.x = tj (tj + 1) / 2 + ti with ti <= tj
    int tj = (int)((sqrtf(8.f * (float)blockIdx.x + 1.f) - 1.f) * 0.5f);
    while ((tj + 1) * (tj + 2) / 2 <= (int)blockIdx.x) ++tj;
    while (tj * (tj + 1) / 2 > (int)blockIdx.x) --tj;
    const int ti = (int)blockIdx.x - tj * (tj + 1) / 2;
    const int row_j0 = tj * T, row_i0 = ti * T;
    const int my_i = wave * 32 + i32;

    const int total = (cols + KC - 1) / KC;
    const int srow = tid >> 2;
    const int scol = (tid & 3) * 4;

    struct Staged {
        f32x4 j0, j1, i0, i1;
    };
    // Branch-free: the same four loads from clamped addresses every time.  Rows are 16-byte
    // aligned and padded to a multiple of 4 columns, so a vector load never leaves its row.
    auto fetch = [&](int step, Staged& g) {
        const int col = step * KC + scol;
        g.j0 = load_row4<true>(Kc, ldk, (int64_t)row_j0 + srow, m, col, cols);
        g.j1 = load_row4<true>(Kc, ldk, (int64_t)row_j0 + srow + 64, m, col, cols);
        g.i0 = load_row4<true>(Kc, ldk, (int64_t)row_i0 + srow, m, col, cols);
        g.i1 = load_row4<true>(Kc, ldk, (int64_t)row_i0 + srow + 64, m, col, cols);
    };
    auto stash = [&](int step, const Staged& g) {
        const int buf = step & 1;
        const int col = step * KC + scol;
        float* jb = js + buf * T * RS;
        float* ib = is + buf * T * RS;
        *reinterpret_cast<f32x4*>(jb + srow * RS + scol) =
            mask_row4(g.j0, row_j0 + srow < m, col, cols, 1.f);
        *reinterpret_cast<f32x4*>(jb + (srow + 64) * RS + scol) =
            mask_row4(g.j1, row_j0 + srow + 64 < m, col, cols, 1.f);
        *reinterpret_cast<f32x4*>(ib + srow * RS + scol) =
            mask_row4(g.i0, row_i0 + srow < m, col, cols, 1.f);
        *reinterpret_cast<f32x4*>(ib + (srow + 64) * RS + scol) =
            mask_row4(g.i1, row_i0 + srow + 64 < m, col, cols, 1.f);
    };

    f32x16 acc[4];
#pragma unroll
    for (int pb = 0; pb < 4; ++pb)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[pb][e] = 0.f;

    Staged set_even, set_odd;
    if (total > 0) {
        fetch(0, set_even);
        stash(0, set_even);
    }
    if (total > 1) fetch(1, set_odd);
    __syncthreads();

    auto run_step = [&](int step, Staged& mine, const Staged& next) {
        const int buf = step & 1;
        fetch(step + 2 < total ? step + 2 : total - 1, mine);  // past the end: a harmless re-load
        const float* jb = js + buf * T * RS;
        const float* ib = is + buf * T * RS;
        f32x4 b[KC / 8], a[KC / 8][4];
#pragma unroll
        for (int g = 0; g < KC / 8; ++g) {
            const int col = g * 8 + h * 4;
            b[g] = *reinterpret_cast<const f32x4*>(ib + my_i * RS + col);
#pragma unroll
            for (int pb = 0; pb < 4; ++pb)
                a[g][pb] = *reinterpret_cast<const f32x4*>(jb + (pb * 32 + i32) * RS + col);
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
        __syncthreads();
    };
    for (int step = 0; step < total; step += 2) {
        run_step(step, set_even, set_odd);
        if (step + 1 < total) run_step(step + 1, set_odd, set_even);
    }

    // register v of block pb: row j = pb*32 + 8*(v/4) + 4*h + v%4 of tile tj, column my_i of tile ti
    const int i = row_i0 + my_i;
    if (i < m) {
#pragma unroll
        for (int pb = 0; pb < 4; ++pb) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int j = row_j0 + pb * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
                if (j < m) A[(int64_t)j * lda + i] += (double)acc[pb][v];
            }
        }
    }
}

}  // namespace

hipError_t launch_zero(double* A, int64_t lda, double* b, int64_t m, hipStream_t stream) {
    const unsigned gy = (unsigned)(m < 4096 ? m : 4096);
    sgpr_zero_kernel<<<dim3((unsigned)((m + 255) / 256), gy), dim3(256), 0, stream>>>(
        A, lda, b, (int)m);
    return hipGetLastError();
}

hipError_t launch_kuf(const float* U, int64_t ldu, const float* X, int64_t ldx, int64_t m,
                      int64_t c0, int64_t cols, int d, float c2, float variance, float* Kc,
                      int64_t ldk, hipStream_t stream) {
    const dim3 grid((unsigned)((cols + 255) / 256),
                    (unsigned)((m + kRowsPerThread - 1) / kRowsPerThread));
    sgpr_kuf_kernel<<<grid, dim3(256), 0, stream>>>(U, ldu, X, ldx, (int)m, c0, (int)cols, d, -c2,
                                                    variance, Kc, ldk);
    return hipGetLastError();
}

hipError_t launch_syrk(const float* Kc, int64_t ldk, int64_t m, int64_t cols, int groups, double* A,
                       int64_t lda, double* copies, int64_t copy_stride, hipStream_t stream) {
    const int64_t T = (m + 127) / 128;
    const size_t lds = (size_t)4 * 128 * knn::kMfmaRowStride * 4;
    // equal runs of whole 16-column steps; the last run takes what is left
    int64_t group_cols = ((cols + groups - 1) / groups + 15) / 16 * 16;
    if (group_cols < 16) group_cols = 16;
    sgpr_syrk_kernel<<<dim3((unsigned)(T * (T + 1) / 2), (unsigned)groups), dim3(256), lds, stream>>>(
        Kc, ldk, (int)m, (int)cols, (int)group_cols, A, lda, copies, copy_stride);
    return hipGetLastError();
}

hipError_t launch_add_copies(double* A, int64_t lda, const double* copies, int64_t copy_stride,
                             int ncopies, int64_t m, hipStream_t stream) {
    const unsigned gy = (unsigned)(m < 4096 ? m : 4096);
    sgpr_add_copies_kernel<<<dim3((unsigned)((m + 255) / 256), gy), dim3(256), 0, stream>>>(
        A, lda, copies, copy_stride, ncopies, (int)m);
    return hipGetLastError();
}

hipError_t launch_kufy(const float* Kc, int64_t ldk, int64_t m, int64_t cols, const float* y,
                       double* b, hipStream_t stream) {
    sgpr_kufy_kernel<<<dim3((unsigned)((m + 3) / 4)), dim3(256), 0, stream>>>(Kc, ldk, (int)m,
                                                                              (int)cols, y, b);
    return hipGetLastError();
}

hipError_t launch_symmetrize(double* A, int64_t lda, int64_t m, hipStream_t stream) {
    const unsigned t = (unsigned)((m + 15) / 16);
    sgpr_symmetrize_kernel<<<dim3(t, t), dim3(256), 0, stream>>>(A, lda, (int)m);
    return hipGetLastError();
}

}  // namespace sgpr
