// Final step of the gfx950 kNN search: merge the per-range partial lists of each query,
// re-evaluate the k winners in fp64 with the plain definition of the metric (paper
// sections 4.1 and 5.2) and write them ordered by (distance, index).
#include <hip/hip_runtime.h>

#include <climits>
#include <cmath>
#include <cstdint>

#include "knn_config.h"
#include "knn_device.h"
#include "knn_kernels.h"

namespace knn {

namespace {

// ---------------------------------------------------------------------------------------
// Merge of the S partial lists, exact re-evaluation, final order.  One wave per query.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ double exact_sqdist(const float* __restrict__ q,
                                               const float* __restrict__ x, int d) {
#pragma clang fp contract(off)
    double acc = 0.0;
    for (int t = 0; t < d; ++t) {
        const double diff = (double)q[t] - (double)x[t];
        acc = acc + diff * diff;
    }
    return acc;
}

// Cosine distance in fp64: 1 - <q,x> / (|q| |x|), clamped at 0; 1 if either vector is zero.
__device__ __forceinline__ double exact_cosdist(const float* __restrict__ q,
                                                const float* __restrict__ x, int d) {
#pragma clang fp contract(off)
    double qq = 0.0, xx = 0.0, qx = 0.0;
    for (int t = 0; t < d; ++t) {
        const double a = (double)q[t], b = (double)x[t];
        qq = qq + a * a;
        xx = xx + b * b;
        qx = qx + a * b;
    }
    if (qq == 0.0 || xx == 0.0) return 1.0;
    const double c = 1.0 - __ddiv_rn(qx, __dsqrt_rn(qq) * __dsqrt_rn(xx));
    return c < 0.0 ? 0.0 : c;
}

// L1 distance in fp64, ascending t.
__device__ __forceinline__ double exact_l1dist(const float* __restrict__ q,
                                               const float* __restrict__ x, int d) {
    double acc = 0.0;
    for (int t = 0; t < d; ++t) acc = acc + fabs((double)q[t] - (double)x[t]);
    return acc;
}

// metric: 0 squared Euclidean, 1 cosine, 2 L1 (the values of knn_metric)
__global__ __launch_bounds__(256) void knn_merge_refine_kernel(
    const float* __restrict__ Q, int64_t ldq, const float* __restrict__ X, int64_t ldx, int rows,
    int n, int d, int k, int S, int metric, int aligned, const float* __restrict__ lk,
    const int* __restrict__ li, int32_t* __restrict__ idx_out, float* __restrict__ dist_out,
    double* __restrict__ d64_out) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int r = blockIdx.x * 4 + wave;
    if (r >= rows) return;  // no workgroup barrier below
    double* wd = reinterpret_cast<double*>(smem) + (size_t)wave * k;
    int* wi = reinterpret_cast<int*>(reinterpret_cast<double*>(smem) + (size_t)4 * k) + (size_t)wave * k;
    float* wk = reinterpret_cast<float*>(reinterpret_cast<int*>(reinterpret_cast<double*>(smem) + (size_t)4 * k) +
                                         (size_t)4 * k) + (size_t)wave * k;  // the winners' list keys

    const size_t rb = (size_t)r * S * k;
    if (S == 1) {
        for (int p = lane; p < k; p += kWave) {
            wi[p] = li[rb + p];
            wk[p] = lk[rb + p];
        }
    } else {
        // rank of an entry = its position in its own list + entries of the other lists
        // that come before it; indices are distinct, so ranks are too
        const int total = S * k;
        for (int e = lane; e < total; e += kWave) {
            const int se = e / k;
            const int p = e - se * k;
            const float key = lk[rb + e];
            const int id = li[rb + e];
            int rank = p;
            for (int s2 = 0; s2 < S && rank < k; ++s2) {
                if (s2 == se) continue;
                const float* k2 = lk + rb + (size_t)s2 * k;
                const int* i2 = li + rb + (size_t)s2 * k;
                int lo = 0, hi = k;
                while (lo < hi) {
                    const int mid = (lo + hi) >> 1;
                    if (before(k2[mid], i2[mid], key, id)) lo = mid + 1;
                    else hi = mid;
                }
                rank += lo;
            }
            if (rank < k) {
                wi[rank] = id;
                wk[rank] = key;
            }
        }
    }
    wave_sync();
    if (metric == 0 && aligned) {
        // Squared-Euclidean distances of rows that are 16-byte aligned: eight lanes per winner, so
        // that a load instruction reads whole 128-byte lines of eight rows (with a lane per winner
        // every instruction touched 64 rows - here every wave of the chip gathers rows at the same
        // time, the case in which that costs half the throughput).  Lane t of a winner adds up the
        // groups of four coordinates t, t + 8, ... in ascending order, one fp64 addition per
        // coordinate and no contraction; the eight partial sums meet in a butterfly (lane distances
        // 1, 2, 4).  Four passes of eight winners have their loads in flight together.
#pragma clang fp contract(off)
        const int part = lane & 7, wl = lane >> 3;
        const int ng = d >> 2;
        const float* qp = Q + (int64_t)r * ldq;
        for (int w0 = 0; w0 < k; w0 += 32) {
            double acc[4];
            const float* xp[4];
            bool ok[4];
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const int w = w0 + 8 * p + wl;
                const int j = w < k ? wi[w] : -1;
                ok[p] = (unsigned)j < (unsigned)n;
                xp[p] = X + (int64_t)(ok[p] ? j : 0) * ldx;
                acc[p] = 0.0;
            }
            for (int g0 = part; g0 < ng; g0 += 16) {
                f32x4 qv[2], xv[4][2];
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int g = g0 + 8 * u;
                    const int gc = g < ng ? g : part;  // a valid group; its value is not used
                    qv[u] = *reinterpret_cast<const f32x4*>(qp + 4 * gc);
#pragma unroll
                    for (int p = 0; p < 4; ++p) xv[p][u] = *reinterpret_cast<const f32x4*>(xp[p] + 4 * gc);
                }
#pragma unroll
                for (int p = 0; p < 4; ++p)
#pragma unroll
                    for (int u = 0; u < 2; ++u) {
                        if (g0 + 8 * u < ng) {
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const double diff = (double)qv[u][e] - (double)xv[p][u][e];
                                acc[p] = acc[p] + diff * diff;
                            }
                        }
                    }
            }
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                acc[p] = acc[p] + __shfl_xor(acc[p], 1);
                acc[p] = acc[p] + __shfl_xor(acc[p], 2);
                acc[p] = acc[p] + __shfl_xor(acc[p], 4);
                const int w = w0 + 8 * p + wl;
                if (part == 0 && w < k) wd[w] = ok[p] ? acc[p] : __builtin_huge_val();
            }
        }
    } else
    for (int w = lane; w < k; w += kWave) {
        const int j = wi[w];
        double dist = __builtin_huge_val();
        if ((unsigned)j < (unsigned)n) {
            const float* qp = Q + (int64_t)r * ldq;
            const float* xp = X + (int64_t)j * ldx;
            dist = metric == 1 ? exact_cosdist(qp, xp, d)
                               : (metric == 2 ? exact_l1dist(qp, xp, d)
                                              : exact_sqdist(qp, xp, d));
        }
        wd[w] = dist;
    }
    wave_sync();
    if (d64_out) {
        // One block of a search over blocks of points (knn_search_host_x): the winners stay in
        // the order of their list keys, with the key in dist_out and the fp64 distance beside
        // it, for knn_fold_keyed_kernel; the final order comes when all blocks are in.
        for (int w = lane; w < k; w += kWave) {
            idx_out[(size_t)r * k + w] = wi[w];
            dist_out[(size_t)r * k + w] = wk[w];
            d64_out[(size_t)r * k + w] = wd[w];
        }
        return;
    }
    for (int w = lane; w < k; w += kWave) {
        const double dw = wd[w];
        const int jw = wi[w];
        // (identical entries can only be the (+inf, no index) fillers of lists that ended up
        // shorter than k; their slot number keeps the ranks distinct)
        int rank = 0;
        for (int v = 0; v < k; ++v)
            rank += (before64(wd[v], wi[v], dw, jw) || (wd[v] == dw && wi[v] == jw && v < w)) ? 1 : 0;
        idx_out[(size_t)r * k + rank] = jw;
        dist_out[(size_t)r * k + rank] = (float)dw;
    }
}

// Running result of a search over blocks of points, kept in the order of the list keys - the
// total order (key, index) in which a resident search merges its point ranges - so that the k
// entries that survive all blocks are the very ones a resident search selects.  One wave per
// query row: running entries (index in idx, key in key, fp64 distance in d64; none yet with
// first != 0) and the block's kb entries (indices + offset) are staged in LDS, every entry finds
// its place by a binary search over the other list, the first k are written back.
__global__ __launch_bounds__(256) void knn_fold_keyed_kernel(
    const int32_t* __restrict__ bidx, const float* __restrict__ bkey, const double* __restrict__ bd64,
    int kb, int offset, int first, int rows, int k, int32_t* __restrict__ idx, float* __restrict__ key,
    double* __restrict__ d64) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    double* ad = reinterpret_cast<double*>(smem) + (size_t)wave * 2 * k;  // running fp64 [k]
    double* bd = ad + k;                                                  // block fp64   [k]
    float* ak = reinterpret_cast<float*>(reinterpret_cast<double*>(smem) + (size_t)4 * 2 * k) + (size_t)wave * 4 * k;
    int* ai = reinterpret_cast<int*>(ak + k);
    float* bk = reinterpret_cast<float*>(ai + k);
    int* bi = reinterpret_cast<int*>(bk + k);
    const int r = blockIdx.x * 4 + wave;
    if (r >= rows) return;  // whole wave; no workgroup barrier below
    const int na = first ? 0 : k;
    const size_t rb = (size_t)r * k;
    for (int p = lane; p < na; p += kWave) {
        ak[p] = key[rb + p];
        ai[p] = idx[rb + p];
        ad[p] = d64[rb + p];
    }
    for (int p = lane; p < kb; p += kWave) {
        bk[p] = bkey[(size_t)r * kb + p];
        const int j = bidx[(size_t)r * kb + p];
        bi[p] = j == kNoIdx ? kNoIdx : j + offset;
        bd[p] = bd64[(size_t)r * kb + p];
    }
    wave_sync();
    for (int p = lane; p < na; p += kWave) {  // behind the block entries that come before it
        int lo = 0, hi = kb;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (before(bk[mid], bi[mid], ak[p], ai[p])) lo = mid + 1;
            else hi = mid;
        }
        const int pos = p + lo;
        if (pos < k) {
            key[rb + pos] = ak[p];
            idx[rb + pos] = ai[p];
            d64[rb + pos] = ad[p];
        }
    }
    for (int p = lane; p < kb; p += kWave) {  // behind the running entries that come before it
        int lo = 0, hi = na;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (before(ak[mid], ai[mid], bk[p], bi[p])) lo = mid + 1;
            else hi = mid;
        }
        const int pos = p + lo;
        if (pos < k) {
            key[rb + pos] = bk[p];
            idx[rb + pos] = bi[p];
            d64[rb + pos] = bd[p];
        }
    }
    for (int p = na + kb + lane; p < k; p += kWave) {  // nothing yet beyond the points seen so far
        key[rb + p] = kInf;
        idx[rb + p] = kNoIdx;
        d64[rb + p] = __builtin_huge_val();
    }
}

// The final order of such a running result: by (fp64 distance, index), as knn_merge_refine_kernel
// orders the winners of a resident search; dist gets the fp64 distance rounded to fp32.
__global__ __launch_bounds__(256) void knn_order_final_kernel(int rows, int k, int32_t* __restrict__ idx,
                                                              float* __restrict__ dist,
                                                              const double* __restrict__ d64) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    double* wd = reinterpret_cast<double*>(smem) + (size_t)wave * k;
    int* wi = reinterpret_cast<int*>(reinterpret_cast<double*>(smem) + (size_t)4 * k) + (size_t)wave * k;
    const int r = blockIdx.x * 4 + wave;
    if (r >= rows) return;
    const size_t rb = (size_t)r * k;
    for (int p = lane; p < k; p += kWave) {
        wd[p] = d64[rb + p];
        wi[p] = idx[rb + p];
    }
    wave_sync();
    for (int w = lane; w < k; w += kWave) {
        const double dw = wd[w];
        const int jw = wi[w];
        int rank = 0;
        for (int v = 0; v < k; ++v)
            rank += (before64(wd[v], wi[v], dw, jw) || (wd[v] == dw && wi[v] == jw && v < w)) ? 1 : 0;
        idx[rb + rank] = jw;
        dist[rb + rank] = (float)dw;
    }
}

}  // namespace

hipError_t launch_fold_keyed(const int32_t* bidx, const float* bkey, const double* bd64, int kb,
                             int64_t offset, int first, int64_t rows, int k, int32_t* idx, float* key,
                             double* d64, hipStream_t stream) {
    const size_t lds = (size_t)4 * k * (2 * sizeof(double) + 4 * sizeof(float));
    hipError_t e = raise_lds_limit(knn_fold_keyed_kernel, lds);
    if (e != hipSuccess) return e;
    knn_fold_keyed_kernel<<<dim3((unsigned)((rows + 3) / 4)), dim3(256), lds, stream>>>(
        bidx, bkey, bd64, kb, (int)offset, first, (int)rows, k, idx, key, d64);
    return hipGetLastError();
}

hipError_t launch_order_final(int64_t rows, int k, int32_t* idx, float* dist, const double* d64,
                              hipStream_t stream) {
    const size_t lds = (size_t)4 * k * (sizeof(double) + sizeof(int));
    hipError_t e = raise_lds_limit(knn_order_final_kernel, lds);
    if (e != hipSuccess) return e;
    knn_order_final_kernel<<<dim3((unsigned)((rows + 3) / 4)), dim3(256), lds, stream>>>((int)rows, k, idx,
                                                                                       dist, d64);
    return hipGetLastError();
}

hipError_t launch_merge_refine(const float* Q, int64_t ldq, const float* X, int64_t ldx,
                               int64_t rows, int64_t n, int d, int k, int S, int metric,
                               const float* lk, const int* li, int32_t* idx, float* dist,
                               hipStream_t stream, double* d64) {
    const size_t lds = (size_t)4 * k * (sizeof(double) + sizeof(int) + sizeof(float));
    hipError_t e = raise_lds_limit(knn_merge_refine_kernel, lds);
    if (e != hipSuccess) return e;
    dim3 grid((unsigned)((rows + 3) / 4));
    const int aligned = (reinterpret_cast<uintptr_t>(Q) % 16 == 0) && (reinterpret_cast<uintptr_t>(X) % 16 == 0) &&
                        (ldq % 4 == 0) && (ldx % 4 == 0) && (d % 4 == 0);
    knn_merge_refine_kernel<<<grid, dim3(256), lds, stream>>>(
        Q, ldq, X, ldx, (int)rows, (int)n, d, k, S, metric, aligned, lk, li, idx, dist, d64);
    return hipGetLastError();
}

}  // namespace knn
