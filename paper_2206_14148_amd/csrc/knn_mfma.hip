// gfx950 (CDNA4, MI355X) matrix-core kNN search kernels (d > 8, and the cosine metric):
// keys come from the expansion  sum x^2 - 2 q.x  of paper section 4.1, evaluated as fp32
// MFMA tiles that never leave the registers (section 4.3: the distance tile is the
// intermediate that must not be materialised).
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
// ---------------------------------------------------------------------------------------
// Matrix-core path: a workgroup of 4 waves owns 128 queries and walks its point range in
// tiles of 128 points.  Data points are the M side and queries the N side of
// v_mfma_f32_32x32x2_f32, so the 16 accumulator values a lane holds per 32x32 block all
// belong to ONE query (column = lane % 32): its threshold is one register and the filter
// is a per-lane compare.  The accumulators start at ||x||^2 and receive (-2 q) . x, which
// gives the key  ||x||^2 - 2 q.x  (the distance minus the per-query constant ||q||^2).
// ---------------------------------------------------------------------------------------
template <bool ALIGNED>
__global__ __launch_bounds__(256, 2) void knn_mfma_kernel(
    const float* __restrict__ Q, int64_t ldq, const float* __restrict__ X, int64_t ldx,
    const float* __restrict__ xn, int cosine, int rows, int n, int d, int k, int S, int split_len,
    int BQ, int BS, float* __restrict__ lk, int* __restrict__ li) {
    constexpr int TQ = kMfmaTileQ, TX = kMfmaTileX, KC = kMfmaKC, RS = kMfmaRowStride;
    constexpr int C = kMfmaCand;
    extern __shared__ __align__(16) unsigned char smem[];
    float* xs = reinterpret_cast<float*>(smem);        // [2][TX][RS]
    float* qs = xs + 2 * TX * RS;                      // [2][TQ][RS]
    float* xns = qs + 2 * TQ * RS;                     // [2][TX] accumulator start values
    float* rns = xns + 2 * TX;                         // [2][TX] row scales (cosine metric)
    float* ck = rns + 2 * TX;                          // [TQ][C]
    int* ci = reinterpret_cast<int*>(ck + TQ * C);     // [TQ][C]
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    MergeScratch sc;
    {
        float* pw = reinterpret_cast<float*>(ci + TQ * C) + (size_t)wave * (2 * kWave + 2 * k);
        sc.cand_key = pw;
        sc.cand_idx = reinterpret_cast<int*>(pw + kWave);
        sc.list_key = pw + 2 * kWave;
        sc.list_idx = reinterpret_cast<int*>(pw + 2 * kWave + k);
    }
    const int i32 = lane & 31;  // query column / point row inside a 32x32 block
    const int h = lane >> 5;    // which half of the wave

    int s, wg_row0;
    if (!xcd_block_map(rows, TQ, S, BQ, BS, s, wg_row0)) return;  // padding (before any barrier)
    const int my_q = wave * 32 + i32;  // query inside the workgroup tile
    const int r = wg_row0 + my_q;
    const bool active = r < rows;

    init_lists32(lk, li, wg_row0 + wave * 32, rows, S, s, k, lane);
    WaveLists wl;
    wl.lk = lk;
    wl.li = li;
    wl.k = k;
    wl.S = S;
    wl.s = s;
    wl.row0 = wg_row0 + wave * 32;
    wl.ck = ck + wave * 32 * C;
    wl.ci = ci + wave * 32 * C;
    wl.sc = sc;
    wl.lane = lane;

    float tau = active ? kInf : -kInf;
    int cnt = 0;  // candidates buffered for this lane's query (same value in both halves)

    const int j0 = s * split_len;
    const int j1 = min(n, j0 + split_len);
    const int ntiles = (j1 > j0) ? (j1 - j0 + TX - 1) / TX : 0;
    const int nch = (d + KC - 1) / KC;
    const int total = ntiles * nch;

    // staging role of this thread: rows srow and srow + 64, four columns at scol
    const int srow = tid >> 2;
    const int scol = (tid & 3) * 4;

    // Global -> register -> LDS staging.  Two register sets alternate: the loads of step s+2
    // are issued at the start of step s and written to LDS at the end of step s+1, so a load
    // has about two steps to come back from beyond the L2 (the step loop is unrolled by two
    // so that the sets are named statically and never copied).
    struct Staged {
        f32x4 x0, x1, q0, q1;
        float xnv;
    };
    // fetch() is branch-free on purpose: every call issues the same five loads, so the
    // compiler can count how many newer loads may still be in flight when an older set is
    // written to LDS (a conditional load would force it to wait for everything).
    auto fetch = [&](int step, Staged& g) {
        const int tile = step / nch;
        const int c = step - tile * nch;
        const int col = c * KC + scol;
        const int64_t jr = (int64_t)j0 + (int64_t)tile * TX + srow;
        g.x0 = load_row4<ALIGNED>(X, ldx, jr, j1, col, d);
        g.x1 = load_row4<ALIGNED>(X, ldx, jr + 64, j1, col, d);
        g.q0 = load_row4<ALIGNED>(Q, ldq, (int64_t)wg_row0 + srow, rows, col, d);
        g.q1 = load_row4<ALIGNED>(Q, ldq, (int64_t)wg_row0 + srow + 64, rows, col, d);
        const int64_t jj = (int64_t)j0 + (int64_t)tile * TX + (tid & (TX - 1));
        g.xnv = xn[jj < j1 ? jj : j1 - 1];
    };
    auto stash = [&](int step, const Staged& g) {
        const int tile = step / nch;
        const int c = step - tile * nch;
        const int buf = step & 1;
        const int col = c * KC + scol;
        const int64_t jr = (int64_t)j0 + (int64_t)tile * TX + srow;
        float* xb = xs + buf * TX * RS;
        float* qb = qs + buf * TQ * RS;
        *reinterpret_cast<f32x4*>(xb + srow * RS + scol) = mask_row4(g.x0, jr < j1, col, d, 1.f);
        *reinterpret_cast<f32x4*>(xb + (srow + 64) * RS + scol) =
            mask_row4(g.x1, jr + 64 < j1, col, d, 1.f);
        *reinterpret_cast<f32x4*>(qb + srow * RS + scol) =
            mask_row4(g.q0, wg_row0 + srow < rows, col, d, -2.f);
        *reinterpret_cast<f32x4*>(qb + (srow + 64) * RS + scol) =
            mask_row4(g.q1, wg_row0 + srow + 64 < rows, col, d, -2.f);
        if (c == 0 && tid < TX) {
            const int64_t jj = (int64_t)j0 + (int64_t)tile * TX + tid;
            // rows past the range get +inf: they can never be accepted.  xn holds |x|^2
            // (start value) for the Euclidean metric, 1/|x| (final scale) for cosine.
            xns[(tile & 1) * TX + tid] = jj < j1 ? (cosine ? 0.f : g.xnv) : kInf;
            rns[(tile & 1) * TX + tid] = (cosine && jj < j1) ? g.xnv : 1.f;
        }
    };

    f32x16 acc[4];

    Staged set_even, set_odd;  // staged data of even / odd steps
    if (total > 0) {
        fetch(0, set_even);
        stash(0, set_even);
    }
    if (total > 1) fetch(1, set_odd);
    __syncthreads();

    // one pipeline step; `mine` holds step+2 afterwards, `next` holds step+1 on entry
    auto run_step = [&](int step, Staged& mine, const Staged& next) {
        const int tile = step / nch;
        const int c = step - tile * nch;
        const int buf = step & 1;
        fetch(step + 2 < total ? step + 2 : total - 1, mine);  // past the end: a harmless re-load

        if (c == 0) {
            const float* xt = xns + (tile & 1) * TX;
#pragma unroll
            for (int pb = 0; pb < 4; ++pb) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const f32x4 v = *reinterpret_cast<const f32x4*>(xt + pb * 32 + g * 8 + h * 4);
                    acc[pb][g * 4 + 0] = v[0];
                    acc[pb][g * 4 + 1] = v[1];
                    acc[pb][g * 4 + 2] = v[2];
                    acc[pb][g * 4 + 3] = v[3];
                }
            }
        }
        {
            // Both K groups of the step are read up front; the write of the next step's
            // data to the other LDS buffer sits between the two MFMA groups so that its
            // LDS traffic and waits overlap with matrix work of this wave.
            const float* xb = xs + buf * TX * RS;
            const float* qb = qs + buf * TQ * RS;
            f32x4 b[KC / 8], a[KC / 8][4];
#pragma unroll
            for (int g = 0; g < KC / 8; ++g) {
                const int col = g * 8 + h * 4;
                b[g] = *reinterpret_cast<const f32x4*>(qb + my_q * RS + col);
#pragma unroll
                for (int pb = 0; pb < 4; ++pb)
                    a[g][pb] = *reinterpret_cast<const f32x4*>(xb + (pb * 32 + i32) * RS + col);
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
            if (cosine) scale_rows(acc, rns + (tile & 1) * TX, h);
            tile_epilogue<C>(acc, wl, j0 + tile * TX, tau, cnt);
        }

        __syncthreads();
    };
    for (int step = 0; step < total; step += 2) {
        run_step(step, set_even, set_odd);
        if (step + 1 < total) run_step(step + 1, set_odd, set_even);
    }
    const uint64_t rest = __builtin_amdgcn_ballot_w64(cnt > 0) & 0xffffffffull;
    if (rest) flush_lists<C>(wl, rest, tau, cnt);
}

// ---------------------------------------------------------------------------------------
// Blocked copy of the points for the register-resident-query kernel: tile t (128 rows) and
// K chunk c (16 columns) become one contiguous 8 KB block, in the order the kernel reads
// them, zero-filled past n and past d.  A workgroup's point stream is then one contiguous
// run (full cache lines, no power-of-two row stride hammering a few L2 sets) that the
// workgroups sharing a range pull through the L2 once.  Needs 4 * ceil(n/128)*128 *
// ceil(d/16)*16 bytes of workspace, so the planner uses it only when the limit has room.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void knn_block_points_kernel(const float* __restrict__ X,
                                                               int64_t ldx, int n, int d,
                                                               f32x4* __restrict__ Xb) {
    constexpr int TX = kMfmaTileX, KC = kMfmaKC;
    const int nch = (d + KC - 1) / KC;
    const int tile = blockIdx.x;
    const int srow = threadIdx.x >> 2;
    const int scol = (threadIdx.x & 3) * 4;
    for (int c = 0; c < nch; ++c) {
        const int col = c * KC + scol;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int64_t row = (int64_t)tile * TX + srow + half * 64;
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
            if (row < n) {
                const float* p = X + row * ldx;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (col + e < d) v[e] = p[col + e];
            }
            Xb[((size_t)tile * nch + c) * 512 + threadIdx.x + half * 256] = v;
        }
    }
}

// ---------------------------------------------------------------------------------------
// Matrix-core path for d <= 16 * NCH <= 256: as knn_mfma_kernel, but the queries never go
// through LDS or the L2 again.  A lane keeps the K values of its query that its half of the
// wave feeds to the MFMAs (d/2 registers, scaled by -2) for the whole kernel, so only the
// point stream is staged: half the global requests, half the LDS writes, and the L2 of an XCD
// holds nothing but the point windows its workgroups share.  The chunk loop of a tile is
// unrolled (together with a second tile when NCH is odd), which also names the two prefetch
// register sets statically.
// ---------------------------------------------------------------------------------------
template <int NCH, bool ALIGNED, bool BLOCKED>
__global__ __launch_bounds__(256, 2) void knn_mfma_qreg_kernel(
    const float* __restrict__ Q, int64_t ldq, const float* __restrict__ X, int64_t ldx,
    const f32x4* __restrict__ Xb, const float* __restrict__ xn, int cosine, int rows, int n, int d,
    int k, int S, int split_len, int BQ, int BS, float* __restrict__ lk, int* __restrict__ li) {
    // the steps (tile, chunk) alternate two LDS buffers and two register sets; the loops are
    // unrolled far enough (two tiles when NCH is odd) for the alternation to be static
    constexpr int TU = (NCH % 2) ? 2 : 1;
    constexpr int TQ = kMfmaTileQ, TX = kMfmaTileX, KC = kMfmaKC, RS = kMfmaRowStride;
    constexpr int C = kMfmaCand;
    extern __shared__ __align__(16) unsigned char smem[];
    float* xs = reinterpret_cast<float*>(smem);     // [2][TX][RS]
    float* xns = xs + 2 * TX * RS;                  // [2][TX] accumulator start values
    float* rns = xns + 2 * TX;                      // [2][TX] row scales (cosine metric)
    float* ck = rns + 2 * TX;                       // [TQ][C]
    int* ci = reinterpret_cast<int*>(ck + TQ * C);  // [TQ][C]
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int i32 = lane & 31;
    const int h = lane >> 5;

    int s, wg_row0;
    if (!xcd_block_map(rows, TQ, S, BQ, BS, s, wg_row0)) return;  // padding (before any barrier)
    const int r = wg_row0 + wave * 32 + i32;
    const bool active = r < rows;

    WaveLists wl;
    wl.lk = lk;
    wl.li = li;
    wl.k = k;
    wl.S = S;
    wl.s = s;
    wl.row0 = wg_row0 + wave * 32;
    wl.ck = ck + wave * 32 * C;
    wl.ci = ci + wave * 32 * C;
    {
        float* pw = reinterpret_cast<float*>(ci + TQ * C) + (size_t)wave * (2 * kWave + 2 * k);
        wl.sc.cand_key = pw;
        wl.sc.cand_idx = reinterpret_cast<int*>(pw + kWave);
        wl.sc.list_key = pw + 2 * kWave;
        wl.sc.list_idx = reinterpret_cast<int*>(pw + 2 * kWave + k);
    }
    wl.lane = lane;
    init_lists32(lk, li, wl.row0, rows, S, s, k, lane);

    // B operand of every MFMA of a tile: K columns 8g + 4h .. 8g + 4h + 3 of this lane's query
    f32x4 qreg[2 * NCH];
#pragma unroll
    for (int g = 0; g < 2 * NCH; ++g) {
        const int col = g * 8 + h * 4;
        qreg[g] = mask_row4(load_row4<ALIGNED>(Q, ldq, r, rows, col, d), active, col, d, -2.f);
    }

    float tau = active ? kInf : -kInf;
    int cnt = 0;

    const int j0 = s * split_len;
    const int j1 = min(n, j0 + split_len);
    const int ntiles = (j1 > j0) ? (j1 - j0 + TX - 1) / TX : 0;
    const int total = ntiles * NCH;

    const int srow = tid >> 2;
    const int scol = (tid & 3) * 4;
    struct Staged {
        f32x4 x0, x1;
        float xnv;
    };
    // branch-free: the same three loads on every call (see knn_mfma_kernel)
    const int nch_real = (d + KC - 1) / KC;  // chunks that exist in the blocked copy
    auto fetch = [&](int step, Staged& g) {
        const int tile = step / NCH;
        const int c = step - tile * NCH;
        if (BLOCKED) {
            // block (tile, chunk): 512 float4, this thread takes entries tid and tid + 256
            const size_t blk = (size_t)(j0 / TX + tile) * nch_real + (c < nch_real ? c : 0);
            g.x0 = Xb[blk * 512 + tid];
            g.x1 = Xb[blk * 512 + tid + 256];
        } else {
            const int col = c * KC + scol;
            const int64_t jr = (int64_t)j0 + (int64_t)tile * TX + srow;
            g.x0 = load_row4<ALIGNED>(X, ldx, jr, j1, col, d);
            g.x1 = load_row4<ALIGNED>(X, ldx, jr + 64, j1, col, d);
        }
        const int64_t jj = (int64_t)j0 + (int64_t)tile * TX + (tid & (TX - 1));
        g.xnv = xn[jj < j1 ? jj : j1 - 1];
    };
    auto stash = [&](int step, const Staged& g) {
        const int tile = step / NCH;
        const int c = step - tile * NCH;
        const int col = c * KC + scol;
        const int64_t jr = (int64_t)j0 + (int64_t)tile * TX + srow;
        float* xb = xs + (step & 1) * TX * RS;
        if (BLOCKED) {  // the copy is zero-filled already; only a whole missing chunk is masked
            const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
            *reinterpret_cast<f32x4*>(xb + srow * RS + scol) = c < nch_real ? g.x0 : zero;
            *reinterpret_cast<f32x4*>(xb + (srow + 64) * RS + scol) = c < nch_real ? g.x1 : zero;
        } else {
            *reinterpret_cast<f32x4*>(xb + srow * RS + scol) =
                mask_row4(g.x0, jr < j1, col, d, 1.f);
            *reinterpret_cast<f32x4*>(xb + (srow + 64) * RS + scol) =
                mask_row4(g.x1, jr + 64 < j1, col, d, 1.f);
        }
        if (c == 0 && tid < TX) {
            const int64_t jj = (int64_t)j0 + (int64_t)tile * TX + tid;
            // +inf: never accepted.  xn is |x|^2 (Euclidean) or 1/|x| (cosine), see above.
            xns[(tile & 1) * TX + tid] = jj < j1 ? (cosine ? 0.f : g.xnv) : kInf;
            rns[(tile & 1) * TX + tid] = (cosine && jj < j1) ? g.xnv : 1.f;
        }
    };

    Staged set_even, set_odd;
    if (total > 0) {
        fetch(0, set_even);
        stash(0, set_even);
        fetch(total > 1 ? 1 : 0, set_odd);
    }
    __syncthreads();

    f32x16 acc[4];
    for (int tile0 = 0; tile0 < ntiles; tile0 += TU) {
#pragma unroll
        for (int tt = 0; tt < TU; ++tt) {
            const int tile = tile0 + tt;
            if (tile >= ntiles) break;  // uniform
            {
                const float* xt = xns + (tile & 1) * TX;
#pragma unroll
                for (int pb = 0; pb < 4; ++pb) {
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const f32x4 v = *reinterpret_cast<const f32x4*>(xt + pb * 32 + g * 8 + h * 4);
                        acc[pb][g * 4 + 0] = v[0];
                        acc[pb][g * 4 + 1] = v[1];
                        acc[pb][g * 4 + 2] = v[2];
                        acc[pb][g * 4 + 3] = v[3];
                    }
                }
            }
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                const int step = tile * NCH + c;
                const int par = (tt * NCH + c) & 1;  // == step & 1, known at compile time
                Staged& mine = par ? set_odd : set_even;        // receives step + 2
                const Staged& next = par ? set_even : set_odd;  // holds step + 1
                fetch(step + 2 < total ? step + 2 : total - 1, mine);
                const float* xb = xs + par * TX * RS;
                f32x4 a[2][4];
#pragma unroll
                for (int g = 0; g < 2; ++g) {
#pragma unroll
                    for (int pb = 0; pb < 4; ++pb)
                        a[g][pb] = *reinterpret_cast<const f32x4*>(xb + (pb * 32 + i32) * RS + g * 8 + h * 4);
                }
#pragma unroll
                for (int g = 0; g < 2; ++g) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
#pragma unroll
                        for (int pb = 0; pb < 4; ++pb)
                            acc[pb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[g][pb][e], qreg[2 * c + g][e],
                                                                           acc[pb], 0, 0, 0);
                    }
                    if (g == 0 && step + 1 < total) stash(step + 1, next);
                }
                if (c == NCH - 1) {
                    if (cosine) scale_rows(acc, rns + (tile & 1) * TX, h);
                    tile_epilogue<C>(acc, wl, j0 + tile * TX, tau, cnt);
                }
                __syncthreads();
            }
        }
    }
    const uint64_t rest = __builtin_amdgcn_ballot_w64(cnt > 0) & 0xffffffffull;
    if (rest) flush_lists<C>(wl, rest, tau, cnt);
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
hipError_t launch_block_points(const float* X, int64_t ldx, int64_t n, int d, void* xblocked,
                               hipStream_t stream) {
    const unsigned tiles = (unsigned)((n + kMfmaTileX - 1) / kMfmaTileX);
    knn_block_points_kernel<<<dim3(tiles), dim3(256), 0, stream>>>(
        X, ldx, (int)n, d, static_cast<f32x4*>(xblocked));
    return hipGetLastError();
}

hipError_t launch_mfma(const float* Q, int64_t ldq, const float* X, int64_t ldx, const float* xn,
                       const void* xblocked, bool cosine, int64_t rows, int64_t n, int d, int k,
                       int S, float* lk, int* li, hipStream_t stream) {
    const size_t lds = (size_t)(2 * kMfmaTileX * kMfmaRowStride + 2 * kMfmaTileQ * kMfmaRowStride +
                                4 * kMfmaTileX + 2 * kMfmaTileQ * kMfmaCand +
                                4 * (2 * kWave + 2 * k)) * 4;
    int64_t split_len = (n + S - 1) / S;
    split_len = (split_len + kMfmaTileX - 1) / kMfmaTileX * kMfmaTileX;
    // block shape for the XCD-aware mapping: BS = a divisor of S, BQ query tiles whose rows
    // (BQ * 128 * d floats) stay within about half of one XCD's 4 MB L2, BQ * BS <= 64
    // (the workgroups one XCD holds at a time)
    const int T = (int)((rows + kMfmaTileQ - 1) / kMfmaTileQ);
    int bq_cap = (int)(2 * 1024 * 1024 / ((int64_t)kMfmaTileQ * d * 4));
    if (bq_cap < 1) bq_cap = 1;
    if (bq_cap > 64) bq_cap = 64;
    const int bs_cap = (64 / bq_cap) > 8 ? (64 / bq_cap) : 8;
    int BS = 1;
    for (int v = 1; v <= S && v <= bs_cap; ++v)
        if (S % v == 0) BS = v;
    int BQ = 64 / BS;
    if (BQ > bq_cap) BQ = bq_cap;
    if (BQ > T) BQ = T;
    if (BQ < 1) BQ = 1;
    const int nQB = (T + BQ - 1) / BQ;
    const int blocks = nQB * (S / BS);
    const unsigned grid_x = (unsigned)((blocks + 7) / 8 * 8 * BQ * BS);
    dim3 grid(grid_x);
    const bool aligned = (reinterpret_cast<uintptr_t>(Q) % 16 == 0) &&
                         (reinterpret_cast<uintptr_t>(X) % 16 == 0) && (ldq % 4 == 0) &&
                         (ldx % 4 == 0) && (d % 4 == 0);
    if (d <= 16 * kMfmaQregMaxChunks) {
        // queries held in registers: only the point stream goes through LDS
        const size_t lds_q = lds - (size_t)2 * kMfmaTileQ * kMfmaRowStride * 4;
        const int nch = (d + kMfmaKC - 1) / kMfmaKC;
#define KNN_QREG_LAUNCH_AB(N, A, B)                                                               \
    do {                                                                                          \
        hipError_t e2 = raise_lds_limit(knn_mfma_qreg_kernel<N, A, B>, lds_q);                    \
        if (e2 != hipSuccess) return e2;                                                          \
        knn_mfma_qreg_kernel<N, A, B><<<grid, dim3(256), lds_q, stream>>>(                        \
            Q, ldq, X, ldx, reinterpret_cast<const f32x4*>(xblocked), xn, cosine ? 1 : 0,         \
            (int)rows, (int)n, d, k, S, (int)split_len, BQ, BS, lk, li);                          \
    } while (0)
#define KNN_QREG_LAUNCH(N)                                                                        \
    do {                                                                                          \
        if (xblocked) {                                                                           \
            if (aligned) KNN_QREG_LAUNCH_AB(N, true, true);                                       \
            else KNN_QREG_LAUNCH_AB(N, false, true);                                              \
        } else {                                                                                  \
            if (aligned) KNN_QREG_LAUNCH_AB(N, true, false);                                      \
            else KNN_QREG_LAUNCH_AB(N, false, false);                                             \
        }                                                                                         \
    } while (0)
        if (nch <= 1) KNN_QREG_LAUNCH(1);
        else if (nch <= 2) KNN_QREG_LAUNCH(2);
        else if (nch <= 4) KNN_QREG_LAUNCH(4);
        else if (nch <= 6) KNN_QREG_LAUNCH(6);
        else if (nch <= 8) KNN_QREG_LAUNCH(8);
        else if (nch <= 12) KNN_QREG_LAUNCH(12);
        else KNN_QREG_LAUNCH(16);
#undef KNN_QREG_LAUNCH_AB
#undef KNN_QREG_LAUNCH
        return hipGetLastError();
    }
    hipError_t e;
    if (aligned) {
        e = raise_lds_limit(knn_mfma_kernel<true>, lds);
        if (e != hipSuccess) return e;
        knn_mfma_kernel<true><<<grid, dim3(256), lds, stream>>>(Q, ldq, X, ldx, xn, cosine ? 1 : 0,
                                                                (int)rows, (int)n, d, k, S,
                                                                (int)split_len, BQ, BS, lk, li);
    } else {
        e = raise_lds_limit(knn_mfma_kernel<false>, lds);
        if (e != hipSuccess) return e;
        knn_mfma_kernel<false><<<grid, dim3(256), lds, stream>>>(Q, ldq, X, ldx, xn, cosine ? 1 : 0,
                                                                 (int)rows, (int)n, d, k, S,
                                                                 (int)split_len, BQ, BS, lk, li);
    }
    return hipGetLastError();
}

}  // namespace knn
