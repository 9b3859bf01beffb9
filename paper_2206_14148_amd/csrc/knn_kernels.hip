// gfx950 (CDNA4, MI355X) kernels for exact brute-force kNN under a memory limit.
//
// Paper section 5.2 defines the result (k closest of n points for each of m queries);
// section 4.1 gives the distance expansion sum x^2 + y^2 - 2xy; section 4.3 (figure 2)
// gives the shape of the computation: a generator (distance tile), a reducer (top-k) and a
// loop over slices, with the big intermediate alive only inside one iteration.  Here the
// intermediate lives in registers: a tile of keys is produced, compared against each
// query's current k-th best and dropped.  The rare survivors go through a small per-query
// candidate buffer in LDS and are merged by one wavefront into the query's sorted list in
// the workspace.
//
// Ordering rule everywhere: (key, index) lexicographic, lower index first on equal keys.
#include <hip/hip_runtime.h>

#include <climits>
#include <cmath>
#include <cstdint>

#include "knn_config.h"
#include "knn_kernels.h"

namespace knn {

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr float kInf = __builtin_huge_valf();
constexpr int kNoIdx = INT_MAX;

__device__ __forceinline__ bool before(float ka, int ia, float kb, int ib) {
    return ka < kb || (ka == kb && ia < ib);
}

__device__ __forceinline__ bool before64(double ka, int ia, double kb, int ib) {
    return ka < kb || (ka == kb && ia < ib);
}

// Make this wave's earlier LDS/global writes visible to its other lanes.
__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

__device__ __forceinline__ float wave_min(float v) {
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) v = fminf(v, __shfl_xor(v, s));
    return v;
}

// Ascending bitonic sort of one (key, idx) per lane across the 64 lanes of a wave.
__device__ __forceinline__ void wave_sort64(float& key, int& idx, int lane) {
#pragma unroll
    for (int size = 2; size <= 64; size <<= 1) {
#pragma unroll
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            const float ok = __shfl_xor(key, stride);
            const int oi = __shfl_xor(idx, stride);
            const bool ascending = (lane & size) == 0;
            const bool low_lane = (lane & stride) == 0;
            const bool keep_min = ascending == low_lane;
            const bool take = keep_min ? before(ok, oi, key, idx) : before(key, idx, ok, oi);
            key = take ? ok : key;
            idx = take ? oi : idx;
        }
    }
}

// Per-wave LDS scratch used while merging candidates into a list.
struct MergeScratch {
    float* list_key;  // [k]   staged copy of the list
    int* list_idx;    // [k]
    float* cand_key;  // [64]  sorted candidates
    int* cand_idx;    // [64]
};

// Merge up to 64 candidates (one per lane; lanes without one pass (+inf, kNoIdx)) into the
// ascending list gk/gi of k entries in global memory.  Returns the key at position k-1 of
// the merged list, i.e. the new acceptance threshold.  All 64 lanes must call it together.
__device__ __noinline__ float wave_merge(float* __restrict__ gk, int* __restrict__ gi, int k, float ckey,
                            int cidx, const MergeScratch& sc, int lane) {
    // A list is read and written only by the wave that owns its query, so wave-level
    // ordering is enough; wave_sync() also orders this wave's earlier global stores to the
    // list before the loads below (same compute unit, same vector L1).
    wave_sync();  // earlier uses of the scratch are finished
    wave_sort64(ckey, cidx, lane);
    sc.cand_key[lane] = ckey;
    sc.cand_idx[lane] = cidx;
    for (int p = lane; p < k; p += kWave) {
        sc.list_key[p] = gk[p];
        sc.list_idx[p] = gi[p];
    }
    wave_sync();
    float tau = kInf;
    // list entries move right by the number of candidates that come before them
    for (int p = lane; p < k; p += kWave) {
        const float ek = sc.list_key[p];
        const int ei = sc.list_idx[p];
        int cnt = 0;
#pragma unroll
        for (int step = 32; step > 0; step >>= 1) {
            const int probe = cnt + step - 1;
            if (before(sc.cand_key[probe], sc.cand_idx[probe], ek, ei)) cnt += step;
        }
        if (before(sc.cand_key[cnt], sc.cand_idx[cnt], ek, ei)) cnt += 1;  // cnt <= 63 here
        const int pos = p + cnt;
        if (pos < k) {
            gk[pos] = ek;
            gi[pos] = ei;
            if (pos == k - 1) tau = ek;
        }
    }
    // candidate c lands after the c candidates before it and the list entries <= it
    {
        int lo = 0, hi = k;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (!before(ckey, cidx, sc.list_key[mid], sc.list_idx[mid])) lo = mid + 1;
            else hi = mid;
        }
        const int pos = lane + lo;
        if (pos < k) {
            gk[pos] = ckey;
            gi[pos] = cidx;
            if (pos == k - 1) tau = ckey;
        }
    }
    tau = wave_min(tau);
    wave_sync();
    return tau;
}

// Bookkeeping of the 32 queries one wave owns in the matrix-core kernels: lane % 32 names the
// query, the two halves of the wave (lane / 32) hold different points of the same query.
struct WaveLists {
    float* lk;        // list keys of the chunk, [rows][S][k]
    int* li;          // list indices
    int k, S, s;      // list length, ranges, this workgroup's range
    int row0;         // first query row (inside the chunk) of this wave
    float* ck;        // candidate keys of this wave, [32][C]
    int* ci;          // candidate indices
    MergeScratch sc;
    int lane;
};

// Merge the buffered candidates of the queries named by bits 0..31 of `mask` into their lists;
// lanes of a merged query get the new threshold and an empty buffer.
template <int C>
__device__ __forceinline__ void flush_lists(const WaveLists& w, uint64_t mask, float& tau,
                                            int& cnt) {
    while (mask) {
        const int L = __builtin_ctzll(mask);
        mask &= mask - 1;
        wave_sync();
        const int c = __shfl(cnt, L);
        float key = kInf;
        int id = kNoIdx;
        if (w.lane < c) {
            key = w.ck[L * C + w.lane];
            id = w.ci[L * C + w.lane];
        }
        const size_t lb = ((size_t)(w.row0 + L) * w.S + w.s) * w.k;
        const float t_new = wave_merge(w.lk + lb, w.li + lb, w.k, key, id, w.sc, w.lane);
        if ((w.lane & 31) == L) {
            tau = t_new;
            cnt = 0;
        }
    }
}

// End of a 128-point tile: acc[pb][e] is the key of query lane % 32 against point
// tile_base + pb*32 + (e/4)*8 + (lane/32)*4 + e%4.  Keys below the query's threshold are
// buffered (the two halves of the wave take consecutive slots), full buffers are merged first.
template <int C>
__device__ __forceinline__ void tile_epilogue(const f32x16 (&acc)[4], const WaveLists& w,
                                              int tile_base, float& tau, int& cnt) {
    float mn = kInf;
#pragma unroll
    for (int pb = 0; pb < 4; ++pb) {
#pragma unroll
        for (int e = 0; e < 16; ++e) mn = fminf(mn, acc[pb][e]);
    }
    if (__builtin_amdgcn_ballot_w64(mn < tau) == 0) return;
    const int i32 = w.lane & 31;
    const int h = w.lane >> 5;
#pragma unroll
    for (int pb = 0; pb < 4; ++pb) {
        int own = 0;
#pragma unroll
        for (int e = 0; e < 16; ++e) own += (acc[pb][e] < tau) ? 1 : 0;
        int oth = __shfl_xor(own, 32);
        const uint64_t need = __builtin_amdgcn_ballot_w64(cnt + own + oth > C) & 0xffffffffull;
        if (need) {
            flush_lists<C>(w, need, tau, cnt);
            own = 0;
#pragma unroll
            for (int e = 0; e < 16; ++e) own += (acc[pb][e] < tau) ? 1 : 0;
            oth = __shfl_xor(own, 32);
        }
        int slot = i32 * C + cnt + (h ? oth : 0);
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            if (acc[pb][e] < tau) {
                w.ck[slot] = acc[pb][e];
                w.ci[slot] = tile_base + pb * 32 + (e >> 2) * 8 + h * 4 + (e & 3);
                ++slot;
            }
        }
        cnt += own + oth;
    }
}

// Cosine metric: the accumulators hold -2 q.x; multiply each by 1/|x| of its point row (rs is
// the tile's 128 row scales in LDS) to get the rank-equivalent key -2 q.x / |x|.
__device__ __forceinline__ void scale_rows(f32x16 (&acc)[4], const float* rs, int h) {
#pragma unroll
    for (int pb = 0; pb < 4; ++pb) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const f32x4 v = *reinterpret_cast<const f32x4*>(rs + pb * 32 + g * 8 + h * 4);
            acc[pb][g * 4 + 0] *= v[0];
            acc[pb][g * 4 + 1] *= v[1];
            acc[pb][g * 4 + 2] *= v[2];
            acc[pb][g * 4 + 3] *= v[3];
        }
    }
}

// Workgroup -> (query tile, point range).  Consecutive workgroup ids go round-robin to the 8
// XCDs, each with its own L2.  The (tile, range) grid is cut into blocks of BQ tiles x BS
// ranges; a block is handed to one XCD as BQ*BS consecutive workgroups of that XCD, so the
// workgroups resident there together re-use BQ query tiles and BS point streams out of its L2
// instead of fetching BQ*BS private ones.  Returns false for a padding workgroup.
__device__ __forceinline__ bool xcd_block_map(int rows, int tile_q, int S, int BQ, int BS, int& s,
                                              int& wg_row0) {
    const int T = (rows + tile_q - 1) / tile_q;
    const int nQB = (T + BQ - 1) / BQ;
    const int nSB = S / BS;  // BS divides S
    const int xcd = blockIdx.x & 7;
    const int slot = blockIdx.x >> 3;
    const int per_block = BQ * BS;
    const int bseq = slot / per_block;
    const int within = slot - bseq * per_block;
    const int b = bseq * 8 + xcd;
    if (b >= nQB * nSB) return false;
    const int sb = b / nQB;
    const int qb = b - sb * nQB;
    const int si = within / BQ;
    const int qi = within - si * BQ;
    const int qtile = qb * BQ + qi;
    if (qtile >= T) return false;
    s = sb * BS + si;
    wg_row0 = qtile * tile_q;
    return true;
}

// Lists of the 32 queries starting at chunk row `row0` begin as k sentinels.
__device__ __forceinline__ void init_lists32(float* __restrict__ lk, int* __restrict__ li, int row0,
                                             int rows, int S, int s, int k, int lane) {
    for (int qq = 0; qq < 32; ++qq) {
        if (row0 + qq >= rows) break;
        const size_t lb = ((size_t)(row0 + qq) * S + s) * k;
        for (int p = lane; p < k; p += kWave) {
            lk[lb + p] = kInf;
            li[lb + p] = kNoIdx;
        }
    }
}

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
// Low-dimensional path: one query per lane, points streamed through uniform (scalar) loads,
// difference-form distance in fp32 on the vector ALU.
// ---------------------------------------------------------------------------------------
template <int D, bool CONTIG>
__global__ __launch_bounds__(kLowdTileQ) void knn_lowd_kernel(
    const float* __restrict__ Q, int64_t ldq, const float* __restrict__ X, int64_t ldx_arg,
    int rows, int n, int k, int S, int split_len, float* __restrict__ lk, int* __restrict__ li) {
    constexpr int U = kLowdUnroll;  // points per filter test
    constexpr int H = 4;            // points pushed between two overflow checks
    constexpr int C = kLowdCand;
    constexpr int CP = C + 1;  // padded row of the candidate buffer
    static_assert(U % H == 0 && C > H, "candidate buffer must hold one push group");
    // rows of X that follow each other without gaps let a whole group be one wide load
    const int64_t ldx = CONTIG ? (int64_t)D : ldx_arg;
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const size_t per_wave = (size_t)(2 * kWave * CP + 2 * k + 2 * kWave) * 4;
    unsigned char* base = smem + (size_t)wave * per_wave;
    float* ck = reinterpret_cast<float*>(base);         // [64][CP]
    int* ci = reinterpret_cast<int*>(ck + kWave * CP);  // [64][CP]
    MergeScratch sc;
    sc.list_key = reinterpret_cast<float*>(ci + kWave * CP);
    sc.list_idx = reinterpret_cast<int*>(sc.list_key + k);
    sc.cand_key = reinterpret_cast<float*>(sc.list_idx + k);
    sc.cand_idx = reinterpret_cast<int*>(sc.cand_key + kWave);

    const int s = blockIdx.y;
    const int wave_row0 = (blockIdx.x * kLowdWaves + wave) * kWave;
    if (wave_row0 >= rows) return;  // whole wave idle; no workgroup barrier is used below
    const int r = wave_row0 + lane;
    const bool active = r < rows;

    // start every list of this wave as k sentinels
    {
        const int nq = min(kWave, rows - wave_row0);
        for (int qq = 0; qq < nq; ++qq) {
            const size_t lb = ((size_t)(wave_row0 + qq) * S + s) * k;
            for (int p = lane; p < k; p += kWave) {
                lk[lb + p] = kInf;
                li[lb + p] = kNoIdx;
            }
        }
    }

    float q[D];
#pragma unroll
    for (int t = 0; t < D; ++t) q[t] = active ? Q[(int64_t)r * ldq + t] : 0.f;
    float tau = active ? kInf : -kInf;  // idle lanes never accept anything
    int cnt = 0;

    auto flush = [&](uint64_t mask) {
        while (mask) {
            const int L = __builtin_ctzll(mask);
            mask &= mask - 1;
            wave_sync();
            const int c = __shfl(cnt, L);
            float key = kInf;
            int id = kNoIdx;
            if (lane < c) {
                key = ck[L * CP + lane];
                id = ci[L * CP + lane];
            }
            const size_t lb = ((size_t)(wave_row0 + L) * S + s) * k;
            const float t_new = wave_merge(lk + lb, li + lb, k, key, id, sc, lane);
            if (lane == L) {
                tau = t_new;
                cnt = 0;
            }
        }
    };
    auto sqdist = [&](const float* __restrict__ xp) {
        float df = q[0] - xp[0];
        float acc = df * df;
#pragma unroll
        for (int t = 1; t < D; ++t) {
            df = q[t] - xp[t];
            acc = fmaf(df, df, acc);
        }
        return acc;
    };

    const int j0 = s * split_len;
    const int j1 = min(n, j0 + split_len);
    int j = j0;
    const float* xp = X + (int64_t)j0 * ldx;  // uniform: the compiler reads it with scalar loads
    for (; j + U <= j1; j += U, xp += U * ldx) {
        float dd[U];
#pragma unroll
        for (int u = 0; u < U; ++u) dd[u] = sqdist(xp + u * ldx);
        float mn = dd[0];
#pragma unroll
        for (int u = 1; u < U; ++u) mn = fminf(mn, dd[u]);
        if (__builtin_amdgcn_ballot_w64(mn < tau) != 0) {
#pragma unroll
            for (int g = 0; g < U / H; ++g) {
#pragma unroll
                for (int u = g * H; u < (g + 1) * H; ++u) {
                    if (dd[u] < tau) {
                        ck[lane * CP + cnt] = dd[u];
                        ci[lane * CP + cnt] = j + u;
                        ++cnt;
                    }
                }
                const uint64_t full = __builtin_amdgcn_ballot_w64(cnt > C - H);
                if (full) flush(full);
            }
        }
    }
    for (; j < j1; ++j, xp += ldx) {
        const float acc = sqdist(xp);
        if (acc < tau) {
            ck[lane * CP + cnt] = acc;
            ci[lane * CP + cnt] = j;
            ++cnt;
        }
        const uint64_t full = __builtin_amdgcn_ballot_w64(cnt > C - H);
        if (full) flush(full);
    }
    const uint64_t rest = __builtin_amdgcn_ballot_w64(cnt > 0);
    if (rest) flush(rest);
}

// ---------------------------------------------------------------------------------------
// L1 metric (the L1 rows of the paper's table): sum |q - x| hides no matrix product, so this
// is a vector-ALU kernel for every d.  One query per lane; a group of 8 points is wave-uniform
// and read with scalar loads; the dimension is walked in chunks of 16 with the query's chunk
// in registers and one running sum per point of the group, so a query value is loaded once
// per 8 points and a point value costs no vector work.  Two VALU ops per pair and dimension
// (subtract, add-absolute).  Sums run in ascending t, whatever the chunking.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(kLowdTileQ) void knn_l1_kernel(
    const float* __restrict__ Q, int64_t ldq, const float* __restrict__ X, int64_t ldx, int rows,
    int n, int d, int k, int S, int split_len, float* __restrict__ lk, int* __restrict__ li) {
    constexpr int P = 8;    // points per group
    constexpr int TC = 16;  // dimensions per register chunk
    constexpr int H = 4;    // points pushed between two overflow checks
    constexpr int C = kLowdCand;
    constexpr int CP = C + 1;
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const size_t per_wave = (size_t)(2 * kWave * CP + 2 * k + 2 * kWave) * 4;
    unsigned char* base = smem + (size_t)wave * per_wave;
    float* ck = reinterpret_cast<float*>(base);         // [64][CP]
    int* ci = reinterpret_cast<int*>(ck + kWave * CP);  // [64][CP]
    MergeScratch sc;
    sc.list_key = reinterpret_cast<float*>(ci + kWave * CP);
    sc.list_idx = reinterpret_cast<int*>(sc.list_key + k);
    sc.cand_key = reinterpret_cast<float*>(sc.list_idx + k);
    sc.cand_idx = reinterpret_cast<int*>(sc.cand_key + kWave);

    const int s = blockIdx.y;
    const int wave_row0 = (blockIdx.x * kLowdWaves + wave) * kWave;
    if (wave_row0 >= rows) return;  // whole wave idle; no workgroup barrier is used below
    const int r = wave_row0 + lane;
    const bool active = r < rows;
    {
        const int nq = min(kWave, rows - wave_row0);
        for (int qq = 0; qq < nq; ++qq) {
            const size_t lb = ((size_t)(wave_row0 + qq) * S + s) * k;
            for (int p = lane; p < k; p += kWave) {
                lk[lb + p] = kInf;
                li[lb + p] = kNoIdx;
            }
        }
    }
    const float* qrow = Q + (int64_t)(active ? r : 0) * ldq;
    const bool qvec = (reinterpret_cast<uintptr_t>(Q) % 16 == 0) && (ldq % 4 == 0);
    float tau = active ? kInf : -kInf;
    int cnt = 0;

    auto flush = [&](uint64_t mask) {
        while (mask) {
            const int L = __builtin_ctzll(mask);
            mask &= mask - 1;
            wave_sync();
            const int c = __shfl(cnt, L);
            float key = kInf;
            int id = kNoIdx;
            if (lane < c) {
                key = ck[L * CP + lane];
                id = ci[L * CP + lane];
            }
            const size_t lb = ((size_t)(wave_row0 + L) * S + s) * k;
            const float t_new = wave_merge(lk + lb, li + lb, k, key, id, sc, lane);
            if (lane == L) {
                tau = t_new;
                cnt = 0;
            }
        }
    };

    const int j0 = s * split_len;
    const int j1 = min(n, j0 + split_len);
    for (int j = j0; j < j1; j += P) {
        float acc[P];
#pragma unroll
        for (int p = 0; p < P; ++p) acc[p] = 0.f;
        for (int t0 = 0; t0 < d; t0 += TC) {
            const bool full = t0 + TC <= d;  // uniform
            float qv[TC];
            if (full && qvec) {  // uniform: whole chunk inside the row and 16-byte aligned
#pragma unroll
                for (int t4 = 0; t4 < TC / 4; ++t4) {
                    const f32x4 v = *reinterpret_cast<const f32x4*>(qrow + t0 + 4 * t4);
                    qv[4 * t4 + 0] = v[0];
                    qv[4 * t4 + 1] = v[1];
                    qv[4 * t4 + 2] = v[2];
                    qv[4 * t4 + 3] = v[3];
                }
            } else {
#pragma unroll
                for (int t = 0; t < TC; ++t) {
                    const int tt = t0 + t;
                    const float v = qrow[tt < d ? tt : d - 1];
                    qv[t] = tt < d ? v : 0.f;
                }
            }
#pragma unroll
            for (int p = 0; p < P; ++p) {
                const int jp = (j + p < j1) ? j + p : j1 - 1;  // uniform; repeats of the last point are masked below
                const float* xp = X + (int64_t)jp * ldx;
                float a = acc[p];
                if (full) {
#pragma unroll
                    for (int t = 0; t < TC; ++t) a += fabsf(qv[t] - xp[t0 + t]);
                } else {
#pragma unroll
                    for (int t = 0; t < TC; ++t) {
                        const int tt = t0 + t;
                        const float xv = xp[tt < d ? tt : d - 1];
                        a += fabsf(qv[t] - (tt < d ? xv : 0.f));
                    }
                }
                acc[p] = a;
            }
        }
        float mn = kInf;
#pragma unroll
        for (int p = 0; p < P; ++p) {
            if (j + p >= j1) acc[p] = kInf;  // past the range
            mn = fminf(mn, acc[p]);
        }
        if (__builtin_amdgcn_ballot_w64(mn < tau) != 0) {
#pragma unroll
            for (int g = 0; g < P / H; ++g) {
#pragma unroll
                for (int p = g * H; p < (g + 1) * H; ++p) {
                    if (acc[p] < tau) {
                        ck[lane * CP + cnt] = acc[p];
                        ci[lane * CP + cnt] = j + p;
                        ++cnt;
                    }
                }
                const uint64_t fullb = __builtin_amdgcn_ballot_w64(cnt > C - H);
                if (fullb) flush(fullb);
            }
        }
    }
    const uint64_t rest = __builtin_amdgcn_ballot_w64(cnt > 0);
    if (rest) flush(rest);
}

// ---------------------------------------------------------------------------------------
// Low-dimensional path on the matrix cores (d <= 3).  The expansion of section 4.1 is used
// only as a FILTER: with points packed as [x0 x1 x2 ||x||^2] and queries as
// [-2q0 -2q1 -2q2 1], two v_mfma_f32_32x32x2_f32 give 32 x 32 keys ||x||^2 - 2 q.x.  A key
// that could still belong to a pair closer than the query's threshold (allowing for the
// rounding of the expansion) sends the pair to the exact test: the same fp32
// difference-form distance as knn_lowd_kernel, compared against the same threshold.  The
// accepted set, the keys and therefore the result are identical to the vector-ALU kernel.
// ---------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void knn_pack_points_kernel(const float* __restrict__ X,
                                                              int64_t ldx, int n,
                                                              f32x4* __restrict__ Xp,
                                                              unsigned* __restrict__ xn_max_bits) {
    const int j = blockIdx.x * 256 + threadIdx.x;
    float nrm = 0.f;
    if (j < n) {
        float v[3] = {0.f, 0.f, 0.f};
#pragma unroll
        for (int t = 0; t < D; ++t) v[t] = X[(int64_t)j * ldx + t];
        nrm = v[0] * v[0];
        nrm = fmaf(v[1], v[1], nrm);
        nrm = fmaf(v[2], v[2], nrm);
        Xp[j] = f32x4{v[0], v[1], v[2], nrm};
    }
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) nrm = fmaxf(nrm, __shfl_xor(nrm, s));
    // non-negative floats order like their bit patterns
    if ((threadIdx.x & 63) == 0) atomicMax(xn_max_bits, __float_as_uint(nrm));
}

__global__ void knn_zero_word_kernel(unsigned* __restrict__ w) { *w = 0u; }

template <int D>
__global__ __launch_bounds__(256, 4) void knn_lowd_mfma_kernel(
    const float* __restrict__ Q, int64_t ldq, const f32x4* __restrict__ Xp,
    const unsigned* __restrict__ xn_max_bits, int rows, int n, int k, int S, int split_len,
    float* __restrict__ lk, int* __restrict__ li) {
    constexpr int C = kPmCand;
    constexpr int UB = 4;        // 32-point blocks per loop iteration
    constexpr int PTS = UB * 32; // points per loop iteration
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int i32 = lane & 31;  // query column (B side) / point row (A side) of the 32x32 block
    const int h = lane >> 5;
    const size_t per_wave = (size_t)(2 * 32 * C + 2 * kWave + 2 * k) * 4;
    float* ck = reinterpret_cast<float*>(smem + (size_t)wave * per_wave);  // [32][C]
    int* ci = reinterpret_cast<int*>(ck + 32 * C);                         // [32][C]
    MergeScratch sc;
    sc.cand_key = reinterpret_cast<float*>(ci + 32 * C);
    sc.cand_idx = reinterpret_cast<int*>(sc.cand_key + kWave);
    sc.list_key = reinterpret_cast<float*>(sc.cand_idx + kWave);
    sc.list_idx = reinterpret_cast<int*>(sc.list_key + k);

    const int s = blockIdx.y;
    const int wave_row0 = (blockIdx.x * 4 + wave) * 32;
    if (wave_row0 >= rows) return;  // whole wave idle; no workgroup barrier is used below
    const int r = wave_row0 + i32;
    const bool active = r < rows;

    for (int qq = 0; qq < 32; ++qq) {
        if (wave_row0 + qq >= rows) break;
        const size_t lb = ((size_t)(wave_row0 + qq) * S + s) * k;
        for (int p = lane; p < k; p += kWave) {
            lk[lb + p] = kInf;
            li[lb + p] = kNoIdx;
        }
    }

    float q[3] = {0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < D; ++t) q[t] = active ? Q[(int64_t)r * ldq + t] : 0.f;
    const float qn = fmaf(q[2], q[2], fmaf(q[1], q[1], q[0] * q[0]));
    // B operand, K order (0, 1 | 2, 3) split over the two halves of the wave
    const float b0 = h ? -2.f * q[2] : -2.f * q[0];
    const float b1 = h ? 1.f : -2.f * q[1];
    const float xmax = __uint_as_float(*xn_max_bits);

    // A pair with exact fp32 distance < tau has key < (tau - qn) + slack: the key and qn each
    // carry a few roundings relative to (||x||^2 + ||q||^2), the distance a few relative to
    // itself; 2^-19 of their sum is several times the worst case.
    float tau = active ? kInf : -kInf;
    auto key_bound = [&](float t) { return (t - qn) + 0x1p-19f * (xmax + qn + t); };
    float tauf = key_bound(tau);
    int cnt = 0;  // candidates buffered for this lane's query (same in both halves)

    auto flush = [&](uint64_t mask) {  // bits 0..31: queries of this wave to merge
        while (mask) {
            const int L = __builtin_ctzll(mask);
            mask &= mask - 1;
            wave_sync();
            const int c = __shfl(cnt, L);
            float key = kInf;
            int id = kNoIdx;
            if (lane < c) {
                key = ck[L * C + lane];
                id = ci[L * C + lane];
            }
            const size_t lb = ((size_t)(wave_row0 + L) * S + s) * k;
            const float t_new = wave_merge(lk + lb, li + lb, k, key, id, sc, lane);
            if (i32 == L) {
                tau = t_new;
                tauf = key_bound(t_new);
                cnt = 0;
            }
        }
    };

    typedef float f32x2 __attribute__((ext_vector_type(2)));
    const f32x2* xp2 = reinterpret_cast<const f32x2*>(Xp);  // point j = entries 2j (x0 x1), 2j+1 (x2 xn)
    const int j0 = s * split_len;
    const int j1 = min(n, j0 + split_len);

    // Rare path of one 32-point block.  Each lane collects the keys that pass the filter in
    // a 16-bit mask and the lanes then work through their own bits in parallel (usually one
    // round).  The coordinates of the point come from the A-operand registers of the lanes
    // that loaded them, not from memory.
    auto examine = [&](const f32x16& keys, const f32x2& apt, int jblock) {
        unsigned bits = 0;  // bit e <=> key e passes; shift-in from the top keeps it to
#pragma unroll          // a compare and an add-with-carry per key
        for (int e = 15; e >= 0; --e) bits = bits + bits + ((keys[e] < tauf) ? 1u : 0u);
        while (__builtin_amdgcn_ballot_w64(bits != 0) != 0) {
            const bool has = bits != 0;
            const int e = __builtin_ctz(bits | 0x10000u);
            bits &= bits - 1;
            const int row = ((e >> 2) * 8 + h * 4 + (e & 3)) & 31;  // point row inside the block
            float xv[3];
            xv[0] = __shfl(apt[0], row);
            xv[1] = __shfl(apt[1], row);
            xv[2] = __shfl(apt[0], row + 32);
            // exact test, same arithmetic as the vector-ALU kernel
            float df = q[0] - xv[0];
            float dd = df * df;
            if (D > 1) {
                df = q[1] - xv[1];
                dd = fmaf(df, df, dd);
            }
            if (D > 2) {
                df = q[2] - xv[2];
                dd = fmaf(df, df, dd);
            }
            bool c = has && dd < tau;
            if (__builtin_amdgcn_ballot_w64(c) == 0) continue;
            int own = c ? 1 : 0;
            int oth = __shfl_xor(own, 32);
            const uint64_t need = __builtin_amdgcn_ballot_w64(cnt + own + oth > C) & 0xffffffffull;
            if (need) {
                flush(need);
                c = c && dd < tau;
                own = c ? 1 : 0;
                oth = __shfl_xor(own, 32);
            }
            if (c) {
                const int slot = i32 * C + cnt + (h ? oth : 0);
                ck[slot] = dd;
                ci[slot] = jblock + row;
            }
            cnt += own + oth;
        }
    };

    // one iteration: UB blocks of 32 points against this wave's 32 queries
    auto process = [&](const f32x2 (&a)[UB], int jb) {
#pragma unroll
        for (int u = 0; u < UB; ++u) {
            f32x16 z;
#pragma unroll
            for (int e = 0; e < 16; ++e) z[e] = 0.f;
            z = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u][0], b0, z, 0, 0, 0);
            z = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u][1], b1, z, 0, 0, 0);
            float m = kInf;  // 8 three-input mins over (inf, 16 keys)
#pragma unroll
            for (int e = 0; e < 16; ++e) m = fminf(m, z[e]);
            if (__builtin_amdgcn_ballot_w64(m < tauf) != 0) examine(z, a[u], jb + u * 32);
        }
    };

    const int nfull = (j1 > j0) ? (j1 - j0) / PTS : 0;
    int jb = j0;
    f32x2 a[UB], an[UB];
#pragma unroll
    for (int u = 0; u < UB; ++u) a[u] = an[u] = f32x2{0.f, 0.f};
    if (nfull > 0) {
#pragma unroll
        for (int u = 0; u < UB; ++u) a[u] = xp2[(size_t)(jb + u * 32 + i32) * 2 + h];
    }
    for (int it = 0; it < nfull; ++it) {
        if (it + 1 < nfull) {
#pragma unroll
            for (int u = 0; u < UB; ++u) an[u] = xp2[(size_t)(jb + PTS + u * 32 + i32) * 2 + h];
        }
        process(a, jb);
#pragma unroll
        for (int u = 0; u < UB; ++u) a[u] = an[u];
        jb += PTS;
    }
    if (jb < j1) {  // ragged tail: rows past the range read a valid row and get ||x||^2 = +inf
#pragma unroll
        for (int u = 0; u < UB; ++u) {
            const int row = jb + u * 32 + i32;
            a[u] = xp2[(size_t)(row < j1 ? row : j1 - 1) * 2 + h];
            if (row >= j1 && h) a[u][1] = kInf;
        }
        process(a, jb);
    }
    const uint64_t rest = __builtin_amdgcn_ballot_w64(cnt > 0) & 0xffffffffull;
    if (rest) flush(rest);
}

// ---------------------------------------------------------------------------------------
// Matrix-core path: a workgroup of 4 waves owns 128 queries and walks its point range in
// tiles of 128 points.  Data points are the M side and queries the N side of
// v_mfma_f32_32x32x2_f32, so the 16 accumulator values a lane holds per 32x32 block all
// belong to ONE query (column = lane % 32): its threshold is one register and the filter
// is a per-lane compare.  The accumulators start at ||x||^2 and receive (-2 q) . x, which
// gives the key  ||x||^2 - 2 q.x  (the distance minus the per-query constant ||q||^2).
// ---------------------------------------------------------------------------------------
// Four consecutive columns of one row, loaded from an address clamped into the matrix so that
// the loads of a pipeline step issue back to back without control flow; mask_row4 zeroes
// what was out of range once the data is used.  ALIGNED: rows are 16-byte aligned and d is
// a multiple of 4, so one vector load covers the four columns.
template <bool ALIGNED>
__device__ __forceinline__ f32x4 load_row4(const float* __restrict__ base, int64_t ld,
                                           int64_t row, int64_t nrows, int col, int d) {
    const float* p = base + (row < nrows ? row : nrows - 1) * ld;
    f32x4 v;
    if (ALIGNED) {
        v = *reinterpret_cast<const f32x4*>(p + (col < d ? col : 0));
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = p[col + e < d ? col + e : 0];
    }
    return v;
}

__device__ __forceinline__ f32x4 mask_row4(f32x4 v, bool row_ok, int col, int d, float scale) {
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = (row_ok && col + e < d) ? v[e] * scale : 0.f;
    return v;
}

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
// unrolled (NCH is even), which also names the two prefetch register sets statically.
// ---------------------------------------------------------------------------------------
template <int NCH, bool ALIGNED, bool BLOCKED>
__global__ __launch_bounds__(256, 2) void knn_mfma_qreg_kernel(
    const float* __restrict__ Q, int64_t ldq, const float* __restrict__ X, int64_t ldx,
    const f32x4* __restrict__ Xb, const float* __restrict__ xn, int cosine, int rows, int n, int d,
    int k, int S, int split_len, int BQ, int BS, float* __restrict__ lk, int* __restrict__ li) {
    static_assert(NCH % 2 == 0, "the chunk loop alternates two LDS buffers and register sets");
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
    for (int tile = 0; tile < ntiles; ++tile) {
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
            Staged& mine = (c & 1) ? set_odd : set_even;        // receives step + 2
            const Staged& next = (c & 1) ? set_even : set_odd;  // holds step + 1
            fetch(step + 2 < total ? step + 2 : total - 1, mine);
            const float* xb = xs + (c & 1) * TX * RS;
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
    const uint64_t rest = __builtin_amdgcn_ballot_w64(cnt > 0) & 0xffffffffull;
    if (rest) flush_lists<C>(wl, rest, tau, cnt);
}

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
    int n, int d, int k, int S, int metric, const float* __restrict__ lk,
    const int* __restrict__ li, int32_t* __restrict__ idx_out, float* __restrict__ dist_out) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int r = blockIdx.x * 4 + wave;
    if (r >= rows) return;  // no workgroup barrier below
    double* wd = reinterpret_cast<double*>(smem) + (size_t)wave * k;
    int* wi = reinterpret_cast<int*>(reinterpret_cast<double*>(smem) + (size_t)4 * k) + (size_t)wave * k;

    const size_t rb = (size_t)r * S * k;
    if (S == 1) {
        for (int p = lane; p < k; p += kWave) wi[p] = li[rb + p];
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
            if (rank < k) wi[rank] = id;
        }
    }
    wave_sync();
    for (int w = lane; w < k; w += kWave) {
        const int j = wi[w];
        double dist = __builtin_huge_val();
        if ((unsigned)j < (unsigned)n) {
            const float* qp = Q + (int64_t)r * ldq;
            const float* xp = X + (int64_t)j * ldx;
            dist = metric == 1 ? exact_cosdist(qp, xp, d)
                               : (metric == 2 ? exact_l1dist(qp, xp, d) : exact_sqdist(qp, xp, d));
        }
        wd[w] = dist;
    }
    wave_sync();
    for (int w = lane; w < k; w += kWave) {
        const double dw = wd[w];
        const int jw = wi[w];
        int rank = 0;
        for (int v = 0; v < k; ++v) rank += before64(wd[v], wi[v], dw, jw) ? 1 : 0;
        idx_out[(size_t)r * k + rank] = jw;
        dist_out[(size_t)r * k + rank] = (float)dw;
    }
}

template <typename F>
hipError_t raise_lds_limit(F kernel, size_t bytes) {
    if (bytes <= 48 * 1024) return hipSuccess;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
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

template <int D>
static hipError_t launch_lowd_d(const float* Q, int64_t ldq, const float* X, int64_t ldx,
                                int64_t rows, int64_t n, int k, int S, float* lk, int* li,
                                hipStream_t stream) {
    const size_t per_wave = (size_t)(2 * kWave * (kLowdCand + 1) + 2 * k + 2 * kWave) * 4;
    const size_t lds = per_wave * kLowdWaves;
    int64_t split_len = (n + S - 1) / S;
    split_len = (split_len + kLowdUnroll - 1) / kLowdUnroll * kLowdUnroll;
    dim3 grid((unsigned)((rows + kLowdTileQ - 1) / kLowdTileQ), (unsigned)S);
    hipError_t e;
    if (ldx == D) {
        e = raise_lds_limit(knn_lowd_kernel<D, true>, lds);
        if (e != hipSuccess) return e;
        knn_lowd_kernel<D, true><<<grid, dim3(kLowdTileQ), lds, stream>>>(
            Q, ldq, X, ldx, (int)rows, (int)n, k, S, (int)split_len, lk, li);
    } else {
        e = raise_lds_limit(knn_lowd_kernel<D, false>, lds);
        if (e != hipSuccess) return e;
        knn_lowd_kernel<D, false><<<grid, dim3(kLowdTileQ), lds, stream>>>(
            Q, ldq, X, ldx, (int)rows, (int)n, k, S, (int)split_len, lk, li);
    }
    return hipGetLastError();
}

hipError_t launch_l1(const float* Q, int64_t ldq, const float* X, int64_t ldx, int64_t rows,
                     int64_t n, int d, int k, int S, float* lk, int* li, hipStream_t stream) {
    const size_t per_wave = (size_t)(2 * kWave * (kLowdCand + 1) + 2 * k + 2 * kWave) * 4;
    const size_t lds = per_wave * kLowdWaves;
    hipError_t e = raise_lds_limit(knn_l1_kernel, lds);
    if (e != hipSuccess) return e;
    int64_t split_len = (n + S - 1) / S;
    split_len = (split_len + 7) / 8 * 8;
    dim3 grid((unsigned)((rows + kLowdTileQ - 1) / kLowdTileQ), (unsigned)S);
    knn_l1_kernel<<<grid, dim3(kLowdTileQ), lds, stream>>>(Q, ldq, X, ldx, (int)rows, (int)n, d, k, S,
                                                           (int)split_len, lk, li);
    return hipGetLastError();
}

hipError_t launch_lowd(const float* Q, int64_t ldq, const float* X, int64_t ldx, int64_t rows,
                       int64_t n, int d, int k, int S, float* lk, int* li, hipStream_t stream) {
    switch (d) {
        case 1: return launch_lowd_d<1>(Q, ldq, X, ldx, rows, n, k, S, lk, li, stream);
        case 2: return launch_lowd_d<2>(Q, ldq, X, ldx, rows, n, k, S, lk, li, stream);
        case 3: return launch_lowd_d<3>(Q, ldq, X, ldx, rows, n, k, S, lk, li, stream);
        case 4: return launch_lowd_d<4>(Q, ldq, X, ldx, rows, n, k, S, lk, li, stream);
        case 5: return launch_lowd_d<5>(Q, ldq, X, ldx, rows, n, k, S, lk, li, stream);
        case 6: return launch_lowd_d<6>(Q, ldq, X, ldx, rows, n, k, S, lk, li, stream);
        case 7: return launch_lowd_d<7>(Q, ldq, X, ldx, rows, n, k, S, lk, li, stream);
        case 8: return launch_lowd_d<8>(Q, ldq, X, ldx, rows, n, k, S, lk, li, stream);
        default: return hipErrorInvalidValue;
    }
}

template <int D>
static hipError_t launch_lowd_mfma_d(const float* Q, int64_t ldq, const float* X, int64_t ldx,
                                     void* packed, int64_t rows, int64_t n, int k, int S,
                                     bool pack, float* lk, int* li, hipStream_t stream) {
    unsigned* xmax = static_cast<unsigned*>(packed);
    f32x4* Xp = reinterpret_cast<f32x4*>(static_cast<unsigned char*>(packed) + kAlign);
    if (pack) {
        knn_zero_word_kernel<<<dim3(1), dim3(1), 0, stream>>>(xmax);
        knn_pack_points_kernel<D><<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream>>>(
            X, ldx, (int)n, Xp, xmax);
        hipError_t e0 = hipGetLastError();
        if (e0 != hipSuccess) return e0;
    }
    if (rows == 0) return hipSuccess;
    const size_t per_wave = (size_t)(2 * 32 * kPmCand + 2 * kWave + 2 * k) * 4;
    const size_t lds = per_wave * 4;
    hipError_t e = raise_lds_limit(knn_lowd_mfma_kernel<D>, lds);
    if (e != hipSuccess) return e;
    int64_t split_len = (n + S - 1) / S;
    split_len = (split_len + 127) / 128 * 128;
    dim3 grid((unsigned)((rows + kPmTileQ - 1) / kPmTileQ), (unsigned)S);
    knn_lowd_mfma_kernel<D><<<grid, dim3(256), lds, stream>>>(
        Q, ldq, Xp, xmax, (int)rows, (int)n, k, S, (int)split_len, lk, li);
    return hipGetLastError();
}

hipError_t launch_lowd_mfma(const float* Q, int64_t ldq, const float* X, int64_t ldx, void* packed,
                            int64_t rows, int64_t n, int d, int k, int S, bool pack, float* lk,
                            int* li, hipStream_t stream) {
    switch (d) {
        case 1: return launch_lowd_mfma_d<1>(Q, ldq, X, ldx, packed, rows, n, k, S, pack, lk, li, stream);
        case 2: return launch_lowd_mfma_d<2>(Q, ldq, X, ldx, packed, rows, n, k, S, pack, lk, li, stream);
        case 3: return launch_lowd_mfma_d<3>(Q, ldq, X, ldx, packed, rows, n, k, S, pack, lk, li, stream);
        default: return hipErrorInvalidValue;
    }
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
        if (nch <= 2) KNN_QREG_LAUNCH(2);
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

hipError_t launch_merge_refine(const float* Q, int64_t ldq, const float* X, int64_t ldx,
                               int64_t rows, int64_t n, int d, int k, int S, int metric,
                               const float* lk, const int* li, int32_t* idx, float* dist,
                               hipStream_t stream) {
    const size_t lds = (size_t)4 * k * (sizeof(double) + sizeof(int));
    hipError_t e = raise_lds_limit(knn_merge_refine_kernel, lds);
    if (e != hipSuccess) return e;
    dim3 grid((unsigned)((rows + 3) / 4));
    knn_merge_refine_kernel<<<grid, dim3(256), lds, stream>>>(
        Q, ldq, X, ldx, (int)rows, (int)n, d, k, S, metric, lk, li, idx, dist);
    return hipGetLastError();
}

}  // namespace knn
