// Device-side helpers shared by the gfx950 kNN kernels: the (key, index) order, the
// wave-cooperative sorted-list merge, the candidate buffers of the running top-k, the
// tile loads of the matrix-core kernels.  Everything sits in an unnamed namespace, so
// each translation unit that includes this header gets its own copy.
//
// Paper section 4.3 (figure 2) gives the shape these serve: a generator (distance tile), a
// reducer (top-k) and a loop over slices, with the big intermediate alive only inside one
// iteration.  Here the intermediate lives in registers: a tile of keys is produced,
// compared against each query's current k-th best and dropped.  The rare survivors go
// through a small per-query candidate buffer in LDS and are merged by one wavefront into
// the query's sorted list in the workspace.
//
// Ordering rule everywhere: (key, index) lexicographic, lower index first on equal keys.
#pragma once
#include <hip/hip_runtime.h>

#include <climits>
#include <cmath>
#include <cstdint>

#include "knn_config.h"

namespace knn {

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr float kInf = __builtin_huge_valf();
constexpr int kNoIdx = INT_MAX;

// (key, index) order; written without short-circuit operators so that it compiles to
// compares and mask arithmetic, not branches
__device__ __forceinline__ bool before(float ka, int ia, float kb, int ib) {
    return (ka < kb) | ((ka == kb) & (ia < ib));
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

__device__ __forceinline__ float wave_min(float v);

// Value of lane (lane ^ S).  Strides below 16 stay inside a row of 16 lanes and use DPP
// (quad permutes; for 4 and 8 a shift left into the low banks and a shift right into the high
// ones: row_shl:n gives lane i the value of lane i + n), which costs VALU moves instead of a
// trip through the LDS crossbar.
template <int S>
__device__ __forceinline__ int lane_xor(int v) {
    if constexpr (S == 1) {
        return __builtin_amdgcn_update_dpp(v, v, 0xB1, 0xF, 0xF, false);  // quad_perm(1,0,3,2)
    } else if constexpr (S == 2) {
        return __builtin_amdgcn_update_dpp(v, v, 0x4E, 0xF, 0xF, false);  // quad_perm(2,3,0,1)
    } else if constexpr (S == 4) {
        const int t = __builtin_amdgcn_update_dpp(v, v, 0x104, 0xF, 0x5, false);  // row_shl:4, banks 0, 2
        return __builtin_amdgcn_update_dpp(t, v, 0x114, 0xF, 0xA, false);         // row_shr:4, banks 1, 3
    } else if constexpr (S == 8) {
        const int t = __builtin_amdgcn_update_dpp(v, v, 0x108, 0xF, 0x3, false);  // row_shl:8, banks 0, 1
        return __builtin_amdgcn_update_dpp(t, v, 0x118, 0xF, 0xC, false);         // row_shr:8, banks 2, 3
    } else if constexpr (S == 32) {
        // v_permlane32_swap exchanges the upper half of its first operand with the lower half
        // of its second: with both set to v the first result holds the lower half twice and
        // the second the upper half twice
        typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
        const u32x2 r = __builtin_amdgcn_permlane32_swap((unsigned)v, (unsigned)v, false, false);
        return (int)((__lane_id() & 32) ? r.x : r.y);
    } else {
        return __shfl_xor(v, S);
    }
}
template <int S>
__device__ __forceinline__ float lane_xor(float v) {
    return __int_as_float(lane_xor<S>(__float_as_int(v)));
}

__device__ __forceinline__ float wave_min(float v) {
    v = fminf(v, lane_xor<32>(v));
    v = fminf(v, lane_xor<16>(v));
    v = fminf(v, lane_xor<8>(v));
    v = fminf(v, lane_xor<4>(v));
    v = fminf(v, lane_xor<2>(v));
    v = fminf(v, lane_xor<1>(v));
    return v;
}

template <int SIZE, int STRIDE>
__device__ __forceinline__ void sort_step(float& key, int& idx, int lane) {
    const float ok = lane_xor<STRIDE>(key);
    const int oi = lane_xor<STRIDE>(idx);
    const bool ascending = (lane & SIZE) == 0;
    const bool low_lane = (lane & STRIDE) == 0;
    const bool keep_min = ascending == low_lane;
    const bool take = keep_min ? before(ok, oi, key, idx) : before(key, idx, ok, oi);
    key = take ? ok : key;
    idx = take ? oi : idx;
}
template <int SIZE, int STRIDE>
__device__ __forceinline__ void sort_size(float& key, int& idx, int lane) {
    sort_step<SIZE, STRIDE>(key, idx, lane);
    if constexpr (STRIDE > 1) sort_size<SIZE, STRIDE / 2>(key, idx, lane);
}
template <int N, int SIZE = 2>
__device__ __forceinline__ void sort_all(float& key, int& idx, int lane) {
    sort_size<SIZE, SIZE / 2>(key, idx, lane);
    if constexpr (SIZE < N) sort_all<N, SIZE * 2>(key, idx, lane);
}

// Ascending bitonic sort of one (key, idx) per lane: across the 64 lanes of a wave, or inside
// each group of 16 lanes (group 0 ascending), which needs DPP strides only.
__device__ __forceinline__ void wave_sort64(float& key, int& idx, int lane) { sort_all<64>(key, idx, lane); }
__device__ __forceinline__ void wave_sort16(float& key, int& idx, int lane) { sort_all<16>(key, idx, lane); }

// Per-wave LDS scratch used while merging candidates into a list.
struct MergeScratch {
    float* list_key;  // [k]   staged copy of the list
    int* list_idx;    // [k]
    float* cand_key;  // [64]  sorted candidates
    int* cand_idx;    // [64]
};

// Merge up to 64 candidates (one per lane; lanes without one pass (+inf, kNoIdx)) into the
// ascending list gk/gi of k entries in global memory.  Returns the key at position k-1 of
// the merged list, i.e. the new acceptance threshold, together with that entry's index: the
// key's bits in the low word, the index in the high word (both stay in registers that way).
// ncand: the candidates sit in lanes 0 .. ncand-1 (wave-uniform; 16 or fewer take a shorter
// network).  All 64 lanes must call it together.
// The first 128 entries of a list as a wave holds them when it has asked for them ahead of a
// merge: entry `lane` and entry 64 + `lane` (values past k are not used).
struct ListHead {
    float k0, k1;
    int i0, i1;
};
__device__ __forceinline__ ListHead load_list_head(const float* __restrict__ gk,
                                                   const int* __restrict__ gi, int k, int lane) {
    ListHead h;
    const int p0 = lane < k ? lane : 0, p1 = lane + kWave < k ? lane + kWave : 0;
    h.k0 = gk[p0];
    h.i0 = gi[p0];
    h.k1 = gk[p1];
    h.i1 = gi[p1];
    return h;
}

template <bool HAVE_HEAD>
__device__ __forceinline__ uint64_t wave_merge_pair_impl(float* __restrict__ gk,
                                                         int* __restrict__ gi, int k, float ckey,
                                                         int cidx, const MergeScratch& sc, int lane,
                                                         int ncand, const ListHead& head, int pos2 = -1,
                                                         float* key2 = nullptr) {
    // (pos2 >= 0: *key2 also gets the key that the merged list holds at position pos2 < k)
    // A list is read and written only by the wave that owns its query, so wave-level
    // ordering is enough; wave_sync() also orders this wave's earlier global stores to the
    // list before the loads below (same compute unit, same vector L1).
    wave_sync();  // earlier uses of the scratch are finished
    const bool few = ncand <= 16;
    if (few) wave_sort16(ckey, cidx, lane);
    else wave_sort64(ckey, cidx, lane);
    sc.cand_key[lane] = ckey;
    sc.cand_idx[lane] = cidx;
    if (HAVE_HEAD) {
        if (lane < k) {
            sc.list_key[lane] = head.k0;
            sc.list_idx[lane] = head.i0;
        }
        if (lane + kWave < k) {
            sc.list_key[lane + kWave] = head.k1;
            sc.list_idx[lane + kWave] = head.i1;
        }
    }
    for (int p = lane + (HAVE_HEAD ? 2 * kWave : 0); p < k; p += kWave) {
        sc.list_key[p] = gk[p];
        sc.list_idx[p] = gi[p];
    }
    wave_sync();
    float tau = kInf;
    int tidx = kNoIdx;
    bool last = false;  // this lane wrote position k-1 (exactly one lane does)
    float t2 = kInf;
    bool hit2 = false;  // this lane wrote position pos2 (exactly one lane does)
    // list entries move right by the number of candidates that come before them
    for (int p = lane; p < k; p += kWave) {
        const float ek = sc.list_key[p];
        const int ei = sc.list_idx[p];
        int cnt = 0;
        for (int step = few ? 8 : 32; step > 0; step >>= 1) {
            const int probe = cnt + step - 1;
            if (before(sc.cand_key[probe], sc.cand_idx[probe], ek, ei)) cnt += step;
        }
        // cnt <= 15 or 63 here; past the candidates the array holds (+inf, kNoIdx)
        if (before(sc.cand_key[cnt], sc.cand_idx[cnt], ek, ei)) cnt += 1;
        const int pos = p + cnt;
        if (pos < k) {
            gk[pos] = ek;
            gi[pos] = ei;
            if (pos == k - 1) {
                tau = ek;
                tidx = ei;
                last = true;
            }
            if (pos == pos2) {
                t2 = ek;
                hit2 = true;
            }
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
            if (pos == k - 1) {
                tau = ckey;
                tidx = cidx;
                last = true;
            }
            if (pos == pos2) {
                t2 = ckey;
                hit2 = true;
            }
        }
    }
    const int src = __builtin_ctzll(__builtin_amdgcn_ballot_w64(last) | (1ull << 63));
    tau = __shfl(tau, src);
    tidx = __shfl(tidx, src);
    if (key2) *key2 = __shfl(t2, __builtin_ctzll(__builtin_amdgcn_ballot_w64(hit2) | (1ull << 63)));
    wave_sync();
    return ((uint64_t)(unsigned)tidx << 32) | __float_as_uint(tau);
}
__device__ __forceinline__ uint64_t wave_merge_pair_inline(float* __restrict__ gk,
                                                           int* __restrict__ gi, int k, float ckey,
                                                           int cidx, const MergeScratch& sc, int lane,
                                                           int ncand) {
    const ListHead none = {0.f, 0.f, 0, 0};
    return wave_merge_pair_impl<false>(gk, gi, k, ckey, cidx, sc, lane, ncand, none);
}
// Out of line: in most kernels the merge is rare and its registers should not count in the
// search loop.  (A kernel whose loop already fills the register file calls the inline form: a
// call would force everything live across it into the callee-saved half of the registers.)
// (The scratch pointers travel by value: a struct passed by reference to a real call has to
// live in the caller's private memory, 48 bytes per lane that the HIP runtime would provide
// for every resident wave behind the workspace accounting.)
__device__ __noinline__ uint64_t wave_merge_pair_call(float* __restrict__ gk, int* __restrict__ gi, int k,
                                                      float ckey, int cidx, float* list_key, int* list_idx,
                                                      float* cand_key, int* cand_idx, int lane, int ncand) {
    MergeScratch sc;
    sc.list_key = list_key;
    sc.list_idx = list_idx;
    sc.cand_key = cand_key;
    sc.cand_idx = cand_idx;
    return wave_merge_pair_inline(gk, gi, k, ckey, cidx, sc, lane, ncand);
}
// The same call with the scratch struct passed by reference: for knn_lowd_bf16_kernel, whose
// register allocation around the call is better that way (measured: 43 against 57 ms on the
// d = 3 workload) and whose private memory the plan accounts for anyway.
__device__ __noinline__ uint64_t wave_merge_pair_ref(float* __restrict__ gk, int* __restrict__ gi, int k,
                                                     float ckey, int cidx, const MergeScratch& sc,
                                                     int lane, int ncand) {
    return wave_merge_pair_inline(gk, gi, k, ckey, cidx, sc, lane, ncand);
}
__device__ __forceinline__ uint64_t wave_merge_pair(float* __restrict__ gk, int* __restrict__ gi, int k,
                                                    float ckey, int cidx, const MergeScratch& sc,
                                                    int lane, int ncand) {
    return wave_merge_pair_call(gk, gi, k, ckey, cidx, sc.list_key, sc.list_idx, sc.cand_key, sc.cand_idx,
                                lane, ncand);
}
__device__ __forceinline__ float merged_key(uint64_t r) { return __uint_as_float((unsigned)r); }
__device__ __forceinline__ int merged_idx(uint64_t r) { return (int)(r >> 32); }

__device__ __forceinline__ float wave_merge(float* __restrict__ gk, int* __restrict__ gi, int k,
                                            float ckey, int cidx, const MergeScratch& sc, int lane,
                                            int ncand = kWave) {
    return merged_key(wave_merge_pair(gk, gi, k, ckey, cidx, sc, lane, ncand));
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
template <typename F>
hipError_t raise_lds_limit(F kernel, size_t bytes) {
    if (bytes <= 48 * 1024) return hipSuccess;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

}  // namespace

}  // namespace knn
