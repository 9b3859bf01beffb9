// gfx950 (CDNA4, MI355X) kNN search for d > 8, squared-Euclidean metric: the expansion
// sum x^2 - 2 q.x of paper section 4.1 as a FILTER on the bf16 matrix cores, in front of an exact
// fp32 test of the few pairs that pass it.
//
// An fp32 MFMA delivers 256 flops per cycle and compute unit, a bf16 MFMA 4096.  The filter takes
// the dot product of the values rounded to bf16 (8 significant bits, relative error <= 2^-8 a
// value): one bf16 MFMA per 16 coordinates.  Its keys are off by at most 1.002 * 2^-6 |x| |q|;
// the filter threshold allows for that and for every fp32 rounding on the way, so no pair at or
// below a query's current k-th distance is lost.  (Two bf16 pieces a value - three MFMAs - give
// an allowance 256 times smaller and were the first design; the pairs the coarser filter lets
// through in addition cost far less than the two MFMAs saved.)  The pairs that pass are buffered
// per query and, when a buffer is full, evaluated exactly (fp32 difference form, fixed summation
// order) and merged into the query's list; the list keys and hence the results do not depend on
// the filter.  The distance tile still never leaves the registers (section 4.3).
#include <hip/hip_runtime.h>

#include <climits>
#include <cmath>
#include <cstdint>

#include "knn_config.h"
#include "knn_device.h"
#include "knn_exact.h"
#include "knn_kernels.h"

namespace knn {

namespace {

// header word 0 of the per-point area: max ||x||^2 (bits of a non-negative float)
__global__ void knn_split_init_kernel(unsigned* __restrict__ hdr) {
    if (threadIdx.x < 2) hdr[threadIdx.x] = 0u;  // (word 1: the largest bf16 rounding residual, path 6)
}

__global__ __launch_bounds__(256) void knn_max_norm_kernel(const float* __restrict__ xn, int64_t n,
                                                           unsigned* __restrict__ hdr) {
    float m = 0.f;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256)
        m = fmaxf(m, xn[i]);
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) m = fmaxf(m, __shfl_xor(m, s));
    if ((threadIdx.x & 63) == 0) atomicMax(hdr, __float_as_uint(m));
}

// B operands of the queries of one chunk: per row and 16-coordinate chunk 32 bytes,
// [bf16(-2 q): coordinates 0..7 | 8..15], zero past d.
template <bool ALIGNED>
__global__ __launch_bounds__(256) void knn_split_queries_kernel(const float* __restrict__ Q,
                                                                int64_t ldq, int rows, int d,
                                                                int nch, uint4* __restrict__ Qs) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)rows * nch) return;
    const int r = (int)(idx / nch);
    const int c = (int)(idx - (int64_t)r * nch);
    uint4 hi[2];
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const int col = c * 16 + half * 8;
        const f32x4 v0 = mask_row4(load_row4<ALIGNED>(Q, ldq, r, rows, col, d), true, col, d, -2.f);
        const f32x4 v1 =
            mask_row4(load_row4<ALIGNED>(Q, ldq, r, rows, col + 4, d), true, col + 4, d, -2.f);
        // (scaling by a power of two and rounding commute)
        hi[half] = uint4{round_pair(v0[0], v0[1]), round_pair(v0[2], v0[3]), round_pair(v1[0], v1[1]),
                         round_pair(v1[2], v1[3])};
    }
    uint4* o = Qs + idx * 2;
    o[0] = hi[0];
    o[1] = hi[1];
}

// Out of line and with everything passed by value, so that the search loop of knn_split_kernel
// keeps its state in registers and pays for the rare path only where it is called.  Two groups
// of a row in flight: every register this path uses is one the search loop has to give up
// around its calls (measured, eight groups in flight were slower: c5 99.6 against 88.9 ms).
template <bool ALIGNED>
__device__ __noinline__ unsigned split_flush_query(const float* __restrict__ qp,
                                                   const float* __restrict__ X, int64_t ldx, int d,
                                                   int jsafe, const int* __restrict__ cbuf, int jbase,
                                                   int cc,
                                                   float* __restrict__ gk, int* __restrict__ gi, int k,
                                                   float* scratch, unsigned* tshr,
                                                   const float* __restrict__ rn, int lane) {
    return flush_query_exact<ALIGNED, 2>(qp, X, ldx, d, jsafe, cbuf, jbase, cc, gk, gi, k, scratch,
                                         tshr, rn, lane);
}

// ---------------------------------------------------------------------------------------
// One workgroup = 256 queries (8 waves x 32) against a range of the points, in tiles of 128
// points.  A pipeline step covers W chunks of 16 coordinates: the workgroup loads a 128 x 16 W
// fp32 piece of X (W float4 per thread), rounds it to bf16 on the way into LDS (laid out as the
// MFMA's A operand: 32 bytes per row and chunk, the lower half-wave reads coordinates 0..7, the
// upper 8..15), and every wave runs W x 4 MFMAs on it; the queries' B operands were rounded once
// per chunk of queries and sit in registers (or come from the workspace, see below).  LDS and
// registers are double-buffered over (tile, step), one workgroup barrier per step, the loads of
// step s + 2 in flight during step s: wide steps are what keeps enough of the point stream in
// flight.
//
// Nothing of X is masked on the way: coordinates past d meet zeros in the B operands, and rows
// past the range get +inf as their norm, so whatever valid (finite) data the clamped loads
// return there cannot make a key pass.
//
// The point ranges of one query run in different workgroups at the same time.  Each publishes
// the k-th key of its own list in tsh[row] (atomic minimum) and reads the others' at every
// tile: a range's k-th best bounds the overall k-th best from above, so pairs beyond it need
// not enter any list.  The lists of a range then hold the range's best entries only as far as
// they can matter; the merged result is the same.
// ---------------------------------------------------------------------------------------
//
// NST > 0 (d <= 16 W NST <= 256): the B operands of all W NST chunks stay in registers for the
// whole kernel, so only the points are streamed; the step loop is unrolled (with a second tile
// when NST is odd, so that the alternation of the two buffers is static).  NST == 0: any d, the
// B operands of the next step are fetched from the workspace in every step.
template <int W, int NST, bool ALIGNED>
__global__ __launch_bounds__(512, 2) void knn_split_kernel(
    const float* __restrict__ Q, int64_t ldq, const float* __restrict__ X, int64_t ldx,
    const uint4* __restrict__ Qs, const float* __restrict__ qnorm, unsigned* tsh,
    const float* __restrict__ xn, const unsigned* __restrict__ hdr, int cosine, int rows, int n,
    int d, int nch_real, int k, int S, int split_len, int BQ, int BS, float* __restrict__ lk,
    int* __restrict__ li) {
    // steps per tile that the pipeline walks, W chunks of 16 coordinates each (the chunks past
    // the real count meet zero B operands)
    const int nst = NST > 0 ? NST : (nch_real + W - 1) / W;
    constexpr int TQ = kSpTileQ, TX = kSpTileX, C = kSpCand;
    extern __shared__ __align__(16) unsigned char smem[];
    uint4* as = reinterpret_cast<uint4*>(smem);  // [2 buffers][W chunks][TX][2 halves of 8 bf16]
    float* xns = reinterpret_cast<float*>(as + 2 * W * TX * 2);  // [2][TX] accumulator start values
    float* rns = xns + 2 * TX;                                   // [2][TX] row scales (cosine)
    int* ci = reinterpret_cast<int*>(rns + 2 * TX);              // [TQ][C] buffered point indices
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int i32 = lane & 31;
    const int h = lane >> 5;

    int s, wg_row0;
    if (!xcd_block_map(rows, TQ, S, BQ, BS, s, wg_row0)) return;  // padding (before any barrier)
    const int wave_row0 = wg_row0 + wave * 32;
    int* wci = ci + wave * 32 * C;
    init_lists32(lk, li, wave_row0, rows, S, s, k, lane);

    const float xmax = __uint_as_float(hdr[0]);
    // Filter keys are  xn_j + bf16(x).bf16(-2 q)  accumulated in fp32; the exact test gives
    // dd = sum (q - x)^2  in fp32.  dd <= tau implies key < (tau - qn) + slack with
    //   rounded operands    sum x~ q~' - sum x q' = sum x~ (q~' - q') + sum (x~ - x) q'  (q' = -2 q),
    //                       at most |x~| |q~' - q'| + |x~ - x| |q'| by Cauchy-Schwarz: the query's
    //                       residual norm is taken below, the largest residual norm of a point
    //                       comes with the header (word 1), |x~| <= sqrt(xmax) + that; 1 % on
    //                       top for the fp32 arithmetic of these norms.  (The worst case, 2^-8 of
    //                       every value, gives 2^-6 |x| |q|: about 2.5 times this on dense data,
    //                       more where many coordinates are zero or exact in bf16.)
    //   fp32 accumulations   one per coordinate (padded), of terms that sum to at most
    //                       2.02 |x| |q| in magnitude
    //   roundings of xn, qn, dd   each below (d / 64 + 8) ulps of the value
    // The constants below cover the first in full and are at least twice the others.
    const float e_acc = (float)(4 * (nst * W * 16) + 32) * 0x1p-24f;
    const float e_dot = 1.01f * 0x1p-6f + e_acc;  // (the worst-case form: cosine metric)
    const float e_sum = (float)(d + 16) * 0x1p-23f;
    // own = k-th key of this range's list (+inf until it is full, -inf for a lane without a
    // query), cap = the lowest k-th key any range of the query has published, tauf = the filter
    // threshold that follows from min(own, cap)
    const int r_mine = wave_row0 + i32;
    const bool active = r_mine < rows;
    const int qrow = active ? r_mine : rows - 1;
    const float qn = qnorm[qrow];
    float cross = 0.f;
    if (!cosine) {
        // |bf16(-2 q) - (-2 q)|^2 of the lane's query: the two halves of the wave share the sum
        const float* qrp = Q + (int64_t)qrow * ldq;
        float rq2 = 0.f;
        if (ALIGNED) {
            for (int g = h; 4 * g < d; g += 2) {
                const f32x4 v = *reinterpret_cast<const f32x4*>(qrp + 4 * g);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float r = bf16_residual(-2.f * v[e]);
                    rq2 = fmaf(r, r, rq2);
                }
            }
        } else {
            for (int t = h; t < d; t += 2) {
                const float r = bf16_residual(-2.f * qrp[t]);
                rq2 = fmaf(r, r, rq2);
            }
        }
        rq2 += lane_xor<32>(rq2);
        const float rxm = sqrtf(__uint_as_float(hdr[1]));
        cross = 1.01f * ((sqrtf(xmax) + rxm) * sqrtf(rq2) + rxm * 2.f * sqrtf(qn)) + e_acc * sqrtf(xmax * qn);
    }
    float own = active ? kInf : -kInf;
    float cap = kInf;
    float tauf = own;
    int cnt = 0, ovf = 0;
    const uint4* const qb = Qs + (size_t)qrow * nch_real * 2 + h;
    // (the smallest normal number keeps the bound strict when every value involved is zero).
    // Cosine metric (xn holds 1 / |x|): filter key = -2 bf16(x).bf16(q) / |x|, exact key
    // = -2 (q.x) / |x| from an fp32 dot product; |x| / |x| = 1 leaves e_dot |q| for the
    // products, and the roundings of 1 / |x|, of the scaling and of the dot product are ulps of
    // values below 2.02 |q|.
    const float cross_cos = (e_dot + 4.f * e_sum) * sqrtf(qn);
    auto key_bound = [&](float t) {
        return cosine ? t + (cross_cos + 0x1p-126f)
                      : (t - qn) + (cross + e_sum * (xmax + qn + t) + 0x1p-126f);
    };

    const int j0 = s * split_len;
    const int j1 = min(n, j0 + split_len);
    const int ntiles = (j1 > j0) ? (j1 - j0 + TX - 1) / TX : 0;
    const int total = ntiles * nst;

    // ---- rare path, only entered while the accumulators are dead (between two tiles) ----
    float* const my_scratch =
        reinterpret_cast<float*>(ci + TQ * C) + (size_t)wave * (2 * kWave + 2 * k);
    // exact keys of cc candidates of query L (its buffer, or with from_range the points
    // jbase ..), merged into its list; the lanes of the query get the new thresholds
    auto flush_one = [&](int L, bool from_range, int jbase, int cc) {
        const int r = wave_row0 + L;
        const size_t lb = ((size_t)r * S + s) * k;
        const unsigned fr = split_flush_query<ALIGNED>(
            Q + (int64_t)r * ldq, X, ldx, d, j0, from_range ? nullptr : wci + L * C, jbase, cc,
            lk + lb, li + lb, k, my_scratch, tsh + r, cosine ? xn : nullptr, lane);
        if (i32 == L) {
            own = __uint_as_float(fr);
            tauf = key_bound(fminf(own, cap));
            if (!from_range) cnt = 0;
        }
    };
    // After a tile: buffers with fewer than kSpRoom free slots are emptied; a query whose
    // buffer could not take all of the tile's candidates (ovf; the part it took was dropped
    // again) gets every point of the tile tested instead.
    auto drain = [&](int tile_base, bool everything) {
        uint64_t full =
            __builtin_amdgcn_ballot_w64(cnt > 0 && (everything || ovf || cnt > C - kSpRoom)) &
            0xffffffffull;
        while (full) {
            const int L = __builtin_ctzll(full);
            full &= full - 1;
            flush_one(L, false, 0, __builtin_amdgcn_readlane(cnt, L));
        }
        uint64_t redo = __builtin_amdgcn_ballot_w64(ovf != 0) & 0xffffffffull;
        while (redo) {
            const int L = __builtin_ctzll(redo);
            redo &= redo - 1;
            for (int b = 0; b < 4; ++b) {
                const int base = tile_base + 32 * b;
                const int cc = min(32, j1 - base);
                if (cc > 0) flush_one(L, true, base, cc);
            }
        }
        ovf = 0;
    };

    // While one wave evaluates candidates the other seven stand at the next barrier, and what it
    // waits for is memory.  So when any wave has a buffer to empty, the whole workgroup empties
    // every buffer that is at least kSpShareMin full, the queries dealt out over the eight waves:
    // the waits overlap, and the next such stop is further away.  (Overflowed queries stay with
    // their own wave, drain() above.)
    int* const co_cnt = reinterpret_cast<int*>(reinterpret_cast<float*>(ci + TQ * C) +
                                               (size_t)kSpWaves * (2 * kWave + 2 * k));  // [TQ]
    unsigned* const co_res = reinterpret_cast<unsigned*>(co_cnt + TQ);                   // [TQ]
    int* const co_queue = reinterpret_cast<int*>(co_res + TQ);                          // [TQ]
    int* const co_n = co_queue + TQ;                                                    // [1]
    // "some wave of the workgroup has a buffer to empty", one word per tile in turn: set before
    // the barrier that ends tile t, read by everybody behind it, cleared behind the barrier of
    // tile t + 1 - three words, so that clearing one never meets a wave that is a tile ahead
    int* const co_stop = co_n + 1;                                                      // [3]
    if (tid < 4) co_n[tid] = 0;  // (a barrier follows before the first use)
    auto shared_drain = [&](int tile_base) {
        const bool mine = !ovf && cnt >= kSpShareMin;
        if (h == 0) {
            const int q = wave * 32 + i32;
            co_cnt[q] = cnt;
            if (mine) co_queue[atomicAdd(co_n, 1)] = q;
        }
        __syncthreads();
        const int nq = *co_n;
        for (int e = wave; e < nq; e += kSpWaves) {
            const int q = co_queue[e];
            const int r = wg_row0 + q;
            const size_t lb = ((size_t)r * S + s) * k;
            const unsigned fr = split_flush_query<ALIGNED>(
                Q + (int64_t)r * ldq, X, ldx, d, j0, ci + q * C, 0, co_cnt[q], lk + lb, li + lb, k,
                my_scratch, tsh + r, cosine ? xn : nullptr, lane);
            if (lane == 0) co_res[q] = fr;
        }
        __syncthreads();
        if (mine) {
            own = __uint_as_float(co_res[wave * 32 + i32]);
            tauf = key_bound(fminf(own, cap));
            cnt = 0;
        }
        if (tid == 0) *co_n = 0;  // the next use is behind the barrier that ends the tile
        if (__builtin_amdgcn_ballot_w64(ovf != 0) != 0) drain(tile_base, false);
    };

    // A query that knows no bound yet (empty list, nothing published by another range) would
    // accept all 128 points of its first tile, overflow its buffer and have the whole tile
    // evaluated exactly.  Instead it takes a bound from the filter keys in the accumulators: if at
    // least k of the tile's keys are <= f, at least k points have exact keys <= f + allowance - an
    // upper bound of the k-th smallest, as good a threshold as one from a full list.  f is
    // narrowed by quartering [lowest, highest finite key] five times while keeping
    // count(<= upper end) >= k; the two halves of the wave hold 64 keys each.  (Counts are kept as
    // floats: their additions are not reassociated, so the compiler forms one short chain per
    // count instead of a tree over 64 compare results at a time.)
    auto seed_from_tile = [&](const f32x16 (&a)[4]) {
        float lo = kInf, hi = -kInf, nv = 0.f;
#pragma unroll
        for (int pb = 0; pb < 4; ++pb)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const float v = a[pb][e];
                const bool fin = v < kInf;  // (rows past the range carry +inf)
                lo = fminf(lo, v);
                hi = fmaxf(hi, fin ? v : -kInf);
                nv += fin ? 1.f : 0.f;
            }
        lo = fminf(lo, lane_xor<32>(lo));
        hi = fmaxf(hi, lane_xor<32>(hi));
        nv += lane_xor<32>(nv);
        const float kf = (float)k;
#pragma nounroll
        for (int it = 0; it < 5; ++it) {
            const float q1 = lo + 0.25f * (hi - lo), q2 = lo + 0.5f * (hi - lo), q3 = lo + 0.75f * (hi - lo);
            float c1 = 0.f, c2 = 0.f, c3 = 0.f;
#pragma unroll
            for (int pb = 0; pb < 4; ++pb)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const float v = a[pb][e];
                    c1 += (v <= q1) ? 1.f : 0.f;
                    c2 += (v <= q2) ? 1.f : 0.f;
                    c3 += (v <= q3) ? 1.f : 0.f;
                }
            c1 += lane_xor<32>(c1);
            c2 += lane_xor<32>(c2);
            c3 += lane_xor<32>(c3);
            if (c1 >= kf) hi = q1;
            else if (c2 >= kf) { lo = q1; hi = q2; }
            else if (c3 >= kf) { lo = q2; hi = q3; }
            else lo = q3;
        }
        // the filter's allowance with the bound itself in place of tau in the rounding term, doubled
        // where it depends on the key (the filter key may be off in either direction)
        const float base = hi + qn;
        const float bound = cosine ? hi + 2.f * (cross_cos + 0x1p-126f)
                                   : base + (cross + 2.f * e_sum * (xmax + qn + fabsf(base) + cross) + 0x1p-126f);
        if (tauf == kInf && nv >= kf && bound < kInf) {
            cap = bound;
            if (h == 0) atomicMin(tsh + qrow, key_word(bound));
            tauf = key_bound(bound);
        }
    };

    // End of a tile, accumulators still live, no calls: keys below the filter threshold are
    // buffered (point index only; the two halves of the wave take consecutive slots).
    // Register e of a lane of half h holds point row 8 (e / 4) + 4 h + e % 4 of its block.
    auto epilogue = [&](const f32x16 (&a)[4], int tile_base) {
        // the smallest key of each block of 32 points first: a block without a key under some
        // lane's threshold costs its 16 minima and one vote
        float mb[4];
#pragma unroll
        for (int pb = 0; pb < 4; ++pb) {
            mb[pb] = a[pb][0];
#pragma unroll
            for (int e = 1; e < 16; ++e) mb[pb] = fminf(mb[pb], a[pb][e]);
        }
        if (__builtin_amdgcn_ballot_w64(fminf(fminf(mb[0], mb[1]), fminf(mb[2], mb[3])) < tauf) == 0)
            return;
        // (not in the one shape whose registers it would overflow: 12 resident chunks of aligned
        // rows; there a first tile is evaluated in full as before)
        constexpr bool kSeedFits = !(W == 4 && NST == 3 && ALIGNED);
        if constexpr (kSeedFits) {
            if (__builtin_amdgcn_ballot_w64(tauf == kInf) != 0) seed_from_tile(a);
        }
        const int cnt0 = cnt;
#pragma unroll
        for (int pb = 0; pb < 4; ++pb) {
            if (__builtin_amdgcn_ballot_w64(mb[pb] < tauf) == 0) continue;
            int mine = 0;
#pragma unroll
            for (int e = 0; e < 16; ++e) mine += (a[pb][e] < tauf) ? 1 : 0;
            const int oth = lane_xor<32>(mine);
            if (cnt + mine + oth > C) ovf = 1;  // the same in both halves of the wave
            if (!ovf) {
                int slot = i32 * C + cnt + (h ? oth : 0);
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    if (a[pb][e] < tauf) {
                        wci[slot] = tile_base + pb * 32 + (e >> 2) * 8 + h * 4 + (e & 3);
                        ++slot;
                    }
                }
                cnt += mine + oth;
            }
        }
        if (ovf) cnt = cnt0;
    };

    // staging of the points: thread -> (row = tid / 4, coordinates 4 (tid % 4) .. + 3 of the chunk)
    const int srow = tid >> 2;
    const int squad = tid & 3;
    struct XS {
        f32x4 x[W];
        float xnv;
    };
    struct QB {
        uint4 b[W];
    };
    int f_tile = 0, f_c = 0;  // (tile, step) of the next fetch
    const float* frow = X + (int64_t)min(j0 + srow, j1 - 1) * ldx;  // this thread's row of tile f_tile
    auto fetchX = [&](XS& g) {
#pragma unroll
        for (int kk = 0; kk < W; ++kk)
            g.x[kk] = load_row4<ALIGNED>(frow, 0, 0, 1, (f_c * W + kk) * 16 + squad * 4, d);
        if (f_c == 0) g.xnv = xn[min(j0 + f_tile * TX + (tid & (TX - 1)), j1 - 1)];
        if (++f_c == nst) {
            f_c = 0;
            if (f_tile + 1 < ntiles) ++f_tile;
            frow = X + (int64_t)min(j0 + f_tile * TX + srow, j1 - 1) * ldx;
        }
    };
    int s_tile = 0, s_c = 0;  // (tile, step) of the next stash
    uint2* const as_w = reinterpret_cast<uint2*>(as) + srow * 4 + squad;
    auto stash = [&](int buf, const XS& g) {
#pragma unroll
        for (int kk = 0; kk < W; ++kk) {
            uint2 hi;
            hi.x = round_pair(g.x[kk][0], g.x[kk][1]);
            hi.y = round_pair(g.x[kk][2], g.x[kk][3]);
            as_w[(buf * W + kk) * TX * 4] = hi;
        }
        if (s_c == 0 && tid < TX) {  // +inf past the range: such a row never passes
            const bool ok = j0 + s_tile * TX + tid < j1;
            // xn is |x|^2, or for the cosine metric 1 / |x|: then the sums start from 0 and are
            // scaled by it at the end of the tile
            xns[(s_tile & 1) * TX + tid] = ok ? (cosine ? 0.f : g.xnv) : kInf;
            rns[(s_tile & 1) * TX + tid] = (ok && cosine) ? g.xnv : 1.f;
        }
        if (++s_c == nst) {
            s_c = 0;
            ++s_tile;
        }
    };
    auto fetchQ = [&](int c, QB& g) {  // the B operands of step c; zero past the real chunks
#pragma unroll
        for (int kk = 0; kk < W; ++kk) {
            const int ch = c * W + kk;
            const uint4 v = qb[(ch < nch_real ? ch : nch_real - 1) * 2];
            const uint4 zero = {0u, 0u, 0u, 0u};
            g.b[kk] = ch < nch_real ? v : zero;
        }
    };

    f32x16 acc[4];
    // accumulators of a tile start from the norms of its points
    auto start_tile = [&](int t) {
        const float* xt = xns + (t & 1) * TX;
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
    };
    XS xe, xo;
    xe.xnv = xo.xnv = 0.f;
    if (total > 0) {
        fetchX(xe);
        stash(0, xe);
        fetchX(xo);
    }
    __syncthreads();
    if (total > 0) start_tile(0);
    int tile = 0, tile3 = 0;  // tile3 = tile % 3
    const uint4* const as_r = as + i32 * 2 + h;
    // one (tile, step) step: MFMAs on LDS buffer `par` with the given B operands, the next
    // step's points go to the other buffer meanwhile; last = the tile's last step
    auto step_fn = [&](int step, int par, bool last, const QB& b, XS& mine, const XS& next) {
        // What the other ranges of the query have reached since the last look: asked for
        // before the step's MFMAs and ahead of the point loads (loads return in order, so the
        // wait for this word at the end of the tile does not wait for those), used behind them.
        unsigned others = 0;
        if (last)
            others = __hip_atomic_load(tsh + qrow, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        fetchX(mine);
        const uint4* ab = as_r + par * (W * TX * 2);
#pragma unroll
        for (int kk = 0; kk < W; ++kk) {
            const bf16x8 bh = __builtin_bit_cast(bf16x8, b.b[kk]);
#pragma unroll
            for (int pb = 0; pb < 4; ++pb) {
                const bf16x8 xh = __builtin_bit_cast(bf16x8, ab[kk * TX * 2 + pb * 64]);
                acc[pb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xh, bh, acc[pb], 0, 0, 0);
            }
            if (kk == (W - 1) / 2 && step + 1 < total) stash(par ^ 1, next);
        }
        if (last) {
            // The last use of this tile's accumulators is the epilogue; they are set again
            // right after the barrier of this branch, so nothing of them is live across the
            // calls in drain().
            const int tile_base = j0 + tile * TX;
            cap = fminf(cap, word_key(others));
            tauf = key_bound(fminf(own, cap));
            if (cosine) scale_rows(acc, rns + (tile & 1) * TX, h);
            epilogue(acc, tile_base);
            // The barrier that ends the step carries the vote on stopping as well.
            const bool need = __builtin_amdgcn_ballot_w64(ovf != 0 || cnt > C - kSpRoom) != 0;
            if (need && lane == 0) co_stop[tile3] = 1;
            __syncthreads();
            if (tid == 0) co_stop[tile3 == 0 ? 2 : tile3 - 1] = 0;  // the previous tile's word
            if (co_stop[tile3] != 0) shared_drain(tile_base);
            ++tile;
            tile3 = tile3 == 2 ? 0 : tile3 + 1;
            if (step + 1 < total) start_tile(tile);
        } else {
            __syncthreads();
        }
    };
    if constexpr (NST == 0) {
        QB be, bo;
        if (total > 0) fetchQ(0, be);
        int c = 0;
        auto body = [&](int step, int par, XS& mine, const XS& next, const QB& bcur, QB& bnext) {
            fetchQ(c + 1 == nst ? 0 : c + 1, bnext);
            const bool last = c == nst - 1;
            c = last ? 0 : c + 1;
            step_fn(step, par, last, bcur, mine, next);
        };
        for (int step = 0; step < total; step += 2) {
            body(step, 0, xe, xo, be, bo);
            if (step + 1 < total) body(step + 1, 1, xo, xe, bo, be);
        }
    } else {
        constexpr int NR = NST > 0 ? NST : 1;
        QB bq[NR];
#pragma unroll
        for (int c = 0; c < NR; ++c) fetchQ(c, bq[c]);
        constexpr int TU = (NR % 2) ? 2 : 1;  // tiles per unrolled iteration
        for (int tile0 = 0; tile0 < ntiles; tile0 += TU) {
#pragma unroll
            for (int tt = 0; tt < TU; ++tt) {
                if (tile0 + tt >= ntiles) break;  // uniform
#pragma unroll
                for (int c = 0; c < NR; ++c) {
                    const int step = (tile0 + tt) * NR + c;
                    if (((tt * NR + c) & 1) == 0)
                        step_fn(step, 0, c == NR - 1, bq[c], xe, xo);
                    else
                        step_fn(step, 1, c == NR - 1, bq[c], xo, xe);
                }
            }
        }
    }
    drain(0, true);
}

__global__ void knn_fill_words_kernel(unsigned* __restrict__ p, int64_t count, unsigned value) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < count) p[i] = value;
}

}  // namespace

hipError_t launch_header_init(void* hdr, hipStream_t stream) {
    knn_split_init_kernel<<<dim3(1), dim3(64), 0, stream>>>(static_cast<unsigned*>(hdr));
    return hipGetLastError();
}

hipError_t launch_max_norm(const float* xn, int64_t n, void* hdr, hipStream_t stream) {
    unsigned* w = static_cast<unsigned*>(hdr);
    int64_t blocks = (n + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    knn_max_norm_kernel<<<dim3((unsigned)blocks), dim3(256), 0, stream>>>(xn, n, w);
    return hipGetLastError();
}

hipError_t launch_fill_words(void* p, int64_t count, unsigned value, hipStream_t stream) {
    if (count > 0)
        knn_fill_words_kernel<<<dim3((unsigned)((count + 255) / 256)), dim3(256), 0, stream>>>(
            static_cast<unsigned*>(p), count, value);
    return hipGetLastError();
}

hipError_t launch_split_queries(const float* Q, int64_t ldq, int64_t rows, int d, void* qs,
                                void* tsh, bool reset_thresholds, hipStream_t stream) {
    const int nch = (d + kSpKC - 1) / kSpKC;
    if (reset_thresholds)
        knn_fill_words_kernel<<<dim3((unsigned)((rows + 255) / 256)), dim3(256), 0, stream>>>(
            static_cast<unsigned*>(tsh), rows, kInfWord);  // +inf: nothing published yet
    const int64_t items = rows * nch;
    const bool aligned = (reinterpret_cast<uintptr_t>(Q) % 16 == 0) && (ldq % 4 == 0) && (d % 4 == 0);
    const dim3 grid((unsigned)((items + 255) / 256));
    if (aligned)
        knn_split_queries_kernel<true><<<grid, dim3(256), 0, stream>>>(Q, ldq, (int)rows, d, nch,
                                                                       static_cast<uint4*>(qs));
    else
        knn_split_queries_kernel<false><<<grid, dim3(256), 0, stream>>>(Q, ldq, (int)rows, d, nch,
                                                                        static_cast<uint4*>(qs));
    return hipGetLastError();
}

hipError_t launch_split(const float* Q, int64_t ldq, const float* X, int64_t ldx, const void* qs,
                        const float* qn, void* tsh, const float* xn, const void* hdr, bool cosine,
                        int64_t rows, int64_t n, int d, int k, int S, float* lk, int* li,
                        hipStream_t stream) {
    const int nch = (d + kSpKC - 1) / kSpKC;
    const size_t lds_fixed = (size_t)4 * kSpTileX * 4 + (size_t)kSpTileQ * kSpCand * 4 +
                             (size_t)kSpWaves * (2 * kWave + 2 * k) * 4 +
                             (size_t)(3 * kSpTileQ + 4) * 4;  // the shared drain's arrays
    int64_t split_len = (n + S - 1) / S;
    split_len = (split_len + kSpTileX - 1) / kSpTileX * kSpTileX;
    // One workgroup per compute unit is resident, so the (tile, range) pairs go to the 8 XCDs
    // round-robin (block shape 1 x 1 of the mapping): consecutive query tiles of one range land
    // on every XCD in turn, each XCD holds at most one pair more than another, and the
    // workgroups that share an XCD's L2 mostly walk the same range of points.
    const int T = (int)((rows + kSpTileQ - 1) / kSpTileQ);
    const int BQ = 1, BS = 1;
    const int blocks = T * S;
    const dim3 grid((unsigned)((blocks + 7) / 8 * 8));
    const bool aligned = (reinterpret_cast<uintptr_t>(Q) % 16 == 0) &&
                         (reinterpret_cast<uintptr_t>(X) % 16 == 0) && (ldq % 4 == 0) &&
                         (ldx % 4 == 0) && (d % 4 == 0);
#define KNN_SPLIT_LAUNCH(W, N, A)                                                                 \
    do {                                                                                          \
        const size_t lds = lds_fixed + (size_t)2 * (W) * kSpTileX * 2 * 16;                       \
        hipError_t e2 = raise_lds_limit(knn_split_kernel<W, N, A>, lds);                          \
        if (e2 != hipSuccess) return e2;                                                          \
        knn_split_kernel<W, N, A><<<grid, dim3(64 * kSpWaves), lds, stream>>>(                    \
            Q, ldq, X, ldx, static_cast<const uint4*>(qs), qn, static_cast<unsigned*>(tsh), xn,   \
            static_cast<const unsigned*>(hdr), cosine ? 1 : 0, (int)rows, (int)n, d, nch, k, S,   \
            (int)split_len, BQ, BS, lk, li);                                                      \
    } while (0)
    // W chunks of 16 coordinates per pipeline step, N steps per tile with the queries resident
    // in registers (up to d = 256; W * N is the chunk count rounded up to a shape that is
    // instantiated), N = 0: any d, queries streamed.  Wide steps keep more bytes of the point
    // stream in flight, which is what the kernel waits for; the shapes are the fastest measured
    // among those that fit the register budget (the element-wise loads of unaligned rows need
    // more registers, so those take narrower steps).
    // (No shape with one step per tile: its loop is unrolled over two tiles and then spills two
    // registers to private memory, which the runtime would have to provide beside the workspace.)
    if (aligned) {
        if (nch <= 2) KNN_SPLIT_LAUNCH(1, 2, true);
        else if (nch <= 4) KNN_SPLIT_LAUNCH(2, 2, true);
        else if (nch <= 6) KNN_SPLIT_LAUNCH(3, 2, true);
        else if (nch <= 8) KNN_SPLIT_LAUNCH(4, 2, true);
        else if (nch <= 9) KNN_SPLIT_LAUNCH(3, 3, true);
        else if (nch <= 12) KNN_SPLIT_LAUNCH(4, 3, true);
        else if (nch <= kSpResidentMaxChunks) KNN_SPLIT_LAUNCH(4, 4, true);
        else KNN_SPLIT_LAUNCH(4, 0, true);
    } else {
        if (nch <= 2) KNN_SPLIT_LAUNCH(1, 2, false);
        else if (nch <= 4) KNN_SPLIT_LAUNCH(2, 2, false);
        else if (nch <= 6) KNN_SPLIT_LAUNCH(2, 3, false);
        else if (nch <= 8) KNN_SPLIT_LAUNCH(2, 4, false);
        else if (nch <= 10) KNN_SPLIT_LAUNCH(2, 5, false);
        else if (nch <= 12) KNN_SPLIT_LAUNCH(2, 6, false);
        else if (nch <= kSpResidentMaxChunks) KNN_SPLIT_LAUNCH(2, 8, false);
        else KNN_SPLIT_LAUNCH(2, 0, false);
    }
#undef KNN_SPLIT_LAUNCH
    return hipGetLastError();
}

}  // namespace knn
