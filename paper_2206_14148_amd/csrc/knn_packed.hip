// gfx950 (CDNA4, MI355X) kNN search for 8 < d <= 256 and many points: the bf16 matrix-core
// filter of knn_split.hip with the roles of the operands swapped.
//
// The expansion sum x^2 - 2 q.x of paper section 4.1 runs on the values rounded to bf16 and only
// filters; what passes is evaluated exactly (knn_exact.h) and merged into the query's list, so
// the distance tile never leaves the registers (section 4.3) and the results do not depend on
// the filter.  What differs from knn_split_kernel is where the operands live:
//   - the points are rounded to bf16 ONCE, by knn_pack_operands_kernel, into a copy in the
//     workspace that is laid out in the order of the MFMA's A operand, so that a wave fetches an
//     operand with one coalesced 1 KB load straight into registers: no conversion, no LDS
//     staging, no workgroup barrier in the search loop;
//   - a workgroup keeps the B operands of up to 16 sets of 32 queries in LDS for its whole
//     life; each of its waves (12 up to d = 128, 8 above) walks its own steps of 64 points, and
//     for every step runs through all query sets: one 1 KB LDS read feeds two MFMAs, and the accumulators start
//     from the points' squared norms through the MFMA's C operand, held in registers per step.
//     A step's operands (up to 128 registers at d = 256) are requested when it begins and are
//     dead when it ends, so three waves of <= 168 registers share a SIMD up to d = 128 and two
//     of <= 256 above, and the others compute while one waits for its operands.
// The waves therefore see different points for the same queries.  Pairs that pass the
// filter go to per-query buffers in LDS that all waves append to (slots reserved with a
// compare-and-swap, all of a wave's pairs for a query and step or none); when a buffer runs
// full the workgroup stops at the next step boundary, the queries with enough buffered pairs are
// dealt out over the waves, evaluated exactly and merged into their lists, and a (wave, query,
// step) that found no room is made good by testing all 64 points of that step.
//
// The thresholds are finite when this kernel starts: knn_seed_kernel has bounded every query's
// k-th distance from the filter keys of a sample of the points (a list that starts from +inf
// would accept everything and spend its time in the stops).
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

// The points of a slab rounded to bf16 in A-operand order: step (64 points) -> row block (32) ->
// chunk of 16 coordinates -> lane: lane (i32, h) holds coordinates 16 c + 8 h .. + 7 of point
// 32 pb + i32, zero past d and past n.  This kernel serves rows that are not 16-byte aligned (one
// thread per (point, chunk, half), element-wise loads); aligned rows take knn_pack_block_kernel.  `scale` (a power of two:
// it commutes with the rounding) is 1 for points and -2 for queries packed as B operands.
__global__ __launch_bounds__(256) void knn_pack_operands_kernel(const float* __restrict__ X,
                                                                int64_t ldx, int n, int d, int nch,
                                                                int j_first, int64_t pieces,
                                                                float scale, uint4* __restrict__ Xp) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= pieces) return;
    const int per_row = nch * 2;
    const int rel = (int)(idx / per_row);
    const int piece = (int)(idx - (int64_t)rel * per_row);
    const int c = piece >> 1, h = piece & 1;
    const int j = j_first + rel;
    const bool ok = j < n;
    const int col = c * 16 + h * 8;
    const f32x4 v0 = mask_row4(load_row4<false>(X, ldx, j, n, col, d), ok, col, d, scale);
    const f32x4 v1 = mask_row4(load_row4<false>(X, ldx, j, n, col + 4, d), ok, col + 4, d, scale);
    const uint4 w = {round_pair(v0[0], v0[1]), round_pair(v0[2], v0[3]), round_pair(v1[0], v1[1]),
                     round_pair(v1[2], v1[3])};
    const int st = rel >> 6, pb = (rel >> 5) & 1, i32 = rel & 31;
    Xp[((size_t)(st * 2 + pb) * nch + c) * 64 + h * 32 + i32] = w;
}

// The same copy for rows that are 16-byte aligned, a row block of 32 points per workgroup, through
// LDS: each of the four waves reads eight rows (32 bytes a lane, whole rows at a stretch) and
// writes their rounded pieces into the block's operands in LDS; the block's operands - nch KB in a
// row in the copy - then go out as whole 1 KB stores.  Rows longer than kPbSeg chunks take several
// passes.  NORMS: the squared norms of the rows (one fma chain per lane over its pieces, lanes added
// up by a butterfly: a fixed order) go to xn, and the largest squared norm of a rounding residual
// x - bf16(x) to hdr[1] - the pass over X that knn_row_norms_kernel would otherwise repeat.
// (With row_scale both are those of the scaled rows; xn may be null.)
constexpr int kPbSeg = 32;               // chunks per pass
constexpr int kPbOperandStride = 64 + 2; // uint4 per operand in LDS (a half of 32 rows + one: no bank conflicts)
template <bool NORMS>
__global__ __launch_bounds__(256) void knn_pack_block_kernel(const float* __restrict__ X, int64_t ldx, int n,
                                                             int d, int nch, int j_first, int nblocks,
                                                             float scale, const float* __restrict__ row_scale,
                                                             uint4* __restrict__ Xp,
                                                             float* __restrict__ xn, unsigned* __restrict__ hdr) {
    __shared__ uint4 ops[kPbSeg * kPbOperandStride];
    __shared__ float wmax[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float worst = 0.f;
    for (int blk = blockIdx.x; blk < nblocks; blk += gridDim.x) {
        float acc[8], res[8];
#pragma unroll
        for (int rr = 0; rr < 8; ++rr) acc[rr] = res[rr] = 0.f;
        for (int c0 = 0; c0 < nch; c0 += kPbSeg) {
            const int cs = min(kPbSeg, nch - c0);
            for (int m = lane; m < 2 * cs; m += 64) {  // piece m of the pass: chunk c0 + m / 2, half m % 2
                const int col = c0 * 16 + m * 8;
                f32x4 v0[8], v1[8];
#pragma unroll
                for (int rr = 0; rr < 8; ++rr) {
                    const int j = j_first + blk * 32 + wave * 8 + rr;
                    v0[rr] = load_row4<true>(X, ldx, j, n, col, d);
                    v1[rr] = load_row4<true>(X, ldx, j, n, col + 4, d);
                }
#pragma unroll
                for (int rr = 0; rr < 8; ++rr) {
                    const int jr = j_first + blk * 32 + wave * 8 + rr;
                    const bool ok = jr < n;
                    // (row_scale: every row times its own factor - the cosine metric's 1 / |x|)
                    const float sc = row_scale ? row_scale[ok ? jr : 0] : scale;
                    const f32x4 a0 = mask_row4(v0[rr], ok, col, d, sc);
                    const f32x4 a1 = mask_row4(v1[rr], ok, col + 4, d, sc);
                    if (NORMS) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            acc[rr] = fmaf(a0[e], a0[e], acc[rr]);
                            const float r = bf16_residual(a0[e]);
                            res[rr] = fmaf(r, r, res[rr]);
                        }
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            acc[rr] = fmaf(a1[e], a1[e], acc[rr]);
                            const float r = bf16_residual(a1[e]);
                            res[rr] = fmaf(r, r, res[rr]);
                        }
                    }
                    const uint4 w = {round_pair(a0[0], a0[1]), round_pair(a0[2], a0[3]), round_pair(a1[0], a1[1]),
                                     round_pair(a1[2], a1[3])};
                    ops[(m >> 1) * kPbOperandStride + (m & 1) * 33 + wave * 8 + rr] = w;
                }
            }
            __syncthreads();
            for (int c = wave; c < cs; c += 4)
                Xp[((size_t)blk * nch + c0 + c) * 64 + lane] = ops[c * kPbOperandStride + (lane >> 5) * 33 + (lane & 31)];
            __syncthreads();
        }
        if (NORMS) {
#pragma unroll
            for (int rr = 0; rr < 8; ++rr) {
                float a = acc[rr], r = res[rr];
#pragma unroll
                for (int sft = 32; sft > 0; sft >>= 1) {
                    a += __shfl_xor(a, sft);
                    r += __shfl_xor(r, sft);
                }
                const int j = j_first + blk * 32 + wave * 8 + rr;
                if (xn && lane == 0 && j < n) xn[j] = a;
                worst = fmaxf(worst, r);
            }
        }
    }
    if (NORMS) {  // one atomic per workgroup (they all go to the same word)
        if (lane == 0) wmax[wave] = worst;
        __syncthreads();
        if (threadIdx.x == 0)
            atomicMax(hdr + 1, __float_as_uint(fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]))));
    }
}

// norms past n (up to the end of the last step) are +inf: such a row never passes the filter
__global__ void knn_pad_norms_kernel(float* __restrict__ xn, int n, int n_pad) {
    const int i = n + blockIdx.x * 64 + threadIdx.x;
    if (i < n_pad) xn[i] = kInf;
}

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

// A first threshold for every query from FILTER keys alone.  The filter key f of a pair and its
// exact key dd differ by at most the filter's allowance (in either direction), so if t is such
// that at least k points of a sample have f <= t, at least k points have dd <= t + qn + allowance:
// an upper bound of the query's k-th smallest distance, as valid a starting threshold as +inf and
// far tighter - without evaluating a single pair exactly.  (Lists that start from +inf accept
// every pair until they hold k entries; with all waves feeding one buffer that phase would be
// spent in stops.)  The sample is `sample_steps` steps of 64 points spread evenly over the packed
// copy.  One workgroup per 32 queries (B operands in registers, every wave a quarter of the
// sample); a first pass finds the lane's lowest
// and highest filter key, then kSeedIters passes quarter the interval [lo, hi] keeping
// count(f <= hi) >= k.  The bound goes into tsh (atomic minimum on the order-preserving word).
constexpr int kSeedIters = 4;
constexpr float kCosUnit = 1.0001f;  // cosine metric: the packed rows are x / |x|, of squared norm below this
constexpr int kSeedSets = 1;  // sets of 32 queries per wave
template <int NCH>
__global__ __launch_bounds__(256, 2) void knn_seed_kernel(const uint4* __restrict__ Xp, const float* __restrict__ xn,
                                                       const uint4* __restrict__ Qs,
                                                       const float* __restrict__ qnorm,
                                                       const unsigned* __restrict__ hdr,
                                                       const float* __restrict__ Q, int64_t ldq,
                                                       unsigned* __restrict__ tsh, int rows, int d,
                                                       int nch_real, int k, int nsteps, int sample_steps,
                                                       int cosine) {
    const int lane = threadIdx.x & 63;
    const int i32 = lane & 31, h = lane >> 5;
    // The four waves of a workgroup serve the same 32 queries and take every fourth step of the
    // sample each; their extremes and counts meet in LDS.  (One wave per 32 queries walking the
    // whole sample left most of the chip idle below 3e4 queries: 0.94 ms of c6's 4.6.)
    const int wv = threadIdx.x >> 6;
    const int row0 = blockIdx.x * (32 * kSeedSets);
    __shared__ float ex_l[4][2][32];
    __shared__ int cnt_l[4][3][32];
    static_assert(kSeedSets == 1, "one query set per workgroup");
    uint4 bq[kSeedSets][NCH];
#pragma unroll
    for (int t = 0; t < kSeedSets; ++t) {
        const int rc = min(row0 + 32 * t + i32, rows - 1);
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            // (loaded from a valid chunk, then selected: a conditional load would be made a load
            // through a selected pointer, with the zeros in private memory)
            const uint4 zero = {0u, 0u, 0u, 0u};
            const uint4 v = Qs[((size_t)rc * nch_real + min(c, nch_real - 1)) * 2 + h];
            bq[t][c] = c < nch_real ? v : zero;
        }
    }
    // keys of one step: acc[t][pb] = query set t against row block pb (as in the search loop of
    // knn_packed_kernel)
    auto keys = [&](int step, f32x16 (&acc)[kSeedSets][2]) {
        const u32x4* p = reinterpret_cast<const u32x4*>(Xp) + (size_t)step * (2 * NCH * 64) + lane;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const f32x4 t0 = *reinterpret_cast<const f32x4*>(xn + (size_t)step * kPkStep + g * 8 + h * 4);
            const f32x4 t1 = *reinterpret_cast<const f32x4*>(xn + (size_t)step * kPkStep + 32 + g * 8 + h * 4);
#pragma unroll
            for (int t = 0; t < kSeedSets; ++t)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    acc[t][0][g * 4 + e] = t0[e];
                    acc[t][1][g * 4 + e] = t1[e];
                }
        }
        // (all of the step's operands are requested before the first is used: one wait a step)
        u32x4 A[2][NCH];
#pragma unroll
        for (int pb = 0; pb < 2; ++pb)
#pragma unroll
            for (int c = 0; c < NCH; ++c) A[pb][c] = p[(pb * NCH + c) * 64];
        __builtin_amdgcn_sched_barrier(0);  // (or the scheduler moves each load down to its use)
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const bf16x8 x0 = __builtin_bit_cast(bf16x8, A[0][c]);
            const bf16x8 x1 = __builtin_bit_cast(bf16x8, A[1][c]);
#pragma unroll
            for (int t = 0; t < kSeedSets; ++t) {
                const bf16x8 b = __builtin_bit_cast(bf16x8, bq[t][c]);
                acc[t][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x0, b, acc[t][0], 0, 0, 0);
                acc[t][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x1, b, acc[t][1], 0, 0, 0);
            }
        }
    };
    auto step_of = [&](int i) { return (int)((int64_t)i * nsteps / sample_steps); };
    float lo[kSeedSets], hi[kSeedSets];
#pragma unroll
    for (int t = 0; t < kSeedSets; ++t) {
        lo[t] = kInf;
        hi[t] = -kInf;
    }
    for (int i = wv; i < sample_steps; i += 4) {
        f32x16 acc[kSeedSets][2];
        keys(step_of(i), acc);
#pragma unroll
        for (int t = 0; t < kSeedSets; ++t)
#pragma unroll
            for (int pb = 0; pb < 2; ++pb)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const float v = acc[t][pb][e];
                    lo[t] = fminf(lo[t], v);
                    hi[t] = fmaxf(hi[t], v < kInf ? v : -kInf);  // (rows past n carry +inf: no points)
                }
    }
#pragma unroll
    for (int t = 0; t < kSeedSets; ++t) {
        lo[t] = fminf(lo[t], lane_xor<32>(lo[t]));
        hi[t] = fmaxf(hi[t], lane_xor<32>(hi[t]));
        if (h == 0) {
            ex_l[wv][0][i32] = lo[t];
            ex_l[wv][1][i32] = hi[t];
        }
        __syncthreads();
        lo[t] = fminf(fminf(ex_l[0][0][i32], ex_l[1][0][i32]), fminf(ex_l[2][0][i32], ex_l[3][0][i32]));
        hi[t] = fmaxf(fmaxf(ex_l[0][1][i32], ex_l[1][1][i32]), fmaxf(ex_l[2][1][i32], ex_l[3][1][i32]));
    }
    // (three thresholds a pass, the quartiles of the interval: two bits of the answer for one
    // walk over the sample, which is what a pass costs - the operands come out of the L2 again)
    for (int it = 0; it < kSeedIters; ++it) {
        float q1[kSeedSets], q2[kSeedSets], q3[kSeedSets];
        int c1[kSeedSets], c2[kSeedSets], c3[kSeedSets];
#pragma unroll
        for (int t = 0; t < kSeedSets; ++t) {
            q1[t] = lo[t] + 0.25f * (hi[t] - lo[t]);
            q2[t] = lo[t] + 0.5f * (hi[t] - lo[t]);
            q3[t] = lo[t] + 0.75f * (hi[t] - lo[t]);
            c1[t] = c2[t] = c3[t] = 0;
        }
        for (int i = wv; i < sample_steps; i += 4) {
            f32x16 acc[kSeedSets][2];
            keys(step_of(i), acc);
#pragma unroll
            for (int t = 0; t < kSeedSets; ++t)
#pragma unroll
                for (int pb = 0; pb < 2; ++pb)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const float v = acc[t][pb][e];
                        c1[t] += (v <= q1[t]) ? 1 : 0;
                        c2[t] += (v <= q2[t]) ? 1 : 0;
                        c3[t] += (v <= q3[t]) ? 1 : 0;
                    }
        }
#pragma unroll
        for (int t = 0; t < kSeedSets; ++t) {
            c1[t] += lane_xor<32>(c1[t]);
            c2[t] += lane_xor<32>(c2[t]);
            c3[t] += lane_xor<32>(c3[t]);
            __syncthreads();  // (the previous pass has read its counts)
            if (h == 0) {
                cnt_l[wv][0][i32] = c1[t];
                cnt_l[wv][1][i32] = c2[t];
                cnt_l[wv][2][i32] = c3[t];
            }
            __syncthreads();
            c1[t] = cnt_l[0][0][i32] + cnt_l[1][0][i32] + cnt_l[2][0][i32] + cnt_l[3][0][i32];
            c2[t] = cnt_l[0][1][i32] + cnt_l[1][1][i32] + cnt_l[2][1][i32] + cnt_l[3][1][i32];
            c3[t] = cnt_l[0][2][i32] + cnt_l[1][2][i32] + cnt_l[2][2][i32] + cnt_l[3][2][i32];
            // the lowest quarter whose upper end still has k keys at or below it
            if (c1[t] >= k) hi[t] = q1[t];
            else if (c2[t] >= k) { lo[t] = q1[t]; hi[t] = q2[t]; }
            else if (c3[t] >= k) { lo[t] = q2[t]; hi[t] = q3[t]; }
            else lo[t] = q3[t];
        }
    }
#pragma unroll
    for (int t = 0; t < kSeedSets; ++t) {
        const int r = row0 + 32 * t + i32;
        if (r < rows && h == 0 && wv == 0) {
            // the allowance of knn_packed_kernel's filter (see there), with the bound itself in
            // place of tau in the rounding term and that term doubled
            const float xmax = cosine ? kCosUnit : __uint_as_float(hdr[0]);
            const float rxm = sqrtf(__uint_as_float(hdr[1]));
            const float qn = qnorm[r];
            float rq2 = 0.f;
            const float* qrow = Q + (int64_t)r * ldq;
            for (int u = 0; u < d; ++u) {
                const float res = bf16_residual(-2.f * qrow[u]);
                rq2 = fmaf(res, res, rq2);
            }
            const float e_acc = (float)(4 * (NCH * 16) + 32) * 0x1p-24f;
            const float e_sum = (float)(d + 16) * 0x1p-23f;
            const float cross = 1.01f * ((sqrtf(xmax) + rxm) * sqrtf(rq2) + rxm * 2.f * sqrtf(qn)) +
                                e_acc * sqrtf(xmax * qn);
            const float base = hi[t] + qn;
            // (cosine metric: the key is -2 q.x / |x| itself, see knn_packed_kernel; twice its allowance)
            const float bound = cosine ? hi[t] + 2.f * (cross + 4.f * e_sum * sqrtf(qn) + 0x1p-126f)
                                       : base + (cross + 2.f * e_sum * (xmax + qn + fabsf(base) + cross) + 0x1p-126f);
            atomicMin(tsh + r, key_word(bound));
        }
    }
}

struct PkArgs {
    const float* Q;
    int64_t ldq;
    const float* X;
    int64_t ldx;
    const uint4* Xp;       // packed points of the slab
    const float* xn;       // squared norms of all points, +inf up to the end of the last step
                           // (cosine metric: zeros, +inf past the points - what the sums start from)
    const float* rn;       // cosine metric: 1 / |x| of all points; else null
    const uint4* Qs;       // B operands of the chunk's queries (knn_split_queries_kernel)
    const float* qnorm;    // their squared norms
    unsigned* tsh;         // [rows] lowest k-th key any range of the query has reached
                           // (order-preserving words)
    unsigned* tsr;         // [rows][S] key at position ceil(k / S) - 1 of each range's list
    const unsigned* hdr;   // word 0: max of xn
    float* lk;
    int* li;
    int rows, n, d, nch_real, k, S, sets, tiles;
    int step_slab0;   // step index of the slab's first step (a step = 64 consecutive points)
    int step_first;   // first step this launch covers
    int step_end;     // one past the last
    int range_steps;  // steps per point range
    int init_from;    // the lists of ranges >= this start empty, the others continue
    int j_valid;      // a valid point index for lanes that hold no candidate
};

enum { kCtlStop = 32, kCtlCount = 33, kCtlDone = 34, kCtlNext = 35 };

template <int NCH, bool ALIGNED, int WV, bool COS>
__global__ __launch_bounds__(64 * WV, WV / 4) void knn_packed_kernel(const PkArgs a) {
    constexpr int kPkWaves = WV;  // 12 or 8 (pk_waves)
    constexpr int C = kPkCand;
    constexpr int NT = 64 * kPkWaves;
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i32 = lane & 31;
    const int h = lane >> 5;
    const int sets = a.sets, Qw = sets * 32, k = a.k, S = a.S;
    // Consecutive workgroups take consecutive query tiles of one range, range after range: with
    // more workgroups than compute units the ranges of a query then run mostly one after the
    // other, and a later range starts under the thresholds the earlier ones have reached (far
    // fewer pairs to evaluate exactly than when all ranges of a query start together: measured
    // at d = 256, S = 8, 75 against 91 ms; the order makes no measurable difference to the
    // point stream, which comes out of the L2 / Infinity Cache either way).
    const int s = blockIdx.x / a.tiles;
    const int wg_row0 = (blockIdx.x - s * a.tiles) * Qw;

    uint4* const Bq = reinterpret_cast<uint4*>(smem);                // [sets][NCH][64]
    int* const cand = reinterpret_cast<int*>(Bq + (size_t)sets * NCH * 64);  // [Qw][C]
    float* const qn_l = reinterpret_cast<float*>(cand + Qw * C);     // [Qw] squared norms
    float* const own_l = qn_l + Qw;      // [Qw] k-th key of the query's list in this range
    // [Qw][3] what the search loop touches of a query, side by side so that one address serves
    // all three (an odd stride in words: no bank conflicts): the filter threshold, the number of
    // buffered pairs, and bit 2 w + p set where wave w found no room in its step of parity p
    int* const hot_l = reinterpret_cast<int*>(own_l + Qw);
    auto tauf_at = [&](int q) -> float& { return *reinterpret_cast<float*>(hot_l + 3 * q); };
    auto alloc_at = [&](int q) -> int& { return hot_l[3 * q + 1]; };
    auto ovf_at = [&](int q) -> int& { return hot_l[3 * q + 2]; };
    int* const queue_l = hot_l + 3 * Qw;  // [Qw] queries a stop has to serve
    float* const cross_l = reinterpret_cast<float*>(queue_l + Qw);  // [Qw] allowance for the rounded operands
    float* const scratch = cross_l + Qw;  // [waves][2 * 64 + 2 k]
    float* const xn_stage = scratch + (size_t)kPkWaves * (2 * kWave + 2 * k);  // [waves][64]
    int* const ctl = reinterpret_cast<int*>(xn_stage + kPkWaves * 64);
    // ctl[2 w + p]: the step wave w walks in its iterations of parity p; then the three words above

    for (int i = tid; i < sets * NCH * 64; i += NT) {
        const int qs = i / (NCH * 64);
        const int rem = i - qs * (NCH * 64);
        const int c = rem >> 6, ln = rem & 63;
        const int row = min(wg_row0 + qs * 32 + (ln & 31), a.rows - 1);
        uint4 v = {0u, 0u, 0u, 0u};
        if (c < a.nch_real) v = a.Qs[((size_t)row * a.nch_real + c) * 2 + (ln >> 5)];
        Bq[i] = v;
    }
    // The filter bound.  The filter key is  xn_j + sum_t bf16(x_jt) bf16(-2 q_it)  accumulated in
    // fp32, the exact test gives dd = sum (q - x)^2 in fp32; dd <= tau implies
    // key < (tau - qn) + slack with
    //   rounded operands    sum x~ q~' - sum x q' = sum x~ (q~' - q') + sum (x~ - x) q'  (q' = -2 q),
    //                       at most |x~| |q~' - q'| + |x~ - x| |q'| by Cauchy-Schwarz: the queries'
    //                       residual norms rq are taken here, the largest residual norm of a
    //                       point comes with the header, |x~| <= sqrt(xmax) + that; 1 % on top
    //                       for the fp32 arithmetic of these norms.  (The worst case, 2^-8 of
    //                       every value, is about 2.5 times this on ordinary data.)
    //   fp32 accumulations   one per coordinate (padded), of terms that sum to at most
    //                       2.02 |x| |q| in magnitude
    //   roundings of xn, qn, dd   each below (d / 64 + 8) ulps of the value
    // The constants below cover the first in full and are at least twice the others.
    // Cosine metric (COS; a.rn = 1 / |x|): the copy holds the rows x / |x| (scaled in fp32, then rounded),
    // the sums start from 0, so the filter key is  sum bf16(x^) bf16(-2 q)  and the exact key
    // -2 (q.x) / |x| from an fp32 dot product (knn_exact.h).  The same two terms bound the rounded
    // operands with |x^| < 1.0001 in place of sqrt(xmax) and the residuals of the scaled rows in
    // the header; the roundings of 1 / |x|, of the scaling and of the dot product are ulps of
    // values below 2.02 |q|: 4 e_sum |q| covers them twice over.  Nothing is subtracted from tau.
    constexpr bool cosine = COS;
    const float xmax = cosine ? kCosUnit : __uint_as_float(a.hdr[0]);
    const float rxm = sqrtf(__uint_as_float(a.hdr[1]));
    const float e_acc = (float)(4 * (NCH * 16) + 32) * 0x1p-24f;
    const float e_sum = (float)(a.d + 16) * 0x1p-23f;
    auto key_bound = [&](float t, float qn, float cross) {
        return cosine ? t + (cross + 4.f * e_sum * sqrtf(qn) + 0x1p-126f)
                      : (t - qn) + (cross + e_sum * (xmax + qn + t) + 0x1p-126f);
    };
    // Thresholds.  A query's S ranges run in different workgroups; any upper bound of the k-th
    // smallest key over ALL points may cut every range's candidates:
    //   own     the k-th key of this range's list;
    //   tsh[r]  the lowest k-th key any range has published;
    //   tsr     every range publishes the key at position p = ceil(k / S) - 1 of its list: the
    //           ranges hold different points, so at least S (p + 1) >= k keys are at or below the
    //           largest of the S published values.  A range that has seen a fraction of the
    //           points finds its (k / S)-th best where the whole stream's k-th best lies, so
    //           this bound is as tight as one list over all points would give.
    const int pos_s = (k + S - 1) / S - 1;
    auto shared_cap = [&](int r) {
        float c = 0.f;
        bool all_finite = true;
        for (int t = 0; t < S; ++t) {
            const float v = word_key(
                __hip_atomic_load(a.tsr + (size_t)r * S + t, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
            all_finite = all_finite && v < kInf;
            c = t == 0 ? v : fmaxf(c, v);
        }
        const float lowest =
            word_key(__hip_atomic_load(a.tsh + r, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        return all_finite ? fminf(c, lowest) : lowest;
    };
    const bool init_mine = s >= a.init_from;
    for (int qq = tid; qq < Qw; qq += NT) {
        const int r = wg_row0 + qq;
        const bool active = r < a.rows;
        const int rc = active ? r : a.rows - 1;
        const float qn = a.qnorm[rc];
        qn_l[qq] = qn;
        // |bf16(-2 q) - (-2 q)|^2 of this query
        float rq2 = 0.f;
        {
            const float* qrow = a.Q + (int64_t)rc * a.ldq;
            for (int t = 0; t < a.d; t += 4) {  // rows are 16-byte aligned, d % 4 == 0
                const f32x4 v = *reinterpret_cast<const f32x4*>(qrow + t);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float r = bf16_residual(-2.f * v[e]);
                    rq2 = fmaf(r, r, rq2);
                }
            }
        }
        const float cross = 1.01f * ((sqrtf(xmax) + rxm) * sqrtf(rq2) + rxm * 2.f * sqrtf(qn)) +
                            e_acc * sqrtf(xmax * qn);
        cross_l[qq] = cross;
        float own = -kInf;  // a row past the chunk: nothing passes
        if (active) {
            const size_t lb = ((size_t)r * S + s) * k;
            own = init_mine ? kInf : a.lk[lb + (k - 1)];
            if (!init_mine)
                __hip_atomic_store(a.tsr + (size_t)r * S + s, key_word(a.lk[lb + pos_s]), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
        }
        own_l[qq] = own;
        tauf_at(qq) = active ? key_bound(fminf(own, shared_cap(rc)), qn, cross) : -kInf;
        alloc_at(qq) = 0;
        ovf_at(qq) = 0;
    }
    if (tid < 64) ctl[tid] = tid == kCtlNext ? a.step_first + s * a.range_steps : 0;
    if (init_mine) {
        for (int e = tid; e < Qw * k; e += NT) {
            const int q = e / k;
            const int r = wg_row0 + q;
            if (r < a.rows) {
                const size_t at = ((size_t)r * S + s) * k + (e - q * k);
                a.lk[at] = kInf;
                a.li[at] = kNoIdx;
            }
        }
    }
    __syncthreads();

    // The range's steps are handed out one at a time (a counter in LDS): the waves of a SIMD do
    // not run at the same pace (the older wave of a pair is served first), and with fixed shares
    // the faster ones would stand idle at the end of the range.
    const int step_lo = a.step_first + s * a.range_steps;
    const int step_hi = min(step_lo + a.range_steps, a.step_end);
    auto take_step = [&]() {
        int v = 0;
        if (lane == 0) v = atomicAdd(ctl + kCtlNext, 1);
        return __builtin_amdgcn_readfirstlane(v);
    };
    u32x4 A[2][NCH];
    f32x16 XN[2];
    auto loadA = [&](int st) {
        const u32x4* p = reinterpret_cast<const u32x4*>(a.Xp) + (size_t)(st - a.step_slab0) * (2 * NCH * 64) + lane;
#pragma unroll
        for (int pb = 0; pb < 2; ++pb)
#pragma unroll
            for (int c = 0; c < NCH; ++c) A[pb][c] = p[(pb * NCH + c) * 64];
    };
    // the step's 64 norms, one per lane, into the accumulator layout: register e of a lane of
    // half h belongs to point row 8 (e / 4) + 4 h + e % 4 of its block
    float* const xs = xn_stage + wave * 64;
    // (the wave's LDS accesses execute in program order, so the reads below see the write
    // without a fence - and a fence would also wait for the A operands that are in flight)
    auto spread_xn = [&](float v) {
        __builtin_amdgcn_wave_barrier();
        xs[lane] = v;
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int pb = 0; pb < 2; ++pb)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const f32x4 t = *reinterpret_cast<const f32x4*>(xs + pb * 32 + g * 8 + h * 4);
                XN[pb][g * 4 + 0] = t[0];
                XN[pb][g * 4 + 1] = t[1];
                XN[pb][g * 4 + 2] = t[2];
                XN[pb][g * 4 + 3] = t[3];
            }
    };

    // Pairs of query q (this lane's, in set qs) under its threshold: nearly always one key of the
    // whole wave, so every accumulator register gets a vote, and a lane whose key passes takes a
    // slot of the query's buffer (a counter in LDS that all waves add to).  A pair that finds
    // the buffer full marks (wave, step parity) for the query: the stop then tests all 64 points
    // of that step for it and drops what the buffer already holds of them.
    auto append = [&](int q, float tq, const f32x16& a0, const f32x16& a1, const float (&g)[8], int st,
                      int parity) {
        bool call = false;
        const int jb = st * kPkStep + h * 4;
        auto one = [&](float key, int off) {
            if (__builtin_amdgcn_ballot_w64(key < tq) == 0) return;
            if (key < tq) {
                // (the index is formed here, behind a barrier to code motion: the 32 sums would
                // otherwise be kept in registers all through the search loop)
                int j = jb;
                asm volatile("" : "+v"(j));
                j += off;
                const int slot = atomicAdd(&alloc_at(q), 1);
                if (slot < C) cand[q * C + slot] = j;
                else atomicOr(&ovf_at(q), 1 << (wave * 2 + parity));
                call = call || slot >= C - kPkRoom;
            }
        };
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (__builtin_amdgcn_ballot_w64(g[u] < tq) == 0) continue;
#pragma unroll
            for (int e = 4 * u; e < 4 * u + 4; ++e) one(a0[e], (e >> 2) * 8 + (e & 3));
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (__builtin_amdgcn_ballot_w64(g[4 + u] < tq) == 0) continue;
#pragma unroll
            for (int e = 4 * u; e < 4 * u + 4; ++e) one(a1[e], 32 + (e >> 2) * 8 + (e & 3));
        }
        if (__builtin_amdgcn_ballot_w64(call) != 0 && lane == 0)
            __hip_atomic_store(ctl + kCtlStop, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    };

    // One query set against the wave's 64 points.
    auto body = [&](int qs, int st, int parity, int ln) {
        const int q = qs * 32 + (ln & 31);
        const float tq = tauf_at(q);
        const uint4* bq = Bq + (size_t)qs * (NCH * 64) + ln;
        f32x16 acc0, acc1;
        // the B operands are read AH chunks ahead of their use
        constexpr int AH = NCH < 4 ? NCH : 4;
        uint4 bw[AH];
#pragma unroll
        for (int c = 0; c < AH; ++c) bw[c] = bq[c * 64];
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const bf16x8 b = __builtin_bit_cast(bf16x8, bw[c % AH]);
            if (c + AH < NCH) bw[c % AH] = bq[(c + AH) * 64];
            acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, A[0][c]), b,
                                                           c == 0 ? XN[0] : acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, A[1][c]), b,
                                                           c == 0 ? XN[1] : acc1, 0, 0, 0);
        }
        // minima of the eight groups of four registers, then of all 32: the rare path below only
        // looks into groups that hold a key under some lane's threshold
        float g[8];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            g[u] = fminf(fminf(fminf(acc0[4 * u], acc0[4 * u + 1]), acc0[4 * u + 2]), acc0[4 * u + 3]);
            g[4 + u] = fminf(fminf(fminf(acc1[4 * u], acc1[4 * u + 1]), acc1[4 * u + 2]), acc1[4 * u + 3]);
        }
        const float m = fminf(fminf(fminf(fminf(g[0], g[1]), g[2]), fminf(fminf(g[3], g[4]), g[5])),
                              fminf(g[6], g[7]));
        if (__builtin_amdgcn_ballot_w64(m < tq) != 0) {
            append(q, tq, acc0, acc1, g, st, parity);
        }
    };

    // A stop: every wave of the workgroup is here, nobody appends.  The queries with enough
    // buffered pairs (everything: all that have any) and those with a step to make good are
    // dealt out over the waves; then every query's filter threshold is brought up to date.
    auto stop_work = [&](bool everything) {
        // The lane index is taken afresh here, in a form the compiler cannot move: everything a
        // stop derives from it (addresses, the sort network's lane tests) would otherwise be
        // computed once before the search loop and occupy some seventy registers all through it.
        int lane;
        asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(lane));
        const int tid = wave * 64 + lane;
        float* const my_scratch = scratch + (size_t)wave * (2 * kWave + 2 * k);
        if (tid == 0) ctl[kCtlStop] = 0;
        const int share = everything ? 1 : kPkShareMin;
        for (int qq = tid; qq < Qw; qq += NT)
            if (alloc_at(qq) >= share || ovf_at(qq) != 0) queue_l[atomicAdd(ctl + kCtlCount, 1)] = qq;
        __syncthreads();
        const int nq = ctl[kCtlCount];
        for (int e = wave; e < nq; e += kPkWaves) {
            const int q = __builtin_amdgcn_readfirstlane(queue_l[e]);
            const int r = wg_row0 + q;
            const size_t lb = ((size_t)r * S + s) * k;
            const int cc = min(C, __builtin_amdgcn_readfirstlane(alloc_at(q)));
            unsigned rem = (unsigned)__builtin_amdgcn_readfirstlane(ovf_at(q));
            unsigned t_bits = __float_as_uint(own_l[q]);
            float key_s = kInf;  // the list's key at position pos_s after the last merge
            bool merged = false;
            // work items: the buffer, then the two row blocks of every step to make good
            // what the buffer holds of a step that is made good in full is dropped (-1: no pair)
            if (rem != 0 && lane < cc) {
                const int j = cand[q * C + lane];
                bool drop = false;
                for (unsigned bits = rem; bits != 0; bits &= bits - 1)
                    drop = drop || (j >> 6) == ctl[__builtin_ctz(bits)];
                if (drop) cand[q * C + lane] = -1;
            }
            int item = 0, half = 0;
            for (;;) {
                const int* cbuf = cand + q * C;
                int jb = 0, n_c = cc;
                if (item != 0) {
                    if (rem == 0) break;
                    const int bit = __builtin_ctz(rem);
                    const int stv = __builtin_amdgcn_readfirstlane(ctl[bit]);
                    cbuf = nullptr;
                    jb = stv * kPkStep + half * 32;
                    n_c = min(32, a.n - jb);
                    if (half == 1) rem &= rem - 1;
                    half ^= 1;
                }
                ++item;
                if (n_c > 0) {
                    t_bits = flush_query_exact<ALIGNED, 8, true>(a.Q + (int64_t)r * a.ldq, a.X, a.ldx, a.d,
                                                           a.j_valid, cbuf, jb, n_c, a.lk + lb, a.li + lb,
                                                           k, my_scratch, a.tsh + r, COS ? a.rn : nullptr, lane, pos_s,
                                                           &key_s);
                    merged = true;
                }
            }
            if (lane == 0) {
                own_l[q] = __uint_as_float(t_bits);
                alloc_at(q) = 0;
                ovf_at(q) = 0;
                if (merged)
                    __hip_atomic_store(a.tsr + (size_t)r * S + s, key_word(key_s), __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        __syncthreads();
        if (tid == 0) ctl[kCtlCount] = 0;
        for (int qq = tid; qq < Qw; qq += NT)
            if (wg_row0 + qq < a.rows)
                tauf_at(qq) = key_bound(fminf(own_l[qq], shared_cap(wg_row0 + qq)), qn_l[qq], cross_l[qq]);
        __syncthreads();
    };

    // A step's A operands and norms are requested when the step begins and are live within it
    // only: the SIMD's other wave has work meanwhile, and registers that carry operands from one
    // iteration of the loop into the next get copies of their own from the compiler (requesting
    // the next step's operands during the last set costs 64 - 128 registers that way and gained
    // nothing measurable at d = 128; at d = 256 it does not fit two waves per SIMD at all).
    // Nothing of them is live across a stop either.
    const int step_any = a.step_first;
    int step = take_step();
    bool have = step < step_hi;
    float xn_next = a.xn[(size_t)(have ? step : step_any) * kPkStep + lane];
    int parity = 0;
    bool announced = false;
    for (;;) {
        if (have) {
            loadA(step);
            spread_xn(xn_next);
            if (lane == 0) ctl[wave * 2 + parity] = step;
            const int taken = take_step();
            const bool has_next = taken < step_hi;
            const int nstep = has_next ? taken : step;
            // (the lane index through an empty asm: the addresses that depend on it are then formed
            // here, step by step, instead of being kept in registers from before the loop)
            int ln = lane;
            asm volatile("" : "+v"(ln));
            xn_next = (a.xn + (size_t)nstep * kPkStep)[(unsigned)ln];
            for (int qs = 0; qs < sets; ++qs) body(qs, step, parity, ln);
            const int stop = __builtin_amdgcn_readfirstlane(
                __hip_atomic_load(ctl + kCtlStop, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
            step = nstep;
            have = has_next;
            parity ^= 1;
            if (stop == 0) continue;
        } else if (!announced) {
            if (lane == 0) atomicAdd(ctl + kCtlDone, 1);
            announced = true;
        }
        __syncthreads();
        const bool all_done = ctl[kCtlDone] == kPkWaves;
        stop_work(all_done);
        if (all_done) break;
    }
}

}  // namespace

hipError_t launch_pack_operands(const float* X, int64_t ldx, int64_t n, int d, int64_t j_first,
                                int64_t points, void* xp, hipStream_t stream, float scale, float* xn,
                                void* hdr, const float* row_scale) {
    const int nch = pk_padded_chunks(d);
    const bool aligned = (reinterpret_cast<uintptr_t>(X) % 16 == 0) && (ldx % 4 == 0) && (d % 4 == 0);
    if ((xn || row_scale) && (!aligned || !hdr)) return hipErrorInvalidValue;
    if (aligned) {
        const int nblocks = (int)(points / 32);
        const dim3 grid((unsigned)(nblocks < 16384 ? nblocks : 16384));
        if (xn || row_scale)
            knn_pack_block_kernel<true><<<grid, dim3(256), 0, stream>>>(X, ldx, (int)n, d, nch, (int)j_first, nblocks,
                                                                         scale, row_scale, static_cast<uint4*>(xp),
                                                                         xn, static_cast<unsigned*>(hdr));
        else
            knn_pack_block_kernel<false><<<grid, dim3(256), 0, stream>>>(X, ldx, (int)n, d, nch, (int)j_first,
                                                                          nblocks, scale, nullptr,
                                                                          static_cast<uint4*>(xp), nullptr, nullptr);
        return hipGetLastError();
    }
    const int64_t pieces = points * nch * 2;
    const dim3 grid((unsigned)((pieces + 255) / 256));
    knn_pack_operands_kernel<<<grid, dim3(256), 0, stream>>>(X, ldx, (int)n, d, nch, (int)j_first,
                                                                    pieces, scale, static_cast<uint4*>(xp));
    return hipGetLastError();
}

hipError_t launch_seed_thresholds(const float* Q, int64_t ldq, const void* xp, const float* xn, const void* qs,
                                  const float* qn, void* tsh, const void* hdr, int64_t rows, int64_t n, int d,
                                  int k, int64_t seed_points, hipStream_t stream, bool cosine) {
    const int nch_real = (d + kSpKC - 1) / kSpKC;
    const int nch = pk_padded_chunks(d);
    const int nsteps = (int)((n + kPkStep - 1) / kPkStep);
    int sample_steps = (int)(seed_points / kPkStep);
    if (sample_steps > nsteps) sample_steps = nsteps;
    if (sample_steps < 1 || (int64_t)sample_steps * kPkStep < k) return hipErrorInvalidValue;
    const dim3 grid((unsigned)((rows + 32 * kSeedSets - 1) / (32 * kSeedSets)));
#define KNN_SEED_LAUNCH(N)                                                                          \
    knn_seed_kernel<N><<<grid, dim3(256), 0, stream>>>(                                             \
        static_cast<const uint4*>(xp), xn, static_cast<const uint4*>(qs), qn,                       \
        static_cast<const unsigned*>(hdr), Q, ldq, static_cast<unsigned*>(tsh), (int)rows, d, nch_real, k, \
        nsteps, sample_steps, cosine ? 1 : 0)
    switch (nch) {
        case 1: KNN_SEED_LAUNCH(1); break;
        case 2: KNN_SEED_LAUNCH(2); break;
        case 3: KNN_SEED_LAUNCH(3); break;
        case 4: KNN_SEED_LAUNCH(4); break;
        case 5: KNN_SEED_LAUNCH(5); break;
        case 6: KNN_SEED_LAUNCH(6); break;
        case 7: KNN_SEED_LAUNCH(7); break;
        case 8: KNN_SEED_LAUNCH(8); break;
        case 10: KNN_SEED_LAUNCH(10); break;
        case 12: KNN_SEED_LAUNCH(12); break;
        case 14: KNN_SEED_LAUNCH(14); break;
        case 16: KNN_SEED_LAUNCH(16); break;
        default: return hipErrorInvalidValue;
    }
#undef KNN_SEED_LAUNCH
    return hipGetLastError();
}

hipError_t launch_pad_norms(float* xn, int64_t n, hipStream_t stream) {
    const int64_t n_pad = (n + kPkStep - 1) / kPkStep * kPkStep;
    if (n_pad > n) knn_pad_norms_kernel<<<dim3(1), dim3(64), 0, stream>>>(xn, (int)n, (int)n_pad);
    return hipGetLastError();
}

bool packed_rows_aligned(const float* Q, int64_t ldq, const float* X, int64_t ldx, int d) {
    return (reinterpret_cast<uintptr_t>(Q) % 16 == 0) && (reinterpret_cast<uintptr_t>(X) % 16 == 0) &&
           (ldq % 4 == 0) && (ldx % 4 == 0) && (d % 4 == 0);
}

hipError_t launch_packed(const float* Q, int64_t ldq, const float* X, int64_t ldx, const void* xp,
                         int64_t slab_first, const void* qs, const float* qn, void* tsh, void* tsr,
                         const float* xn, const void* hdr, int64_t rows, int64_t n, int d, int k, int S,
                         int sets, int64_t j_first, int64_t j_end, int init_from, float* lk, int* li,
                         hipStream_t stream, const float* rn) {
    const int nch_real = (d + kSpKC - 1) / kSpKC;
    const int nch = pk_padded_chunks(d);
    if (d > kPkMaxD || sets < 1 || sets > pk_max_sets(nch, k) || !packed_rows_aligned(Q, ldq, X, ldx, d) ||
        j_first % kPkStep != 0 || slab_first % kPkStep != 0 || j_first < slab_first || j_end <= j_first ||
        j_end > n)
        return hipErrorInvalidValue;
    PkArgs a;
    a.Q = Q;
    a.ldq = ldq;
    a.X = X;
    a.ldx = ldx;
    a.Xp = static_cast<const uint4*>(xp);
    a.xn = xn;
    a.rn = rn;
    a.Qs = static_cast<const uint4*>(qs);
    a.qnorm = qn;
    a.tsh = static_cast<unsigned*>(tsh);
    a.tsr = static_cast<unsigned*>(tsr);
    a.hdr = static_cast<const unsigned*>(hdr);
    a.lk = lk;
    a.li = li;
    a.rows = (int)rows;
    a.n = (int)n;
    a.d = d;
    a.nch_real = nch_real;
    a.k = k;
    a.S = S;
    a.sets = sets;
    a.tiles = (int)((rows + sets * 32 - 1) / (sets * 32));
    a.step_slab0 = (int)(slab_first / kPkStep);
    a.step_first = (int)(j_first / kPkStep);
    a.step_end = (int)((j_end + kPkStep - 1) / kPkStep);
    // ranges of a multiple of eight steps
    const int steps = a.step_end - a.step_first;
    int per = (steps + S - 1) / S;
    per = (per + 7) / 8 * 8;
    a.range_steps = per;
    a.init_from = init_from;
    a.j_valid = (int)j_first;
    const size_t lds = (size_t)pk_lds_bytes(nch, k, sets);
    const dim3 grid((unsigned)(a.tiles * S));
    const int waves = pk_waves(nch, k);
#define KNN_PACKED_LAUNCH_W(N, W)                                                              \
    do {                                                                                       \
        if (rn) {                                                                              \
            hipError_t e2 = raise_lds_limit(knn_packed_kernel<N, true, W, true>, lds);         \
            if (e2 != hipSuccess) return e2;                                                   \
            knn_packed_kernel<N, true, W, true><<<grid, dim3(64 * W), lds, stream>>>(a);       \
        } else {                                                                               \
            hipError_t e2 = raise_lds_limit(knn_packed_kernel<N, true, W, false>, lds);        \
            if (e2 != hipSuccess) return e2;                                                   \
            knn_packed_kernel<N, true, W, false><<<grid, dim3(64 * W), lds, stream>>>(a);      \
        }                                                                                      \
    } while (0)
#define KNN_PACKED_LAUNCH(N)                                                                   \
    do {                                                                                       \
        if (waves == 12) KNN_PACKED_LAUNCH_W(N, 12);                                           \
        else KNN_PACKED_LAUNCH_W(N, 8);                                                        \
    } while (0)
    switch (nch) {
        case 1: KNN_PACKED_LAUNCH(1); break;
        case 2: KNN_PACKED_LAUNCH(2); break;
        case 3: KNN_PACKED_LAUNCH(3); break;
        case 4: KNN_PACKED_LAUNCH(4); break;
        case 5: KNN_PACKED_LAUNCH(5); break;
        case 6: KNN_PACKED_LAUNCH(6); break;
        case 7: KNN_PACKED_LAUNCH(7); break;
        case 8: KNN_PACKED_LAUNCH(8); break;
        case 10: KNN_PACKED_LAUNCH_W(10, 8); break;
        case 12: KNN_PACKED_LAUNCH_W(12, 8); break;
        case 14: KNN_PACKED_LAUNCH_W(14, 8); break;
        case 16: KNN_PACKED_LAUNCH_W(16, 8); break;
        default: return hipErrorInvalidValue;
    }
#undef KNN_PACKED_LAUNCH_W
#undef KNN_PACKED_LAUNCH
    return hipGetLastError();
}

}  // namespace knn
