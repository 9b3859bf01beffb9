// gfx950 (CDNA4, MI355X) kNN search for d > 256 and many points, squared-Euclidean metric: the
// bf16 matrix-core filter of knn_split.hip on tiles of 512 queries x 128 points, both operands
// rounded to bf16 once and kept in the workspace in the order of the MFMA's operands.
//
// The expansion sum x^2 - 2 q.x of paper section 4.1 runs on the rounded values and only
// filters; what passes is evaluated exactly (knn_exact.h) and merged into the query's list, so
// the distance tile never leaves the registers (section 4.3) and the results do not depend on
// the filter.  With hundreds of coordinates neither operand of a tile fits registers or LDS for
// the whole contraction, so both are streamed chunk by chunk (16 coordinates), and what a
// workgroup fetches per pair falls with the size of its tile:
//   - a workgroup of 8 waves holds 512 x 128 accumulators (a wave: two sets of 32 queries against
//     four row blocks of 32 points, 128 registers), twice the queries of knn_split_kernel, so the
//     point stream - the part that comes from HBM - is read half as often, and as bf16 it is half
//     as long;
//   - the points of a stage (two chunks) go through LDS, fetched as 1 KB operands by one wave
//     each and read by all eight; a wave's own B operands come straight from the packed copy of
//     the queries into registers (they stay in the L2: a few query tiles per XCD), a stage ahead;
//   - one 1 KB LDS read feeds two MFMAs, one workgroup barrier per stage of 16 MFMAs a wave.
// List maintenance is that of knn_split_kernel (per-query candidate buffers in LDS, the workgroup
// stops between two tiles when a buffer runs full and deals the queries out over its waves), with
// two additions: the point ranges of a query bound each other through the key at position
// ceil(k / S) - 1 of their lists (as in knn_packed.hip), and a list that knows no bound yet takes
// one from the filter keys of its first tile instead of evaluating all of that tile exactly.
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

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

struct WdArgs {
    const float* Q;
    int64_t ldq;
    const float* X;
    int64_t ldx;
    const u32x4* Xp;      // packed points of the slab: [step of 64][row block][chunk][lane] 16 B
    const float* xn;      // squared norms of all points
    const u32x4* Qp;      // packed B operands bf16(-2 q) of the chunk's queries: [set of 32][chunk][lane]
    const float* qnorm;   // their squared norms
    unsigned* tsh;        // [rows] lowest upper bound of the query's k-th key anybody has published
    unsigned* tsr;        // [rows][S] key at position ceil(k / S) - 1 of each range's list
    const unsigned* hdr;  // word 0: max of xn, word 1: largest squared bf16 residual norm of a point
    float* lk;
    int* li;
    int rows, n, d, nch, k, S, tiles;
    int qsets;            // sets of 32 rows the packed queries hold
    int j_slab0;          // first point of the packed copy
    int slab_steps;       // steps of 64 points it holds
    int j_first, j_end;   // points this launch covers
    int range_len;        // points per range (a multiple of 128)
    int init_from;        // the lists of ranges >= this start empty, the others continue
    int q_stage;          // 1: the LDS has room for one query row per wave (the stops' exact keys read it there)
};

__global__ __launch_bounds__(64 * kWdWaves, 1) void knn_wide_kernel(const WdArgs a) {
    constexpr int TQ = kWdTileQ, TX = kWdTileX, C = kWdCand, W = kWdW, NT = kWdSets;
    static_assert(4 * W == kWdWaves, "one A operand per wave and stage");
    extern __shared__ __align__(16) unsigned char smem[];
    u32x4* const as = reinterpret_cast<u32x4*>(smem);                 // [2 buffers][W][4 row blocks][64]
    float* const xns = reinterpret_cast<float*>(as + 2 * W * 4 * 64);  // [2][TX] accumulator start values
    int* const ci = reinterpret_cast<int*>(xns + 2 * TX);             // [TQ][C] buffered point indices
    float* const qn_l = reinterpret_cast<float*>(ci + TQ * C);        // [TQ] squared norms of the queries
    float* const cross_l = qn_l + TQ;   // [TQ] allowance for the rounded operands
    float* const own_l = cross_l + TQ;  // [TQ] k-th key of the query's list in this range
    float* const cap_l = own_l + TQ;    // [TQ] lowest bound of the query's k-th key seen in tsh
    float* const fbest_l = cap_l + TQ;  // [TQ] smallest filter key the query has met in this range
    int* const co_cnt = reinterpret_cast<int*>(fbest_l + TQ);  // [TQ] what a stop has to do for the query
    int* const co_queue = co_cnt + TQ;                       // [TQ]
    int* const co_n = co_queue + TQ;                         // [1]
    int* const co_stop = co_n + 1;                           // [3]
    float* const scratch0 = reinterpret_cast<float*>(co_n + 16);  // [waves][2 * 64 + 2 k]
    // [waves][d] the row of the query a wave is evaluating at a stop (a.q_stage)
    float* const qstage0 = scratch0 + (size_t)kWdWaves * (2 * kWave + 2 * a.k);
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i32 = lane & 31;
    const int h = lane >> 5;
    const int k = a.k, S = a.S;
    // Workgroups go to the eight XCDs in turn.  The (query tile, range) pairs, tile by tile, are
    // dealt out in eight runs, one per XCD, so that the workgroups sharing an L2 work on as few
    // query tiles as possible: the tiles' B operands (re-read for every 128 points) then stay there.
    int s, wg_row0;
    {
        const int total_wgs = a.tiles * S, xcd = blockIdx.x & 7;
        const int pair = xcd * (total_wgs >> 3) + min(xcd, total_wgs & 7) + (blockIdx.x >> 3);
        const int qt = pair / S;
        s = pair - qt * S;
        wg_row0 = qt * TQ;
    }
    const int wave_q0 = wave * (32 * NT);  // the wave's first query within the workgroup
    const int wave_row0 = wg_row0 + wave_q0;

    const int j0 = a.j_first + s * a.range_len;
    const int j1 = min(a.j_end, j0 + a.range_len);
    const int ntiles = j1 > j0 ? (j1 - j0 + TX - 1) / TX : 0;
    const int nst = a.nch / W;
    const int pos_s = (k + S - 1) / S - 1;

    // lists: empty, or continued from an earlier launch over other points
    const bool init_mine = s >= a.init_from;
    if (init_mine) {
#pragma unroll
        for (int t = 0; t < NT; ++t) init_lists32(a.lk, a.li, wave_row0 + 32 * t, a.rows, S, s, k, lane);
    }
    if (tid < 4) co_n[tid] = 0;  // (a barrier follows before the first use)

    // The filter bound, as in knn_split_kernel: dd <= tau implies key < (tau - qn) + slack with
    //   rounded operands    |x~| |q~' - q'| + |x~ - x| |q'|  (q' = -2 q) by Cauchy-Schwarz, from the
    //                       query's residual norm (taken below) and the largest residual norm of
    //                       a point (header word 1), 1 % on top for the fp32 arithmetic of these norms
    //   fp32 accumulations   one per coordinate (padded), of terms that sum to at most 2.02 |x| |q|
    //   roundings of xn, qn, dd   each below (d / 64 + 8) ulps of the value
    const float xmax = __uint_as_float(a.hdr[0]);
    const float e_sum = (float)(a.d + 16) * 0x1p-23f;
    auto key_bound = [&](float tau, float qn, float cross) {
        return (tau - qn) + (cross + e_sum * (xmax + qn + tau) + 0x1p-126f);
    };
    // Per lane and query set only the filter threshold and the fill of the query's buffer stay in
    // registers; what they follow from sits in LDS (both halves of a wave hold the same values).
    float tauf[NT];
    int cnt[NT];
    int ovf = 0;  // bit t: the buffer of the lane's query in set t could not take a tile's candidates
    {
        const float rxm = sqrtf(__uint_as_float(a.hdr[1]));
        const float e_acc = (float)(4 * (a.nch * 16) + 32) * 0x1p-24f;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int q = wave_q0 + 32 * t + i32;
            const int r = wg_row0 + q;
            const bool active = r < a.rows;
            const int rc = active ? r : a.rows - 1;
            const float qn = a.qnorm[rc];
            // |bf16(-2 q) - (-2 q)|^2 of the lane's query: the two halves of the wave share the sum
            const float* qrp = a.Q + (int64_t)rc * a.ldq;
            float rq2 = 0.f;
            for (int g = h; 4 * g < a.d; g += 2) {  // rows are 16-byte aligned, d % 4 == 0
                const f32x4 v = *reinterpret_cast<const f32x4*>(qrp + 4 * g);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float res = bf16_residual(-2.f * v[e]);
                    rq2 = fmaf(res, res, rq2);
                }
            }
            rq2 += lane_xor<32>(rq2);
            const float cross = 1.01f * ((sqrtf(xmax) + rxm) * sqrtf(rq2) + rxm * 2.f * sqrtf(qn)) +
                                e_acc * sqrtf(xmax * qn);
            float own = active ? kInf : -kInf;  // a row past the chunk: nothing passes
            if (active && !init_mine) {
                const size_t lb = ((size_t)r * S + s) * k;
                own = a.lk[lb + (k - 1)];
                if (h == 0) atomicMin(a.tsr + (size_t)r * S + s, key_word(a.lk[lb + pos_s]));
            }
            const float cap =
                word_key(__hip_atomic_load(a.tsh + rc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
            if (h == 0) {
                qn_l[q] = qn;
                cross_l[q] = cross;
                own_l[q] = own;
                cap_l[q] = cap;
                fbest_l[q] = kInf;
            }
            tauf[t] = key_bound(fminf(own, cap), qn, cross);
            cnt[t] = 0;
        }
    }

    // Row indices for the rare paths are passed through this: addresses formed from them are then
    // computed where they are used instead of once before the search loop, where each would
    // occupy two registers all through it.
    auto here = [](int v) {
        asm volatile("" : "+v"(v));
        return v;
    };
    // An upper bound of a pair's exact key from its filter key fk: the allowance of the filter with
    // the bound itself in place of tau in the rounding term and that term doubled (the filter key
    // may be off in either direction).
    auto exact_bound = [&](float fk, float qn, float cross) {
        const float base = fk + qn;
        return base + (cross + 2.f * e_sum * (xmax + qn + fabsf(base) + cross) + 0x1p-126f);
    };
    // What the S ranges of query r know together.  Range s' publishes in tsr an upper bound b_s' of
    // the key at position pos_s of its list - pos_s + 1 of its points lie at or below it - and the
    // ranges hold different points, so with need = ceil(k / (pos_s + 1)) <= S the need-th smallest
    // of the S values has at least k points at or below it: an upper bound of the k-th smallest
    // key over all points, as tight as one list over everything the ranges have seen would give
    // (a range finds its (k / S)-th best where the whole stream's k-th best lies).  The whole
    // wave calls this; `mine` is this range's own value; +inf: not enough ranges have published.
    const int need_s = (k + pos_s) / (pos_s + 1);
    auto union_bound = [&](int r, float mine, int ln) {
        float v = kInf;
        if (ln < S) {
            v = word_key(__hip_atomic_load(a.tsr + (size_t)r * S + ln, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
            if (ln == s) v = fminf(v, mine);
        }
        int rank = 0;
        for (int t2 = 0; t2 < S; ++t2) {
            const float o = __shfl(v, t2);
            rank += (o < v || (o == v && t2 < ln)) ? 1 : 0;
        }
        const uint64_t hit = __builtin_amdgcn_ballot_w64(ln < S && rank == need_s - 1);
        return __shfl(v, __builtin_ctzll(hit | (1ull << 63)));  // (lane 63 holds +inf unless S = 64)
    };

    // The same per lane, for the periodic look at the other ranges between stops: the need-th
    // smallest of S values is the (S - need + 1)-th largest, found by keeping the four largest
    // (shapes that would need more keep to the stops' refresh).
    const int m_top = S - need_s + 1;
    auto union_bound_lane = [&](int r) {
        float t1 = -kInf, t2 = -kInf, t3 = -kInf, t4 = -kInf;
        const unsigned* p = a.tsr + (size_t)r * S;
        for (int s2 = 0; s2 < S; s2 += 4) {
            float v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float w =
                    word_key(__hip_atomic_load(p + min(s2 + i, S - 1), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
                v[i] = s2 + i < S ? w : -kInf;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float c = v[i], n;
                n = fmaxf(t1, c); c = fminf(t1, c); t1 = n;
                n = fmaxf(t2, c); c = fminf(t2, c); t2 = n;
                n = fmaxf(t3, c); c = fminf(t3, c); t3 = n;
                t4 = fmaxf(t4, c);
            }
        }
        return m_top == 1 ? t1 : m_top == 2 ? t2 : m_top == 3 ? t3 : t4;
    };

    // ---- the stop: between two tiles, accumulators dead, every wave of the workgroup here ----
    // Queries with at least `share` buffered pairs (everything: any) and those whose buffer
    // overflowed in the tile that just ended are dealt out over the eight waves: exact keys of
    // the buffered pairs, for an overflowed query then of all points of the tile (what the
    // buffer took of that tile was dropped again), merged into the list; the range's new key at
    // position pos_s goes to tsr, and the bound that follows from all ranges' values there
    // (union_bound) to tsh.
    auto stop_work = [&](int tile_base, bool everything) __attribute__((always_inline)) {
        // The lane index is taken afresh here, in a form the compiler cannot move: what a stop
        // derives from it would otherwise be computed before the search loop and occupy
        // registers all through it.
        int ln;
        asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(ln));
        float* const my_scratch = scratch0 + (size_t)wave * (2 * kWave + 2 * k);
        const int share = everything ? 1 : kWdShareMin;
        if ((ln >> 5) == 0) {
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const int q = wave_q0 + 32 * t + (ln & 31);
                const int o = (ovf >> t) & 1;
                co_cnt[q] = cnt[t] | (o << 8);
                if (cnt[t] >= share || o) co_queue[atomicAdd(co_n, 1)] = q;
            }
        }
        __syncthreads();
        const int nq = *co_n;
        for (int e = wave; e < nq; e += kWdWaves) {
            const int q = __builtin_amdgcn_readfirstlane(co_queue[e]);
            const int r = wg_row0 + q;
            const size_t lb = ((size_t)r * S + s) * k;
            const int v = __builtin_amdgcn_readfirstlane(co_cnt[q]);
            const int cc = v & 255;
            const bool o = (v >> 8) != 0;
            unsigned t_bits = 0;
            float key_s = kInf;
            bool merged = false;
            // An exact key is a chain of round trips, one per U groups of four coordinates of the
            // candidates' rows (98 groups a lane at d = 784), and the query's row would take half
            // of the registers that are in flight: staged in LDS (behind the first trip's
            // requests, knn_exact.h) it leaves them all to the candidates - sixteen groups a trip
            // instead of eight, the same sums.
            const float* qrow = a.Q + (int64_t)r * a.ldq;
            float* const qst = qstage0 + (size_t)wave * a.d;
            for (int item = 0; item < (o ? 5 : 1); ++item) {
                const int* cbuf = item == 0 ? ci + q * C : nullptr;
                const int jb = tile_base + 32 * (item - 1);
                const int n_c = item == 0 ? cc : min(32, j1 - jb);
                if (n_c > 0) {
                    if (a.q_stage)
                        t_bits = flush_query_exact<true, 16, true, 2>(qrow, a.X, a.ldx, a.d, j0, cbuf, jb, n_c,
                                                                      a.lk + lb, a.li + lb, k, my_scratch,
                                                                      a.tsh + r, nullptr, ln, pos_s, &key_s, qst);
                    else
                        t_bits = flush_query_exact<true, 8, true>(qrow, a.X, a.ldx, a.d, j0, cbuf, jb, n_c,
                                                                  a.lk + lb, a.li + lb, k, my_scratch, a.tsh + r,
                                                                  nullptr, ln, pos_s, &key_s);
                    merged = true;
                }
            }
            if (merged) {
                if (ln == 0) {
                    own_l[q] = __uint_as_float(t_bits);
                    atomicMin(a.tsr + (size_t)r * S + s, key_word(key_s));
                }
                const float m = union_bound(r, key_s, ln);
                if (ln == 0 && m < kInf) atomicMin(a.tsh + r, key_word(m));
            }
        }
        __syncthreads();
        if (wave == 0 && ln == 0) *co_n = 0;  // the next use is behind the barrier that ends a tile
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int q = wave_q0 + 32 * t + (ln & 31);
            if (cnt[t] >= share || ((ovf >> t) & 1)) cnt[t] = 0;
            const int rc = min(wg_row0 + q, a.rows - 1);
            const float cap = fminf(cap_l[q], word_key(__hip_atomic_load(a.tsh + rc, __ATOMIC_RELAXED,
                                                                        __HIP_MEMORY_SCOPE_AGENT)));
            if ((ln >> 5) == 0) cap_l[q] = cap;
            tauf[t] = key_bound(fminf(own_l[q], cap), qn_l[q], cross_l[q]);
        }
        ovf = 0;
    };

    // A query that knows no bound yet (empty list, nothing published) takes one from the filter
    // keys of the tile in the accumulators: if at least k of them are <= f, at least k points have
    // exact keys <= f + qn + allowance - an upper bound of the k-th smallest, as good a threshold
    // as one from a full list.  f is narrowed by quartering [lowest, highest finite key] five
    // times while keeping count(<= upper end) >= k; the two halves of the wave hold 64 keys each.
    // The same search for pos_s + 1 keys gives the value this range publishes in tsr until its
    // list has entries.
    auto seed_from_tile = [&](int t, const f32x16 (&acc)[4]) {
        // (counts are kept as floats: their additions are not reassociated, so the compiler
        // forms one short chain per count instead of a tree over 64 compare results at a time)
        float lo = kInf, hi = -kInf, nv = 0.f;
#pragma unroll
        for (int pb = 0; pb < 4; ++pb)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const float v = acc[pb][e];
                const bool fin = v < kInf;  // (rows past the range start from +inf)
                lo = fminf(lo, v);
                hi = fmaxf(hi, fin ? v : -kInf);
                nv += fin ? 1.f : 0.f;
            }
        lo = fminf(lo, lane_xor<32>(lo));
        hi = fmaxf(hi, lane_xor<32>(hi));
        nv += lane_xor<32>(nv);
        const float kf = (float)k;
        const float lo0 = lo, hi0 = hi;
        float f[2];  // f[0]: at least k keys are <= it; f[1]: at least pos_s + 1 keys are
#pragma nounroll
        for (int which = 0; which < 2; ++which) {
            const float want = which == 0 ? kf : (float)(pos_s + 1);
            lo = lo0;
            hi = hi0;
#pragma nounroll
            for (int it = 0; it < 5; ++it) {
                const float q1 = lo + 0.25f * (hi - lo), q2 = lo + 0.5f * (hi - lo), q3 = lo + 0.75f * (hi - lo);
                float c1 = 0.f, c2 = 0.f, c3 = 0.f;
#pragma unroll
                for (int pb = 0; pb < 4; ++pb)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const float v = acc[pb][e];
                        c1 += (v <= q1) ? 1.f : 0.f;
                        c2 += (v <= q2) ? 1.f : 0.f;
                        c3 += (v <= q3) ? 1.f : 0.f;
                    }
                c1 += lane_xor<32>(c1);
                c2 += lane_xor<32>(c2);
                c3 += lane_xor<32>(c3);
                if (c1 >= want) hi = q1;
                else if (c2 >= want) { lo = q1; hi = q2; }
                else if (c3 >= want) { lo = q2; hi = q3; }
                else lo = q3;
            }
            f[which] = hi;
        }
        if (pos_s == 0) f[1] = lo0;  // (the tile's smallest key itself)
        const int q = wave_q0 + 32 * t + i32;
        const float qn = qn_l[q], cross = cross_l[q];
        const float bound = exact_bound(f[0], qn, cross);
        if (tauf[t] == kInf && nv >= kf && bound < kInf) {
            if (h == 0) {
                const int r = here(wg_row0 + q);  // (tauf == +inf: the lane holds a query)
                cap_l[q] = bound;
                atomicMin(a.tsh + r, key_word(bound));
                // and what the other ranges may count on: pos_s + 1 points of this range at or below
                atomicMin(a.tsr + (size_t)r * S + s, key_word(exact_bound(f[1], qn, cross)));
            }
            tauf[t] = key_bound(bound, qn, cross);
        }
    };

    // End of a tile, accumulators live: keys below the filter threshold are buffered (point
    // index only; the two halves of the wave take consecutive slots).  Register e of a lane of
    // half h holds point row 8 (e / 4) + 4 h + e % 4 of its block.
    auto epilogue = [&](int t, const f32x16 (&acc)[4], int tile_base) {
        float mb[4];
#pragma unroll
        for (int pb = 0; pb < 4; ++pb) {
            mb[pb] = acc[pb][0];
#pragma unroll
            for (int e = 1; e < 16; ++e) mb[pb] = fminf(mb[pb], acc[pb][e]);
        }
        if (__builtin_amdgcn_ballot_w64(fminf(fminf(mb[0], mb[1]), fminf(mb[2], mb[3])) < tauf[t]) == 0) return;
        if (__builtin_amdgcn_ballot_w64(tauf[t] == kInf) != 0) seed_from_tile(t, acc);
        if (pos_s == 0) {
            // Ranges that publish the bound of their BEST key (k <= S): a smaller filter key than any
            // before bounds it anew, without waiting for the pair's exact evaluation.
            float tm = fminf(fminf(mb[0], mb[1]), fminf(mb[2], mb[3]));
            tm = fminf(tm, lane_xor<32>(tm));
            const int q = wave_q0 + 32 * t + i32;
            if (h == 0 && tm < fbest_l[q]) {
                fbest_l[q] = tm;
                atomicMin(a.tsr + (size_t)here(min(wg_row0 + q, a.rows - 1)) * S + s,
                          key_word(exact_bound(tm, qn_l[q], cross_l[q])));
            }
        }
        int* const wci = ci + (wave_q0 + 32 * t) * C;
        // (formed here, behind a barrier to code motion: the compiler would otherwise keep the
        // sums of h * 4 and the 64 row offsets in registers all through the search loop)
        int jb = tile_base + h * 4;
        asm volatile("" : "+v"(jb));
        const int cnt0 = cnt[t];
        bool over = false;
#pragma unroll
        for (int pb = 0; pb < 4; ++pb) {
            if (__builtin_amdgcn_ballot_w64(mb[pb] < tauf[t]) == 0) continue;
            int mine = 0;
#pragma unroll
            for (int e = 0; e < 16; ++e) mine += (acc[pb][e] < tauf[t]) ? 1 : 0;
            const int oth = lane_xor<32>(mine);
            if (cnt[t] + mine + oth > C) over = true;  // the same in both halves of the wave
            if (!over) {
                int slot = i32 * C + cnt[t] + (h ? oth : 0);
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    if (acc[pb][e] < tauf[t]) {
                        wci[slot] = jb + (pb * 32 + (e >> 2) * 8 + (e & 3));
                        ++slot;
                    }
                }
                cnt[t] += mine + oth;
            }
        }
        if (over) {
            cnt[t] = cnt0;
            ovf |= 1 << t;
        }
    };

    // ---- the stream: a stage covers W chunks; wave w fetches operand (row block w & 3, chunk
    // w >> 2) of it, two stages ahead, and writes it to LDS one stage ahead ----
    const int step0 = (j0 - a.j_slab0) / kPkStep;
    const int rb = wave & 3, kk_mine = wave >> 2;
    int f_tile = 0, f_c = 0;  // (tile, stage) of the next fetch
    struct XS {
        u32x4 x;
        float xnv;
    };
    struct QB {
        u32x4 b[W][NT];
    };
    auto fetchX = [&](XS& g) {
        // (a tile's second step may lie past the copy: any valid operand will do, its rows carry +inf)
        const int st = min(step0 + 2 * f_tile + (rb >> 1), a.slab_steps - 1);
        g.x = a.Xp[((size_t)(st * 2 + (rb & 1)) * a.nch + f_c * W + kk_mine) * 64 + lane];
        if (f_c == 0) g.xnv = a.xn[min(j0 + f_tile * TX + (tid & (TX - 1)), j1 - 1)];
        if (++f_c == nst) {
            f_c = 0;
            if (f_tile + 1 < ntiles) ++f_tile;
        }
    };
    int s_tile = 0, s_c = 0;  // (tile, stage) of the next stash
    auto stash = [&](int buf, const XS& g) {
        as[((buf * W + kk_mine) * 4 + rb) * 64 + lane] = g.x;
        if (s_c == 0 && tid < TX)  // +inf past the range: such a row never passes
            xns[(s_tile & 1) * TX + tid] = j0 + s_tile * TX + tid < j1 ? g.xnv : kInf;
        if (++s_c == nst) {
            s_c = 0;
            ++s_tile;
        }
    };
    // (sets past the packed queries - a last, partly filled tile - read the last set: their lanes
    // hold no query)
    const u32x4* qb[NT];  // (uniform: the lane is added as a 32-bit offset at the loads)
#pragma unroll
    for (int t = 0; t < NT; ++t) qb[t] = a.Qp + (size_t)min(wave_row0 / 32 + t, a.qsets - 1) * a.nch * 64;
    auto fetchQ = [&](int c, QB& g) {
#pragma unroll
        for (int kk = 0; kk < W; ++kk)
#pragma unroll
            for (int t = 0; t < NT; ++t) g.b[kk][t] = qb[t][(c * W + kk) * 64 + lane];
    };

    f32x16 acc[NT][4];
    // Accumulators of a tile start from the norms of its points.  (Each query set reads them
    // from LDS for itself, through an offset the compiler cannot see through: one read shared
    // by both sets would hold 64 registers beside the 128 accumulators.)
    auto start_tile = [&](int tl) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            int off = (tl & 1) * TX + h * 4;
            asm volatile("" : "+v"(off));
#pragma unroll
            for (int pb = 0; pb < 4; ++pb)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const f32x4 v = *reinterpret_cast<const f32x4*>(xns + off + pb * 32 + g * 8);
                    acc[t][pb][g * 4 + 0] = v[0];
                    acc[t][pb][g * 4 + 1] = v[1];
                    acc[t][pb][g * 4 + 2] = v[2];
                    acc[t][pb][g * 4 + 3] = v[3];
                }
        }
    };
    if (ntiles == 0) return;  // (the whole workgroup: a range past the end of the points)
    XS xe, xo;
    xe.xnv = xo.xnv = 0.f;
    QB be, bo;
    fetchQ(0, be);
    fetchX(xe);
    stash(0, xe);
    fetchX(xo);
    __syncthreads();
    const u32x4* const as_r = as + lane;
    // One stage: MFMAs on LDS buffer `par` with B operands b; the B operands of the next stage
    // (chunks from c_next on) and the A operand of the stage after it are requested, the A operand
    // of the next stage goes to the other buffer.
    auto stage = [&](int par, int c_next, const QB& b, QB& bn, XS& mine, const XS& next) {
        fetchQ(c_next, bn);
        fetchX(mine);
#pragma unroll
        for (int kk = 0; kk < W; ++kk) {
            bf16x8 av[4];
#pragma unroll
            for (int pb = 0; pb < 4; ++pb)
                av[pb] = __builtin_bit_cast(bf16x8, as_r[((par * W + kk) * 4 + pb) * 64]);
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const bf16x8 bb = __builtin_bit_cast(bf16x8, b.b[kk][t]);
#pragma unroll
                for (int pb = 0; pb < 4; ++pb)
                    acc[t][pb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[pb], bb, acc[t][pb], 0, 0, 0);
            }
            if (kk == (W - 1) / 2) stash(par ^ 1, next);
        }
    };
    // The stages of one tile, the register sets (be, bo) and (xe, xo) taking turns.  After an odd
    // number of stages the roles would be exchanged for the next tile; instead the tile's end
    // moves the two sets that are still needed (bo: the next stage's B operands, xe: the A operand
    // of the stage after it) into the places where a tile expects them.
    unsigned others[NT];
    auto ask_others = [&]() {
        // What the other ranges of the lane's queries have reached since the last look: asked for
        // ahead of the tile's last stage, used behind it.
#pragma unroll
        for (int t = 0; t < NT; ++t)
            others[t] = __hip_atomic_load(a.tsh + here(min(wave_row0 + 32 * t + i32, a.rows - 1)), __ATOMIC_RELAXED,
                                          __HIP_MEMORY_SCOPE_AGENT);
    };
    int par0 = 0;  // LDS buffer of the tile's first stage
    int tile3 = 0;  // tile % 3
    for (int tile = 0; tile < ntiles; ++tile) {
        start_tile(tile);
        int c = 0;
        for (; c + 2 <= nst; c += 2) {
            stage(par0, c + 1, be, bo, xe, xo);
            __syncthreads();
            if (c + 2 == nst) ask_others();
            stage(par0 ^ 1, c + 2 == nst ? 0 : c + 2, bo, be, xo, xe);
            if (c + 2 < nst) __syncthreads();
        }
        if (c < nst) {
            ask_others();
            stage(par0, 0, be, bo, xe, xo);
        }
        // (the tile's last stage has no barrier of its own yet: the one below ends it)
        const int tile_base = j0 + tile * TX;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int q = wave_q0 + 32 * t + i32;
            const float cap = fminf(cap_l[q], word_key(others[t]));
            if (h == 0) cap_l[q] = cap;
            tauf[t] = key_bound(fminf(own_l[q], cap), qn_l[q], cross_l[q]);
        }
#pragma unroll
        for (int t = 0; t < NT; ++t) epilogue(t, acc[t], tile_base);
        if (((tile & 7) == 7 || tile == 1) && m_top <= 4) {
            // After the second tile (every range has left its first value in tsr by then: they
            // start together) and every eighth tile from there on, accumulators dead: what all
            // ranges of the lane's queries have published by now.  The lower half of the wave
            // looks for the first query set, the upper for the second.
            static_assert(NT == 2, "one query set per half wave");
            const float mine = union_bound_lane(here(min(wave_row0 + 32 * h + i32, a.rows - 1)));
            const float oth = lane_xor<32>(mine);
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const int q = wave_q0 + 32 * t + i32;
                const float cap = fminf(cap_l[q], (h == t) ? mine : oth);
                if (h == 0) cap_l[q] = cap;
                tauf[t] = key_bound(fminf(own_l[q], cap), qn_l[q], cross_l[q]);
            }
        }
        if (tile == 1 && m_top > 4) {
            // (shapes the per-lane form does not cover: the same look after the second tile,
            // one query at a time, the wave's lanes reading the S words)
            for (int qq = 0; qq < 32 * NT; ++qq) {
                const int r = wave_row0 + qq;
                if (r >= a.rows) break;
                const float mine = word_key(
                    __hip_atomic_load(a.tsr + (size_t)r * S + s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
                const float m = union_bound(r, mine, lane);
                if (lane == 0 && m < kInf) atomicMin(a.tsh + r, key_word(m));
            }
        }
        // The barrier that ends the tile carries the vote on stopping as well: one word per tile
        // in turn, set before the barrier, read behind it, cleared behind the next one.  The
        // range's last tile ends with a stop that empties every buffer.
        const bool end = tile + 1 == ntiles;
        bool full = ovf != 0 || end;
#pragma unroll
        for (int t = 0; t < NT; ++t) full = full || cnt[t] > C - kWdRoom;
        if (__builtin_amdgcn_ballot_w64(full) != 0 && lane == 0) co_stop[tile3] = 1;
        __syncthreads();
        if (tid == 0) co_stop[tile3 == 0 ? 2 : tile3 - 1] = 0;
        if (co_stop[tile3] != 0) stop_work(tile_base, end);
        tile3 = tile3 == 2 ? 0 : tile3 + 1;
        if (nst & 1) {
            be = bo;
            xo = xe;
            par0 ^= 1;
        }
    }
}

}  // namespace

hipError_t launch_wide(const float* Q, int64_t ldq, const float* X, int64_t ldx, const void* xp,
                       int64_t slab_first, int64_t slab_points, const void* qp, const float* qn, void* tsh,
                       void* tsr, const float* xn, const void* hdr, int64_t rows, int64_t n, int d, int k,
                       int S, int64_t j_first, int64_t j_end, int init_from, float* lk, int* li,
                       hipStream_t stream) {
    const int nch = pk_padded_chunks(d);
    if (nch % kWdW != 0 || S < 1 || S > kWave || !packed_rows_aligned(Q, ldq, X, ldx, d) ||
        j_first % kPkStep != 0 || slab_first % kPkStep != 0 || slab_points % kPkStep != 0 ||
        j_first < slab_first || j_end <= j_first || j_end > n || j_end > slab_first + slab_points)
        return hipErrorInvalidValue;
    WdArgs a;
    a.Q = Q;
    a.ldq = ldq;
    a.X = X;
    a.ldx = ldx;
    a.Xp = static_cast<const u32x4*>(xp);
    a.xn = xn;
    a.Qp = static_cast<const u32x4*>(qp);
    a.qnorm = qn;
    a.tsh = static_cast<unsigned*>(tsh);
    a.tsr = static_cast<unsigned*>(tsr);
    a.hdr = static_cast<const unsigned*>(hdr);
    a.lk = lk;
    a.li = li;
    a.rows = (int)rows;
    a.n = (int)n;
    a.d = d;
    a.nch = nch;
    a.k = k;
    a.S = S;
    a.tiles = (int)((rows + kWdTileQ - 1) / kWdTileQ);
    a.qsets = (int)((rows + kPkStep - 1) / kPkStep * 2);
    a.j_slab0 = (int)slab_first;
    a.slab_steps = (int)(slab_points / kPkStep);
    a.j_first = (int)j_first;
    a.j_end = (int)j_end;
    const int64_t span = j_end - j_first;
    int64_t per = (span + S - 1) / S;
    per = (per + kWdTileX - 1) / kWdTileX * kWdTileX;
    a.range_len = (int)per;
    a.init_from = init_from;
    // (room left in the LDS for one query row per wave: the stops stage the row they work on)
    a.q_stage = wd_lds_bytes(k) + (int64_t)kWdWaves * d * 4 <= kPkLdsBytes ? 1 : 0;
    const size_t lds = (size_t)wd_lds_bytes(k) + (a.q_stage ? (size_t)kWdWaves * d * 4 : 0);
    hipError_t e = raise_lds_limit(knn_wide_kernel, lds);
    if (e != hipSuccess) return e;
    knn_wide_kernel<<<dim3((unsigned)(a.tiles * S)), dim3(64 * kWdWaves), lds, stream>>>(a);
    return hipGetLastError();
}

}  // namespace knn
