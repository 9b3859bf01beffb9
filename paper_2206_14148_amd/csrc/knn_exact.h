// Exact fp32 keys of the pairs that a bf16 matrix-core filter lets through, and their merge into
// a query's list: shared by the gfx950 search kernels for d > 8 (knn_split.hip, knn_packed.hip, knn_wide.hip).
// The expansion of paper section 4.1 only filters there; the keys that enter the lists are the
// difference form sum_t (q_t - x_t)^2 evaluated here, in one fixed summation order, so that a
// key is the same bits whichever kernel, tiling or memory limit produced it.
#pragma once
#include <hip/hip_runtime.h>

#include "knn_config.h"
#include "knn_device.h"

namespace knn {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// bf16 (round to nearest even) of two floats in one word, the first in the low half
__device__ __forceinline__ unsigned round_pair(float a, float b) {
    const f32x2 p = {a, b};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(p, bf16x2));
}

// float - its bf16 rounding (exact in fp32)
__device__ __forceinline__ float bf16_residual(float v) {
    return v - __uint_as_float(round_pair(v, 0.f) << 16);
}

// floats <-> unsigned words with the same order (for atomicMin on keys of either sign)
__device__ __forceinline__ unsigned key_word(float f) {
    const unsigned u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float word_key(unsigned w) {
    return __uint_as_float((w & 0x80000000u) ? (w & 0x7fffffffu) : ~w);
}
constexpr unsigned kInfWord = 0xff800000u;  // key_word(+inf)

// One lane's share of the exact key of a candidate - sum_t (q_t - x_t)^2, or with DOT the
// product sum_t q_t x_t of the cosine metric: the groups of four
// coordinates g = part, part + 2, ... in ascending order, one fma chain.  The loads of two groups
// are issued before the first is used (U = 2), or of U groups: more in flight shorten the wait
// for a long row and cost registers, which the caller may or may not have to spare.  U does not
// change the order of the additions.
// QMODE (aligned rows) 1: the query's groups are read where they are used instead of together with
// the candidate's - for a query row that the caller has staged in LDS (qp), so that all U groups
// in flight are the candidate's.  2: the same with the staging done here: the wave copies the
// row qp to qst (LDS, d floats) behind the requests for the candidate's first U groups, so that
// the copy shares their round trip.
template <bool ALIGNED, bool DOT, int U, int QMODE = 0>
__device__ __forceinline__ float exact_partial(const float* __restrict__ qp, const float* __restrict__ xp,
                                               int d, int part, float* qst = nullptr, int lane = 0) {
    static_assert(QMODE == 0 || ALIGNED, "late query reads: aligned rows only");
    float sum = 0.f;
    const int ng = (d + 3) >> 2;  // groups of four coordinates (the last may be ragged)
    const float* const qsrc = QMODE == 2 ? qst : qp;
    int trip = 0;
    for (int g0 = part; g0 < ng; g0 += 2 * U, ++trip) {
        f32x4 xv[U], qv[QMODE ? 1 : U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int g = g0 + 2 * u;
            const int gc = g < ng ? g : part;  // a valid group; its value is not used
            if (ALIGNED) {
                xv[u] = *reinterpret_cast<const f32x4*>(xp + 4 * gc);
                if (!QMODE) qv[u] = *reinterpret_cast<const f32x4*>(qp + 4 * gc);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int t = 4 * gc + e < d ? 4 * gc + e : 0;
                    xv[u][e] = xp[t];
                    qv[u][e] = qp[t];
                }
            }
        }
        if (QMODE == 2 && trip == 0) {
            for (int g = lane; g < ng; g += kWave)
                *reinterpret_cast<f32x4*>(qst + 4 * g) = *reinterpret_cast<const f32x4*>(qp + 4 * g);
            wave_sync();
        }
        // A coordinate past the row's end (or a group past it) leaves the sum as it is: its x is
        // replaced by q (a zero difference), for the dot product by 0, and sum + 0 = sum exactly -
        // a select on the operand, so that the chain stays one straight run of fused multiply-adds
        // (a select on the sum was compiled into a branch per coordinate).
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int g = g0 + 2 * u;
            const bool ok_g = g < ng;
            const f32x4 qg = QMODE ? *reinterpret_cast<const f32x4*>(qsrc + 4 * (ok_g ? g : part)) : qv[QMODE ? 0 : u];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bool ok = ALIGNED ? ok_g : (ok_g && 4 * g + e < d);  // (aligned rows: d % 4 == 0)
                const float qe = qg[e];
                const float xe = ok ? xv[u][e] : (DOT ? 0.f : qe);
                const float df = qe - xe;
                sum = DOT ? fmaf(qe, xe, sum) : fmaf(df, df, sum);
            }
        }
    }
    return sum;
}

// The rare path of the filter kernels for one query.  The cc <= 32 candidates are the point indices cbuf[0 .. cc-1], or, with cbuf null,
// the points jbase .. jbase + cc - 1.  Two lanes per
// candidate: lane 2c + p sums the groups of four coordinates g = p, p + 2, ... (exact_partial),
// the two partial sums are added; that order is part of the key's definition.  The keys are
// merged into the query's list gk/gi, the list's k-th key is published in *tshr (atomic
// minimum on order-preserving words).  rn != null selects the cosine metric: the key of point j
// is -2 (q . x_j) rn[j] with the dot product summed in the same order.  Returns the list's new
// k-th key as float bits; with pos2 >= 0, *key2 gets the key at position pos2 of the merged list.
// QMODE 2: the query's row is staged in LDS first (exact_partial) - in qst, or in the scratch, which
// must then hold d floats.
template <bool ALIGNED, int U, bool HEAD_AHEAD = false, int QMODE = 0>
__device__ __forceinline__ unsigned flush_query_exact(const float* __restrict__ qp,
                                                   const float* __restrict__ X, int64_t ldx, int d,
                                                   int jsafe, const int* __restrict__ cbuf, int jbase,
                                                   int cc,
                                                   float* __restrict__ gk, int* __restrict__ gi, int k,
                                                   float* scratch, unsigned* tshr,
                                                   const float* __restrict__ rn, int lane, int pos2 = -1,
                                                   float* key2 = nullptr, float* qst = nullptr) {
    MergeScratch sc;
    sc.cand_key = scratch;
    sc.cand_idx = reinterpret_cast<int*>(scratch + kWave);
    sc.list_key = scratch + 2 * kWave;
    sc.list_idx = reinterpret_cast<int*>(scratch + 2 * kWave + k);
    wave_sync();
    // HEAD_AHEAD: the list is asked for first and used last, so that its round trip runs beside
    // the rows' (four more registers all through the evaluation: not for callers that are short
    // of them)
    ListHead head = {0.f, 0.f, 0, 0};
    if (HEAD_AHEAD) head = load_list_head(gk, gi, k, lane);
    const int cand = lane >> 1, part = lane & 1;
    const int j = cand < cc ? (cbuf ? cbuf[cand] : jbase + cand) : -1;
    const int jl = j < 0 ? jsafe : j;
    float sum;
    if (rn) {
        sum = exact_partial<ALIGNED, true, U, QMODE>(qp, X + (int64_t)jl * ldx, d, part, qst ? qst : scratch, lane);
        sum += lane_xor<1>(sum);
        sum = (-2.f * sum) * rn[jl];
    } else {
        sum = exact_partial<ALIGNED, false, U, QMODE>(qp, X + (int64_t)jl * ldx, d, part, qst ? qst : scratch, lane);
        sum += lane_xor<1>(sum);
    }
    // candidate c sits in lanes 2c, 2c + 1; the merge wants it in lane c
    const int src = (2 * lane) & 63;
    float key = __shfl(sum, src);
    int id = __shfl(j, src);
    if (lane >= cc || id < 0) {  // (a buffer entry may have been struck out: -1)
        key = kInf;
        id = kNoIdx;
    }
    const uint64_t mr = wave_merge_pair_impl<HEAD_AHEAD>(gk, gi, k, key, id, sc, lane, cc, head, pos2, key2);
    const unsigned t_bits = (unsigned)mr;
    // no value returned: nothing waits for the round trip
    if (lane == 0) atomicMin(tshr, key_word(__uint_as_float(t_bits)));
    return t_bits;
}

}  // namespace

}  // namespace knn
