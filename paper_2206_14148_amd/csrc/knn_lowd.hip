// gfx950 (CDNA4, MI355X) kNN search kernels for low-dimensional points and for the L1
// metric: paper section 5.2 defines the result, section 4.1 the squared distance; these
// kernels evaluate the difference form directly (d <= 8, L1) or use an MFMA filter in
// front of it (d <= 3 with packed points).
#include <hip/hip_runtime.h>

#include <climits>
#include <cmath>
#include <cstdint>
#include <type_traits>

#include "knn_config.h"
#include "knn_device.h"
#include "knn_kernels.h"

namespace knn {

namespace {

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
            const float t_new = wave_merge(lk + lb, li + lb, k, key, id, sc, lane, c);
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
// The queries are read from a transposed copy, blocks of 64 rows x 4 coordinates with a
// lane's four values side by side (zeros past the rows and past d): a wave's load of a chunk
// is then four fully coalesced 1 KB reads (read from their own rows, every lane touched a
// different cache line: 64 tag look-ups per load instruction, the vector L1 busy all the time).
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void knn_l1_transpose_kernel(const float* __restrict__ Q,
                                                               int64_t ldq, int rows, int d,
                                                               f32x4* __restrict__ Qt) {
    const int d4 = (d + 3) / 4;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;  // (block of 64 rows, t / 4, lane)
    const int64_t total = (int64_t)((rows + kWave - 1) / kWave) * d4 * kWave;
    if (i >= total) return;
    const int lane = (int)(i % kWave);
    const int t4 = (int)(i / kWave % d4);
    const int64_t r = i / ((int64_t)kWave * d4) * kWave + lane;
    f32x4 v = {0.f, 0.f, 0.f, 0.f};
    if (r < rows) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (4 * t4 + e < d) v[e] = Q[r * ldq + 4 * t4 + e];
    }
    Qt[i] = v;
}

__global__ __launch_bounds__(kLowdTileQ) void knn_l1_kernel(
    const f32x4* __restrict__ Qt, const float* __restrict__ X, int64_t ldx, int rows, int n, int d,
    int k, int S, int split_len, float* __restrict__ lk, int* __restrict__ li) {
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
    // this lane's query: coordinates 4 t4 .. 4 t4 + 3 are qt[t4 * 64]
    const f32x4* qt = Qt + (size_t)(wave_row0 / kWave) * ((d + 3) / 4) * kWave + lane;
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
            const float t_new = wave_merge(lk + lb, li + lb, k, key, id, sc, lane, c);
            if (lane == L) {
                tau = t_new;
                cnt = 0;
            }
        }
    };

    const int j0 = s * split_len;
    const int j1 = min(n, j0 + split_len);
    // The query's next TC values are asked for one piece ahead (at the end of a row: those of
    // the row's start, for the next group of points).
    struct QV {
        f32x4 v[TC / 4];
    };
    const int d4 = (d + 3) / 4;
    auto load_q = [&](QV& q, int t) {
        const int g0 = (t < d ? t : 0) / 4;
#pragma unroll
        for (int t4 = 0; t4 < TC / 4; ++t4) q.v[t4] = qt[(size_t)min(g0 + t4, d4 - 1) * kWave];
    };
    QV qa, qb;
    load_q(qa, 0);
    float ahead = 0.f;
    for (int j = j0; j < j1; j += P) {
        float acc[P];
#pragma unroll
        for (int p = 0; p < P; ++p) acc[p] = 0.f;
        // N dimensions t0 .. t0 + N - 1 for the P points of the group; masked: some of them
        // lie past d (only the last, shorter piece of a row)
        // cur: the query's values from t0 on; nxt receives those of the piece after this one
        auto piece = [&](auto n_tag, int t0, bool masked, const QV& cur, QV& nxt) {
            constexpr int N = decltype(n_tag)::value;
            load_q(nxt, t0 + N);
            // What the piece after this one will read of its points is asked for now through
            // the vector memory path (one word at each end of a point's span, lane l for
            // point l % 8; the value is not used, it only has to be waited for, one piece
            // later): that brings the lines into the L2, so the scalar loads that touch them
            // then wait for the L2 and not for HBM.
            if (N == TC) {
                asm volatile("" ::"v"(ahead));
                const bool wrap = t0 + N >= d;
                const int tn = wrap ? 0 : t0 + N;
                const int jn = (wrap ? j + P : j) + (lane & (P - 1));
                const int tw = (lane & P) ? tn : min(tn + N - 1, d - 1);
                ahead = X[(int64_t)min(jn, j1 - 1) * ldx + tw];
            }
            float qv[N];
#pragma unroll
            for (int t = 0; t < N; ++t) qv[t] = cur.v[t / 4][t % 4];
            // Scalar loads return in any order, so every wait is for all of them, and the 64
            // bytes a piece reads of a point are one or two cache lines that nobody has touched
            // before: left alone, the P loads of a piece miss one after the other, each in
            // front of its point's arithmetic.  Asking for the last word of every point's span
            // first (and the first word at the start of a row; later pieces share that line
            // with the piece before) brings the lines in side by side, one wait for all.
            if (N == TC) {
                static_assert(P == 8, "one operand per load below");
                const int tl = min(t0 + N - 1, d - 1);
                float w[P];
                if (t0 == 0) {
#pragma unroll
                    for (int p = 0; p < P; ++p) w[p] = X[(int64_t)((j + p < j1) ? j + p : j1 - 1) * ldx];
                    asm volatile("" ::"s"(w[0]), "s"(w[1]), "s"(w[2]), "s"(w[3]), "s"(w[4]), "s"(w[5]),
                                 "s"(w[6]), "s"(w[7]));
                }
#pragma unroll
                for (int p = 0; p < P; ++p) w[p] = X[(int64_t)((j + p < j1) ? j + p : j1 - 1) * ldx + tl];
                asm volatile("" ::"s"(w[0]), "s"(w[1]), "s"(w[2]), "s"(w[3]), "s"(w[4]), "s"(w[5]),
                             "s"(w[6]), "s"(w[7])
                             : "memory");
            }
            if (N == TC) {
                // A wait for scalar data is a wait for all of it, so the next point's values
                // can be on their way only while this point's are being used: ask for them
                // right behind the first use (which is where the wait sits), not later.
                float xv[2][N];
                auto load_x = [&](float(&dst)[N], int p) {
                    const float* xp = X + (int64_t)((j + p < j1) ? j + p : j1 - 1) * ldx + t0;
#pragma unroll
                    for (int t = 0; t < N; ++t) dst[t] = xp[t];
                };
                load_x(xv[0], 0);
#pragma unroll
                for (int p = 0; p < P; ++p) {
                    float a = acc[p] + fabsf(qv[0] - xv[p & 1][0]);
                    if (p + 1 < P) {
                        // (the sum threads through both statements, so the arithmetic before
                        // and after them stays where it is written)
                        asm volatile("" : "+v"(a)::"memory");
                        load_x(xv[(p + 1) & 1], p + 1);
                        asm volatile("" : "+v"(a)::"memory");
                    }
#pragma unroll
                    for (int t = 1; t < N; ++t) a += fabsf(qv[t] - xv[p & 1][t]);
                    acc[p] = a;
                }
                return;
            }
#pragma unroll
            for (int p = 0; p < P; ++p) {
                const int jp = (j + p < j1) ? j + p : j1 - 1;  // uniform; repeats of the last point are masked below
                const float* xp = X + (int64_t)jp * ldx;
                float a = acc[p];
                if (!masked) {
#pragma unroll
                    for (int t = 0; t < N; ++t) a += fabsf(qv[t] - xp[t0 + t]);
                } else {
#pragma unroll
                    for (int t = 0; t < N; ++t) {
                        const int tt = t0 + t;
                        const float xv = xp[tt < d ? tt : d - 1];
                        a += fabsf(qv[t] - (tt < d ? xv : 0.f));
                    }
                }
                acc[p] = a;
            }
        };
        // whole chunks of TC dimensions, then pieces of 4, then what is left (ascending t throughout)
        // (chunks in pairs, so that the two sets of query registers swap roles without copies)
        constexpr std::integral_constant<int, TC> whole{};
        constexpr std::integral_constant<int, 4> four{};
        int t0 = 0;
        for (; t0 + 2 * TC <= d; t0 += 2 * TC) {
            piece(whole, t0, false, qa, qb);
            piece(whole, t0 + TC, false, qb, qa);
        }
        if (t0 + TC <= d) {
            piece(whole, t0, false, qa, qb);
            qa = qb;
            t0 += TC;
        }
        for (; t0 + 4 <= d; t0 += 4) {
            piece(four, t0, false, qa, qb);
            qa = qb;
        }
        if (t0 < d) {
            piece(four, t0, true, qa, qb);
            qa = qb;
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

    // A pair with exact fp32 distance <= tau has key < (tau - qn) + slack: the key and qn each
    // carry a few roundings relative to (||x||^2 + ||q||^2), the distance a few relative to
    // itself; 2^-19 of their sum is several times the worst case.
    float tau = active ? kInf : -kInf;
    int taui = active ? kNoIdx : -1;  // (tau, taui): key and index of the current k-th best
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
            const uint64_t mr = wave_merge_pair(lk + lb, li + lb, k, key, id, sc, lane, c);
            const float t_new = merged_key(mr);
            if (i32 == L) {
                tau = t_new;
                taui = merged_idx(mr);
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
            // the halves of the wave hold interleaved runs of four rows, so pairs do not come
            // in index order: compare on (key, index) with the current k-th best
            bool c = has && before(dd, jblock + row, tau, taui);
            if (__builtin_amdgcn_ballot_w64(c) == 0) continue;
            int own = c ? 1 : 0;
            int oth = __shfl_xor(own, 32);
            const uint64_t need = __builtin_amdgcn_ballot_w64(cnt + own + oth > C) & 0xffffffffull;
            if (need) {
                flush(need);
                c = c && before(dd, jblock + row, tau, taui);
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
    // wave-uniform base + constant lane offset + immediate: no vector address arithmetic
    const f32x2* xb = xp2 + (size_t)j0 * 2;
    const int loff = i32 * 2 + h;
    if (nfull > 0) {
#pragma unroll
        for (int u = 0; u < UB; ++u) a[u] = xb[loff + u * 64];
    }
    for (int it = 0; it < nfull; ++it) {
        xb += PTS * 2;
        if (it + 1 < nfull) {
#pragma unroll
            for (int u = 0; u < UB; ++u) an[u] = xb[loff + u * 64];
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
// Low-dimensional path with a bf16 filter (d <= 3, room for 32 bytes per point).  The filter
// of the kernel above costs two fp32 MFMAs (128 cycles) per 32 x 32 keys; one
// v_mfma_f32_32x32x16_bf16 (32 cycles) gives keys that are nearly as sharp if every fp32 value
// is cut into bf16 pieces and the cross products that matter are spread over the 16 K slots:
//     x = xh + xl + xr,  |xl| <= 2^-8 |x|,  |xr| <= 2^-17 |x|  (round to nearest, 8 significant
//     bits a piece),  q likewise,  ||x||^2 = nh + nm + nl exactly
//     key = sum_t  xh_t (-2 qh_t) + xh_t (-2 ql_t) + xl_t (-2 qh_t) + xl_t (-2 ql_t)
//           +  (nh + nm + nl) * 1
// (15 of 16 slots at d = 3, products of two bf16 values are exact in fp32).  What is left out,
// -2 (xr q + x qr - xr qr), is at most 2^-15 (1 + 2^-16) ||x|| ||q||, which the filter bound
// allows for; d = 4 and d = 8 have no slots for xl ql, there the bound is twice that plus
// 2^-15.  Points and queries are first
// moved by the midpoint of the points' bounding box, so that bound scales with the spread of
// the data, not with its offset from the origin.  The filter only decides which pairs go to
// the exact test; that test reads the point's original fp32 coordinates from X and is the
// same arithmetic as knn_lowd_kernel, so keys, accepted sets and results are identical.
// ---------------------------------------------------------------------------------------
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// round-to-nearest-even bf16 of a finite fp32 value, as its 16 bits
__device__ __forceinline__ unsigned bf16_bits(float x) {
    unsigned u = __float_as_uint(x);
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}
__device__ __forceinline__ float bf16_value(unsigned bits) { return __uint_as_float(bits << 16); }

// floats <-> unsigned keys with the same order (for atomicMin / atomicMax)
__device__ __forceinline__ unsigned ordered_bits(float f) {
    const unsigned u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float ordered_value(unsigned k) {
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

// header words of the packed area: 0 max ||x - c||^2 (bits of a non-negative float),
// 1 .. kPbMaxD per-dimension minimum, kPbMaxD + 1 .. 2 kPbMaxD per-dimension maximum (ordered keys)
__global__ void knn_bbox_init_kernel(unsigned* __restrict__ hdr) {
    const int t = threadIdx.x;
    if (t == 0) hdr[0] = 0u;
    if (t >= 1 && t <= kPbMaxD) hdr[t] = 0xffffffffu;
    if (t > kPbMaxD && t <= 2 * kPbMaxD) hdr[t] = 0u;
}

template <int D>
__global__ __launch_bounds__(256) void knn_bbox_kernel(const float* __restrict__ X, int64_t ldx,
                                                       int n, unsigned* __restrict__ hdr) {
    // grid-stride over the points, one running box per thread, then wave and workgroup
    // reductions, so that a workgroup sends 2 D atomics however many points it saw
    __shared__ float box[4][2 * D];
    float lo[D], hi[D];
#pragma unroll
    for (int t = 0; t < D; ++t) {
        lo[t] = kInf;
        hi[t] = -kInf;
    }
    for (int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x; j < n; j += (int64_t)gridDim.x * 256) {
#pragma unroll
        for (int t = 0; t < D; ++t) {
            const float v = X[j * ldx + t];
            lo[t] = fminf(lo[t], v);
            hi[t] = fmaxf(hi[t], v);
        }
    }
#pragma unroll
    for (int t = 0; t < D; ++t) {
#pragma unroll
        for (int s = 32; s > 0; s >>= 1) {
            lo[t] = fminf(lo[t], __shfl_xor(lo[t], s));
            hi[t] = fmaxf(hi[t], __shfl_xor(hi[t], s));
        }
        if ((threadIdx.x & 63) == 0) {
            box[threadIdx.x >> 6][t] = lo[t];
            box[threadIdx.x >> 6][D + t] = hi[t];
        }
    }
    __syncthreads();
    if (threadIdx.x < D) {
        const int t = threadIdx.x;
        const float l = fminf(fminf(box[0][t], box[1][t]), fminf(box[2][t], box[3][t]));
        const float u = fmaxf(fmaxf(box[0][D + t], box[1][D + t]), fmaxf(box[2][D + t], box[3][D + t]));
        if (l <= u) {  // the workgroup saw at least one point
            atomicMin(hdr + 1 + t, ordered_bits(l));
            atomicMax(hdr + 1 + kPbMaxD + t, ordered_bits(u));
        }
    }
}

template <int D>
__device__ __forceinline__ void bbox_centre(const unsigned* __restrict__ hdr, float (&c)[D]) {
#pragma unroll
    for (int t = 0; t < D; ++t)
        c[t] = 0.5f * ordered_value(hdr[1 + t]) + 0.5f * ordered_value(hdr[1 + kPbMaxD + t]);
}

// ---------------------------------------------------------------------------------------
// Threshold seed (D <= kSeedMaxD).  The points are counted into a grid of G^D cells over their
// bounding box.  A query finds the smallest block of cells around its own cell (own cell, then
// 3^D, then 5^D cells) that holds at least k points: each of those points lies inside the block,
// so the squared distance from the query to the block's farthest corner bounds the query's k-th
// smallest distance from above, and its list can start from that threshold instead of +inf.
// Pairs beyond the bound never reach the exact test, which takes most of the list warm-up away;
// results do not change, because every pair at or below the true k-th distance still passes.
// ---------------------------------------------------------------------------------------
template <int D>
struct SeedGrid {
    float mn[D], inv_w[D], w[D], slack[D];
    int G;
};

template <int D>
__device__ __forceinline__ SeedGrid<D> seed_grid(const unsigned* __restrict__ hdr, int G) {
    SeedGrid<D> g;
    g.G = G;
#pragma unroll
    for (int t = 0; t < D; ++t) {
        const float mn = ordered_value(hdr[1 + t]);
        const float mx = ordered_value(hdr[1 + kPbMaxD + t]);
        float rg = mx - mn;
        if (!(rg > 1e-30f)) rg = 1.f;  // all points share this coordinate: one cell holds them
        g.mn[t] = mn;
        g.inv_w[t] = (float)G / rg;
        g.w[t] = rg / (float)G;
        // A point whose computed cell number is c lies in mn + [c w, (c + 1) w] up to the
        // roundings of (x - mn) * inv_w, of w and of the two ends: under 16 ulps of the
        // magnitudes involved; the slack is twice that.
        g.slack[t] = 0x1p-19f * (fabsf(mn) + fabsf(mx) + rg);
    }
    return g;
}

// cell number along axis t, the same expression for points and queries (queries outside the
// box land in the nearest cell)
template <int D>
__device__ __forceinline__ int seed_cell(const SeedGrid<D>& g, int t, float x) {
    const float u = (x - g.mn[t]) * g.inv_w[t];
    return (int)fminf(fmaxf(u, 0.f), (float)(g.G - 1));  // NaN -> 0
}

__global__ void knn_zero_ints_kernel(int* __restrict__ p, int count) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < count) p[i] = 0;
}

template <int D>
__device__ __forceinline__ int seed_cell_of(const SeedGrid<D>& g, const float* __restrict__ x) {
    int cell = 0;
#pragma unroll
    for (int t = D - 1; t >= 0; --t) cell = cell * g.G + seed_cell<D>(g, t, x[t]);
    return cell;
}

template <int D>
__global__ __launch_bounds__(256) void knn_cell_count_kernel(const float* __restrict__ X, int64_t ldx,
                                                             int n, const unsigned* __restrict__ hdr,
                                                             int G, int* __restrict__ counts) {
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= n) return;
    const SeedGrid<D> g = seed_grid<D>(hdr, G);
    atomicAdd(counts + seed_cell_of<D>(g, X + (int64_t)j * ldx), 1);
}

// starts[c] = number of points in the cells before c (starts[ncell] = n); the counts are set
// back to zero, to serve as the cells' fill cursors.  One workgroup: ncell <= kSeedMaxCells.
__global__ __launch_bounds__(256) void knn_cell_scan_kernel(int* __restrict__ counts, int ncell,
                                                            int* __restrict__ starts) {
    __shared__ int part[256];
    const int t = threadIdx.x;
    const int per = (ncell + 255) / 256;
    const int c0 = min(t * per, ncell), c1 = min(c0 + per, ncell);
    int sum = 0;
    for (int c = c0; c < c1; ++c) sum += counts[c];
    part[t] = sum;
    __syncthreads();
    if (t == 0) {
        int run = 0;
        for (int i = 0; i < 256; ++i) {
            const int v = part[i];
            part[i] = run;
            run += v;
        }
        starts[ncell] = run;
    }
    __syncthreads();
    int run = part[t];
    for (int c = c0; c < c1; ++c) {
        starts[c] = run;
        run += counts[c];
        counts[c] = 0;
    }
}

// the points in cell order: (x0, x1, x2, index bits) at sorted[starts[cell] ...]; the order
// inside a cell is whatever the atomics give (only sets of points are read from it)
template <int D>
__global__ __launch_bounds__(256) void knn_cell_fill_kernel(const float* __restrict__ X, int64_t ldx,
                                                            int n, const unsigned* __restrict__ hdr,
                                                            int G, const int* __restrict__ starts,
                                                            int* __restrict__ cursor,
                                                            f32x4* __restrict__ sorted) {
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= n) return;
    const SeedGrid<D> g = seed_grid<D>(hdr, G);
    const float* x = X + (int64_t)j * ldx;
    const int cell = seed_cell_of<D>(g, x);
    const int pos = starts[cell] + atomicAdd(cursor + cell, 1);
    f32x4 v = {0.f, 0.f, 0.f, __int_as_float(j)};
#pragma unroll
    for (int t = 0; t < D; ++t) v[t] = x[t];
    sorted[pos] = v;
}

// The smallest block of cells around q's cell (own cell, 3^D, 5^D cells) that holds at least k
// points; false when even 5^D cells hold fewer.
template <int D>
__device__ __forceinline__ bool seed_block(const SeedGrid<D>& g, const int* __restrict__ starts,
                                           const float (&q)[D], int k, int (&c0)[3], int (&c1)[3]) {
    static_assert(D <= 3, "block walk below is written for up to three axes");
    int cq[3] = {0, 0, 0};
#pragma unroll
    for (int t = 0; t < D; ++t) cq[t] = seed_cell<D>(g, t, q[t]);
    const int G = g.G;
    for (int R = 0; R <= 2; ++R) {
#pragma unroll
        for (int t = 0; t < 3; ++t) {
            c0[t] = t < D ? max(cq[t] - R, 0) : 0;
            c1[t] = t < D ? min(cq[t] + R, G - 1) : 0;
        }
        int count = 0;
        for (int z = c0[2]; z <= c1[2]; ++z)
            for (int y = c0[1]; y <= c1[1]; ++y) {
                const int row = (z * G + y) * G;  // cells of one row are neighbours in memory
                count += starts[row + c1[0] + 1] - starts[row + c0[0]];
            }
        if (count >= k) return true;
    }
    return false;
}

// upper bound of the k-th smallest fp32 difference-form squared distance from q to the counted
// points: all points of the block lie inside it, so the distance to its farthest corner
template <int D>
__device__ __forceinline__ float seed_bound(const SeedGrid<D>& g, const float (&q)[D],
                                            const int (&c0)[3], const int (&c1)[3]) {
    float b = 0.f;
#pragma unroll
    for (int t = 0; t < D; ++t) {
        const float lo = (g.mn[t] + (float)c0[t] * g.w[t]) - g.slack[t];
        const float hi = (g.mn[t] + (float)(c1[t] + 1) * g.w[t]) + g.slack[t];
        const float far = fmaxf(fabsf(q[t] - lo), fabsf(hi - q[t]));
        b = fmaf(far, far, b);
    }
    // roundings of the bound itself and of the distance it is compared with
    return b * (1.f + 0x1p-17f);
}

// The k-th smallest key among the points of the block itself, k <= K: the keys are those of the
// exact test (same arithmetic), so at least k pairs are at or below the value returned and it
// can start the list's threshold.  K running minima in registers, 2 K operations per point.
template <int D, int K>
__device__ __forceinline__ float seed_exact(const SeedGrid<D>& g, const int* __restrict__ starts,
                                            const f32x4* __restrict__ sorted, const float (&q)[D],
                                            int k, const int (&c0)[3], const int (&c1)[3]) {
    float best[K];
#pragma unroll
    for (int i = 0; i < K; ++i) best[i] = kInf;
    const int G = g.G;
    for (int z = c0[2]; z <= c1[2]; ++z)
        for (int y = c0[1]; y <= c1[1]; ++y) {
            const int row = (z * G + y) * G;
            const int p1 = starts[row + c1[0] + 1];
            for (int p = starts[row + c0[0]]; p < p1; ++p) {
                const f32x4 x = sorted[p];
                float df = q[0] - x[0];
                float v = df * df;
#pragma unroll
                for (int t = 1; t < D; ++t) {
                    df = q[t] - x[t];
                    v = fmaf(df, df, v);
                }
#pragma unroll
                for (int i = 0; i < K; ++i) {  // v sinks to its place, the largest falls out
                    const float lo = fminf(best[i], v);
                    v = fmaxf(best[i], v);
                    best[i] = lo;
                }
            }
        }
    float r = kInf;
#pragma unroll
    for (int i = 0; i < K; ++i) r = (i == k - 1) ? best[i] : r;
    return r;
}

// K slots of the filter's contraction for dimension D, padded with zeros to NM MFMAs of 16
// slots: slot s < D pairs xh_s with -2 qh_s, D <= s < 2D pairs xh with -2 ql, 2D <= s < 3D pairs
// xl with -2 qh; where 4 D + 3 slots fit into the same number of MFMAs (all D but 4 and 8) the
// slots 3D <= s < 4D pair xl with -2 ql as well; the three pieces of the squared norm meet 1.
template <int D>
struct FilterSlots {
    static constexpr int kMfmas = (3 * D + 3 + 15) / 16;  // 1 for D <= 4, 2 for D <= 8
    static constexpr bool kLowLow = 4 * D + 3 <= 16 * kMfmas;
    static constexpr int kProducts = (kLowLow ? 4 : 3) * D;  // slots before the norm pieces
    static constexpr int kUsed = kProducts + 3;
};

// A-operand piece of slot s: xh / xl are the bf16 pieces of the moved coordinates, np the three
// pieces of the squared norm
template <int D>
__device__ __forceinline__ unsigned slot_a(int s, const unsigned (&xh)[D], const unsigned (&xl)[D],
                                           const unsigned (&np)[3]) {
    constexpr int P = FilterSlots<D>::kProducts;
    if (s < 2 * D) return xh[s < D ? s : s - D];
    if (s < P) return xl[s < 3 * D ? s - 2 * D : s - 3 * D];
    if (s < P + 3) return np[s - P];
    return 0u;
}
// B-operand piece of slot s: qh / ql hold the bf16 bits of -2 qh_t and -2 ql_t
template <int D>
__device__ __forceinline__ unsigned slot_b(int s, const unsigned (&qh)[D], const unsigned (&ql)[D]) {
    constexpr int P = FilterSlots<D>::kProducts;
    if (s < D) return qh[s];
    if (s < 2 * D) return ql[s - D];
    if (s < 3 * D) return qh[s - 2 * D];
    if (s < P) return ql[s - 3 * D];
    if (s < P + 3) return 0x3f80u;  // 1.0
    return 0u;
}

// 32 bytes per point and MFMA: 16 for the lanes 0..31 of the A operand (K slots 0..7 of that
// MFMA), 16 for the lanes 32..63 (slots 8..15).  Record (j, i, half) is Xp[(j * NM + i) * 2 + half].
template <int D>
__global__ __launch_bounds__(256) void knn_pack_bf16_kernel(const float* __restrict__ X,
                                                            int64_t ldx, int n,
                                                            uint4* __restrict__ Xp,
                                                            unsigned* __restrict__ hdr) {
    constexpr int NM = FilterSlots<D>::kMfmas;
    const int j = blockIdx.x * 256 + threadIdx.x;
    float c[D];
    bbox_centre<D>(hdr, c);
    float nrm = 0.f;
    if (j < n) {
        float v[D];
#pragma unroll
        for (int t = 0; t < D; ++t) v[t] = X[(int64_t)j * ldx + t] - c[t];
        nrm = v[0] * v[0];
#pragma unroll
        for (int t = 1; t < D; ++t) nrm = fmaf(v[t], v[t], nrm);
        unsigned xh[D], xl[D], np[3];
#pragma unroll
        for (int t = 0; t < D; ++t) {
            xh[t] = bf16_bits(v[t]);
            xl[t] = bf16_bits(v[t] - bf16_value(xh[t]));
        }
        np[0] = bf16_bits(nrm);
        const float r1 = nrm - bf16_value(np[0]);
        np[1] = bf16_bits(r1);
        np[2] = bf16_bits(r1 - bf16_value(np[1]));
#pragma unroll
        for (int i = 0; i < NM; ++i) {
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                unsigned w[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int s0 = 16 * i + 8 * half + 2 * e;
                    w[e] = slot_a<D>(s0, xh, xl, np) | (slot_a<D>(s0 + 1, xh, xl, np) << 16);
                }
                Xp[((size_t)j * NM + i) * 2 + half] = uint4{w[0], w[1], w[2], w[3]};
            }
        }
    }
#pragma unroll
    for (int s = 32; s > 0; s >>= 1) nrm = fmaxf(nrm, __shfl_xor(nrm, s));
    if ((threadIdx.x & 63) == 0) atomicMax(hdr, __float_as_uint(nrm));
}

template <int D>
__global__ __launch_bounds__(256, FilterSlots<D>::kMfmas == 1 ? 4 : 3) void knn_lowd_bf16_kernel(
    const float* __restrict__ Q, int64_t ldq, const float* __restrict__ X, int64_t ldx,
    const uint4* __restrict__ Xp, const unsigned* __restrict__ hdr, const int* __restrict__ starts,
    const f32x4* __restrict__ sorted, int seed_cells, int rows, int n, int k, int S, int split_len,
    float* __restrict__ lk,
    int* __restrict__ li) {
    constexpr int C = kPbCand;
    constexpr int NS = kPbSets;  // query sets of 32 per wave: one A-operand load feeds NS MFMAs
    constexpr int NM = FilterSlots<D>::kMfmas;  // MFMAs (of 16 K slots) per 32 x 32 keys
    constexpr int UB = 4 / NM;   // 32-point blocks per loop iteration
    constexpr int PTS = UB * 32; // points per loop iteration
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int i32 = lane & 31;  // query column (B side) / point row (A side) of the 32x32 block
    const int h = lane >> 5;
    const size_t per_wave = (size_t)(2 * NS * 32 * C + 2 * kWave + 2 * k) * 4;
    float* ck = reinterpret_cast<float*>(smem + (size_t)wave * per_wave);  // [NS * 32][C]
    int* ci = reinterpret_cast<int*>(ck + NS * 32 * C);                    // [NS * 32][C]
    MergeScratch sc;
    sc.cand_key = reinterpret_cast<float*>(ci + NS * 32 * C);
    sc.cand_idx = reinterpret_cast<int*>(sc.cand_key + kWave);
    sc.list_key = reinterpret_cast<float*>(sc.cand_idx + kWave);
    sc.list_idx = reinterpret_cast<int*>(sc.list_key + k);

    const int s = blockIdx.y;
    const int wave_row0 = (blockIdx.x * 4 + wave) * (NS * 32);
    if (wave_row0 >= rows) return;  // whole wave idle; no workgroup barrier is used below

    for (int qq = 0; qq < NS * 32; ++qq) {
        if (wave_row0 + qq >= rows) break;
        const size_t lb = ((size_t)(wave_row0 + qq) * S + s) * k;
        for (int p = lane; p < k; p += kWave) {
            lk[lb + p] = kInf;
            li[lb + p] = kNoIdx;
        }
    }

    // the filter sees points and queries moved by the midpoint of the points' bounding box
    float c[D];
    bbox_centre<D>(hdr, c);
    const float xmax = __uint_as_float(hdr[0]);

    // per query set: the query (original coordinates, for the exact test), the B operands, the
    // thresholds and the number of buffered candidates (same value in both halves of the wave)
    float q[NS][D];
    bf16x8 bq[NS][NM];
    float qn[NS], cross[NS], tau[NS], tauf[NS];
    int taui[NS], cnt[NS];  // (tau, taui): key and index of the query's current k-th best
    float tcap[NS];         // upper bound of the k-th smallest distance known before the scan
    // A pair with exact fp32 distance <= tau has a filter key below (tau - qn) + slack: the cross
    // terms the bf16 pieces leave out (<= kCross ||x'|| ||q'|| <= kCross sqrt(xmax qn)), the
    // fp32 roundings of the accumulation (16 NM additions of terms whose magnitudes sum to at
    // most 2.01 (xmax + qn): 2^-19 NM of that sum if the matrix core rounds after every one), of
    // qn, of the moved coordinates and of the distance itself (a few 2^-24 each): kSum of
    // ||x'||^2 + ||q'||^2 + tau covers twice their total.
    // (with the xl ql products: 2 (2^-17 + 2^-17 + 2^-34); without: 2 2^-16 (1 + 2^-7) more)
    constexpr float kCross = FilterSlots<D>::kLowLow ? 0x1p-15f * 1.001f : 0x1p-14f * 1.006f;
    constexpr float kSum = NM == 1 ? 0x1p-18f : 0x1p-17f;
    auto key_bound = [&](int st, float t) {
        return (t - qn[st]) + (cross[st] + kSum * (xmax + qn[st] + t));
    };
#pragma unroll
    for (int st = 0; st < NS; ++st) {
        const int r = wave_row0 + st * 32 + i32;
        const bool active = r < rows;
        float qc[D];
#pragma unroll
        for (int t = 0; t < D; ++t) {
            q[st][t] = active ? Q[(int64_t)r * ldq + t] : 0.f;
            qc[t] = active ? q[st][t] - c[t] : 0.f;
        }
        qn[st] = qc[0] * qc[0];
#pragma unroll
        for (int t = 1; t < D; ++t) qn[st] = fmaf(qc[t], qc[t], qn[st]);
        cross[st] = kCross * sqrtf(xmax * qn[st]);
        // B operands: the pieces -2 qh, -2 ql and 1 in the slot order of FilterSlots; a lane of
        // half h holds slots 8h .. 8h + 7 of each MFMA
        unsigned qh[D], ql[D];
#pragma unroll
        for (int t = 0; t < D; ++t) {
            const unsigned hb = bf16_bits(qc[t]);
            const float hv = bf16_value(hb);
            qh[t] = bf16_bits(-2.f * hv);                                 // exact
            ql[t] = bf16_bits(-2.f * bf16_value(bf16_bits(qc[t] - hv)));  // exact
        }
#pragma unroll
        for (int i = 0; i < NM; ++i) {
            unsigned w[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int s0 = 16 * i + 2 * e;  // slot of the lower half-wave
                const unsigned lo = slot_b<D>(s0, qh, ql) | (slot_b<D>(s0 + 1, qh, ql) << 16);
                const unsigned hi = slot_b<D>(s0 + 8, qh, ql) | (slot_b<D>(s0 + 9, qh, ql) << 16);
                w[e] = h ? hi : lo;
            }
            bq[st][i] = __builtin_bit_cast(bf16x8, uint4{w[0], w[1], w[2], w[3]});
        }
        tcap[st] = kInf;
        tau[st] = active ? kInf : -kInf;
        taui[st] = active ? kNoIdx : -1;
        cnt[st] = 0;
    }
    // Threshold seed: the lanes of half h work for the queries of set h, then the halves swap
    // what they found.  Up to k = 32 the k-th smallest exact key inside the block of cells, above
    // that the distance to the block's farthest corner.
    if constexpr (D <= kSeedMaxD) {
        static_assert(NS == 2, "one query set per half of the wave");
        if (seed_cells > 0) {
            float mine = kInf;
            const int r = wave_row0 + h * 32 + i32;
            if (r < rows) {
                float qm[D];
#pragma unroll
                for (int t = 0; t < D; ++t) qm[t] = h ? q[1][t] : q[0][t];
                const SeedGrid<D> g = seed_grid<D>(hdr, seed_cells);
                int c0[3], c1[3];
                if (seed_block<D>(g, starts, qm, k, c0, c1)) {
                    if (k <= 16) mine = seed_exact<D, 16>(g, starts, sorted, qm, k, c0, c1);
                    else if (k <= 32) mine = seed_exact<D, 32>(g, starts, sorted, qm, k, c0, c1);
                    else mine = seed_bound<D>(g, qm, c0, c1);
                }
            }
            const float other = lane_xor<32>(mine);
            tcap[0] = h ? other : mine;
            tcap[1] = h ? mine : other;
#pragma unroll
            for (int st = 0; st < NS; ++st)
                if (wave_row0 + st * 32 + i32 < rows) tau[st] = tcap[st];
        }
    }
#pragma unroll
    for (int st = 0; st < NS; ++st) tauf[st] = key_bound(st, tau[st]);

    // bits 0..31 of mask: queries of set st to merge
    auto flush = [&](int st, uint64_t mask) {
        while (mask) {
            const int L = __builtin_ctzll(mask);
            mask &= mask - 1;
            wave_sync();
            const int cc = __shfl(cnt[st], L);
            float key = kInf;
            int id = kNoIdx;
            if (lane < cc) {
                key = ck[(st * 32 + L) * C + lane];
                id = ci[(st * 32 + L) * C + lane];
            }
            const size_t lb = ((size_t)(wave_row0 + st * 32 + L) * S + s) * k;
            const uint64_t mr = wave_merge_pair_ref(lk + lb, li + lb, k, key, id, sc, lane, cc);
            // a list that is not full yet returns +inf: the seed bound stays the threshold
            const bool capped = !(merged_key(mr) <= tcap[st]);
            const float t_new = capped ? tcap[st] : merged_key(mr);
            if (i32 == L) {
                tau[st] = t_new;
                taui[st] = capped ? kNoIdx : merged_idx(mr);
                tauf[st] = key_bound(st, t_new);
                cnt[st] = 0;
            }
        }
    };

    const int j0 = s * split_len;
    const int j1 = min(n, j0 + split_len);

    // Rare path of one 32-point block and one query set (about one block in five at n = 1e6,
    // k = 16, nearly always for a single key).  Sixteen compares leave one lane mask per
    // accumulator register in scalar registers; everything that picks the registers with a set
    // bit is scalar work, and one copy of the exact test handles them one register at a time.
    // Register e of the lanes' half h holds point row 8 (e / 4) + 4 h + e % 4 of the block; the
    // point's coordinates are read from X.
    const int h4 = 4 * h;
    auto examine = [&](int st, const f32x16& keys, int jblock) {
        unsigned nz = 0;  // registers in which some lane passes the filter
#pragma unroll
        for (int e = 0; e < 16; ++e)
            nz |= __builtin_amdgcn_ballot_w64(keys[e] < tauf[st]) ? (1u << e) : 0u;
        while (nz) {
            const int e = __builtin_ctz(nz);  // wave-uniform register number
            nz &= nz - 1;
            const bool pass = keys[e] < tauf[st];
            const int row = 8 * (e >> 2) + (e & 3) + h4;
            float dd = kInf;
            if (pass) {  // only these lanes touch X, so no index leaves the matrix
                const float* __restrict__ xr = X + (int64_t)(jblock + row) * ldx;
                // exact test, same arithmetic as the vector-ALU kernel
                float df = q[st][0] - xr[0];
                dd = df * df;
#pragma unroll
                for (int t = 1; t < D; ++t) {
                    df = q[st][t] - xr[t];
                    dd = fmaf(df, df, dd);
                }
            }
            // The two halves of the wave hold interleaved runs of four rows, so pairs do not
            // reach this test in index order: the comparison with the current k-th best is on
            // (key, index), or a pair could lose a tie against a higher index merged earlier.
            bool cnd = pass && before(dd, jblock + row, tau[st], taui[st]);
            if (__builtin_amdgcn_ballot_w64(cnd) == 0) continue;
            int own = cnd ? 1 : 0;
            int oth = lane_xor<32>(own);
            const uint64_t need =
                __builtin_amdgcn_ballot_w64(cnt[st] + own + oth > C) & 0xffffffffull;
            if (need) {
                flush(st, need);
                cnd = cnd && before(dd, jblock + row, tau[st], taui[st]);
                own = cnd ? 1 : 0;
                oth = lane_xor<32>(own);
            }
            if (cnd) {
                const int slot = (st * 32 + i32) * C + cnt[st] + (h ? oth : 0);
                ck[slot] = dd;
                ci[slot] = jblock + row;
            }
            cnt[st] += own + oth;
        }
    };

    auto process = [&](const uint4 (&a)[UB][NM], int jb) {
#pragma unroll
        for (int u = 0; u < UB; ++u) {
#pragma unroll
            for (int st = 0; st < NS; ++st) {
                f32x16 z;
#pragma unroll
                for (int e = 0; e < 16; ++e) z[e] = 0.f;
#pragma unroll
                for (int i = 0; i < NM; ++i)
                    z = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[u][i]),
                                                                bq[st][i], z, 0, 0, 0);
                float m = kInf;  // 8 three-input mins over (inf, 16 keys)
#pragma unroll
                for (int e = 0; e < 16; ++e) m = fminf(m, z[e]);
                if (__builtin_amdgcn_ballot_w64(m < tauf[st]) != 0) examine(st, z, jb + u * 32);
            }
        }
    };

    // Two statically named sets of A operands alternate (the loop is unrolled by two), so the
    // loads of the next iteration land in registers that are never copied.
    const int nfull = (j1 > j0) ? (j1 - j0) / PTS : 0;
    int jb = j0;
    uint4 a_even[UB][NM], a_odd[UB][NM];
#pragma unroll
    for (int u = 0; u < UB; ++u)
#pragma unroll
        for (int i = 0; i < NM; ++i) a_even[u][i] = a_odd[u][i] = uint4{0u, 0u, 0u, 0u};
    // wave-uniform base + constant lane offset + immediate: no vector address arithmetic.
    // Record (point, MFMA i, half) sits at uint4 index (point * NM + i) * 2 + half.
    const uint4* xb = Xp + (size_t)j0 * (2 * NM);
    const int loff = i32 * (2 * NM) + h;
    auto fetch = [&](uint4 (&dst)[UB][NM]) {
#pragma unroll
        for (int u = 0; u < UB; ++u)
#pragma unroll
            for (int i = 0; i < NM; ++i) dst[u][i] = xb[loff + u * (64 * NM) + 2 * i];
    };
    if (nfull > 0) fetch(a_even);
    for (int it = 0; it < nfull; it += 2) {
        xb += PTS * 2 * NM;
        if (it + 1 < nfull) fetch(a_odd);
        process(a_even, jb);
        jb += PTS;
        if (it + 1 < nfull) {
            xb += PTS * 2 * NM;
            if (it + 2 < nfull) fetch(a_even);
            process(a_odd, jb);
            jb += PTS;
        }
    }
    if (jb < j1) {  // ragged tail: rows past the range read a valid row and get ||x||^2 = +inf
        constexpr int kNormSlot = FilterSlots<D>::kProducts;  // leading piece of the squared norm
#pragma unroll
        for (int u = 0; u < UB; ++u) {
            const int row = jb + u * 32 + i32;
#pragma unroll
            for (int i = 0; i < NM; ++i) {
                uint4 v = Xp[((size_t)(row < j1 ? row : j1 - 1) * NM + i) * 2 + h];
                if (row >= j1 && i == kNormSlot / 16 && h == (kNormSlot % 16) / 8) {
                    unsigned* w = reinterpret_cast<unsigned*>(&v);
                    constexpr int e = kNormSlot % 8;
                    w[e / 2] = (e % 2) ? ((w[e / 2] & 0x0000ffffu) | 0x7f800000u)
                                       : ((w[e / 2] & 0xffff0000u) | 0x00007f80u);
                }
                a_even[u][i] = v;
            }
        }
        process(a_even, jb);
    }
#pragma unroll
    for (int st = 0; st < NS; ++st) {
        const uint64_t rest = __builtin_amdgcn_ballot_w64(cnt[st] > 0) & 0xffffffffull;
        if (rest) flush(st, rest);
    }
}

}  // namespace

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

hipError_t launch_l1(const float* Q, int64_t ldq, const float* X, int64_t ldx, void* qt,
                     int64_t rows, int64_t n, int d, int k, int S, float* lk, int* li,
                     hipStream_t stream) {
    {
        const int64_t total = (rows + kWave - 1) / kWave * ((d + 3) / 4) * kWave;
        knn_l1_transpose_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream>>>(
            Q, ldq, (int)rows, d, static_cast<f32x4*>(qt));
        hipError_t e0 = hipGetLastError();
        if (e0 != hipSuccess) return e0;
    }
    const size_t per_wave = (size_t)(2 * kWave * (kLowdCand + 1) + 2 * k + 2 * kWave) * 4;
    const size_t lds = per_wave * kLowdWaves;
    hipError_t e = raise_lds_limit(knn_l1_kernel, lds);
    if (e != hipSuccess) return e;
    int64_t split_len = (n + S - 1) / S;
    split_len = (split_len + 7) / 8 * 8;
    dim3 grid((unsigned)((rows + kLowdTileQ - 1) / kLowdTileQ), (unsigned)S);
    knn_l1_kernel<<<grid, dim3(kLowdTileQ), lds, stream>>>(static_cast<const f32x4*>(qt), X, ldx,
                                                           (int)rows, (int)n, d, k, S,
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

template <int D>
static hipError_t launch_lowd_bf16_d(const float* Q, int64_t ldq, const float* X, int64_t ldx,
                                     void* packed, int64_t rows, int64_t n, int k, int S,
                                     bool pack, int seed_cells, float* lk, int* li,
                                     hipStream_t stream) {
    constexpr int NM = FilterSlots<D>::kMfmas;
    unsigned* hdr = static_cast<unsigned*>(packed);
    uint4* Xp = reinterpret_cast<uint4*>(static_cast<unsigned char*>(packed) + kAlign);
    // the threshold seed's data follow the packed points: cell starts (ncell + 1 words), fill
    // cursors (ncell words), the points in cell order (16 bytes each)
    if (D > kSeedMaxD) seed_cells = 0;
    int ncell = 1;
    for (int t = 0; t < D && seed_cells > 0; ++t) ncell *= seed_cells;
    unsigned char* seed_base =
        static_cast<unsigned char*>(packed) + kAlign + align_up((uint64_t)n * 32 * NM);
    int* starts = reinterpret_cast<int*>(seed_base);
    int* cursor = reinterpret_cast<int*>(seed_base + align_up((uint64_t)(ncell + 1) * 4));
    f32x4* sorted = reinterpret_cast<f32x4*>(reinterpret_cast<unsigned char*>(cursor) +
                                             align_up((uint64_t)ncell * 4));
    const dim3 pgrid((unsigned)((n + 255) / 256));
    if (pack) {
        knn_bbox_init_kernel<<<dim3(1), dim3(64), 0, stream>>>(hdr);
        const unsigned bgrid = pgrid.x < 1024u ? pgrid.x : 1024u;
        knn_bbox_kernel<D><<<dim3(bgrid), dim3(256), 0, stream>>>(X, ldx, (int)n, hdr);
        knn_pack_bf16_kernel<D><<<pgrid, dim3(256), 0, stream>>>(X, ldx, (int)n, Xp, hdr);
        if constexpr (D <= kSeedMaxD) {
            if (seed_cells > 0) {
                knn_zero_ints_kernel<<<dim3((unsigned)((ncell + 255) / 256)), dim3(256), 0, stream>>>(
                    cursor, ncell);
                knn_cell_count_kernel<D><<<pgrid, dim3(256), 0, stream>>>(X, ldx, (int)n, hdr,
                                                                          seed_cells, cursor);
                knn_cell_scan_kernel<<<dim3(1), dim3(256), 0, stream>>>(cursor, ncell, starts);
                knn_cell_fill_kernel<D><<<pgrid, dim3(256), 0, stream>>>(
                    X, ldx, (int)n, hdr, seed_cells, starts, cursor, sorted);
            }
        }
        hipError_t e0 = hipGetLastError();
        if (e0 != hipSuccess) return e0;
    }
    if (rows == 0) return hipSuccess;
    const size_t per_wave = (size_t)(2 * kPbSets * 32 * kPbCand + 2 * kWave + 2 * k) * 4;
    const size_t lds = per_wave * 4;
    hipError_t e = raise_lds_limit(knn_lowd_bf16_kernel<D>, lds);
    if (e != hipSuccess) return e;
    int64_t split_len = (n + S - 1) / S;
    split_len = (split_len + 127) / 128 * 128;
    dim3 grid((unsigned)((rows + kPbTileQ - 1) / kPbTileQ), (unsigned)S);
    knn_lowd_bf16_kernel<D><<<grid, dim3(256), lds, stream>>>(
        Q, ldq, X, ldx, Xp, hdr, starts, sorted, seed_cells, (int)rows, (int)n, k, S, (int)split_len,
        lk, li);
    return hipGetLastError();
}

hipError_t launch_lowd_bf16(const float* Q, int64_t ldq, const float* X, int64_t ldx, void* packed,
                            int64_t rows, int64_t n, int d, int k, int S, bool pack, int seed_cells,
                            float* lk, int* li, hipStream_t stream) {
    switch (d) {
        case 1: return launch_lowd_bf16_d<1>(Q, ldq, X, ldx, packed, rows, n, k, S, pack, seed_cells, lk, li, stream);
        case 2: return launch_lowd_bf16_d<2>(Q, ldq, X, ldx, packed, rows, n, k, S, pack, seed_cells, lk, li, stream);
        case 3: return launch_lowd_bf16_d<3>(Q, ldq, X, ldx, packed, rows, n, k, S, pack, seed_cells, lk, li, stream);
        case 4: return launch_lowd_bf16_d<4>(Q, ldq, X, ldx, packed, rows, n, k, S, pack, seed_cells, lk, li, stream);
        case 5: return launch_lowd_bf16_d<5>(Q, ldq, X, ldx, packed, rows, n, k, S, pack, seed_cells, lk, li, stream);
        case 6: return launch_lowd_bf16_d<6>(Q, ldq, X, ldx, packed, rows, n, k, S, pack, seed_cells, lk, li, stream);
        case 7: return launch_lowd_bf16_d<7>(Q, ldq, X, ldx, packed, rows, n, k, S, pack, seed_cells, lk, li, stream);
        case 8: return launch_lowd_bf16_d<8>(Q, ldq, X, ldx, packed, rows, n, k, S, pack, seed_cells, lk, li, stream);
        default: return hipErrorInvalidValue;
    }
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

}  // namespace knn
