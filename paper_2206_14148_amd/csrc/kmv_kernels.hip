// gfx950 (CDNA4, MI355X) kernels for the kernel matrix-vector product  y = K v  with the
// squared-exponential kernel (paper section 5.1; kernel formula in the appendix).  The
// n x m matrix K is the intermediate that section 4.3 keeps from being materialised: here
// a lane owns one row of K, produces its entries a few at a time in registers, multiplies
// them by v and adds them up, so K costs no memory at all.
//
// Summation order of one y_i, whatever the launch shape: points in ascending j inside
// groups of 64 (fp32, one fused multiply-add per point), groups in ascending order (fp64),
// point ranges in ascending order (fp64).
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <type_traits>
#include <utility>

#include "kmv_kernels.h"
#include "knn_config.h"
#include "knn_device.h"

namespace kmv {

namespace {

using knn::f32x16;
using knn::f32x4;
using knn::kInf;
using knn::load_row4;
using knn::mask_row4;

__global__ __launch_bounds__(256) void kmv_scaled_norms_kernel(const float* __restrict__ Z,
                                                               int64_t ldz, int64_t m, int d,
                                                               float c2, float* __restrict__ zn) {
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    for (int64_t j = wave; j < m; j += nwaves) {
        const float* p = Z + j * ldz;
        float acc = 0.f;
        for (int t = lane; t < d; t += 64) acc = fmaf(p[t], p[t], acc);
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) acc += __shfl_xor(acc, o);
        if (lane == 0) zn[j] = -c2 * acc;
    }
}

__global__ __launch_bounds__(256) void kmv_zero_kernel(double* __restrict__ y, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) y[i] = 0.0;
}

__global__ __launch_bounds__(256) void kmv_reduce_kernel(const double* __restrict__ partials, int S,
                                                         int64_t n, double* __restrict__ y) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    double acc = partials[i];
    for (int s = 1; s < S; ++s) acc += partials[(int64_t)s * n + i];
    y[i] = acc;
}

// ---------------------------------------------------------------------------------------
// d <= 8: one row x_i per lane in registers; the points z_j and the values v_j are the same
// for the whole wave, so they arrive through scalar loads and cost no vector work.  Per pair:
// d subtractions, d multiply-adds, one multiply by -c2, one hardware exp2, one multiply-add.
// ---------------------------------------------------------------------------------------
template <int D, bool CONTIG>
__global__ __launch_bounds__(kLowdTileRows) void kmv_lowd_kernel(
    const float* __restrict__ X, int64_t ldx, const float* __restrict__ Z, int64_t ldz_arg,
    const float* __restrict__ v, int n, int m, int split_len, float negc2, double variance,
    double* __restrict__ out) {
    constexpr int U = 8;
    const int64_t ldz = CONTIG ? (int64_t)D : ldz_arg;
    const int s = blockIdx.y;
    const int i = blockIdx.x * kLowdTileRows + threadIdx.x;
    const bool active = i < n;
    float x[D];
#pragma unroll
    for (int t = 0; t < D; ++t) x[t] = active ? X[(int64_t)i * ldx + t] : 0.f;

    auto term = [&](const float* __restrict__ zp, float vj, float part) {
        float df = x[0] - zp[0];
        float sq = df * df;
#pragma unroll
        for (int t = 1; t < D; ++t) {
            df = x[t] - zp[t];
            sq = fmaf(df, df, sq);
        }
        return fmaf(__builtin_amdgcn_exp2f(sq * negc2), vj, part);
    };

    const int j0 = s * split_len;  // split_len is a multiple of kGroup
    const int j1 = min(m, j0 + split_len);
    const float* zp = Z + (int64_t)j0 * ldz;  // uniform: read with scalar loads
    const float* vp = v + j0;
    double total = 0.0;
    int j = j0;
    for (; j + kGroup <= j1; j += kGroup) {
        float part = 0.f;
        for (int g = 0; g < kGroup; g += U, zp += U * ldz, vp += U) {
#pragma unroll
            for (int u = 0; u < U; ++u) part = term(zp + u * ldz, vp[u], part);
        }
        total += (double)part;
    }
    if (j < j1) {
        float part = 0.f;
        for (; j < j1; ++j, zp += ldz, ++vp) part = term(zp, vp[0], part);
        total += (double)part;
    }
    if (active) out[(int64_t)s * n + i] = variance * total;
}

// ---------------------------------------------------------------------------------------
// d > 8: a workgroup of 4 waves owns 128 rows of X and walks its point range in tiles of 128
// points, on the bf16 matrix cores.  Points are the M side and rows of X the N side of
// v_mfma_f32_32x32x16_bf16, so the 16 accumulator values a lane holds per 32x32 block belong
// to ONE row x_i (column = lane % 32) and 16 different points.  The accumulators start at
// -c2 |z_j|^2 and receive (2 c2 x_i) . z_j; adding -c2 |x_i|^2 gives the exponent
// -c2 |x_i - z_j|^2 of the expansion in section 4.1.
//
// Every fp32 value is cut into three bf16 pieces, hi + mid + lo = the value exactly (3 x 8
// significant bits); of the nine piece products of a pair of values the six of weight >= 2^-16
// are kept, each exact in the fp32 accumulator, so a product is off by about 2^-23 of its
// size, the rounding an fp32 multiply would have made.  Six bf16 MFMAs per 16 coordinates
// take 192 cycles against 512 for the sixteen v_mfma_f32_32x32x2_f32 of an fp32 contraction.
// The points are cut while they are staged into LDS (double buffered, the global loads of
// step s+2 in flight during step s).  NCH > 0 (d <= 16 NCH): the pieces of this lane's row are
// made once and stay in registers.  NCH = 0: the rows of X stream through LDS like the points.
// Inputs must be finite with squares that fit fp32.
// ---------------------------------------------------------------------------------------
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ void split3_pair(float a, float b, unsigned& hi, unsigned& mid,
                                            unsigned& lo) {
    const f32x2 p = {a, b};
    const bf16x2 hb = __builtin_convertvector(p, bf16x2);
    const f32x2 r1 = p - __builtin_convertvector(hb, f32x2);
    const bf16x2 mb = __builtin_convertvector(r1, bf16x2);
    const f32x2 r2 = r1 - __builtin_convertvector(mb, f32x2);
    const bf16x2 lb = __builtin_convertvector(r2, bf16x2);
    hi = __builtin_bit_cast(unsigned, hb);
    mid = __builtin_bit_cast(unsigned, mb);
    lo = __builtin_bit_cast(unsigned, lb);
}

__device__ __forceinline__ void split3_row8(const f32x4& x0, const f32x4& x1, uint4& hi, uint4& mid,
                                            uint4& lo) {
    split3_pair(x0[0], x0[1], hi.x, mid.x, lo.x);
    split3_pair(x0[2], x0[3], hi.y, mid.y, lo.y);
    split3_pair(x1[0], x1[1], hi.z, mid.z, lo.z);
    split3_pair(x1[2], x1[3], hi.w, mid.w, lo.w);
}

template <int NCH, bool ALIGNED>
__global__ __launch_bounds__(256, 2) void kmv_mfma_kernel(
    const float* __restrict__ X, int64_t ldx, const float* __restrict__ Z, int64_t ldz,
    const float* __restrict__ v, const float* __restrict__ zn, int n, int m, int d, int split_len,
    float c2, double variance, double* __restrict__ out) {
    constexpr int TR = kMfmaTileRows, TZ = 128, KC = kMfmaKC;
    constexpr bool RES = NCH > 0;
    // One piece of a staged tile: per block of 32 rows the 16-byte words of the rows' first
    // halves (coordinates 0..7 of the chunk), 8 words of padding, then the second halves.  A
    // wave's read of an MFMA operand (lane = row, upper lanes the second half) then covers
    // consecutive words, and the two words a pair of staging threads writes for one row lie
    // 640 bytes apart, in different halves of the banks: no bank conflicts either way.
    constexpr int BLK = 32 + 8 + 32;       // words per block of 32 rows
    constexpr int HALF = 32 + 8;           // offset of the second halves inside a block
    constexpr int PIECE = (TZ / 32) * BLK;  // words of one piece of a staged tile (TR == TZ)
    static_assert(TR == TZ, "one staging layout for both operands");
    extern __shared__ __align__(16) unsigned char smem[];
    uint4* zs = reinterpret_cast<uint4*>(smem);      // [2][3 pieces][PIECE]
    float* zns = reinterpret_cast<float*>(zs + 2 * 3 * PIECE);  // [2][TZ] accumulator start values
    float* vs = zns + 2 * TZ;                        // [2][TZ] pieces of v
    uint4* xs = reinterpret_cast<uint4*>(vs + 2 * TZ);  // NCH = 0 only: [2][3 pieces][PIECE]
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int i32 = lane & 31;
    const int h = lane >> 5;
    const int s = blockIdx.y;
    const int wg_row0 = blockIdx.x * TR;
    const int my_row = wave * 32 + i32;
    const int r = wg_row0 + my_row;
    const bool active = r < n;
    const float bscale = 2.f * c2;
    const int nch = RES ? NCH : (d + KC - 1) / KC;

    // this lane's row: -c2 |x_i|^2, summed in ascending t, and (NCH > 0) the pieces of
    // 2 c2 x_i for the coordinates 8h .. 8h+7 of every chunk
    float nxn = 0.f;
    bf16x8 bx[RES ? NCH : 1][3];
    {
        const int64_t rr = active ? r : n - 1;
        if (active) {
            const float* p = X + rr * ldx;
            float acc = 0.f;
            for (int t = 0; t < d; ++t) acc = fmaf(p[t], p[t], acc);
            nxn = -c2 * acc;
        }
        if constexpr (RES) {
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                const int col = c * KC + h * 8;
                uint4 ph, pm, pl;
                split3_row8(
                    mask_row4(load_row4<ALIGNED>(X, ldx, rr, n, col, d), active, col, d, bscale),
                    mask_row4(load_row4<ALIGNED>(X, ldx, rr, n, col + 4, d), active, col + 4, d, bscale),
                    ph, pm, pl);
                bx[c][0] = __builtin_bit_cast(bf16x8, ph);
                bx[c][1] = __builtin_bit_cast(bf16x8, pm);
                bx[c][2] = __builtin_bit_cast(bf16x8, pl);
            }
        }
    }

    const int j0 = s * split_len;  // split_len is a multiple of TZ
    const int j1 = min(m, j0 + split_len);
    const int ntiles = (j1 > j0) ? (j1 - j0 + TZ - 1) / TZ : 0;
    const int total = ntiles * nch;

    const int srow = tid >> 1;        // staging: this thread cuts 8 coordinates of one row
    const int scol = (tid & 1) * 8;

    struct Staged {
        f32x4 z0, z1, x0, x1;
        float znv, vv;
    };
    // Branch-free on purpose: every call issues the same loads from clamped addresses, so the
    // compiler can count the newer loads still in flight when an older set is consumed.
    auto fetch = [&](int step, Staged& g) {
        const int tile = step / nch;
        const int c = step - tile * nch;
        const int col = c * KC + scol;
        const int64_t jr = (int64_t)j0 + (int64_t)tile * TZ + srow;
        g.z0 = load_row4<ALIGNED>(Z, ldz, jr, j1, col, d);
        g.z1 = load_row4<ALIGNED>(Z, ldz, jr, j1, col + 4, d);
        if constexpr (!RES) {
            g.x0 = load_row4<ALIGNED>(X, ldx, (int64_t)wg_row0 + srow, n, col, d);
            g.x1 = load_row4<ALIGNED>(X, ldx, (int64_t)wg_row0 + srow, n, col + 4, d);
        }
        const int64_t jj = (int64_t)j0 + (int64_t)tile * TZ + (tid & (TZ - 1));
        const int64_t jc = jj < j1 ? jj : j1 - 1;
        g.znv = zn[jc];
        g.vv = v[jc];
    };
    auto stash = [&](int step, const Staged& g) {
        const int tile = step / nch;
        const int c = step - tile * nch;
        const int buf = step & 1;
        const int col = c * KC + scol;
        const int64_t jr = (int64_t)j0 + (int64_t)tile * TZ + srow;
        uint4 ph, pm, pl;
        split3_row8(mask_row4(g.z0, jr < j1, col, d, 1.f), mask_row4(g.z1, jr < j1, col + 4, d, 1.f),
                    ph, pm, pl);
        const int slot = (srow >> 5) * BLK + (tid & 1) * HALF + (srow & 31);
        uint4* zb = zs + buf * 3 * PIECE + slot;
        zb[0] = ph;
        zb[PIECE] = pm;
        zb[2 * PIECE] = pl;
        if constexpr (!RES) {
            const bool ok = wg_row0 + srow < n;
            split3_row8(mask_row4(g.x0, ok, col, d, bscale), mask_row4(g.x1, ok, col + 4, d, bscale),
                        ph, pm, pl);
            uint4* xb = xs + buf * 3 * PIECE + slot;
            xb[0] = ph;
            xb[PIECE] = pm;
            xb[2 * PIECE] = pl;
        }
        if (c == 0 && tid < TZ) {
            const int64_t jj = (int64_t)j0 + (int64_t)tile * TZ + tid;
            // points past the range: exponent -inf and weight 0, so they add exactly 0
            zns[(tile & 1) * TZ + tid] = jj < j1 ? g.znv : -kInf;
            vs[(tile & 1) * TZ + tid] = jj < j1 ? g.vv : 0.f;
        }
    };

    f32x16 acc[4];
    double sum = 0.0;

    Staged set_even, set_odd;
    if (total > 0) {
        fetch(0, set_even);
        stash(0, set_even);
    }
    if (total > 1) fetch(1, set_odd);
    __syncthreads();

    // cc: the chunk, tbc: tile & 1 -- integral constants when NCH > 0 (so bx[c] is a register),
    // plain ints otherwise; parc: step & 1, always a constant (which staging set is whose)
    auto run_step = [&](int step, auto cc, auto parc, auto tbc) {
        constexpr int buf = decltype(parc)::value;
        const int c = cc;
        const int tbuf = tbc;
        Staged& mine = buf ? set_odd : set_even;
        const Staged& next = buf ? set_even : set_odd;
        fetch(step + 2 < total ? step + 2 : total - 1, mine);  // past the end: a harmless re-load

        if (c == 0) {
            const float* zt = zns + tbuf * TZ;
#pragma unroll
            for (int pb = 0; pb < 4; ++pb) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const f32x4 w = *reinterpret_cast<const f32x4*>(zt + pb * 32 + g * 8 + h * 4);
                    acc[pb][g * 4 + 0] = w[0];
                    acc[pb][g * 4 + 1] = w[1];
                    acc[pb][g * 4 + 2] = w[2];
                    acc[pb][g * 4 + 3] = w[3];
                }
            }
        }
        {
            bf16x8 b[3];
            if constexpr (RES) {
                constexpr int C = decltype(cc)::value;
                b[0] = bx[C][0];
                b[1] = bx[C][1];
                b[2] = bx[C][2];
            } else {
                const uint4* xb = xs + buf * 3 * PIECE + wave * BLK + h * HALF + i32;
#pragma unroll
                for (int p = 0; p < 3; ++p) b[p] = __builtin_bit_cast(bf16x8, xb[p * PIECE]);
            }
            const uint4* zb = zs + buf * 3 * PIECE + h * HALF + i32;
            bf16x8 a[4][3];
#pragma unroll
            for (int pb = 0; pb < 4; ++pb)
#pragma unroll
                for (int p = 0; p < 3; ++p)
                    a[pb][p] = __builtin_bit_cast(bf16x8, zb[p * PIECE + pb * BLK]);
#pragma unroll
            for (int pb = 0; pb < 4; ++pb) {
                // smallest products first: lo.hi, hi.lo, mid.mid, then mid.hi, hi.mid, hi.hi
                acc[pb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[pb][2], b[0], acc[pb], 0, 0, 0);
                acc[pb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[pb][0], b[2], acc[pb], 0, 0, 0);
                acc[pb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[pb][1], b[1], acc[pb], 0, 0, 0);
                acc[pb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[pb][1], b[0], acc[pb], 0, 0, 0);
                acc[pb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[pb][0], b[1], acc[pb], 0, 0, 0);
                acc[pb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[pb][0], b[0], acc[pb], 0, 0, 0);
                if (pb == 1 && step + 1 < total) stash(step + 1, next);
            }
        }

        if (c == nch - 1) {
            // This lane's 64 points of the tile, in ascending j: block pb, register group g,
            // element e is point pb*32 + g*8 + h*4 + e.  The two halves of the wave hold
            // interleaved runs of 4 points; they are added at the very end.
            const float* vt = vs + tbuf * TZ;
            float part = 0.f;
#pragma unroll
            for (int pb = 0; pb < 4; ++pb) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const f32x4 w = *reinterpret_cast<const f32x4*>(vt + pb * 32 + g * 8 + h * 4);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float arg = fminf(acc[pb][g * 4 + e] + nxn, 0.f);
                        part = fmaf(__builtin_amdgcn_exp2f(arg), w[e], part);
                    }
                }
            }
            sum += (double)part;
        }
        __syncthreads();
    };
    using std::integral_constant;
    if constexpr (RES) {
        // two tiles per trip, so that the parity of a step is a constant whatever NCH is
        auto run_tile = [&](int tile, auto ttc) {
            constexpr int tt = decltype(ttc)::value;
            run_step(tile * NCH, integral_constant<int, 0>{}, integral_constant<int, (tt * NCH) & 1>{}, ttc);
            if constexpr (NCH > 1)
                run_step(tile * NCH + 1, integral_constant<int, 1>{},
                         integral_constant<int, (tt * NCH + 1) & 1>{}, ttc);
            if constexpr (NCH > 2)
                run_step(tile * NCH + 2, integral_constant<int, 2>{},
                         integral_constant<int, (tt * NCH + 2) & 1>{}, ttc);
            if constexpr (NCH > 3)
                run_step(tile * NCH + 3, integral_constant<int, 3>{},
                         integral_constant<int, (tt * NCH + 3) & 1>{}, ttc);
            static_assert(NCH <= 4, "one run_step per chunk is written out up to four");
        };
        for (int tile0 = 0; tile0 < ntiles; tile0 += 2) {
            run_tile(tile0, integral_constant<int, 0>{});
            if (tile0 + 1 < ntiles) run_tile(tile0 + 1, integral_constant<int, 1>{});
        }
    } else {
        int tile = 0, c = 0;
        auto advance = [&]() {
            if (++c == nch) {
                c = 0;
                ++tile;
            }
        };
        for (int step = 0; step < total; step += 2) {
            run_step(step, c, integral_constant<int, 0>{}, tile & 1);
            advance();
            if (step + 1 < total) {
                run_step(step + 1, c, integral_constant<int, 1>{}, tile & 1);
                advance();
            }
        }
    }
    const double other = __shfl_xor(sum, 32);
    if (active && h == 0) out[(int64_t)s * n + r] = variance * (sum + other);
}

// ---------------------------------------------------------------------------------------
// fp64 variant, d <= 8: the low-d kernel with every operation in fp64 and the library's exp.
// The sum runs over j ascending in one fp64 accumulator.
// ---------------------------------------------------------------------------------------
template <int D, bool CONTIG>
__global__ __launch_bounds__(kLowdTileRows) void kmv_lowd_f64_kernel(
    const double* __restrict__ X, int64_t ldx, const double* __restrict__ Z, int64_t ldz_arg,
    const double* __restrict__ v, int n, int m, int split_len, double negc, double variance,
    double* __restrict__ out) {
    constexpr int U = 4;
    const int64_t ldz = CONTIG ? (int64_t)D : ldz_arg;
    const int s = blockIdx.y;
    const int i = blockIdx.x * kLowdTileRows + threadIdx.x;
    const bool active = i < n;
    double x[D];
#pragma unroll
    for (int t = 0; t < D; ++t) x[t] = active ? X[(int64_t)i * ldx + t] : 0.0;

    auto term = [&](const double* __restrict__ zp, double vj, double total) {
        double df = x[0] - zp[0];
        double sq = df * df;
#pragma unroll
        for (int t = 1; t < D; ++t) {
            df = x[t] - zp[t];
            sq = fma(df, df, sq);
        }
        return fma(exp(sq * negc), vj, total);
    };

    const int j0 = s * split_len;
    const int j1 = min(m, j0 + split_len);
    const double* zp = Z + (int64_t)j0 * ldz;  // uniform: read with scalar loads
    const double* vp = v + j0;
    double total = 0.0;
    int j = j0;
    for (; j + U <= j1; j += U, zp += U * ldz, vp += U) {
#pragma unroll
        for (int u = 0; u < U; ++u) total = term(zp + u * ldz, vp[u], total);
    }
    for (; j < j1; ++j, zp += ldz, ++vp) total = term(zp, vp[0], total);
    if (active) out[(int64_t)s * n + i] = variance * total;
}

// ---------------------------------------------------------------------------------------
// fp64 variant, any d: one row per lane; a group of 8 wave-uniform points (scalar loads)
// keeps one running squared distance each while the row is walked in chunks of 4 columns,
// so a row value is loaded once per 8 points.  Columns in ascending order, points in
// ascending order, one fp64 accumulator.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(kLowdTileRows) void kmv_anyd_f64_kernel(
    const double* __restrict__ X, int64_t ldx, const double* __restrict__ Z, int64_t ldz,
    const double* __restrict__ v, int n, int m, int d, int split_len, double negc, double variance,
    double* __restrict__ out) {
    constexpr int P = 8, TC = 4;
    const int s = blockIdx.y;
    const int i = blockIdx.x * kLowdTileRows + threadIdx.x;
    const bool active = i < n;
    const double* __restrict__ xrow = X + (int64_t)(active ? i : n - 1) * ldx;  // in bounds for idle lanes
    const int j0 = s * split_len;
    const int j1 = min(m, j0 + split_len);
    const double* zp = Z + (int64_t)j0 * ldz;  // uniform
    const double* vp = v + j0;
    double total = 0.0;
    int j = j0;
    for (; j + P <= j1; j += P, zp += P * ldz, vp += P) {
        double sq[P];
#pragma unroll
        for (int p = 0; p < P; ++p) sq[p] = 0.0;
        int c = 0;
        for (; c + TC <= d; c += TC) {
            double xr[TC];
#pragma unroll
            for (int t = 0; t < TC; ++t) xr[t] = xrow[c + t];
#pragma unroll
            for (int p = 0; p < P; ++p) {
#pragma unroll
                for (int t = 0; t < TC; ++t) {
                    const double df = xr[t] - zp[p * ldz + c + t];
                    sq[p] = fma(df, df, sq[p]);
                }
            }
        }
        for (; c < d; ++c) {
            const double xr = xrow[c];
#pragma unroll
            for (int p = 0; p < P; ++p) {
                const double df = xr - zp[p * ldz + c];
                sq[p] = fma(df, df, sq[p]);
            }
        }
#pragma unroll
        for (int p = 0; p < P; ++p) total = fma(exp(sq[p] * negc), vp[p], total);
    }
    for (; j < j1; ++j, zp += ldz, ++vp) {
        double sq = 0.0;
        for (int c = 0; c < d; ++c) {
            const double df = xrow[c] - zp[c];
            sq = fma(df, df, sq);
        }
        total = fma(exp(sq * negc), vp[0], total);
    }
    if (active) out[(int64_t)s * n + i] = variance * total;
}

int64_t split_length(int64_t m, int S, int tile) {
    int64_t len = (m + S - 1) / S;
    return (len + tile - 1) / tile * tile;
}

}  // namespace

hipError_t launch_scaled_norms(const float* Z, int64_t ldz, int64_t m, int d, float c2, float* zn,
                               hipStream_t stream) {
    if (m == 0) return hipSuccess;
    int64_t blocks = (m + 3) / 4;
    if (blocks > 16384) blocks = 16384;
    kmv_scaled_norms_kernel<<<dim3((unsigned)blocks), dim3(256), 0, stream>>>(Z, ldz, m, d, c2, zn);
    return hipGetLastError();
}

hipError_t launch_zero(double* y, int64_t n, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    kmv_zero_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream>>>(y, n);
    return hipGetLastError();
}

hipError_t launch_reduce(const double* partials, int S, int64_t n, double* y, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    kmv_reduce_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream>>>(partials, S, n, y);
    return hipGetLastError();
}

template <int D>
static hipError_t launch_lowd_d(const float* X, int64_t ldx, const float* Z, int64_t ldz,
                                const float* v, int64_t n, int64_t m, float c2, double variance,
                                int S, double* out, hipStream_t stream) {
    const dim3 grid((unsigned)((n + kLowdTileRows - 1) / kLowdTileRows), (unsigned)S);
    const int split_len = (int)split_length(m, S, kGroup);
    if (ldz == D) {
        kmv_lowd_kernel<D, true><<<grid, dim3(kLowdTileRows), 0, stream>>>(
            X, ldx, Z, ldz, v, (int)n, (int)m, split_len, -c2, variance, out);
    } else {
        kmv_lowd_kernel<D, false><<<grid, dim3(kLowdTileRows), 0, stream>>>(
            X, ldx, Z, ldz, v, (int)n, (int)m, split_len, -c2, variance, out);
    }
    return hipGetLastError();
}

hipError_t launch_lowd(const float* X, int64_t ldx, const float* Z, int64_t ldz, const float* v,
                       int64_t n, int64_t m, int d, float c2, double variance, int S, double* out,
                       hipStream_t stream) {
    if (n == 0) return hipSuccess;
    switch (d) {
        case 1: return launch_lowd_d<1>(X, ldx, Z, ldz, v, n, m, c2, variance, S, out, stream);
        case 2: return launch_lowd_d<2>(X, ldx, Z, ldz, v, n, m, c2, variance, S, out, stream);
        case 3: return launch_lowd_d<3>(X, ldx, Z, ldz, v, n, m, c2, variance, S, out, stream);
        case 4: return launch_lowd_d<4>(X, ldx, Z, ldz, v, n, m, c2, variance, S, out, stream);
        case 5: return launch_lowd_d<5>(X, ldx, Z, ldz, v, n, m, c2, variance, S, out, stream);
        case 6: return launch_lowd_d<6>(X, ldx, Z, ldz, v, n, m, c2, variance, S, out, stream);
        case 7: return launch_lowd_d<7>(X, ldx, Z, ldz, v, n, m, c2, variance, S, out, stream);
        case 8: return launch_lowd_d<8>(X, ldx, Z, ldz, v, n, m, c2, variance, S, out, stream);
        default: return hipErrorInvalidValue;
    }
}

template <int D>
static hipError_t launch_f64_d(const double* X, int64_t ldx, const double* Z, int64_t ldz,
                               const double* v, int64_t n, int64_t m, double negc, double variance,
                               int S, double* out, hipStream_t stream) {
    const dim3 grid((unsigned)((n + kLowdTileRows - 1) / kLowdTileRows), (unsigned)S);
    const int split_len = (int)split_length(m, S, kGroup);
    if (ldz == D) {
        kmv_lowd_f64_kernel<D, true><<<grid, dim3(kLowdTileRows), 0, stream>>>(
            X, ldx, Z, ldz, v, (int)n, (int)m, split_len, negc, variance, out);
    } else {
        kmv_lowd_f64_kernel<D, false><<<grid, dim3(kLowdTileRows), 0, stream>>>(
            X, ldx, Z, ldz, v, (int)n, (int)m, split_len, negc, variance, out);
    }
    return hipGetLastError();
}

hipError_t launch_f64(const double* X, int64_t ldx, const double* Z, int64_t ldz, const double* v,
                      int64_t n, int64_t m, int d, double negc, double variance, int S, double* out,
                      hipStream_t stream) {
    if (n == 0) return hipSuccess;
    switch (d) {
        case 1: return launch_f64_d<1>(X, ldx, Z, ldz, v, n, m, negc, variance, S, out, stream);
        case 2: return launch_f64_d<2>(X, ldx, Z, ldz, v, n, m, negc, variance, S, out, stream);
        case 3: return launch_f64_d<3>(X, ldx, Z, ldz, v, n, m, negc, variance, S, out, stream);
        case 4: return launch_f64_d<4>(X, ldx, Z, ldz, v, n, m, negc, variance, S, out, stream);
        case 5: return launch_f64_d<5>(X, ldx, Z, ldz, v, n, m, negc, variance, S, out, stream);
        case 6: return launch_f64_d<6>(X, ldx, Z, ldz, v, n, m, negc, variance, S, out, stream);
        case 7: return launch_f64_d<7>(X, ldx, Z, ldz, v, n, m, negc, variance, S, out, stream);
        case 8: return launch_f64_d<8>(X, ldx, Z, ldz, v, n, m, negc, variance, S, out, stream);
        default: break;
    }
    const dim3 grid((unsigned)((n + kLowdTileRows - 1) / kLowdTileRows), (unsigned)S);
    const int split_len = (int)split_length(m, S, kGroup);
    kmv_anyd_f64_kernel<<<grid, dim3(kLowdTileRows), 0, stream>>>(
        X, ldx, Z, ldz, v, (int)n, (int)m, d, split_len, negc, variance, out);
    return hipGetLastError();
}

hipError_t launch_mfma(const float* X, int64_t ldx, const float* Z, int64_t ldz, const float* v,
                       const float* zn, int64_t n, int64_t m, int d, float c2, double variance, int S,
                       double* out, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    const dim3 grid((unsigned)((n + kMfmaTileRows - 1) / kMfmaTileRows), (unsigned)S);
    const int split_len = (int)split_length(m, S, 128);
    const bool aligned = (reinterpret_cast<uintptr_t>(X) % 16 == 0) &&
                         (reinterpret_cast<uintptr_t>(Z) % 16 == 0) && (ldx % 4 == 0) &&
                         (ldz % 4 == 0) && (d % 4 == 0);
    const int nch = (d + kMfmaKC - 1) / kMfmaKC;
    const int variant = nch <= kMfmaResidentChunks ? nch : 0;
    // staged pieces of a tile of points (and of rows, when they stream), start values, v
    const size_t tile_bytes = (size_t)2 * 3 * (128 / 32) * (32 + 8 + 32) * 16;
    const size_t lds = tile_bytes * (variant == 0 ? 2 : 1) + 4 * 128 * 4;
    hipError_t err = hipSuccess;
    auto go = [&](auto kernel) {
        err = knn::raise_lds_limit(kernel, lds);
        if (err != hipSuccess) return;
        kernel<<<grid, dim3(256), lds, stream>>>(X, ldx, Z, ldz, v, zn, (int)n, (int)m, d, split_len,
                                                 c2, variance, out);
        err = hipGetLastError();
    };
    switch (variant * 2 + (aligned ? 1 : 0)) {
        case 0: go(kmv_mfma_kernel<0, false>); break;
        case 1: go(kmv_mfma_kernel<0, true>); break;
        case 2: go(kmv_mfma_kernel<1, false>); break;
        case 3: go(kmv_mfma_kernel<1, true>); break;
        case 4: go(kmv_mfma_kernel<2, false>); break;
        case 5: go(kmv_mfma_kernel<2, true>); break;
        case 6: go(kmv_mfma_kernel<3, false>); break;
        case 7: go(kmv_mfma_kernel<3, true>); break;
        case 8: go(kmv_mfma_kernel<4, false>); break;
        default: go(kmv_mfma_kernel<4, true>); break;
    }
    return err;
}

}  // namespace kmv
