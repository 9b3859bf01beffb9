// Internal launcher interface between the C ABI (api.hip) and the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace knn {

// Partial k-lists of one query chunk live in the workspace as two arrays of
// rows * S * k entries: keys (fp32) and point indices (int32).  The list of chunk row r
// and point range s starts at ((r * S) + s) * k and is ascending by (key, index).

// xn[j] = sum_t X[j][t]^2 in fp32 (the sum x^2 term of paper section 4.1); inverse = true writes
// 1 / sqrt(that) instead (0 for a zero row), the row scale of the cosine metric.
// resid != null (a word zeroed beforehand, launch_header_init): it also gets the bits of
// max_j |x_j - bf16(x_j)|^2.
hipError_t launch_row_norms(const float* X, int64_t ldx, int64_t n, int d, bool inverse, float* xn,
                            hipStream_t stream, void* resid = nullptr);

// d <= kLowdMaxD: key = fp32 difference-form squared distance.
hipError_t launch_lowd(const float* Q, int64_t ldq, const float* X, int64_t ldx, int64_t rows,
                       int64_t n, int d, int k, int S, float* lk, int* li, hipStream_t stream);

// L1 metric, any d: key = fp32 sum of absolute differences.  qt = room for the transposed
// queries, ceil(rows / 64) * 64 * ceil(d / 4) * 16 bytes (written here, read by the search).
hipError_t launch_l1(const float* Q, int64_t ldq, const float* X, int64_t ldx, void* qt,
                     int64_t rows, int64_t n, int d, int k, int S, float* lk, int* li,
                     hipStream_t stream);

// d <= kPmMaxD with room for the packed points: the same keys as launch_lowd, found through an
// MFMA filter.  `packed` = kAlign bytes (max ||x||^2 word) + 16 n bytes ([x0 x1 x2 ||x||^2] per
// point); pack = true (re)builds it from X first; rows == 0 only packs.
hipError_t launch_lowd_mfma(const float* Q, int64_t ldq, const float* X, int64_t ldx, void* packed,
                            int64_t rows, int64_t n, int d, int k, int S, bool pack, float* lk,
                            int* li, hipStream_t stream);

// d <= kPbMaxD with room for 32 n bytes (d <= 4) or 64 n bytes: the same keys again, found through
// a bf16 MFMA filter on points and queries moved by the midpoint of the points' bounding box.
// `packed` = kAlign bytes (header: max moved norm, bounding box) + the packed points; pack /
// rows == 0 as above.  seed_cells > 0 (d <= kSeedMaxD only): the area continues with
// seed_cells^d ints, the points counted into a grid of that many cells per axis, from which
// every query's list gets a finite starting threshold.
hipError_t launch_lowd_bf16(const float* Q, int64_t ldq, const float* X, int64_t ldx, void* packed,
                            int64_t rows, int64_t n, int d, int k, int S, bool pack, int seed_cells,
                            float* lk, int* li, hipStream_t stream);

// d > kPbMaxD, and the cosine metric at any d: bf16 matrix-core filter on split values, exact
// fp32 test of what passes it (knn_split.hip).
//   launch_header_init   hdr words 0 and 1 = 0 (hdr: kAlign bytes)
//   launch_max_norm      hdr word 0 = max of xn[0..n), after launch_header_init
//   launch_split_queries qs = the B operands of `rows` queries: ceil(d / 16) * 64 bytes per row;
//                        tsh = [rows] words, the thresholds the ranges share: set to +inf, or
//                        (reset_thresholds false) kept from an earlier search of other points
//                        for the same queries and the same k
//   launch_split         the search; qn = squared norms of the chunk's queries (fp32, [rows]);
//                        cosine: xn holds 1 / |x| and the keys are -2 q.x / |x|
hipError_t launch_header_init(void* hdr, hipStream_t stream);
hipError_t launch_max_norm(const float* xn, int64_t n, void* hdr, hipStream_t stream);
hipError_t launch_split_queries(const float* Q, int64_t ldq, int64_t rows, int d, void* qs,
                                void* tsh, bool reset_thresholds, hipStream_t stream);
hipError_t launch_split(const float* Q, int64_t ldq, const float* X, int64_t ldx, const void* qs,
                        const float* qn, void* tsh, const float* xn, const void* hdr, bool cosine,
                        int64_t rows, int64_t n, int d, int k, int S, float* lk, int* li,
                        hipStream_t stream);

// 8 < d <= 256 with the points rounded to bf16 in the workspace (knn_packed.hip).
//   launch_pack_operands  xp = `points` points from j_first on (j_first and points multiples of
//                         64; rows past n are zero), pk_padded_chunks(d) x 32 bytes per point;
//                         scale = -2 packs queries as B operands (n = their number); xn != null
//                         (16-byte aligned rows only): the same pass also writes the rows'
//                         squared norms to xn[j_first ..] and raises hdr word 1 to the largest
//                         squared norm of a rounding residual, as launch_row_norms would;
//                         row_scale != null (aligned rows, hdr != null): row j is multiplied by
//                         row_scale[j] before it is rounded (the cosine metric's x / |x|), and
//                         the residuals (and norms, if xn != null) are those of the scaled rows
//   launch_pad_norms      xn[n .. next multiple of 64) = +inf
//   launch_packed         the search of points [j_first, j_end) (j_first a multiple of 64) out of
//                         the copy xp whose first point is slab_first, for queries whose B
//                         operands, norms and shared thresholds are those of launch_split;
//                         sets = query sets of 32 per workgroup (<= pk_max_sets); the lists of
//                         ranges < init_from continue (an earlier launch filled them from
//                         other points), the others start empty; tsr = [rows][S] words, set to
//                         0xff800000 (+inf) beforehand: the key at position ceil(k / S) - 1 of
//                         every range's list, through which the ranges bound each other.
//                         Rows must be 16-byte aligned (packed_rows_aligned).
//                         Cosine metric: rn = 1 / |x| of all points, xp packed with row_scale =
//                         rn, xn = zeros (+inf from n to the next multiple of 64), and
//                         launch_seed_thresholds with cosine = true.
hipError_t launch_pack_operands(const float* X, int64_t ldx, int64_t n, int d, int64_t j_first,
                                int64_t points, void* xp, hipStream_t stream, float scale = 1.f,
                                float* xn = nullptr, void* hdr = nullptr, const float* row_scale = nullptr);
hipError_t launch_pad_norms(float* xn, int64_t n, hipStream_t stream);
//   launch_seed_thresholds  tsh[r] = min(tsh[r], an upper bound of query r's k-th smallest distance
//                         found from the filter keys of seed_points points spread over the packed
//                         copy xp (of all n points)); after launch_split_queries, the queries'
//                         norms and the header
hipError_t launch_seed_thresholds(const float* Q, int64_t ldq, const void* xp, const float* xn, const void* qs,
                                  const float* qn, void* tsh, const void* hdr, int64_t rows, int64_t n, int d,
                                  int k, int64_t seed_points, hipStream_t stream, bool cosine = false);
bool packed_rows_aligned(const float* Q, int64_t ldq, const float* X, int64_t ldx, int d);
hipError_t launch_packed(const float* Q, int64_t ldq, const float* X, int64_t ldx, const void* xp,
                         int64_t slab_first, const void* qs, const float* qn, void* tsh, void* tsr,
                         const float* xn, const void* hdr, int64_t rows, int64_t n, int d, int k, int S,
                         int sets, int64_t j_first, int64_t j_end, int init_from, float* lk, int* li,
                         hipStream_t stream, const float* rn = nullptr);
// d > 256 with both operands rounded to bf16 in the workspace (knn_wide.hip).
//   launch_wide   the search of points [j_first, j_end) (j_first a multiple of 64) out of the copy
//                 xp (launch_pack_operands) that holds slab_points points from slab_first on, for
//                 queries whose B operands qp were packed by launch_pack_operands with scale -2
//                 (rows rounded up to 64), qn / tsh / tsr / xn / hdr / init_from as for
//                 launch_packed.  S <= 64.  Rows must be 16-byte aligned (packed_rows_aligned).
hipError_t launch_wide(const float* Q, int64_t ldq, const float* X, int64_t ldx, const void* xp,
                       int64_t slab_first, int64_t slab_points, const void* qp, const float* qn, void* tsh,
                       void* tsr, const float* xn, const void* hdr, int64_t rows, int64_t n, int d, int k,
                       int S, int64_t j_first, int64_t j_end, int init_from, float* lk, int* li,
                       hipStream_t stream);
// p[0 .. count) = value (32-bit words)
hipError_t launch_fill_words(void* p, int64_t count, unsigned value, hipStream_t stream);

// Merge the S lists of each row, re-evaluate the k winners in fp64 (metric: knn_metric value),
// order by (distance, index) and write idx / dist rows.  d64 != null (one block of a search over
// blocks of points): the winners are left in the order of their list keys, dist gets the KEYS and
// d64 the fp64 distances, for launch_fold_keyed.
hipError_t launch_merge_refine(const float* Q, int64_t ldq, const float* X, int64_t ldx,
                               int64_t rows, int64_t n, int d, int k, int S, int metric,
                               const float* lk, const int* li, int32_t* idx, float* dist,
                               hipStream_t stream, double* d64 = nullptr);

// Running result of a search over blocks of points: idx / key / d64 [rows][k], ascending by
// (list key, index) - the order in which a resident search merges its point ranges - absorb one
// block's [rows][kb] results in the same order, whose indices get `offset` added.  first != 0: the
// running result is empty.  launch_order_final then orders every row by (fp64 distance, index)
// and writes the distances rounded to fp32 over the keys.
hipError_t launch_fold_keyed(const int32_t* bidx, const float* bkey, const double* bd64, int kb,
                             int64_t offset, int first, int64_t rows, int k, int32_t* idx, float* key,
                             double* d64, hipStream_t stream);
hipError_t launch_order_final(int64_t rows, int k, int32_t* idx, float* dist, const double* d64,
                              hipStream_t stream);

}  // namespace knn
