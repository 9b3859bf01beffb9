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
hipError_t launch_row_norms(const float* X, int64_t ldx, int64_t n, int d, bool inverse, float* xn,
                            hipStream_t stream);

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
//   launch_max_norm      hdr word 0 = max of xn[0..n) (hdr: kAlign bytes)
//   launch_split_queries qs = the B operands of `rows` queries: ceil(d / 16) * 64 bytes per row;
//                        tsh = [rows] words, the thresholds the ranges share: set to +inf, or
//                        (reset_thresholds false) kept from an earlier search of other points
//                        for the same queries and the same k
//   launch_split         the search; qn = squared norms of the chunk's queries (fp32, [rows]);
//                        cosine: xn holds 1 / |x| and the keys are -2 q.x / |x|
hipError_t launch_max_norm(const float* xn, int64_t n, void* hdr, hipStream_t stream);
hipError_t launch_split_queries(const float* Q, int64_t ldq, int64_t rows, int d, void* qs,
                                void* tsh, bool reset_thresholds, hipStream_t stream);
hipError_t launch_split(const float* Q, int64_t ldq, const float* X, int64_t ldx, const void* qs,
                        const float* qn, void* tsh, const float* xn, const void* hdr, bool cosine,
                        int64_t rows, int64_t n, int d, int k, int S, float* lk, int* li,
                        hipStream_t stream);

// Merge the S lists of each row, re-evaluate the k winners in fp64 (metric: knn_metric value),
// order by (distance, index) and write idx / dist rows.
hipError_t launch_merge_refine(const float* Q, int64_t ldq, const float* X, int64_t ldx,
                               int64_t rows, int64_t n, int d, int k, int S, int metric,
                               const float* lk, const int* li, int32_t* idx, float* dist,
                               hipStream_t stream);

// Running result of a search over blocks of points: idx/dist [rows][k] (ascending by fp32
// distance) absorb one block's [rows][kb] results, whose indices get `offset` added.  On equal
// distances the running entries (earlier blocks, lower indices) stay in front.  first != 0:
// the running result is empty (the block becomes the result, padded with +inf / INT_MAX).
hipError_t launch_fold_block(const int32_t* bidx, const float* bdist, int kb, int64_t offset,
                             int first, int64_t rows, int k, int32_t* idx, float* dist,
                             hipStream_t stream);

}  // namespace knn
