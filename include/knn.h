/*
 * knn.h - C ABI of the MI355X (gfx950) exact brute-force k-nearest-neighbour
 * library with a caller-given device-memory limit.
 *
 * Operation (paper section 5.2, "K-Nearest Neighbours"): for each of m query
 * points select the k closest of n data points.  Distances are squared
 * Euclidean.  The expansion of section 4.1 (sum x^2 + y^2 - 2xy, whose largest
 * operand is m x n instead of m x n x d) runs on the matrix cores and decides
 * which pairs can still matter to a query; those pairs are then evaluated in
 * the difference form in fp32, and the k winners once more in fp64.
 * The m x n matrix itself is never stored: it is produced tile by tile and
 * reduced on the fly to each query's k smallest, in the spirit of the
 * generator / reducer loop of section 4.3 (figure 2, algorithm 1).  All
 * library-owned device memory is one workspace whose size never exceeds the
 * caller's limit; section 4.4 notes that a limit-unaware allocator can still
 * overflow, so this library allocates nothing itself.
 *
 * Conventions shared by every entry point
 *   - Row-major fp32 matrices with a leading dimension in ELEMENTS (ld >= d).
 *   - "DEVICE" pointers are HIP device memory of the current device; "HOST"
 *     pointers are ordinary process memory.  The library never takes ownership
 *     of, frees or reallocates a pointer it is given.
 *   - Byte sizes with unit suffixes are DECIMAL (1GB = 1e9 bytes), as the
 *     paper's appendix example implies (125e6 fp64 values = "1GB").
 *   - Result rows are ascending by (distance, index): equal distances are
 *     ordered by the lower point index.  The paper leaves ties unspecified.
 *   - Inputs must be finite; behaviour for NaN/Inf entries is unspecified.
 */
#ifndef KNN_MI355X_H
#define KNN_MI355X_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    KNN_OK = 0,
    KNN_ERR_INVALID_ARG = 1,         /* null pointer, m<0, n<1, d<1, k<1, k>n, ld<d */
    KNN_ERR_MEM_LIMIT_TOO_SMALL = 2, /* limit below knn_plan_t.min_limit_bytes      */
    KNN_ERR_WORKSPACE_TOO_SMALL = 3, /* workspace_bytes < plan.workspace_bytes      */
    KNN_ERR_UNSUPPORTED = 4,         /* n > 2^31 - 65536 (int32 indices) or k > KNN_MAX_K */
    KNN_ERR_HIP = 5,                 /* a HIP call or kernel launch failed          */
    KNN_ERR_STATIC_SCRATCH_TOO_SMALL = 6 /* knn_search_static: no plan of this shape fits
                                        KNN_STATIC_SCRATCH_BYTES                     */
} knn_status;

#define KNN_MAX_K 1024

/*
 * Distance (section 5.2 and the appendix table report squared-Euclidean, L1 and cosine rows).
 *   KNN_METRIC_L2SQ    sum_t (q_t - x_t)^2
 *   KNN_METRIC_COSINE  max(0, 1 - <q, x> / (|q| |x|)); 1 if either vector is zero.
 *                      Always runs on the matrix-core path (path 5), whatever d.
 *   KNN_METRIC_L1      sum_t |q_t - x_t|.  Vector-ALU path 3, whatever d.
 */
typedef enum { KNN_METRIC_L2SQ = 0, KNN_METRIC_COSINE = 1, KNN_METRIC_L1 = 2 } knn_metric;

/* kernel families (knn_plan_t.path) */
#define KNN_PATH_LOWD 0 /* d <= 8: difference-form distances on the vector ALU  */
#define KNN_PATH_L1 3   /* L1 metric: absolute differences on the vector ALU, any d   */
#define KNN_PATH_LOWD_MFMA 2 /* d <= 3 and room for 16 n bytes of packed points:
                                matrix-core filter + the same exact test as path 0 */
#define KNN_PATH_LOWD_BF16 4 /* d <= 8 and room for 32 n bytes (d <= 4) or 64 n bytes: the filter
                                in bf16 pieces on points moved by their bounding box's midpoint,
                                same exact test */
#define KNN_PATH_MFMA_SPLIT 5 /* d > 8, and the cosine metric at any d: -2 Q X^T (plus norms)
                                 from the values rounded to bf16, one matrix-core product per
                                 coordinate, as a filter whose threshold allows for the
                                 rounding; exact fp32 test of the pairs that pass.  (Number 1
                                 was this path's fp32 matrix-core predecessor.) */

#define KNN_PATH_MFMA_PACKED 6 /* 8 < d <= 256 squared-Euclidean, d <= 256 cosine (on the rows x / |x|, whole copy
                                  only), m >= 64 (2048 up to d = 16), n >= 65536 and room for the
                                  points rounded to bf16 (32 bytes per point and 16 coordinates):
                                  the filter of path 5 with the queries resident in LDS and the
                                  points read from that copy in matrix-core operand order; the
                                  lists start under thresholds found from a sample's filter keys.
                                  Same exact test, same keys, same results as path 5. */
#define KNN_PATH_MFMA_WIDE 7 /* d > 256, squared-Euclidean, k <= 512, m >= 16, n >= 65536 and room for
                                the points rounded to bf16: the filter of path 5 on tiles of 512
                                queries x 128 points, both operands read from bf16 copies in
                                matrix-core operand order; a list without a bound takes its first
                                threshold from the filter keys of its first tile.  Same exact test,
                                same keys, same results as path 5. */

/*
 * The plan: how the call is cut into pieces (section 4.3: split the largest
 * splittable axis so that each piece stays under the limit; the loop body
 * produces a slice of the final result).  Queries are processed in q_chunks
 * chunks of at most chunk_rows rows; inside a chunk the points are cut into
 * n_splits ranges that are searched concurrently and merged afterwards.
 */
typedef struct {
    int64_t m, n;
    int32_t d, k;
    int32_t path;        /* KNN_PATH_*                                          */
    int32_t tile_q;      /* query rows per workgroup                            */
    int32_t tile_x;      /* data points per inner tile                          */
    int32_t n_splits;    /* ranges the point axis is cut into                   */
    int64_t chunk_rows;  /* query rows per chunk (multiple of tile_q, or m)     */
    int64_t q_chunks;    /* ceil(m / chunk_rows); 0 when m == 0                 */
    int32_t streams;     /* HIP streams used.  1: the caller's.  2 (more than one query chunk and
                            room for two sets of lists): merge and exact re-evaluation of a
                            chunk run on an internal stream while the next chunk is searched */
    int32_t seed_points; /* path 6: every query's first threshold comes from the filter keys of
                            this many points spread over X (no exact evaluation); else 0 */
    int32_t metric;      /* knn_metric                                          */
    int32_t seed_cells;  /* path 4, d <= 3: cells per axis of the grid the points are sorted
                            into to give every list a finite starting threshold (up to k = 32
                            the k-th smallest distance among a query's neighbouring cells,
                            above that the distance to their farthest corner); 0: none */
    uint64_t norms_bytes;     /* workspace: per-point data. path 2: packed points
                                 [x0 x1 x2 |x|^2]; path 5: squared norms (cosine: 1 / norm)
                                 and a 256-byte header; paths 6, 7: the same (norms padded to a
                                 multiple of 64 points) and slab_points points rounded to bf16
                                 (path 6, cosine: and as many words again, zeros); path 4: a 256-byte header, 32 bytes
                                 per point and 16 K slots, and with seed_cells the grid's cell
                                 starts and cursors and the points in cell order (16 bytes each);
                                 paths 0, 3: nothing                                   */
    uint64_t query_bytes;     /* workspace: per-query data of one chunk. path 5: the queries
                                 rounded to bf16 (32 bytes per row and 16 coordinates), their
                                 squared norms and shared thresholds (paths 6, 7: and a word per
                                 query and point range; path 7: rows rounded up to 64); path 3: the queries
                                 transposed in blocks of 64 rows (16 bytes per row and 4
                                 coordinates); else 0                                  */
    uint64_t lists_bytes;     /* workspace: partial k-lists of one chunk (streams == 2: of two) */
    uint64_t workspace_bytes; /* total device workspace needed, <= mem_limit    */
    uint64_t min_limit_bytes; /* smallest limit any plan for this shape fits in */
    uint64_t private_bytes;   /* device memory the plan's kernels use beside the workspace: their
                                 private (register spill) segment, which the HIP runtime provides.
                                 Bytes per lane x 64 lanes x the waves that can be resident on
                                 the 256 compute units.  0 on every path except path 4 (at
                                 most 64 bytes per lane, 16 waves per compute unit); the
                                 planner takes that path only where workspace_bytes +
                                 private_bytes stays within the limit.  Not part of
                                 workspace_bytes: the caller does not allocate it. */
    int64_t slab_points;      /* paths 6, 7: points the bf16 copy holds at a time (n rounded up to 64
                                 when all of them fit under the limit, else a multiple of 8192:
                                 the points are then packed and searched slab after slab, the
                                 lists carrying over); else 0 */
} knn_plan_t;

/*
 * knn_plan - pure host arithmetic, no HIP call; usable without a GPU.
 * Fills *out for the shape and limit given.  On KNN_ERR_MEM_LIMIT_TOO_SMALL
 * *out still carries min_limit_bytes.  m == 0 gives an empty plan and KNN_OK.
 */
knn_status knn_plan(int64_t m, int64_t n, int32_t d, int32_t k,
                    uint64_t mem_limit_bytes, knn_plan_t *out /* HOST */);

/* Same for a given metric (knn_plan is the squared-Euclidean case). */
knn_status knn_plan_metric(int64_t m, int64_t n, int32_t d, int32_t k, knn_metric metric,
                           uint64_t mem_limit_bytes, knn_plan_t *out /* HOST */);

/* workspace_bytes of the plan above, or 0 if there is none (error or m == 0). */
uint64_t knn_workspace_bytes(int64_t m, int64_t n, int32_t d, int32_t k,
                             uint64_t mem_limit_bytes);

/*
 * knn_search - the whole path: norms, tiled distances, running top-k, merge of
 * the point ranges, exact re-evaluation of the winners, output.
 *
 *   Q [m, d], ldq      DEVICE in, row-major fp32 queries
 *   X [n, d], ldx      DEVICE in, row-major fp32 data points (Q may alias X)
 *   k                  neighbours per query, 1 <= k <= min(n, KNN_MAX_K)
 *   mem_limit_bytes    upper bound for library-owned device memory.  It covers
 *                      the workspace only, not Q, X, idx, dist (the caller's).
 *   workspace          DEVICE scratch of workspace_bytes >= plan.workspace_bytes,
 *                      256-byte aligned, caller-allocated, contents undefined
 *                      before and after.  The library touches no byte beyond
 *                      plan.workspace_bytes and allocates nothing itself.
 *   idx  [m, k]        DEVICE out, int32, contiguous; point indices
 *   dist [m, k]        DEVICE out, fp32, contiguous; squared distances >= 0,
 *                      the fp64 difference-form value rounded to fp32
 *   hip_stream         hipStream_t (NULL = default stream).  The work is enqueued
 *                      there (with plan.streams == 2 partly on one internal stream
 *                      of default priority, forked from and joined back into
 *                      hip_stream with events); outputs are valid once the caller
 *                      has synchronised hip_stream.
 *
 * Argument and plan errors are returned synchronously and leave the outputs
 * untouched.  The result does not depend on mem_limit_bytes: every limit that
 * admits a plan gives bit-identical idx and dist.  Nor does it depend on how
 * the launch is scheduled: on path 5 the point ranges of a query tell each
 * other their current k-th distance while they run, which changes how many
 * pairs each of them looks at more closely, never which ones win.
 */
knn_status knn_search(const float *Q, int64_t ldq, const float *X, int64_t ldx,
                      int64_t m, int64_t n, int32_t d, int32_t k,
                      uint64_t mem_limit_bytes,
                      void *workspace, uint64_t workspace_bytes,
                      int32_t *idx, float *dist, void *hip_stream);

/*
 * knn_search_metric - knn_search for a given metric; every other argument as above.  For
 * KNN_METRIC_COSINE dist holds the fp64 cosine distance rounded to fp32, and the workspace
 * must satisfy knn_plan_metric(..., KNN_METRIC_COSINE, ...).
 */
knn_status knn_search_metric(const float *Q, int64_t ldq, const float *X, int64_t ldx,
                             int64_t m, int64_t n, int32_t d, int32_t k, knn_metric metric,
                             uint64_t mem_limit_bytes,
                             void *workspace, uint64_t workspace_bytes,
                             int32_t *idx, float *dist, void *hip_stream);

/* Plan and workspace size of this thread's last successful knn_search. */
knn_status knn_last_stats(knn_plan_t *plan_out /* HOST */,
                          uint64_t *peak_workspace_bytes /* HOST */);

/* Static string for a status code. */
const char *knn_status_string(knn_status s);

/*
 * knn_parse_size - "64MB", "1GB", "500KB", "123" -> bytes, DECIMAL multipliers
 * (KB = 1e3, MB = 1e6, GB = 1e9, TB = 1e12), matching the size options of the
 * paper's section 4.3 listing as read through the appendix example.
 * Returns KNN_ERR_INVALID_ARG for anything else.
 */
knn_status knn_parse_size(const char *text /* HOST */, uint64_t *bytes_out /* HOST */);

/*
 * knn_chunk_rows - rows of row_bytes each that fit in limit_bytes:
 * floor(limit_bytes / row_bytes), the chunk length rule of algorithm 1 as it
 * appears in the appendix example (1GB / (1e6 * 8 B) = 125 rows).
 */
int64_t knn_chunk_rows(uint64_t limit_bytes, uint64_t row_bytes);

/*
 * Kernel timing for benchmarks (section 5 reports elapsed time next to memory use).
 * knn_profile_enable(1) makes every later knn_search on this thread bracket its kernels
 * with HIP events recorded on the caller's stream: [norms] [search] [merge+refine] per
 * query chunk.  knn_profile_read waits for those events, adds the elapsed milliseconds of
 * all searches since the last read into the three HOST outputs (any may be NULL), stores
 * the number of search-kernel launches, and resets the tally.  Events are host objects; no
 * device memory is allocated.  Off by default; knn_profile_enable(0) frees the events.
 * The other entry points of the library use the same three slots: kmv_apply(_f64) puts its
 * main kernel into the search slot; sgpr_accumulate puts the kernel-matrix chunks into the
 * norms slot, the chunk products into the search slot and the products with y into the third.
 */
knn_status knn_profile_enable(int32_t on);
knn_status knn_profile_read(float *norms_ms /* HOST */, float *search_ms /* HOST */,
                            float *refine_ms /* HOST */, int64_t *search_launches /* HOST */);

/*
 * knn_measure_mfma_peak - what the matrix cores of this GPU sustain: a kernel of nothing but
 * MFMAs (one workgroup of 8 waves per compute unit, about 15 ms, run three times, the last two
 * timed with HIP events on hip_stream; the call waits for them).  Section 5 reports measured
 * times; a roofline fraction needs a peak to stand against, and under matrix-core load the chip
 * does not hold the clock its published peak assumes.
 *   dtype        0: v_mfma_f32_32x32x16_bf16 (published 2.5 PFLOP/s), 1: v_mfma_f32_32x32x2_f32
 *                (published 157.3 TFLOP/s)
 *   scratch      DEVICE, at least 512 KiB, contents undefined afterwards
 *   tflops_out   HOST
 */
knn_status knn_measure_mfma_peak(int32_t dtype, void *scratch /* DEVICE */, uint64_t scratch_bytes,
                                 void *hip_stream, float *tflops_out /* HOST */);

/*
 * Data points in HOST memory, streamed through the workspace.
 *
 * Section 5.1 reports data set sizes "far beyond" the device's memory capacity once every
 * intermediate is bounded.  Here the n x d matrix X itself may stay in host memory: it is cut
 * into blocks of block_rows rows; block b+1 is copied host-to-device into one of two staging
 * buffers (inside the workspace, so they count against the limit) by an internal copy stream
 * while block b is searched on the caller's stream with the kernels of knn_search; each block's
 * k best per query (exact fp64 re-evaluation included, done while the block is on the device)
 * are folded into the running result held in idx / dist.
 *
 * The plan: workspace = staging (two buffers of block_rows x d fp32, one if n_blocks == 1)
 *           + block_out (one block's indices, list keys and fp64 distances and the running
 *           result's fp64 distances, m x k each) + the workspace of `inner`,
 *           the knn_plan_metric of one full block under inner_limit_bytes.
 */
typedef struct {
    int64_t m, n;
    int32_t d, k;
    int32_t metric, reserved;
    int64_t block_rows;         /* rows of X per staged block (the last may be shorter) */
    int64_t n_blocks;
    uint64_t staging_bytes;
    uint64_t block_out_bytes;
    uint64_t inner_limit_bytes; /* limit handed to the plan of a block */
    uint64_t workspace_bytes;   /* <= mem_limit_bytes */
    uint64_t min_limit_bytes;
    knn_plan_t inner;           /* plan of one full block: (m, block_rows, d, min(k, block_rows)) */
} knn_host_plan_t;

/* HOST.  Errors as knn_plan_metric. */
knn_status knn_plan_host_x(int64_t m, int64_t n, int32_t d, int32_t k, knn_metric metric,
                           uint64_t mem_limit_bytes, knn_host_plan_t *out /* HOST */);

/*
 * knn_search_host_x - knn_search_metric with X in HOST memory.
 *   X [n, d], ldx   HOST in, row-major fp32; pinned memory (hipHostMalloc) lets the copies
 *                   overlap the search, pageable memory works but serialises them.  Must stay
 *                   valid and unchanged until the caller has synchronised hip_stream.
 *   Q, idx, dist, workspace   DEVICE, as in knn_search; workspace_bytes >=
 *                   knn_plan_host_x(...).workspace_bytes
 * Result: bit for bit what knn_search_metric gives on a device copy of X.  The blocks' winners
 * are folded in the order of their list keys (key, index) - the order in which a resident
 * search merges its point ranges - with their fp64 distances carried along, and the final
 * order by (fp64 distance, index) is written when the last block is in; until then dist holds
 * list keys.
 * The call enqueues work on hip_stream and on one internal stream (created on first use, default
 * priority) ordered against it with events; it returns without waiting for the GPU when X is
 * pinned.  It allocates no device memory.  Calls of one host thread that share a workspace
 * must be made on the same hip_stream or be synchronised by the caller.
 */
knn_status knn_search_host_x(const float *Q, int64_t ldq, const float *X /* HOST */, int64_t ldx,
                             int64_t m, int64_t n, int32_t d, int32_t k, knn_metric metric,
                             uint64_t mem_limit_bytes, void *workspace, uint64_t workspace_bytes,
                             int32_t *idx, float *dist, void *hip_stream);

/*
 * knn_search_static - knn_search for callers that cannot allocate device memory and have no
 * workspace to hand over: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same kernels, same result (bit for bit) as knn_search; the workspace is a
 * buffer of KNN_STATIC_SCRATCH_BYTES that is part of the library's device image (one copy per
 * GPU the library runs on, held until the process ends), and the plan is the one knn_plan gives
 * for mem_limit_bytes = KNN_STATIC_SCRATCH_BYTES (all of it on hip_stream: no internal stream
 * is created).  The call allocates nothing (no hipMalloc,
 * hipFree or allocating library routine); the first call on a device looks up that device's
 * address of the buffer.
 *   Q, X, idx, dist, hip_stream   as in knn_search (DEVICE pointers of the current device)
 * Errors: those of knn_search, and KNN_ERR_STATIC_SCRATCH_TOO_SMALL (outputs untouched) when
 * the smallest plan of the shape needs more than KNN_STATIC_SCRATCH_BYTES - for d > 8 that is
 * 4 n bytes of norms plus one query tile of lists, so n up to about 8e6.
 * Every call on a GPU uses that GPU's one buffer: calls that overlap in time on one GPU (other
 * streams, other host threads) race and must be serialised by the caller.  The buffer keeps
 * the last call's contents; every kernel initialises what it reads.
 */
#define KNN_STATIC_SCRATCH_BYTES 33554432ull /* 32 MiB */
knn_status knn_search_static(const float *Q, int64_t ldq, const float *X, int64_t ldx,
                             int64_t m, int64_t n, int32_t d, int32_t k,
                             int32_t *idx, float *dist, void *hip_stream);

/* Last HIP error text seen by this thread ("" if none). */
const char *knn_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* KNN_MI355X_H */
