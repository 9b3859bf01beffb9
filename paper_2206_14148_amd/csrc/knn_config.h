// Compile-time shape constants shared by the host planner and the gfx950 kernels.
#pragma once
#include <cstdint>

namespace knn {

constexpr int kWave = 64;            // CDNA wavefront width
constexpr int kNumCU = 256;          // MI355X compute units (8 XCDs x 32)

// d <= kLowdMaxD: one query per lane, difference-form distances on the vector ALU.
constexpr int kLowdMaxD = 8;
constexpr int kLowdWaves = 4;                    // waves per workgroup
constexpr int kLowdTileQ = kLowdWaves * kWave;   // 256 query rows per workgroup
constexpr int kLowdUnroll = 8;                   // points examined per filter test
constexpr int kLowdCand = 16;                    // candidate slots per query (LDS)

// d <= kPmMaxD (and workspace room for packed points): MFMA filter + exact test, 4 waves, each
// wave owns 32 queries.
constexpr int kPmMaxD = 3;
constexpr int kPmTileQ = 128;
constexpr int kPmCand = 32;                      // candidate slots per query (LDS)

// the same with a bf16 filter, d <= kPbMaxD (room for 32 bytes per point up to d = 4, 64 above):
// each wave owns kPbSets sets of 32 queries, so one load of a block of points feeds kPbSets
// MFMAs per 16 K slots.
constexpr int kPbMaxD = 8;
constexpr int kPbSets = 2;
constexpr int kPbTileQ = 4 * 32 * kPbSets;       // query rows per workgroup
constexpr int kPbCand = 16;                      // candidate slots per query (LDS)
// threshold seed of that path, d <= kSeedMaxD: the points are counted into a grid of at most
// kSeedMaxCells cells, about 1.5 k points per cell (n * 2 / (3 k) cells): measured best between
// 1 k (own cell too often short of k points) and 2 k (looser bound) at n = 1e6, k = 16 and 64
constexpr int kSeedMaxD = 3;
constexpr int kSeedMaxCells = 32768;
constexpr int kSeedCellsPerPointNum = 2;
constexpr int kSeedCellsPerPointDen = 3;

// fp32 MFMA tiles of the SGPR sums (sgpr_kernels.hip): LDS staging of 128-row tiles
constexpr int kMfmaKC = 16;          // K columns staged in LDS per pipeline step
constexpr int kMfmaRowStride = 20;   // floats per staged row (16 + 4 pad, keeps 16 B alignment)

// d > kPbMaxD, and the cosine metric: bf16 matrix-core filter on rounded values + exact fp32 test,
// 8 waves, each wave owns 32 queries x 128 points.
constexpr int kSpWaves = 8;
constexpr int kSpTileQ = 32 * kSpWaves;
constexpr int kSpTileX = 128;
constexpr int kSpKC = 16;            // coordinates per chunk (one MFMA's K slots); a step takes 1..4
constexpr int kSpCand = 32;          // buffered point indices per query (LDS)
constexpr int kSpResidentMaxChunks = 16;  // d <= 256: the queries' B operands stay in registers
constexpr int kSpShareMin = 20;      // when the workgroup stops to empty buffers: all with at least this many entries
constexpr int kSpRoom = 4;           // a buffer with fewer free slots than this is emptied after the tile

// 8 < d <= 256, squared-Euclidean metric, many points, and room in the workspace for the points
// rounded to bf16 in matrix-core operand order: the same filter with the roles swapped.  A
// workgroup keeps the B operands of up to 16 sets of 32 queries in LDS for its whole life; each of
// its waves streams its own steps of 64 points from the packed copy straight into registers.
constexpr int kPkStep = 64;              // points per wave step (two MFMA row blocks)
constexpr int kPkMaxD = 256;
constexpr int kPkMaxSets = 16;           // 512 queries: one thread per query in the stops
constexpr int kPkCand = 32;              // buffered point indices per query (LDS)
constexpr int kPkShareMin = 20;          // a stop empties every buffer with at least this many entries
constexpr int kPkRoom = 4;               // a buffer with fewer free slots than this calls a stop
// (swept at d = 128, k = 100: 12 / 8 250.6 ms, 16 / 8 247.9, 16 / 4 248.0, 20 / 4 245.1, 24 / 4 246.3, 8 / 8 257.5)
constexpr int kPkLdsBytes = 160 * 1024;  // LDS of a gfx950 compute unit
constexpr int kPkSeedMin = 8192;         // sample of max(this, 8 k) points for the first thresholds
constexpr int64_t kPkMinPoints = 65536;  // fewer points: not worth packing
constexpr int64_t kPkSlabGrain = 8192;   // slabs of the packed copy are multiples of this many points
constexpr int64_t kPkMinQueries = 64;    // fewer queries: packing all points costs more than it saves
                                         // (n = 1e6, ms on path 6 against path 5: 64 queries d = 64, k = 10: 1.45 / 1.69;
                                         // d = 128, k = 100: 3.3 / 9.3; d = 256, k = 32: 3.0 / 5.6; 1000 queries: 1.9 / 2.1,
                                         // 4.1 / 15.0, 3.2 / 7.7)
constexpr int64_t kPkMinQueriesOneChunk = 2048;  // the same for d <= 16 (n = 1e6, d = 16, k = 10, ms on path 6 / path 5:
                                                 // 1000 queries 1.59 / 1.37, 1e4 2.21 / 3.40, 1e5 8.6 / 23.1)
// the chunk counts the kernel is instantiated for (1 .. 8 and the even ones up to 16); others are
// padded up with zero operands
constexpr inline int pk_padded_chunks(int d) {
    const int nch = (d + kSpKC - 1) / kSpKC;
    return nch <= 8 ? nch : (nch + 1) / 2 * 2;
}
// Waves per workgroup.  A wave's state is what it holds of a step - A operands (8 registers a
// chunk), norms, two accumulators - and fits 168 registers up to 8 chunks (d <= 128): three waves
// per SIMD; above, up to 256: two.  Every wave has its own merge scratch in LDS (2 k + 128 words),
// which the query sets pay for: where twelve of them would take more than half the LDS (k > 789)
// the workgroup has eight waves at every d (measured at d = 128, m = 2e4, n = 1e6, ms with 12 / 8
// waves: k = 10 .. 700 faster with twelve - 21.3 / 23.5, 17.0 / 19.8 at k = 256, 86.7 / 90.8 at
// k = 700 - but k = 1024, 4 sets instead of 6: 258 / 169).
constexpr inline int pk_waves(int nch_padded, int k) {
    return nch_padded <= 8 && 12 * (2 * kWave + 2 * (int64_t)k) * 4 <= kPkLdsBytes / 2 ? 12 : 8;
}
// LDS bytes of a workgroup with `sets` query sets: B operands, candidate buffers, seven words of
// state per query, the merge scratch of each wave, a few control words
constexpr inline int64_t pk_lds_bytes(int nch_padded, int k, int sets) {
    return (int64_t)sets * nch_padded * 1024 + (int64_t)sets * 32 * (kPkCand * 4 + 28) +
           (int64_t)pk_waves(nch_padded, k) * (2 * kWave + 2 * k) * 4 + (int64_t)pk_waves(nch_padded, k) * 256 + 256;
}
// most query sets a workgroup can hold (0: the shape does not fit)
constexpr inline int pk_max_sets(int nch_padded, int k) {
    int sets = 0;
    while (sets < kPkMaxSets && pk_lds_bytes(nch_padded, k, sets + 1) <= kPkLdsBytes) ++sets;
    return sets;
}
// Points whose filter keys give every query its first threshold on path 6 (knn_seed_kernel).
// The path needs n >= 4 x the smallest sample, max(8192, 8 k) points; the sample grows with k up
// to 160 k (at most a quarter of the points, at most 65536): a list's first threshold passes
// about k / sample of the points, and c4 (k = 100, ms for preparation + search on one box):
// 8192 points 4.7 + 218.2, 16000 6.5 + 211.8, 32000 10.2 + 207.2; c5 (k = 32): 4096 1.7 + 45.1,
// 8192 2.7 + 44.3, 16384 4.6 + 43.7.
constexpr inline int64_t pk_seed_points_min(int k) {
    const int64_t w = 8 * (int64_t)k;
    return ((w > kPkSeedMin ? w : kPkSeedMin) + kPkStep - 1) / kPkStep * kPkStep;
}
constexpr inline int64_t pk_seed_points(int k, int64_t n) {
    int64_t w = 160 * (int64_t)k;
    if (w > 65536) w = 65536;
    if (w > n / 4) w = n / 4;
    w = w / kPkStep * kPkStep;
    const int64_t least = pk_seed_points_min(k);
    return w > least ? w : least;
}

// d > 256, squared-Euclidean metric, many points, room for the points rounded to bf16:
// tiles of 512 queries x 128 points with both operands streamed from packed bf16 copies
// (knn_wide.hip).  A workgroup has 8 waves of two query sets each; a pipeline stage covers two
// chunks of 16 coordinates.
constexpr int kWdWaves = 8;
constexpr int kWdSets = 2;                            // query sets of 32 per wave
constexpr int kWdTileQ = 32 * kWdSets * kWdWaves;     // 512
constexpr int kWdTileX = 128;
constexpr int kWdW = 2;                               // chunks per pipeline stage
constexpr int kWdCand = 32;                           // buffered point indices per query (LDS)
constexpr int kWdShareMin = 20;                       // a stop empties every buffer with at least this many entries
constexpr int kWdRoom = 4;                            // a buffer with fewer free slots than this calls a stop
constexpr int64_t kWdMinPoints = 65536;               // fewer points or queries: the split path
constexpr int64_t kWdMinQueries = 16;                 // (n = 1e6, d = 784: one query 3.6 ms against the split path's
                                                      // 3.4, 16 queries 3.9 against 5.7, 256 queries 5.6 against 10.6)
constexpr int kWdMaxSplits = 64;                      // (a wave's lanes read the ranges' words of a query)
constexpr int kWdMaxK = 512;                          // larger k: the split path (LDS)
// LDS bytes of a workgroup: two stage buffers of the points' operands, two tiles of norms, the
// candidate buffers, seven words of state per query, a few control words, the merge scratch of each wave
constexpr inline int64_t wd_lds_bytes(int k) {
    return (int64_t)2 * kWdW * 4 * 1024 + 2 * kWdTileX * 4 + (int64_t)kWdTileQ * kWdCand * 4 +
           7 * kWdTileQ * 4 + 64 + (int64_t)kWdWaves * (2 * kWave + 2 * k) * 4;
}
static_assert(wd_lds_bytes(kWdMaxK) <= kPkLdsBytes, "the largest k must fit the LDS");

// Workgroups the chip holds at once (LDS-limited): the planner sizes launches in rounds of these.
constexpr int kLowdResidentWorkgroups = 4 * kNumCU;
constexpr int kSpResidentWorkgroups = kNumCU;   // 8 waves of up to 256 registers: one per CU
constexpr int kWarmupPointsPerK = 64;     // list warm-up of one point range, in point-equivalents per k
// the same for the low-d filter kernels, per k and per unit of 1 + ln(range / k): measured
// ~370 cycles per accepted pair against ~5 (bf16, 64 queries per wave) or ~7 (fp32 filter, 32
// queries per wave) cycles per scanned point and wave
constexpr int kWarmupPointsPerKBf16 = 4700;
constexpr int kWarmupPointsPerKFilter = 1800;
constexpr int kMaxSplits = 64;
constexpr int64_t kMaxPoints = ((int64_t)1 << 31) - 65536;
constexpr int64_t kMaxChunkRows = 1 << 22;  // keeps per-launch row counts and grids in int range
constexpr int kMinSplitPoints = 2048;    // a point range shorter than this is not worth a split
constexpr int kSpMinSplitPoints = 512;   // the same on the split path

// Private memory of knn_lowd_bf16_kernel (its out-of-line list merge takes the scratch pointers
// as a struct in the caller's stack frame, and up to d = 4 a few registers spill under the cap
// of 128): at most this many bytes per lane, and the bound the plan reports for it (64 lanes, up
// to 16 resident waves on each compute unit)
constexpr int kPbPrivateBytesPerLane = 64;
constexpr uint64_t kPbPrivateBytes = (uint64_t)kPbPrivateBytesPerLane * kWave * 16 * kNumCU;

constexpr uint64_t kAlign = 256;
constexpr inline uint64_t align_up(uint64_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

}  // namespace knn
