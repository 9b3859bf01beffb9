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

constexpr uint64_t kAlign = 256;
constexpr inline uint64_t align_up(uint64_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

}  // namespace knn
