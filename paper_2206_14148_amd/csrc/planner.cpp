// Host-side planner: turns (m, n, d, k, mem_limit) into tile, split and chunk sizes.
//
// Paper section 4.3 / algorithm 1: the largest splittable axis is cut so that each piece
// stays under the size limit and the loop body yields a slice of the result.  For kNN the
// query axis is freely splittable (rows are independent) and the point axis becomes
// splittable because the reduction is a mergeable running top-k instead of a sort.
// Section 4.4: every concurrently live buffer counts, so the plan sums all library-owned
// device memory (norms + every partial list of a chunk) and keeps the sum under the limit.
#include <cctype>
#include <cmath>
#include <cstring>

#include "../../include/knn.h"
#include "knn_config.h"

using namespace knn;

extern "C" int64_t knn_chunk_rows(uint64_t limit_bytes, uint64_t row_bytes) {
    if (row_bytes == 0) return 0;
    uint64_t rows = limit_bytes / row_bytes;
    return rows > (uint64_t)INT64_MAX ? INT64_MAX : (int64_t)rows;
}

extern "C" knn_status knn_parse_size(const char* text, uint64_t* bytes_out) {
    if (!text || !bytes_out) return KNN_ERR_INVALID_ARG;
    while (*text && isspace((unsigned char)*text)) ++text;
    if (!isdigit((unsigned char)*text)) return KNN_ERR_INVALID_ARG;
    uint64_t value = 0;
    while (isdigit((unsigned char)*text)) {
        uint64_t digit = (uint64_t)(*text - '0');
        if (value > (UINT64_MAX - digit) / 10) return KNN_ERR_INVALID_ARG;
        value = value * 10 + digit;
        ++text;
    }
    char unit[4] = {0, 0, 0, 0};
    int len = 0;
    while (*text && !isspace((unsigned char)*text)) {
        if (len >= 2) return KNN_ERR_INVALID_ARG;
        unit[len++] = (char)toupper((unsigned char)*text++);
    }
    while (*text && isspace((unsigned char)*text)) ++text;
    if (*text) return KNN_ERR_INVALID_ARG;
    uint64_t mult;
    if (len == 0 || !strcmp(unit, "B")) mult = 1ull;
    else if (!strcmp(unit, "KB")) mult = 1000ull;
    else if (!strcmp(unit, "MB")) mult = 1000000ull;
    else if (!strcmp(unit, "GB")) mult = 1000000000ull;
    else if (!strcmp(unit, "TB")) mult = 1000000000000ull;
    else return KNN_ERR_INVALID_ARG;
    if (value > UINT64_MAX / mult) return KNN_ERR_INVALID_ARG;
    *bytes_out = value * mult;
    return KNN_OK;
}

extern "C" const char* knn_status_string(knn_status s) {
    switch (s) {
        case KNN_OK: return "ok";
        case KNN_ERR_INVALID_ARG: return "invalid argument";
        case KNN_ERR_MEM_LIMIT_TOO_SMALL: return "memory limit below the smallest feasible plan";
        case KNN_ERR_WORKSPACE_TOO_SMALL: return "workspace smaller than the plan requires";
        case KNN_ERR_UNSUPPORTED: return "unsupported size (n >= 2^31 or k > KNN_MAX_K)";
        case KNN_ERR_HIP: return "HIP runtime error";
        case KNN_ERR_STATIC_SCRATCH_TOO_SMALL:
            return "no plan of this shape fits the static scratch buffer (KNN_STATIC_SCRATCH_BYTES)";
    }
    return "unknown status";
}

namespace {

// bytes of the two list arrays (keys fp32, indices int32) for `rows` queries and S ranges
uint64_t lists_bytes_for(uint64_t rows, uint64_t S, uint64_t k) {
    return 2 * align_up(rows * S * k * 4);
}

// per-query data of a chunk besides its lists.  kind 1 (path 5): the queries' split B operands
// (qrow = 32 bytes per 16 coordinates), their squared norms and the thresholds their point
// ranges share (a word each); kind 2 (L1 path): the queries transposed in blocks of 64 rows
// (qrow = 16 bytes per 4 coordinates); kind 0: nothing.
uint64_t query_bytes_for(uint64_t rows, uint64_t qrow, int kind, uint64_t S = 1) {
    if (kind == 1) return align_up(rows * qrow) + 2 * align_up(rows * 4);
    // kind 3 (path 6): as kind 1, and a word per query and point range
    if (kind == 3) return align_up(rows * qrow) + 2 * align_up(rows * 4) + align_up(rows * S * 4);
    // kind 4 (path 7): as kind 3 with the B operands of rows rounded up to 64
    if (kind == 4) return align_up((rows + 63) / 64 * 64 * qrow) + 2 * align_up(rows * 4) + align_up(rows * S * 4);
    if (kind == 2) return align_up((rows + 63) / 64 * 64 * qrow);
    return 0;
}

// largest row count whose lists (S ranges) and per-query data fit in `avail` bytes
int64_t rows_fitting(uint64_t avail, uint64_t S, uint64_t k, uint64_t qrow, int kind) {
    if (kind == 0) {
        // 2 * align_up(x) <= avail  <=>  x <= floor(floor(avail / 2) / kAlign) * kAlign
        uint64_t usable = avail / 2 / kAlign * kAlign;
        return knn_chunk_rows(usable, S * k * 4);
    }
    auto need = [&](uint64_t rows) {
        return lists_bytes_for(rows, S, k) + query_bytes_for(rows, qrow, kind, S);
    };
    const uint64_t per_row =
        2 * S * k * 4 + qrow + (kind == 1 ? 8 : 0) + (kind == 3 || kind == 4 ? 8 + S * 4 : 0);  // exact, roundings aside
    // the roundings (six to kAlign, one to 64 rows) add less than this: start below the
    // answer, then step up to it
    const uint64_t slack = 6 * kAlign + 64 * qrow;
    uint64_t rows = avail > slack ? (avail - slack) / per_row : 0;
    while (need(rows + 1) <= avail) ++rows;
    return (int64_t)rows;
}

// More than one query chunk: the merge and exact re-evaluation of a chunk can run on a second
// stream while the next chunk is searched, if each of the two has lists of its own.  Both sets
// are live at once, so both count (section 4.4): the chunk is shortened until two sets of lists
// fit beside everything else; where not even one query tile fits twice, the chunks stay serial.
void plan_two_streams(knn_plan_t* out, int64_t m, uint64_t mem_limit_bytes, uint64_t qrow, int qkind) {
    if (out->q_chunks <= 1) return;
    const uint64_t S = (uint64_t)out->n_splits, k = (uint64_t)out->k;
    const uint64_t fixed = out->norms_bytes + out->private_bytes;
    const int64_t tile = out->tile_q;
    auto need = [&](int64_t rows) {
        return fixed + query_bytes_for((uint64_t)rows, qrow, qkind, S) + 2 * lists_bytes_for((uint64_t)rows, S, k);
    };
    int64_t rows = out->chunk_rows / 2 / tile * tile;
    while (rows >= tile && need(rows) > mem_limit_bytes) rows -= tile;
    if (rows < tile) return;
    while (rows + tile < m && rows + tile <= kMaxChunkRows && need(rows + tile) <= mem_limit_bytes) rows += tile;
    out->streams = 2;
    out->chunk_rows = rows;
    out->q_chunks = (m + rows - 1) / rows;
    out->query_bytes = query_bytes_for((uint64_t)rows, qrow, qkind, S);
    out->lists_bytes = 2 * lists_bytes_for((uint64_t)rows, S, k);
    out->workspace_bytes = out->norms_bytes + out->query_bytes + out->lists_bytes;
}

}  // namespace

extern "C" knn_status knn_plan(int64_t m, int64_t n, int32_t d, int32_t k,
                               uint64_t mem_limit_bytes, knn_plan_t* out) {
    return knn_plan_metric(m, n, d, k, KNN_METRIC_L2SQ, mem_limit_bytes, out);
}

extern "C" knn_status knn_plan_metric(int64_t m, int64_t n, int32_t d, int32_t k, knn_metric metric,
                                      uint64_t mem_limit_bytes, knn_plan_t* out) {
    if (!out) return KNN_ERR_INVALID_ARG;
    memset(out, 0, sizeof(*out));
    if (metric != KNN_METRIC_L2SQ && metric != KNN_METRIC_COSINE && metric != KNN_METRIC_L1)
        return KNN_ERR_INVALID_ARG;
    out->metric = (int32_t)metric;
    if (m < 0 || n < 1 || d < 1 || k < 1 || (int64_t)k > n) return KNN_ERR_INVALID_ARG;
    // int32 indices, with headroom so that range ends rounded up to a tile stay representable
    if (n > kMaxPoints || k > KNN_MAX_K) return KNN_ERR_UNSUPPORTED;
    out->m = m;
    out->n = n;
    out->d = d;
    out->k = k;
    out->streams = 1;
    // the cosine keys come from the matrix-core kernels only
    // (lowd also stands for the L1 kernel: same workgroup shape, no per-point workspace; its
    // queries are kept transposed per chunk)
    const bool lowd = (d <= kLowdMaxD && metric == KNN_METRIC_L2SQ) || metric == KNN_METRIC_L1;
    // d > 8, or the cosine metric at any d: the bf16 filter on split values + exact test
    const bool split = !lowd;
    // smallest plan of all: the vector-ALU path (no per-point workspace) or a matrix-core path
    out->path = metric == KNN_METRIC_L1 ? KNN_PATH_L1 : (lowd ? KNN_PATH_LOWD : KNN_PATH_MFMA_SPLIT);
    out->tile_q = lowd ? kLowdTileQ : kSpTileQ;
    out->tile_x = lowd ? kLowdUnroll : kSpTileX;
    out->norms_bytes = lowd ? 0 : align_up((uint64_t)n * 4) + (split ? kAlign : 0);
    const bool l1 = metric == KNN_METRIC_L1;
    const int qkind = split ? 1 : (l1 ? 2 : 0);
    const uint64_t qrow = split ? 32ull * (((uint64_t)d + kSpKC - 1) / kSpKC)
                                : (l1 ? 16ull * (((uint64_t)d + 3) / 4) : 0);
    {
        const int64_t t0 = out->tile_q;
        const int64_t min_rows = m < t0 ? (m > 0 ? m : 1) : t0;
        out->min_limit_bytes = out->norms_bytes + lists_bytes_for((uint64_t)min_rows, 1, (uint64_t)k) +
                               query_bytes_for((uint64_t)min_rows, qrow, qkind);
    }
    if (m == 0) return KNN_OK;
    if (mem_limit_bytes < out->min_limit_bytes) return KNN_ERR_MEM_LIMIT_TOO_SMALL;
    if (d <= kPbMaxD && metric == KNN_METRIC_L2SQ) {
        // the matrix-core filters need the points packed into the workspace; take one when the
        // limit has room for that and at least one query tile of lists
        if (d <= kPmMaxD) {
            const uint64_t packed = kAlign + align_up((uint64_t)n * 16);
            const int64_t min_rows = m < kPmTileQ ? m : kPmTileQ;
            if (mem_limit_bytes >= packed + lists_bytes_for((uint64_t)min_rows, 1, (uint64_t)k)) {
                out->path = KNN_PATH_LOWD_MFMA;
                out->tile_q = kPmTileQ;
                out->tile_x = 32;
                out->norms_bytes = packed;
            }
        }
        // with 32 bytes per point and 16 K slots (one MFMA up to d = 4, two up to d = 8) the
        // filter runs in bf16 pieces, four times cheaper per MFMA
        const uint64_t per_point = 32ull * ((3 * (uint64_t)d + 3 + 15) / 16);
        const uint64_t packed16 = kAlign + align_up((uint64_t)n * per_point);
        const int64_t min_rows16 = m < kPbTileQ ? m : kPbTileQ;
        // (section 4.4: everything that is live counts - this kernel uses a little private
        // memory, which the runtime provides beside the workspace)
        const uint64_t priv = kPbPrivateBytes;
        if (mem_limit_bytes >= packed16 + priv + lists_bytes_for((uint64_t)min_rows16, 1, (uint64_t)k)) {
            out->path = KNN_PATH_LOWD_BF16;
            out->private_bytes = priv;
            out->tile_q = kPbTileQ;
            out->tile_x = 32;
            out->norms_bytes = packed16;
            // threshold seed: a grid with about 1.5 k points per cell, when the grid is worth
            // having (two cells or more per axis) and its counts fit as well
            if (d <= kSeedMaxD) {
                const int64_t want = n * kSeedCellsPerPointNum / ((int64_t)kSeedCellsPerPointDen * k);
                int64_t G = 1;
                auto cells_of = [&](int64_t g) {
                    int64_t c = 1;
                    for (int t = 0; t < d; ++t) c *= g;
                    return c;
                };
                while (cells_of(G + 1) <= want && cells_of(G + 1) <= kSeedMaxCells) ++G;
                // cell starts, fill cursors and the points in cell order (16 bytes each)
                const uint64_t seed = align_up(((uint64_t)cells_of(G) + 1) * 4) +
                                      align_up((uint64_t)cells_of(G) * 4) + align_up((uint64_t)n * 16);
                if (G >= 2 && mem_limit_bytes >= packed16 + priv + seed +
                                                     lists_bytes_for((uint64_t)min_rows16, 1, (uint64_t)k)) {
                    out->seed_cells = (int32_t)G;
                    out->norms_bytes = packed16 + seed;
                }
            }
        }
    }
    // 8 < d <= 256 and many points: with room for the points rounded to bf16 in operand order
    // the search runs with the queries resident in LDS (knn_packed.hip).  Its workspace is that
    // of path 5 plus the packed copy, so a call whose rows turn out not to be 16-byte aligned
    // still runs under this plan, on path 5's kernel.
    // The cosine metric runs there too, on a copy of the rows x / |x|, with one more array of n
    // words (what the sums start from; the first holds 1 / |x|) and the whole copy only, no slabs.
    const bool cosine6 = metric == KNN_METRIC_COSINE;
    if (split && (metric == KNN_METRIC_L2SQ || cosine6) && d <= kPkMaxD &&
        n >= kPkMinPoints && n >= 4 * pk_seed_points_min(k) &&
        m >= (d <= kSpKC ? kPkMinQueriesOneChunk : kPkMinQueries)) {
        const int nch_p = pk_padded_chunks(d);
        const int sets_max = pk_max_sets(nch_p, k);
        const uint64_t n64 = ((uint64_t)n + kPkStep - 1) / kPkStep * kPkStep;
        // norms of all points and the header stay for the whole call; the bf16 copy holds one SLAB
        // of the points at a time - all of them if the limit has room, else the largest slab that
        // leaves the lists a place: the point axis is cut by the limit as well (section 4.3), each
        // slab is packed into the same buffer and searched, and the lists carry over.
        const uint64_t fixed = align_up(n64 * 4) * (cosine6 ? 2 : 1) + kAlign;
        const int64_t min_rows = m < 64 ? m : 64;
        double best = 0.0;
        int best_sets = 0;
        int64_t best_S = 0, best_r = 0, best_slab = 0;
        for (int64_t slab = (int64_t)n64;
             sets_max >= 2 && (slab == (int64_t)n64 || (slab >= 2 * kPkMinPoints && !cosine6));
             slab = (slab / 2 + kPkSlabGrain - 1) / kPkSlabGrain * kPkSlabGrain) {
            const uint64_t copy = align_up((uint64_t)slab * (uint64_t)nch_p * 32);
            if (mem_limit_bytes >= fixed + copy + lists_bytes_for((uint64_t)min_rows, 1, (uint64_t)k) +
                                       query_bytes_for((uint64_t)min_rows, qrow, 3, 1)) {
                // Query sets per workgroup and point ranges: a launch runs in rounds of one
                // workgroup per compute unit, a workgroup's time goes with sets x (range + a
                // start-up allowance), and there is one launch per slab and query chunk.
                const uint64_t avail6 = mem_limit_bytes - fixed - copy;
                const int64_t nslabs = ((int64_t)n64 + slab - 1) / slab;
                for (int sets = sets_max; sets >= 2 && sets >= sets_max - 6; --sets) {
                    const int64_t tile6 = 32 * sets;
                    for (int64_t S = 1; S <= 32; ++S) {
                        if (slab / S < 8 * kPkStep * 16) break;  // ranges of >= 16 rounds of the waves
                        int64_t rows = rows_fitting(avail6, (uint64_t)S, (uint64_t)k, qrow, 3);
                        if (rows > kMaxChunkRows) rows = kMaxChunkRows;
                        if (rows >= m) rows = m;
                        else rows = rows / tile6 * tile6;
                        if (rows < 1) continue;
                        const int64_t chunks = (m + rows - 1) / rows;
                        // (a slab is packed again for every query chunk, and small tiles make
                        // poor use of it: slabs only where all queries fit one chunk of large tiles)
                        if (nslabs > 1 && (chunks > 1 || sets < sets_max - 3)) continue;
                        const int64_t wgs = (rows + tile6 - 1) / tile6 * S;
                        const int64_t rounds = (wgs + kNumCU - 1) / kNumCU;
                        const double range = (double)((slab + S - 1) / S);
                        // larger tiles re-read the points less often: a mild preference
                        // and fewer ranges mean fewer lists to fill and to merge.  One list per
                        // query in a launch that fits the chip at once (S = 1, one round) always
                        // works under its own latest threshold and ends with one merge per
                        // query, which pays with k: measured (ms for search + merge, S = 1 in one
                        // round against the plan without this term) c5, k = 32: 40.5 + 0.24 / 42.0 +
                        // 0.75; m = 6e4, n = 2e6, d = 128, k = 50: 26.3 + 0.24 / 27.6 + 0.54; but
                        // m = 5e4, n = 4e6, d = 128, k = 10: 38.3 + 0.08 / 36.6 + 0.21, and over
                        // several rounds the choice loses (m = 2e5, n = 1e6, d = 128: 43.5 / 41.3).
                        const double kk = 0.004 * (double)k;
                        const double order = (S == 1 && rounds == 1) ? 1.0 - (kk < 0.12 ? kk : 0.12) : 1.0;
                        const double cost = (double)chunks * (double)nslabs * (double)rounds * (double)sets *
                                            (range + 4096.0 + 64.0 * (double)k) * (1.0 + 0.5 / (double)sets) *
                                            (1.0 + 0.005 * (double)S) * order;
                        if (best_sets == 0 || cost < best) {
                            best = cost;
                            best_sets = sets;
                            best_S = S;
                            best_r = rows;
                            best_slab = slab;
                        }
                    }
                }
            }
        }
        if (best_sets != 0) {
            out->path = KNN_PATH_MFMA_PACKED;
            out->seed_points = (int32_t)pk_seed_points(k, n);
            out->slab_points = best_slab;
            out->tile_q = 32 * best_sets;
            out->tile_x = kPkStep;
            out->norms_bytes = fixed + align_up((uint64_t)best_slab * (uint64_t)nch_p * 32);
            out->n_splits = (int32_t)best_S;
            out->chunk_rows = best_r;
            out->q_chunks = (m + best_r - 1) / best_r;
            out->lists_bytes = lists_bytes_for((uint64_t)best_r, (uint64_t)best_S, (uint64_t)k);
            out->query_bytes = query_bytes_for((uint64_t)best_r, qrow, 3, (uint64_t)best_S);
            out->workspace_bytes = out->norms_bytes + out->query_bytes + out->lists_bytes;
            plan_two_streams(out, m, mem_limit_bytes, qrow, 3);
            return KNN_OK;
        }
    }
    // d > 256 with many points and queries: tiles of 512 queries x 128 points on bf16 copies of
    // both operands (knn_wide.hip).  The workspace is path 5's plus the packed points (all of them,
    // or one slab at a time as on path 6) with the queries' B operands in operand order, so a
    // call whose rows turn out not to be 16-byte aligned still runs under this plan on path 5's
    // kernel.
    if (split && metric == KNN_METRIC_L2SQ && d > kPkMaxD && k <= kWdMaxK && n >= kWdMinPoints &&
        m >= kWdMinQueries) {
        const int nch_p = pk_padded_chunks(d);
        const uint64_t qrow7 = 32ull * (uint64_t)nch_p;
        const uint64_t n64 = ((uint64_t)n + kPkStep - 1) / kPkStep * kPkStep;
        const uint64_t fixed = align_up(n64 * 4) + kAlign;
        const int64_t min_rows = 64;
        double best = 0.0;
        int64_t best_S = 0, best_r = 0, best_slab = 0;
        for (int64_t slab = (int64_t)n64; slab == (int64_t)n64 || slab >= 2 * kWdMinPoints;
             slab = (slab / 2 + kPkSlabGrain - 1) / kPkSlabGrain * kPkSlabGrain) {
            const uint64_t copy = align_up((uint64_t)slab * (uint64_t)nch_p * 32);
            if (mem_limit_bytes < fixed + copy + lists_bytes_for((uint64_t)min_rows, 1, (uint64_t)k) +
                                      query_bytes_for((uint64_t)min_rows, qrow7, 4, 1))
                continue;
            const uint64_t avail7 = mem_limit_bytes - fixed - copy;
            const int64_t nslabs = ((int64_t)n64 + slab - 1) / slab;
            for (int64_t S = 1; S <= kWdMaxSplits; ++S) {
                if (S > 1 && slab / S < 16 * kWdTileX) break;  // ranges of at least 16 tiles
                int64_t rows = rows_fitting(avail7, (uint64_t)S, (uint64_t)k, qrow7, 4);
                if (rows > kMaxChunkRows) rows = kMaxChunkRows;
                if (rows >= m) rows = m;
                else rows = rows / kWdTileQ * kWdTileQ;
                if (rows < 1) continue;
                const int64_t chunks = (m + rows - 1) / rows;
                // (a slab is packed again for every query chunk)
                if (nslabs > 1 && chunks > 1) continue;
                const int64_t wgs = (rows + kWdTileQ - 1) / kWdTileQ * S;
                const int64_t rounds = (wgs + kNumCU - 1) / kNumCU;
                const double range = (double)((slab + S - 1) / S);
                // one workgroup per compute unit at a time; a range costs its tiles plus the start
                // of its lists (a first tile, and about 64 k points' worth of exact evaluations)
                const double cost = (double)chunks * (double)nslabs * (double)rounds *
                                    (range + 2048.0 + 64.0 * (double)k) * (1.0 + 0.005 * (double)S);
                if (best_S == 0 || cost < best) {
                    best = cost;
                    best_S = S;
                    best_r = rows;
                    best_slab = slab;
                }
            }
            if (best_S != 0) break;  // the largest slab that fits
        }
        if (best_S != 0) {
            out->path = KNN_PATH_MFMA_WIDE;
            out->slab_points = best_slab;
            out->tile_q = kWdTileQ;
            out->tile_x = kWdTileX;
            out->norms_bytes = fixed + align_up((uint64_t)best_slab * (uint64_t)nch_p * 32);
            out->n_splits = (int32_t)best_S;
            out->chunk_rows = best_r;
            out->q_chunks = (m + best_r - 1) / best_r;
            out->lists_bytes = lists_bytes_for((uint64_t)best_r, (uint64_t)best_S, (uint64_t)k);
            out->query_bytes = query_bytes_for((uint64_t)best_r, qrow7, 4, (uint64_t)best_S);
            out->workspace_bytes = out->norms_bytes + out->query_bytes + out->lists_bytes;
            plan_two_streams(out, m, mem_limit_bytes, qrow7, 4);
            return KNN_OK;
        }
    }
    const int64_t tile = out->tile_q;
    const uint64_t avail = mem_limit_bytes - out->norms_bytes - out->private_bytes;

    // Number of point ranges S.  More ranges mean more workgroups (tiles x S), each walking
    // n / S points, but also more list warm-up and merge work.  Estimated run time of a
    // plan: chunks x rounds of resident workgroups x points per workgroup (+ a warm-up
    // allowance); a larger S must beat a smaller one by 10 %.
    // (on the split path the ranges of a query share their thresholds, so short ranges cost
    // little list warm-up: they may be shorter)
    int64_t s_max = n / (split ? kSpMinSplitPoints : kMinSplitPoints);
    if (s_max < 1) s_max = 1;
    if (s_max > kMaxSplits) s_max = kMaxSplits;
    const int64_t slots = lowd ? kLowdResidentWorkgroups : kSpResidentWorkgroups;
    int64_t best_s = 0, best_rows = 0;
    double best_cost = 0.0;
    for (int64_t S = 1; S <= s_max; S = (S < 8 ? S + 1 : S + 8)) {
        int64_t rows = rows_fitting(avail, (uint64_t)S, (uint64_t)k, qrow, qkind);
        if (rows > kMaxChunkRows) rows = kMaxChunkRows;
        if (rows >= m) rows = m;
        else rows = rows / tile * tile;
        if (rows < 1) continue;
        const int64_t chunks = (m + rows - 1) / rows;
        const int64_t wgs = (rows + tile - 1) / tile * S;
        const int64_t rounds = (wgs + slots - 1) / slots;
        const double range = (double)((n + S - 1) / S);
        double warm = (double)kWarmupPointsPerK * (double)k;
        if (out->path == KNN_PATH_LOWD_BF16 || out->path == KNN_PATH_LOWD_MFMA) {
            // The filter kernels scan a point in a few cycles per wave, while every accepted
            // pair (about k (1 + ln(range / k)) per query and range) costs a few hundred, so a
            // range's list warm-up is worth on the order of a million scanned points there.
            const double per_k = out->path == KNN_PATH_LOWD_BF16 ? kWarmupPointsPerKBf16
                                                                 : kWarmupPointsPerKFilter;
            const double ratio = range > (double)k ? range / (double)k : 1.0;
            warm = per_k * (double)k * (1.0 + log(ratio));
        }
        const double per_wg = range + warm;
        const double cost = (double)chunks * (double)rounds * per_wg;
        if (best_s == 0 || cost < 0.9 * best_cost) {
            best_cost = cost;
            best_s = S;
            best_rows = rows;
        }
    }
    if (best_s == 0) return KNN_ERR_MEM_LIMIT_TOO_SMALL;
    out->n_splits = (int32_t)best_s;
    out->chunk_rows = best_rows;
    out->q_chunks = (m + best_rows - 1) / best_rows;
    out->lists_bytes = lists_bytes_for((uint64_t)best_rows, (uint64_t)best_s, (uint64_t)k);
    out->query_bytes = query_bytes_for((uint64_t)best_rows, qrow, qkind);
    out->workspace_bytes = out->norms_bytes + out->query_bytes + out->lists_bytes;
    plan_two_streams(out, m, mem_limit_bytes, qrow, qkind);
    return KNN_OK;
}

// Host-resident points: the limit pays for two staging buffers, one block's results and the
// plan of a block.  Staging gets at most half of what is left after the block results, so
// that the block's own lists keep at least as much; blocks are as long as that allows.
extern "C" knn_status knn_plan_host_x(int64_t m, int64_t n, int32_t d, int32_t k, knn_metric metric,
                                      uint64_t mem_limit_bytes, knn_host_plan_t* out) {
    if (!out) return KNN_ERR_INVALID_ARG;
    memset(out, 0, sizeof(*out));
    knn_plan_t probe;
    // argument checks (and the empty plan for m == 0) are those of the resident search
    knn_status st = knn_plan_metric(m, n, d, k, metric, UINT64_MAX / 4, &probe);
    if (st != KNN_OK) return st;
    out->m = m;
    out->n = n;
    out->d = d;
    out->k = k;
    out->metric = (int32_t)metric;
    if (m == 0) return KNN_OK;
    const uint64_t row = (uint64_t)d * 4;
    // a block's winners (index, list key, fp64 distance) and the running result's fp64 distances
    // (its indices and keys live in the caller's idx and dist until the final order is written)
    const uint64_t outb = 2 * align_up((uint64_t)m * (uint64_t)k * 4) + 2 * align_up((uint64_t)m * (uint64_t)k * 8);
    const int64_t b_floor = n < 1024 ? n : ((int64_t)k > 1024 ? (int64_t)k : 1024);  // shortest block
    {
        knn_plan_t smallest;
        knn_plan_metric(m, b_floor, d, k < b_floor ? k : (int32_t)b_floor, metric, 0, &smallest);
        const uint64_t bufs = b_floor < n ? 2 : 1;
        out->min_limit_bytes = outb + bufs * align_up((uint64_t)b_floor * row) + smallest.min_limit_bytes;
    }
    out->block_out_bytes = outb;
    if (mem_limit_bytes < out->min_limit_bytes) return KNN_ERR_MEM_LIMIT_TOO_SMALL;
    const uint64_t half = (mem_limit_bytes - outb) / 2;
    // candidate block lengths, longest first: everything at once, what half of the room
    // stages twice, the shortest block; the first whose block plans fit is taken
    int64_t cand[3];
    int ncand = 0;
    if (align_up((uint64_t)n * row) <= half) cand[ncand++] = n;
    {
        int64_t B = (int64_t)(half / 2 / kAlign * kAlign / row);
        if (B >= 4096) B = B / 4096 * 4096;
        else if (B >= 128) B = B / 128 * 128;
        if (B < b_floor) B = b_floor;
        if (B > n) B = n;
        if (ncand == 0 || B < cand[ncand - 1]) cand[ncand++] = B;
    }
    if (b_floor < cand[ncand - 1]) cand[ncand++] = b_floor;
    st = KNN_ERR_MEM_LIMIT_TOO_SMALL;
    uint64_t inner_ws = 0;
    for (int c = 0; c < ncand; ++c) {
        const int64_t B = cand[c];
        const int64_t nb = (n + B - 1) / B;
        const uint64_t staging = (nb > 1 ? 2 : 1) * align_up((uint64_t)B * row);
        if (staging + outb > mem_limit_bytes) continue;
        const uint64_t inner_limit = mem_limit_bytes - outb - staging;
        knn_plan_t full, tail;
        if (knn_plan_metric(m, B, d, (int64_t)k < B ? k : (int32_t)B, metric, inner_limit, &full) !=
            KNN_OK)
            continue;
        inner_ws = full.workspace_bytes;
        const int64_t last = n - (nb - 1) * B;
        if (last != B) {
            if (knn_plan_metric(m, last, d, (int64_t)k < last ? k : (int32_t)last, metric,
                                inner_limit, &tail) != KNN_OK)
                continue;
            if (tail.workspace_bytes > inner_ws) inner_ws = tail.workspace_bytes;
        }
        out->block_rows = B;
        out->n_blocks = nb;
        out->staging_bytes = staging;
        out->inner_limit_bytes = inner_limit;
        out->inner = full;
        st = KNN_OK;
        break;
    }
    if (st != KNN_OK) return st;
    out->workspace_bytes = out->staging_bytes + outb + inner_ws;
    return KNN_OK;
}

extern "C" uint64_t knn_workspace_bytes(int64_t m, int64_t n, int32_t d, int32_t k,
                                        uint64_t mem_limit_bytes) {
    knn_plan_t p;
    if (knn_plan(m, n, d, k, mem_limit_bytes, &p) != KNN_OK) return 0;
    return p.workspace_bytes;
}
