// C ABI entry points that touch the GPU (see include/knn.h for the contract).
//
// knn_search is the loop of paper section 4.3 written by hand: the query axis is cut into
// chunks whose partial lists fit the workspace, each chunk is one "generator + reducer"
// launch over all point ranges followed by the merge that writes a slice of the final
// result.  Nothing is allocated here: the only device memory the library uses is the
// caller's workspace, so its footprint is bounded by the limit by construction (the
// limit-unaware allocator is the overflow risk section 4.4 describes).
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstring>
#include <mutex>
#include <vector>

#include "../../include/knn.h"
#include "knn_config.h"
#include "knn_kernels.h"

namespace {

thread_local knn_plan_t g_last_plan;
thread_local uint64_t g_last_peak = 0;
thread_local bool g_have_last = false;
thread_local char g_hip_error[256] = "";

// Event brackets of the profiled searches since the last knn_profile_read.
struct Bracket {
    hipEvent_t begin, end;
    int kind;  // 0 norms, 1 search, 2 merge+refine
};
thread_local bool g_profile = false;
thread_local std::vector<Bracket> g_brackets;
thread_local std::vector<hipEvent_t> g_event_pool;

hipEvent_t take_event() {
    hipEvent_t ev = nullptr;
    if (!g_event_pool.empty()) {
        ev = g_event_pool.back();
        g_event_pool.pop_back();
    } else if (hipEventCreate(&ev) != hipSuccess) {
        ev = nullptr;
    }
    return ev;
}

// Records an event on the stream when profiling is on; returns nullptr otherwise.
hipEvent_t mark(hipStream_t stream) {
    if (!g_profile) return nullptr;
    hipEvent_t ev = take_event();
    if (ev && hipEventRecord(ev, stream) != hipSuccess) {
        g_event_pool.push_back(ev);
        ev = nullptr;
    }
    return ev;
}

// Gives back the opening event of a bracket whose launch failed.
void drop_bracket(hipEvent_t begin) {
    if (begin) g_event_pool.push_back(begin);
}

void close_bracket(hipEvent_t begin, hipStream_t stream, int kind) {
    if (!begin) return;
    hipEvent_t end = mark(stream);
    if (!end) {
        g_event_pool.push_back(begin);
        return;
    }
    g_brackets.push_back({begin, end, kind});
}

knn_status hip_fail(hipError_t e, const char* what) {
    snprintf(g_hip_error, sizeof(g_hip_error), "%s: %s", what, hipGetErrorString(e));
    return KNN_ERR_HIP;
}

}  // namespace

namespace knn {
// Lets the other C ABI sources of the library record into the same per-thread message and
// into the same event brackets (kind 0: preparation, 1: the dominant kernel, 2: the rest).
void set_last_hip_error(hipError_t e, const char* what) { hip_fail(e, what); }
hipEvent_t profile_mark(hipStream_t stream) { return mark(stream); }
void profile_close(hipEvent_t begin, hipStream_t stream, int kind) { close_bracket(begin, stream, kind); }
void profile_drop(hipEvent_t begin) { drop_bracket(begin); }
}  // namespace knn

extern "C" const char* knn_last_hip_error(void) { return g_hip_error; }

extern "C" knn_status knn_profile_enable(int32_t on) {
    g_profile = on != 0;
    if (!g_profile) {
        for (auto& b : g_brackets) {
            g_event_pool.push_back(b.begin);
            g_event_pool.push_back(b.end);
        }
        g_brackets.clear();
        for (hipEvent_t ev : g_event_pool) (void)hipEventDestroy(ev);
        g_event_pool.clear();
    }
    return KNN_OK;
}

extern "C" knn_status knn_profile_read(float* norms_ms, float* search_ms, float* refine_ms,
                                       int64_t* search_launches) {
    float sum[3] = {0.f, 0.f, 0.f};
    int64_t launches = 0;
    knn_status st = KNN_OK;
    for (auto& b : g_brackets) {
        float ms = 0.f;
        hipError_t e = hipEventSynchronize(b.end);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, b.begin, b.end);
        if (e != hipSuccess) st = hip_fail(e, "profile event");
        else sum[b.kind] += ms;
        if (b.kind == 1) ++launches;
        g_event_pool.push_back(b.begin);
        g_event_pool.push_back(b.end);
    }
    g_brackets.clear();
    if (norms_ms) *norms_ms = sum[0];
    if (search_ms) *search_ms = sum[1];
    if (refine_ms) *refine_ms = sum[2];
    if (search_launches) *search_launches = launches;
    return st;
}

extern "C" knn_status knn_last_stats(knn_plan_t* plan_out, uint64_t* peak_workspace_bytes) {
    if (!g_have_last) return KNN_ERR_INVALID_ARG;
    if (plan_out) *plan_out = g_last_plan;
    if (peak_workspace_bytes) *peak_workspace_bytes = g_last_peak;
    return KNN_OK;
}

extern "C" knn_status knn_search(const float* Q, int64_t ldq, const float* X, int64_t ldx,
                                 int64_t m, int64_t n, int32_t d, int32_t k,
                                 uint64_t mem_limit_bytes, void* workspace,
                                 uint64_t workspace_bytes, int32_t* idx, float* dist,
                                 void* hip_stream) {
    return knn_search_metric(Q, ldq, X, ldx, m, n, d, k, KNN_METRIC_L2SQ, mem_limit_bytes,
                             workspace, workspace_bytes, idx, dist, hip_stream);
}

namespace {

// Second stream of a search in several query chunks (one per host thread and device, created on
// first use, default priority): merge and exact re-evaluation of chunk c run there while the
// caller's stream searches chunk c + 1.
struct ChunkStreamState {
    int device = -1;
    hipStream_t side = nullptr;
    hipEvent_t searched[2] = {nullptr, nullptr};  // lists of buffer b are complete
    hipEvent_t merged[2] = {nullptr, nullptr};    // lists of buffer b are free again
};
thread_local ChunkStreamState g_chunk;

hipError_t chunk_state_init() {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (g_chunk.side && g_chunk.device == dev) return hipSuccess;
    ChunkStreamState fresh;
    fresh.device = dev;
    e = hipStreamCreateWithFlags(&fresh.side, hipStreamNonBlocking);
    if (e != hipSuccess) return e;
    hipEvent_t* all[4] = {&fresh.searched[0], &fresh.searched[1], &fresh.merged[0], &fresh.merged[1]};
    for (hipEvent_t* ev : all) {
        e = hipEventCreateWithFlags(ev, hipEventDisableTiming);
        if (e != hipSuccess) return e;
    }
    g_chunk = fresh;  // a set made for another device is left alone: it belongs to that device
    return hipSuccess;
}

// The search of one resident point set under a given plan: norms / packing, then per query
// chunk the search kernel over all point ranges and the merge + exact re-evaluation.
// keep_thresholds (path 5, one query chunk): the thresholds that an earlier call with the same
// plan left in the workspace - k-th keys of the same queries against OTHER points, lists of
// the same length k - bound this call's lists from the start.
knn_status run_search(const knn_plan_t& plan, const float* Q, int64_t ldq, const float* X,
                      int64_t ldx, int64_t m, int64_t n, int32_t d, int32_t k, knn_metric metric,
                      unsigned char* ws, int32_t* idx, float* dist, hipStream_t stream,
                      bool keep_thresholds = false, bool one_stream = false, double* block_d64 = nullptr) {
    using namespace knn;
    float* xn = reinterpret_cast<float*>(ws);
    // path 5: [squared norms][header: their maximum] | [split queries][query norms][shared
    // thresholds] | lists; L1 path: [transposed queries] | lists
    const bool wide_plan = plan.path == KNN_PATH_MFMA_WIDE;
    const bool packed_plan = plan.path == KNN_PATH_MFMA_PACKED || wide_plan;
    const uint64_t n64 = ((uint64_t)n + kPkStep - 1) / kPkStep * kPkStep;
    unsigned char* hdr = ws + align_up((packed_plan ? n64 : (uint64_t)n) * 4);
    unsigned char* xp = hdr + kAlign;  // paths 6, 7: the points rounded to bf16
    // paths 6, 7 need 16-byte aligned rows; other calls run their plans on path 5's kernel
    const bool packed = packed_plan && packed_rows_aligned(Q, ldq, X, ldx, d);
    unsigned char* qs = ws + plan.norms_bytes;
    // (path 7: the B operands in operand order, rows rounded up to 64, chunks to an even count)
    const uint64_t qs_bytes =
        wide_plan ? ((uint64_t)plan.chunk_rows + 63) / 64 * 64 * 32 * (uint64_t)pk_padded_chunks(d)
                  : (uint64_t)plan.chunk_rows * 32 * (((uint64_t)d + kSpKC - 1) / kSpKC);
    float* qn = reinterpret_cast<float*>(qs + align_up(qs_bytes));
    unsigned char* tsh = reinterpret_cast<unsigned char*>(qn) + align_up((uint64_t)plan.chunk_rows * 4);
    unsigned char* tsr = tsh + align_up((uint64_t)plan.chunk_rows * 4);  // path 6: [rows][S] words
    unsigned char* lists = ws + plan.norms_bytes + plan.query_bytes;
    // plan.streams == 2: two sets of lists, used by the chunks in turn
    const int nbuf = plan.streams == 2 ? 2 : 1;
    const uint64_t set_bytes = plan.lists_bytes / nbuf;
    const bool overlap = nbuf == 2 && !one_stream;
    if (overlap) {
        hipError_t e0 = chunk_state_init();
        if (e0 != hipSuccess) return hip_fail(e0, "second stream / events");
    }
    const int S = plan.n_splits;
    const bool cosine = metric == KNN_METRIC_COSINE;
    // path 6, cosine metric: xn holds 1 / |x|, the copy the rows x / |x|, and behind the copy lie
    // the values the filter's sums start from (zeros, +inf from n to the end of the last step)
    float* const sum0 =
        (cosine && plan.path == KNN_PATH_MFMA_PACKED)
            ? reinterpret_cast<float*>(xp + align_up((uint64_t)plan.slab_points * (uint64_t)pk_padded_chunks(d) * 32))
            : xn;

    hipError_t e;
    if (plan.path == KNN_PATH_MFMA_SPLIT || packed_plan) {
        hipEvent_t t0 = mark(stream);
        // (the header's second word: the points' largest bf16 rounding residual, which the
        // filters' allowance is built from; not used by the cosine metric)
        e = launch_header_init(hdr, stream);
        // (one slab: the copy is made here, once for all query chunks, and the pass that makes it
        // takes the norms and the largest rounding residual along)
        const bool copy_now = packed && plan.slab_points >= (int64_t)n64;
        if (e == hipSuccess && copy_now && !cosine)
            e = launch_pack_operands(X, ldx, n, d, 0, (int64_t)n64, xp, stream, 1.f, xn, hdr);
        if (e == hipSuccess && (!copy_now || cosine))
            e = launch_row_norms(X, ldx, n, d, cosine, xn, stream, cosine ? nullptr : hdr + 4);
        if (e == hipSuccess) e = launch_max_norm(xn, n, hdr, stream);
        if (e == hipSuccess && packed && cosine) {  // (plans of the cosine metric hold the whole copy)
            e = launch_pack_operands(X, ldx, n, d, 0, (int64_t)n64, xp, stream, 1.f, nullptr, hdr, xn);
            if (e == hipSuccess) e = launch_fill_words(sum0, (int64_t)n64, 0u, stream);
        }
        if (e == hipSuccess && packed) e = launch_pad_norms(sum0, n, stream);
        if (e != hipSuccess) {
            drop_bracket(t0);
            return hip_fail(e, "row norms launch");
        }
        close_bracket(t0, stream, 0);
    } else if (plan.path == KNN_PATH_LOWD_MFMA || plan.path == KNN_PATH_LOWD_BF16) {
        hipEvent_t t0 = mark(stream);
        e = plan.path == KNN_PATH_LOWD_BF16
                ? launch_lowd_bf16(Q, ldq, X, ldx, ws, 0, n, d, k, S, true, plan.seed_cells, nullptr, nullptr, stream)
                : launch_lowd_mfma(Q, ldq, X, ldx, ws, 0, n, d, k, S, true, nullptr, nullptr, stream);
        if (e != hipSuccess) {
            drop_bracket(t0);
            return hip_fail(e, "point packing launch");
        }
        close_bracket(t0, stream, 0);
    }
    for (int64_t c = 0; c < plan.q_chunks; ++c) {
        const int buf = (int)(c % nbuf);
        float* lk = reinterpret_cast<float*>(lists + buf * set_bytes);
        int* li = reinterpret_cast<int*>(lists + buf * set_bytes + set_bytes / 2);
        if (overlap && c >= 2) {  // the merge that read this set of lists two chunks ago
            e = hipStreamWaitEvent(stream, g_chunk.merged[buf], 0);
            if (e != hipSuccess) return hip_fail(e, "waiting for a set of lists");
        }
        const int64_t row0 = c * plan.chunk_rows;
        const int64_t rows = (m - row0 < plan.chunk_rows) ? (m - row0) : plan.chunk_rows;
        const float* Qc = Q + row0 * ldq;
        hipEvent_t t1 = mark(stream);
        if (plan.path == KNN_PATH_LOWD)
            e = launch_lowd(Qc, ldq, X, ldx, rows, n, d, k, S, lk, li, stream);
        else if (plan.path == KNN_PATH_L1)
            e = launch_l1(Qc, ldq, X, ldx, qs, rows, n, d, k, S, lk, li, stream);
        else if (plan.path == KNN_PATH_LOWD_MFMA)
            e = launch_lowd_mfma(Qc, ldq, X, ldx, ws, rows, n, d, k, S, false, lk, li, stream);
        else if (plan.path == KNN_PATH_LOWD_BF16)
            e = launch_lowd_bf16(Qc, ldq, X, ldx, ws, rows, n, d, k, S, false, plan.seed_cells, lk,
                                 li, stream);
        else if (plan.path == KNN_PATH_MFMA_SPLIT || packed_plan) {
            if (wide_plan && packed) {
                // the queries' B operands bf16(-2 q) in operand order; thresholds start from +inf
                e = launch_pack_operands(Qc, ldq, rows, d, 0, (rows + kPkStep - 1) / kPkStep * kPkStep, qs,
                                         stream, -2.f);
                if (e == hipSuccess && !keep_thresholds) e = launch_fill_words(tsh, rows, 0xff800000u, stream);  // (the word of +inf)
            } else {
                e = launch_split_queries(Qc, ldq, rows, d, qs, tsh, !keep_thresholds, stream);
            }
            if (e == hipSuccess) e = launch_row_norms(Qc, ldq, rows, d, false, qn, stream);
            if (e == hipSuccess && !packed)
                e = launch_split(Qc, ldq, X, ldx, qs, qn, tsh, xn, hdr, cosine, rows, n, d, k, S, lk,
                                 li, stream);
            // path 6: the thresholds start from the filter keys of a sample of the first slab
            // (preparation in the event brackets), then the packed kernel searches the points slab
            // after slab, S ranges each; the lists of slab b + 1 continue those of slab b
            if (e == hipSuccess && packed) {
                const int64_t slab = plan.slab_points;
                const bool one = slab >= (int64_t)n64;
                for (int64_t j0 = 0; j0 < (int64_t)n64 && e == hipSuccess; j0 += slab) {
                    const int64_t pts = (int64_t)n64 - j0 < slab ? (int64_t)n64 - j0 : slab;
                    const int64_t j1 = j0 + pts < n ? j0 + pts : n;
                    if (!one) {
                        if (j0 > 0) {
                            close_bracket(t1, stream, 1);
                            t1 = mark(stream);
                        }
                        e = launch_pack_operands(X, ldx, n, d, j0, pts, xp, stream);
                    }
                    if (j0 == 0) {
                        // (thresholds kept from an earlier block of a host-streamed search are
                        // tighter than a sample of this block would make them; path 7 takes its
                        // first thresholds inside the search kernel)
                        if (e == hipSuccess && !keep_thresholds && !wide_plan)
                            e = launch_seed_thresholds(Qc, ldq, xp, sum0, qs, qn, tsh, hdr, rows, j1, d, k,
                                                       plan.seed_points, stream, cosine);
                        if (e == hipSuccess) e = launch_fill_words(tsr, rows * S, 0xff800000u, stream);
                    }
                    if (e != hipSuccess) break;
                    close_bracket(t1, stream, 0);
                    t1 = mark(stream);
                    if (wide_plan)
                        e = launch_wide(Qc, ldq, X, ldx, xp, j0, pts, qs, qn, tsh, tsr, xn, hdr, rows, n, d, k,
                                        S, j0, j1, j0 == 0 ? 0 : S, lk, li, stream);
                    else
                        e = launch_packed(Qc, ldq, X, ldx, xp, j0, qs, qn, tsh, tsr, sum0, hdr, rows, n, d, k, S,
                                          plan.tile_q / 32, j0, j1, j0 == 0 ? 0 : S, lk, li, stream,
                                          cosine ? xn : nullptr);
                }
            }
        } else
            e = hipErrorInvalidValue;  // no such path
        if (e != hipSuccess) {
            drop_bracket(t1);
            return hip_fail(e, "search launch");
        }
        close_bracket(t1, stream, 1);
        hipStream_t ms = stream;
        if (overlap) {
            ms = g_chunk.side;
            e = hipEventRecord(g_chunk.searched[buf], stream);
            if (e == hipSuccess) e = hipStreamWaitEvent(ms, g_chunk.searched[buf], 0);
            if (e != hipSuccess) return hip_fail(e, "ordering the second stream");
        }
        hipEvent_t t2 = mark(ms);
        e = launch_merge_refine(Qc, ldq, X, ldx, rows, n, d, k, S, (int)metric, lk, li,
                                idx + row0 * k, dist + row0 * k, ms, block_d64 ? block_d64 + row0 * k : nullptr);
        if (e != hipSuccess) {
            drop_bracket(t2);
            return hip_fail(e, "merge/refine launch");
        }
        close_bracket(t2, ms, 2);
        if (overlap) {
            e = hipEventRecord(g_chunk.merged[buf], ms);
            if (e != hipSuccess) return hip_fail(e, "ordering the second stream");
        }
    }
    if (overlap) {  // the caller's stream ends behind the last merges
        const int64_t last = plan.q_chunks - 1;
        for (int64_t c = last > 0 ? last - 1 : 0; c <= last; ++c) {
            e = hipStreamWaitEvent(stream, g_chunk.merged[c % 2], 0);
            if (e != hipSuccess) return hip_fail(e, "joining the second stream");
        }
    }
    return KNN_OK;
}

}  // namespace

extern "C" knn_status knn_search_metric(const float* Q, int64_t ldq, const float* X, int64_t ldx,
                                        int64_t m, int64_t n, int32_t d, int32_t k,
                                        knn_metric metric, uint64_t mem_limit_bytes,
                                        void* workspace, uint64_t workspace_bytes, int32_t* idx,
                                        float* dist, void* hip_stream) {
    using namespace knn;
    if (m < 0 || n < 1 || d < 1 || k < 1 || (int64_t)k > n) return KNN_ERR_INVALID_ARG;
    if (ldq < d || ldx < d) return KNN_ERR_INVALID_ARG;
    if (!X) return KNN_ERR_INVALID_ARG;
    if (m > 0 && (!Q || !idx || !dist)) return KNN_ERR_INVALID_ARG;
    knn_plan_t plan;
    knn_status st = knn_plan_metric(m, n, d, k, metric, mem_limit_bytes, &plan);
    if (st != KNN_OK) return st;
    if (m == 0) {
        g_last_plan = plan;
        g_last_peak = 0;
        g_have_last = true;
        return KNN_OK;
    }
    if (!workspace || reinterpret_cast<uintptr_t>(workspace) % kAlign != 0)
        return KNN_ERR_INVALID_ARG;
    if (workspace_bytes < plan.workspace_bytes) return KNN_ERR_WORKSPACE_TOO_SMALL;

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    st = run_search(plan, Q, ldq, X, ldx, m, n, d, k, metric, static_cast<unsigned char*>(workspace),
                    idx, dist, stream);
    if (st != KNN_OK) return st;
    g_last_plan = plan;
    g_last_peak = plan.workspace_bytes;
    g_have_last = true;
    return KNN_OK;
}

// Workspace of knn_search_static: part of the device image, so no call ever allocates it.  In
// host code this name is only a handle for hipGetSymbolAddress; the address kernels can use is
// looked up once per device and kept in g_static_ptr.
static __device__ __align__(256) unsigned char scratch[KNN_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_static_mutex;
unsigned char* g_static_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (each GPU holds its own copy).
knn_status static_scratch(unsigned char** out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return KNN_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (!g_static_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return hip_fail(e, "hipGetSymbolAddress(scratch)");
        g_static_ptr[dev] = static_cast<unsigned char*>(p);
    }
    *out = g_static_ptr[dev];
    return KNN_OK;
}

}  // namespace

extern "C" knn_status knn_search_static(const float* Q, int64_t ldq, const float* X, int64_t ldx,
                                        int64_t m, int64_t n, int32_t d, int32_t k, int32_t* idx,
                                        float* dist, void* hip_stream) {
    if (m < 0 || n < 1 || d < 1 || k < 1 || (int64_t)k > n) return KNN_ERR_INVALID_ARG;
    if (ldq < d || ldx < d) return KNN_ERR_INVALID_ARG;
    if (!X) return KNN_ERR_INVALID_ARG;
    if (m > 0 && (!Q || !idx || !dist)) return KNN_ERR_INVALID_ARG;
    knn_plan_t plan;
    knn_status st = knn_plan_metric(m, n, d, k, KNN_METRIC_L2SQ, KNN_STATIC_SCRATCH_BYTES, &plan);
    if (st == KNN_ERR_MEM_LIMIT_TOO_SMALL) return KNN_ERR_STATIC_SCRATCH_TOO_SMALL;
    if (st != KNN_OK) return st;
    if (m > 0) {
        if (plan.workspace_bytes > KNN_STATIC_SCRATCH_BYTES) return KNN_ERR_STATIC_SCRATCH_TOO_SMALL;
        unsigned char* ws = nullptr;
        st = static_scratch(&ws);
        if (st != KNN_OK) return st;
        // (no second stream here: creating one may allocate)
        st = run_search(plan, Q, ldq, X, ldx, m, n, d, k, KNN_METRIC_L2SQ, ws, idx, dist,
                        static_cast<hipStream_t>(hip_stream), false, true);
        if (st != KNN_OK) return st;
    }
    g_last_plan = plan;
    g_last_peak = m > 0 ? plan.workspace_bytes : 0;
    g_have_last = true;
    return KNN_OK;
}

namespace {

// Copy stream and events of the host-streamed search, one set per host thread and device.
struct HostStreamState {
    int device = -1;
    hipStream_t copy = nullptr;
    hipEvent_t start = nullptr;
    hipEvent_t copied[2] = {nullptr, nullptr};
    hipEvent_t consumed[2] = {nullptr, nullptr};
};
thread_local HostStreamState g_host;

hipError_t host_state_init() {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (g_host.copy && g_host.device == dev) return hipSuccess;
    HostStreamState fresh;
    fresh.device = dev;
    e = hipStreamCreateWithFlags(&fresh.copy, hipStreamNonBlocking);
    if (e != hipSuccess) return e;
    hipEvent_t* all[5] = {&fresh.start, &fresh.copied[0], &fresh.copied[1], &fresh.consumed[0],
                          &fresh.consumed[1]};
    for (hipEvent_t* ev : all) {
        e = hipEventCreateWithFlags(ev, hipEventDisableTiming);
        if (e != hipSuccess) return e;
    }
    g_host = fresh;  // a set made for another device is left alone: it belongs to that device
    return hipSuccess;
}

}  // namespace

extern "C" knn_status knn_search_host_x(const float* Q, int64_t ldq, const float* X, int64_t ldx,
                                        int64_t m, int64_t n, int32_t d, int32_t k,
                                        knn_metric metric, uint64_t mem_limit_bytes,
                                        void* workspace, uint64_t workspace_bytes, int32_t* idx,
                                        float* dist, void* hip_stream) {
    using namespace knn;
    if (m < 0 || n < 1 || d < 1 || k < 1 || (int64_t)k > n) return KNN_ERR_INVALID_ARG;
    if (ldq < d || ldx < d) return KNN_ERR_INVALID_ARG;
    if (!X) return KNN_ERR_INVALID_ARG;
    if (m > 0 && (!Q || !idx || !dist)) return KNN_ERR_INVALID_ARG;
    knn_host_plan_t hp;
    knn_status st = knn_plan_host_x(m, n, d, k, metric, mem_limit_bytes, &hp);
    if (st != KNN_OK) return st;
    if (m == 0) return KNN_OK;
    if (!workspace || reinterpret_cast<uintptr_t>(workspace) % kAlign != 0)
        return KNN_ERR_INVALID_ARG;
    if (workspace_bytes < hp.workspace_bytes) return KNN_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipError_t e = host_state_init();
    if (e != hipSuccess) return hip_fail(e, "copy stream / events");

    // workspace: [staging 0 | staging 1] [block idx | block keys | block fp64 | running fp64]
    // [workspace of the block's plan]
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    const uint64_t stage_bytes = hp.staging_bytes / (hp.n_blocks > 1 ? 2 : 1);
    float* stage[2] = {reinterpret_cast<float*>(ws), reinterpret_cast<float*>(ws + stage_bytes)};
    const uint64_t a4 = align_up((uint64_t)m * (uint64_t)k * 4), a8 = align_up((uint64_t)m * (uint64_t)k * 8);
    int32_t* bidx = reinterpret_cast<int32_t*>(ws + hp.staging_bytes);
    float* bdist = reinterpret_cast<float*>(ws + hp.staging_bytes + a4);
    double* bd64 = reinterpret_cast<double*>(ws + hp.staging_bytes + 2 * a4);
    double* rd64 = reinterpret_cast<double*>(ws + hp.staging_bytes + 2 * a4 + a8);
    unsigned char* inner_ws = ws + hp.staging_bytes + hp.block_out_bytes;

    // the staging buffers may still be in use by earlier work on the caller's stream
    e = hipEventRecord(g_host.start, stream);
    if (e == hipSuccess) e = hipStreamWaitEvent(g_host.copy, g_host.start, 0);
    if (e != hipSuccess) return hip_fail(e, "ordering the copy stream");

    const size_t row_bytes = (size_t)d * 4;
    for (int64_t b = 0; b < hp.n_blocks; ++b) {
        const int buf = (int)(b & 1);
        const int64_t j0 = b * hp.block_rows;
        const int64_t nb = (n - j0 < hp.block_rows) ? (n - j0) : hp.block_rows;
        const int32_t kb = (int64_t)k < nb ? k : (int32_t)nb;
        if (b >= 2) {  // the block searched out of this buffer two steps ago must be done with it
            e = hipStreamWaitEvent(g_host.copy, g_host.consumed[buf], 0);
            if (e != hipSuccess) return hip_fail(e, "waiting for a staging buffer");
        }
        e = hipMemcpy2DAsync(stage[buf], row_bytes, X + j0 * ldx, (size_t)ldx * 4, row_bytes,
                             (size_t)nb, hipMemcpyHostToDevice, g_host.copy);
        if (e == hipSuccess) e = hipEventRecord(g_host.copied[buf], g_host.copy);
        if (e == hipSuccess) e = hipStreamWaitEvent(stream, g_host.copied[buf], 0);
        if (e != hipSuccess) return hip_fail(e, "host-to-device copy of a block");

        knn_plan_t plan = hp.inner;
        if (nb != hp.block_rows) {
            st = knn_plan_metric(m, nb, d, kb, metric, hp.inner_limit_bytes, &plan);
            if (st != KNN_OK) return st;
        }
        // From the second full block on, a block's lists start under the thresholds the
        // blocks before it reached (every earlier block is a full one with lists of length k,
        // so its k-th key bounds the overall k-th key) instead of warming up again.
        const bool keep = b > 0 && nb == hp.block_rows &&
                          (plan.path == KNN_PATH_MFMA_SPLIT || plan.path == KNN_PATH_MFMA_PACKED ||
                           plan.path == KNN_PATH_MFMA_WIDE) &&
                          plan.q_chunks == 1;
        st = run_search(plan, Q, ldq, stage[buf], d, m, nb, d, kb, metric, inner_ws, bidx, bdist,
                        stream, keep, false, bd64);
        if (st != KNN_OK) return st;
        // (until the final order below, dist holds the running result's list keys)
        e = launch_fold_keyed(bidx, bdist, bd64, kb, j0, b == 0 ? 1 : 0, m, k, idx, dist, rd64, stream);
        if (e == hipSuccess) e = hipEventRecord(g_host.consumed[buf], stream);
        if (e != hipSuccess) return hip_fail(e, "folding a block into the result");
    }
    e = launch_order_final(m, k, idx, dist, rd64, stream);
    if (e != hipSuccess) return hip_fail(e, "final order of the folded result");
    g_last_plan = hp.inner;
    g_last_peak = hp.workspace_bytes;
    g_have_last = true;
    return KNN_OK;
}
