// C ABI of the SGPR accumulations (see include/sgpr.h for the contract).
//
// The loop of paper section 4.3 over the data axis, written by hand: per chunk of data points
// make the m x chunk piece of K_uf in the workspace, add its product with its own transpose
// into A and its product with the chunk of y into b, then reuse the workspace.  Memory the
// library keeps: that one piece, whatever n is.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>

#include "../../include/sgpr.h"
#include "knn_config.h"
#include "sgpr_kernels.h"

namespace knn {  // api.hip
void set_last_hip_error(hipError_t e, const char* what);
hipEvent_t profile_mark(hipStream_t stream);
void profile_close(hipEvent_t begin, hipStream_t stream, int kind);
void profile_drop(hipEvent_t begin);
}  // namespace knn

namespace {

knn_status hip_fail(hipError_t e, const char* what) {
    knn::set_last_hip_error(e, what);
    return KNN_ERR_HIP;
}

}  // namespace

extern "C" knn_status sgpr_plan(int64_t m, int64_t n, int32_t d, uint64_t mem_limit_bytes,
                                sgpr_plan_t* out) {
    if (!out) return KNN_ERR_INVALID_ARG;
    std::memset(out, 0, sizeof(*out));
    if (m < 1 || n < 0 || d < 1) return KNN_ERR_INVALID_ARG;
    if (m > (1 << 17) || n > knn::kMaxPoints) return KNN_ERR_UNSUPPORTED;
    out->m = m;
    out->n = n;
    out->d = d;
    out->min_limit_bytes = knn::align_up((uint64_t)m * 16 * 4);
    if (mem_limit_bytes < out->min_limit_bytes) return KNN_ERR_MEM_LIMIT_TOO_SMALL;
    // columns of fp32 that fit: the whole allocation is rounded up to the alignment
    int64_t cols = (int64_t)(mem_limit_bytes / knn::kAlign * knn::kAlign / ((uint64_t)m * 4));
    cols = cols / 16 * 16;
    if (cols > SGPR_MAX_CHUNK_COLS) cols = SGPR_MAX_CHUNK_COLS;
    const int64_t n16 = (n + 15) / 16 * 16;
    if (cols > n16) cols = n16 > 0 ? n16 : 16;
    out->chunk_ld = cols;
    out->chunk_cols = cols < n ? cols : n;
    out->n_chunks = n > 0 ? (n + cols - 1) / cols : 0;
    const uint64_t chunk_bytes = knn::align_up((uint64_t)m * (uint64_t)cols * 4);
    // Few tiles of A: spread a chunk's columns over several groups of workgroups, each with
    // its own copy of A, while a group keeps at least 256 columns and the copies fit.
    const int64_t T = (m + 127) / 128;
    const int64_t tiles = T * (T + 1) / 2;
    const uint64_t copy_bytes = knn::align_up((uint64_t)m * (uint64_t)m * 8);
    int G = 1;
    while (G < 8 && tiles * G < 2048 && cols / (2 * G) >= 256 && (cols / (2 * G)) % 16 == 0 &&
           chunk_bytes + (uint64_t)(2 * G - 1) * copy_bytes <= mem_limit_bytes)
        G *= 2;
    out->col_groups = G;
    out->workspace_bytes = chunk_bytes + (uint64_t)(G - 1) * copy_bytes;
    return KNN_OK;
}

extern "C" knn_status sgpr_accumulate(const float* U, int64_t ldu, const float* X, int64_t ldx,
                                      const float* y, int64_t m, int64_t n, int32_t d,
                                      double variance, double lengthscale,
                                      uint64_t mem_limit_bytes, void* workspace,
                                      uint64_t workspace_bytes, double* A, int64_t lda, double* b,
                                      void* hip_stream) {
    sgpr_plan_t plan;
    knn_status st = sgpr_plan(m, n, d, mem_limit_bytes, &plan);
    if (st != KNN_OK) return st;
    if (!(variance >= 0.0) || !(lengthscale > 0.0) || !std::isfinite(variance) ||
        !std::isfinite(lengthscale))
        return KNN_ERR_INVALID_ARG;
    if (!U || !A || !b || ldu < d || ldx < d || lda < m) return KNN_ERR_INVALID_ARG;
    if (n > 0 && (!X || !y)) return KNN_ERR_INVALID_ARG;
    if (!workspace || reinterpret_cast<uintptr_t>(workspace) % knn::kAlign != 0)
        return KNN_ERR_INVALID_ARG;
    if (workspace_bytes < plan.workspace_bytes) return KNN_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    float* Kc = static_cast<float*>(workspace);
    const float c2 = (float)(0.5 / (lengthscale * lengthscale) * 1.4426950408889634);

    const int G = plan.col_groups;
    const uint64_t chunk_bytes = knn::align_up((uint64_t)m * (uint64_t)plan.chunk_ld * 4);
    const uint64_t copy_bytes = knn::align_up((uint64_t)m * (uint64_t)m * 8);
    double* copies = reinterpret_cast<double*>(static_cast<unsigned char*>(workspace) + chunk_bytes);
    hipError_t e = sgpr::launch_zero(A, lda, b, m, stream);
    for (int g = 1; g < G && e == hipSuccess; ++g)
        e = sgpr::launch_zero(copies + (size_t)(g - 1) * (copy_bytes / 8), m, nullptr, m, stream);
    if (e != hipSuccess) return hip_fail(e, "sgpr zero kernel");
    for (int64_t c = 0; c < plan.n_chunks; ++c) {
        const int64_t c0 = c * plan.chunk_cols;
        const int64_t cols = n - c0 < plan.chunk_cols ? n - c0 : plan.chunk_cols;
        hipEvent_t t0 = knn::profile_mark(stream);
        e = sgpr::launch_kuf(U, ldu, X, ldx, m, c0, cols, d, c2, (float)variance, Kc, plan.chunk_ld,
                             stream);
        if (e != hipSuccess) {
            knn::profile_drop(t0);
            return hip_fail(e, "sgpr kernel-matrix chunk");
        }
        knn::profile_close(t0, stream, 0);
        hipEvent_t t1 = knn::profile_mark(stream);
        e = sgpr::launch_syrk(Kc, plan.chunk_ld, m, cols, G, A, lda, copies, (int64_t)(copy_bytes / 8),
                              stream);
        if (e != hipSuccess) {
            knn::profile_drop(t1);
            return hip_fail(e, "sgpr chunk product");
        }
        knn::profile_close(t1, stream, 1);
        hipEvent_t t2 = knn::profile_mark(stream);
        e = sgpr::launch_kufy(Kc, plan.chunk_ld, m, cols, y + c0, b, stream);
        if (e != hipSuccess) {
            knn::profile_drop(t2);
            return hip_fail(e, "sgpr chunk times y");
        }
        knn::profile_close(t2, stream, 2);
    }
    if (G > 1) {
        e = sgpr::launch_add_copies(A, lda, copies, (int64_t)(copy_bytes / 8), G - 1, m, stream);
        if (e != hipSuccess) return hip_fail(e, "sgpr add-copies kernel");
    }
    e = sgpr::launch_symmetrize(A, lda, m, stream);
    if (e != hipSuccess) return hip_fail(e, "sgpr symmetrize kernel");
    return KNN_OK;
}
