// C ABI of the kernel matrix-vector product (see include/kmv.h for the contract).
//
// The loop that paper section 4.3 generates for y = K v is here a fixed launch shape: the rows
// of K are spread over workgroups, the point axis is cut into ranges only to fill the GPU,
// and the only memory the library needs is one partial sum per row and range (plus the
// scaled norms of Z on the matrix-core path), all inside the caller's workspace.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstring>

#include "../../include/kmv.h"
#include "kmv_kernels.h"
#include "knn_config.h"

namespace knn {  // api.hip
void set_last_hip_error(hipError_t e, const char* what);
hipEvent_t profile_mark(hipStream_t stream);
void profile_close(hipEvent_t begin, hipStream_t stream, int kind);
void profile_drop(hipEvent_t begin);
}  // namespace knn

namespace {

int64_t align_up(int64_t v) { return (v + knn::kAlign - 1) / knn::kAlign * knn::kAlign; }

knn_status hip_fail(hipError_t e, const char* what) {
    knn::set_last_hip_error(e, what);
    return KNN_ERR_HIP;
}

}  // namespace

namespace {

int plan_impl(int64_t n, int64_t m, int32_t d, int64_t mem_limit_bytes, bool f64, kmv_plan_t* out) {
    if (!out) return KNN_ERR_INVALID_ARG;
    std::memset(out, 0, sizeof(*out));
    if (n < 0 || m < 0 || d < 1 || mem_limit_bytes < 0) return KNN_ERR_INVALID_ARG;
    if (n > knn::kMaxPoints || m > knn::kMaxPoints) return KNN_ERR_UNSUPPORTED;
    out->n = n;
    out->m = m;
    out->d = d;
    const bool valu = f64 || d <= kmv::kLowdMaxD;  // vector-ALU kernels: one row per lane
    const bool lowd = valu;
    out->path = d <= kmv::kLowdMaxD ? KMV_PATH_LOWD : (f64 ? KMV_PATH_VALU : KMV_PATH_MFMA);
    out->tile_rows = valu ? kmv::kLowdTileRows : kmv::kMfmaTileRows;
    out->n_splits = 1;
    out->norms_bytes = valu ? 0 : align_up(4 * m);
    out->min_limit_bytes = out->norms_bytes;
    if (mem_limit_bytes < out->min_limit_bytes) return KNN_ERR_MEM_LIMIT_TOO_SMALL;
    const int64_t tiles = (n + out->tile_rows - 1) / out->tile_rows;
    int S = 1;
    if (lowd) {
        // Ranges: double until the launch has enough workgroups for every CU to hold its share
        // (the low-d kernel runs 4 workgroups per CU), as long as a range keeps at least 2048
        // points and the partial sums fit under the limit.
        const int64_t want = 4 * (int64_t)knn::kNumCU;
        while (tiles > 0 && tiles * S < want && 2 * S <= kmv::kMaxSplits && m / (2 * S) >= 2048 &&
               out->norms_bytes + align_up(8 * n * (2 * S)) <= mem_limit_bytes)
            S *= 2;
    } else if (tiles > 0) {
        // The matrix-core kernel holds few workgroups per CU (2 or 3, by its registers), all of
        // the same length, so a launch runs in rounds and the last one may be nearly empty:
        // 1563 workgroups on 768 places take three rounds for two rounds' worth of work.
        // Ranges make the rounds shorter.  Cost of S ranges = rounds x (points per range + a
        // fixed start-up worth about 512 points); the smallest S within 4 % of the best is
        // taken, among those whose ranges keep 2048 points and whose partial sums fit.
        const int nch = (d + kmv::kMfmaKC - 1) / kmv::kMfmaKC;
        const int64_t places = (int64_t)knn::kNumCU * (nch <= 2 ? 3 : 2);
        auto cost = [&](int64_t s) {
            const int64_t rounds = (tiles * s + places - 1) / places;
            return (double)rounds * (double)((m + s - 1) / s + 512);
        };
        auto allowed = [&](int64_t s) {
            return s == 1 || (s <= kmv::kMaxSplits && m / s >= 2048 &&
                              out->norms_bytes + align_up(8 * n * s) <= mem_limit_bytes);
        };
        static const int kCandidates[] = {1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 48, 64};
        double best = cost(1);
        for (int s : kCandidates)
            if (allowed(s) && cost(s) < best) best = cost(s);
        for (int s : kCandidates)
            if (allowed(s) && cost(s) <= 1.04 * best) {
                S = s;
                break;
            }
    }
    out->n_splits = S;
    out->partials_bytes = S > 1 ? align_up(8 * n * S) : 0;
    out->workspace_bytes = out->norms_bytes + out->partials_bytes;
    return KNN_OK;
}

}  // namespace

extern "C" int kmv_plan(int64_t n, int64_t m, int32_t d, int64_t mem_limit_bytes, kmv_plan_t* out) {
    return plan_impl(n, m, d, mem_limit_bytes, false, out);
}

extern "C" int kmv_plan_f64(int64_t n, int64_t m, int32_t d, int64_t mem_limit_bytes,
                            kmv_plan_t* out) {
    return plan_impl(n, m, d, mem_limit_bytes, true, out);
}

extern "C" int kmv_apply(const float* X, int64_t ldx, const float* Z, int64_t ldz, const float* v,
                         int64_t n, int64_t m, int32_t d, double variance, double lengthscale,
                         int64_t mem_limit_bytes, void* workspace, int64_t workspace_bytes,
                         double* y, void* stream_v) {
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    kmv_plan_t plan;
    const int rc = kmv_plan(n, m, d, mem_limit_bytes, &plan);
    if (rc != KNN_OK) return rc;
    if (!(variance >= 0.0) || !(lengthscale > 0.0) || !std::isfinite(variance) ||
        !std::isfinite(lengthscale))
        return KNN_ERR_INVALID_ARG;
    if (ldx < d || ldz < d) return KNN_ERR_INVALID_ARG;
    if (n == 0) return KNN_OK;
    if (!y || !X) return KNN_ERR_INVALID_ARG;
    if (m > 0 && (!Z || !v)) return KNN_ERR_INVALID_ARG;
    if (plan.workspace_bytes > 0) {
        if (!workspace || reinterpret_cast<uintptr_t>(workspace) % knn::kAlign != 0)
            return KNN_ERR_INVALID_ARG;
        if (workspace_bytes < plan.workspace_bytes) return KNN_ERR_WORKSPACE_TOO_SMALL;
    }
    hipError_t e;
    if (m == 0) {
        e = kmv::launch_zero(y, n, stream);
        return e == hipSuccess ? KNN_OK : hip_fail(e, "kmv zero");
    }
    // K = variance * exp2(-c2 * sqdist)
    const float c2 = (float)(0.5 / (lengthscale * lengthscale) * 1.4426950408889634);
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    float* zn = reinterpret_cast<float*>(ws);
    double* partials = reinterpret_cast<double*>(ws + plan.norms_bytes);
    const int S = plan.n_splits;
    double* target = S > 1 ? partials : y;
    if (plan.path == KMV_PATH_LOWD) {
        hipEvent_t t1 = knn::profile_mark(stream);
        e = kmv::launch_lowd(X, ldx, Z, ldz, v, n, m, d, c2, variance, S, target, stream);
        if (e != hipSuccess) {
            knn::profile_drop(t1);
            return hip_fail(e, "kmv low-d kernel");
        }
        knn::profile_close(t1, stream, 1);
    } else {
        e = kmv::launch_scaled_norms(Z, ldz, m, d, c2, zn, stream);
        if (e != hipSuccess) return hip_fail(e, "kmv norms kernel");
        hipEvent_t t1 = knn::profile_mark(stream);
        e = kmv::launch_mfma(X, ldx, Z, ldz, v, zn, n, m, d, c2, variance, S, target, stream);
        if (e != hipSuccess) {
            knn::profile_drop(t1);
            return hip_fail(e, "kmv matrix-core kernel");
        }
        knn::profile_close(t1, stream, 1);
    }
    if (S > 1) {
        e = kmv::launch_reduce(partials, S, n, y, stream);
        if (e != hipSuccess) return hip_fail(e, "kmv reduce kernel");
    }
    return KNN_OK;
}

extern "C" int kmv_apply_f64(const double* X, int64_t ldx, const double* Z, int64_t ldz,
                             const double* v, int64_t n, int64_t m, int32_t d, double variance,
                             double lengthscale, int64_t mem_limit_bytes, void* workspace,
                             int64_t workspace_bytes, double* y, void* stream_v) {
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    kmv_plan_t plan;
    const int rc = kmv_plan_f64(n, m, d, mem_limit_bytes, &plan);
    if (rc != KNN_OK) return rc;
    if (!(variance >= 0.0) || !(lengthscale > 0.0) || !std::isfinite(variance) ||
        !std::isfinite(lengthscale))
        return KNN_ERR_INVALID_ARG;
    if (ldx < d || ldz < d) return KNN_ERR_INVALID_ARG;
    if (n == 0) return KNN_OK;
    if (!y || !X) return KNN_ERR_INVALID_ARG;
    if (m > 0 && (!Z || !v)) return KNN_ERR_INVALID_ARG;
    if (plan.workspace_bytes > 0) {
        if (!workspace || reinterpret_cast<uintptr_t>(workspace) % knn::kAlign != 0)
            return KNN_ERR_INVALID_ARG;
        if (workspace_bytes < plan.workspace_bytes) return KNN_ERR_WORKSPACE_TOO_SMALL;
    }
    hipError_t e;
    if (m == 0) {
        e = kmv::launch_zero(y, n, stream);
        return e == hipSuccess ? KNN_OK : hip_fail(e, "kmv zero");
    }
    const double negc = -0.5 / (lengthscale * lengthscale);
    double* partials = static_cast<double*>(workspace);
    const int S = plan.n_splits;
    hipEvent_t t1 = knn::profile_mark(stream);
    e = kmv::launch_f64(X, ldx, Z, ldz, v, n, m, d, negc, variance, S, S > 1 ? partials : y, stream);
    if (e != hipSuccess) {
        knn::profile_drop(t1);
        return hip_fail(e, "kmv fp64 kernel");
    }
    knn::profile_close(t1, stream, 1);
    if (S > 1) {
        e = kmv::launch_reduce(partials, S, n, y, stream);
        if (e != hipSuccess) return hip_fail(e, "kmv reduce kernel");
    }
    return KNN_OK;
}
