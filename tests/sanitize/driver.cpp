// Host-side sanitizer run: the planner (planner.cpp) and the CPU oracle (oracle/knn_oracle.c)
// built with AddressSanitizer and UndefinedBehaviorSanitizer, driven over seeded random shapes.
// Planner: every plan the planner accepts must account for its workspace and stay under the limit
// (paper section 4.4: every live buffer counts); oracle: heap selection and the written-out
// definition (all distances, one sort) must agree on tiny inputs.  Any sanitizer report aborts.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../../include/knn.h"

extern "C" {
int oracle_knn_metric(const float*, int64_t, const float*, int64_t, int64_t, int32_t, int32_t, const int64_t*,
                      int64_t, int64_t*, double*, double*, int32_t, int32_t);
int oracle_knn_fullsort_metric(const float*, int64_t, const float*, int64_t, int64_t, int32_t, int32_t,
                               const int64_t*, int64_t, int64_t*, double*, double*, int32_t);
double oracle_sqdist(const float*, const float*, int32_t);
}

static uint64_t state = 0x9E3779B97F4A7C15ull;
static uint64_t rnd() {
    state ^= state << 13;
    state ^= state >> 7;
    state ^= state << 17;
    return state;
}
static int64_t pick(const int64_t* v, int n) { return v[rnd() % (uint64_t)n]; }

#define CHECK(c)                                                               \
    do {                                                                       \
        if (!(c)) {                                                            \
            fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #c);    \
            return 1;                                                          \
        }                                                                      \
    } while (0)

int main() {
    // ---- planner fuzz ----
    const int64_t ms[] = {0, 1, 7, 255, 256, 257, 5000, 100000, 1000000};
    const int64_t ns[] = {1, 2, 63, 64, 65, 4096, 65536, 70001, 1000000, 10000000, 2147418111};
    const int64_t ds[] = {1, 2, 3, 4, 8, 9, 16, 17, 100, 128, 129, 256, 257, 784, 5000};
    const int64_t ks[] = {1, 2, 10, 16, 32, 100, 1024};
    const uint64_t extra[] = {0, 1, 255, 4096, 1000000, 100000000, 10000000000ull, 1ull << 40};
    int plans = 0, refused = 0;
    for (int it = 0; it < 20000; ++it) {
        const int64_t m = pick(ms, 9), n = pick(ns, 11);
        const int32_t d = (int32_t)pick(ds, 15), k = (int32_t)pick(ks, 7);
        const knn_metric metric = (knn_metric)(rnd() % 3);
        knn_plan_t big;
        knn_status st = knn_plan_metric(m, n, d, k, metric, UINT64_MAX / 4, &big);
        if (k > n) {
            CHECK(st == KNN_ERR_INVALID_ARG);
            continue;
        }
        CHECK(st == KNN_OK);
        const uint64_t limit = big.min_limit_bytes + extra[rnd() % 8];
        knn_plan_t p;
        st = knn_plan_metric(m, n, d, k, metric, limit, &p);
        CHECK(st == KNN_OK);
        ++plans;
        if (m == 0) continue;
        CHECK(p.workspace_bytes == p.norms_bytes + p.query_bytes + p.lists_bytes);
        CHECK(p.workspace_bytes + p.private_bytes <= limit);
        CHECK(p.chunk_rows >= 1 && p.q_chunks * p.chunk_rows >= m && (p.q_chunks - 1) * p.chunk_rows < m);
        CHECK(p.lists_bytes >= (uint64_t)p.chunk_rows * (uint64_t)p.n_splits * (uint64_t)k * 8);
        CHECK(p.n_splits >= 1 && p.tile_q >= 1);
        if (big.min_limit_bytes > 0) {
            knn_plan_t q;
            if (knn_plan_metric(m, n, d, k, metric, big.min_limit_bytes - 1, &q) != KNN_OK) ++refused;
        }
        knn_host_plan_t hp;
        st = knn_plan_host_x(m, n, d, k, metric, limit, &hp);
        if (st == KNN_OK) CHECK(hp.workspace_bytes <= limit && hp.n_blocks * hp.block_rows >= n);
        else CHECK(st == KNN_ERR_MEM_LIMIT_TOO_SMALL);
    }
    CHECK(refused > 0);
    uint64_t bytes = 0;
    CHECK(knn_parse_size("1GB", &bytes) == KNN_OK && bytes == 1000000000ull);
    CHECK(knn_parse_size("12XB", &bytes) == KNN_ERR_INVALID_ARG);
    CHECK(knn_chunk_rows(1000000000ull, 8000000ull) == 125);  // the appendix example
    // ---- oracle: heap selection against the definition, all three metrics ----
    int rows_checked = 0;
    for (int it = 0; it < 300; ++it) {
        const int64_t n = 1 + (int64_t)(rnd() % 40), m = 1 + (int64_t)(rnd() % 6);
        const int32_t d = 1 + (int32_t)(rnd() % 9);
        const int32_t k = 1 + (int32_t)(rnd() % (uint64_t)n);
        const int64_t ld = d + (int64_t)(rnd() % 3);
        std::vector<float> X((size_t)(n * ld)), Q((size_t)(m * ld));
        for (auto& v : X) v = (float)((int)(rnd() % 9) - 4) * 0.5f;  // a coarse grid: many ties
        for (auto& v : Q) v = (float)((int)(rnd() % 9) - 4) * 0.5f;
        for (int32_t metric = 0; metric < 3; ++metric) {
            std::vector<int64_t> i1((size_t)(m * k)), i2((size_t)(m * k));
            std::vector<double> d1((size_t)(m * k)), d2((size_t)(m * k)), n1((size_t)m), n2((size_t)m);
            CHECK(oracle_knn_metric(Q.data(), ld, X.data(), ld, n, d, k, nullptr, m, i1.data(), d1.data(),
                                    n1.data(), 2, metric) == 0);
            CHECK(oracle_knn_fullsort_metric(Q.data(), ld, X.data(), ld, n, d, k, nullptr, m, i2.data(),
                                             d2.data(), n2.data(), metric) == 0);
            for (size_t e = 0; e < i1.size(); ++e) CHECK(i1[e] == i2[e] && d1[e] == d2[e]);
            for (int64_t r = 0; r < m; ++r) CHECK(n1[(size_t)r] == n2[(size_t)r] || (std::isinf(n1[(size_t)r]) && std::isinf(n2[(size_t)r])));
            rows_checked += (int)m;
        }
    }
    const float a[3] = {1.f, 2.f, 3.f}, b[3] = {4.f, 6.f, 3.f};
    CHECK(oracle_sqdist(a, b, 3) == 25.0);
    printf("sanitizer driver ok: %d plans, %d limits refused one byte below the minimum, %d oracle rows\n",
           plans, refused, rows_checked);
    return 0;
}
