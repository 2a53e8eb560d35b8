// Walk through every entry point of the C ABI on nine problem sizes (both recurrence kernels,
// every flag, the B sweep, table construction, the equal-layer restriction, placement,
// operator clustering, two error paths), meant to be built with the host code under
// AddressSanitizer and run on a GPU machine:
//
//   hipcc --offload-arch=gfx950 -O1 -g -std=c++17 -Xarch_host -fsanitize=address \
//         -Xclang -target-feature -Xclang -packed-fp32-ops -Iinclude \
//         -o asan_driver tests/asan_driver.cpp paper_2201_12023_amd/csrc/*.hip
//   ASAN_OPTIONS=detect_leaks=0 ./asan_driver
//
// It checks return codes only (results are the parity tests' business) and prints "ALL OK".
#include "../include/alpa_dp.h"
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>
#include <random>
#include <unistd.h>
#define CK(x) do { int rc_ = (x); if (rc_) { printf("FAIL %s -> %d (%s)\n", #x, rc_, alpa_dp_last_error()); return 1; } } while (0)
static std::vector<alpa_shape_t> shapes_of(int N, int M) {
    std::vector<alpa_shape_t> s;
    for (int m = 1; m <= M; m *= 2) s.push_back({1, m});
    for (int n = 2; n <= N; ++n) s.push_back({n, M});
    return s;
}
int main() {
    std::mt19937 rng(7);
    struct Case { int K, N, M, B; } cases[] = {{1,1,1,1},{7,1,4,3},{24,2,8,32},{64,8,8,128},{70,3,8,5},{40,16,8,9},{100,9,8,4},{130,2,4,2},{20,40,8,2}};
    for (auto c : cases) {
        auto sh = shapes_of(c.N, c.M); int S = (int)sh.size();
        printf("case K=%d %dx%d S=%d\n", c.K, c.N, c.M, S); fflush(stdout);
        std::vector<int32_t> tab((size_t)c.K * c.K * c.K * S);
        for (auto &v : tab) v = (rng() % 5 == 0) ? ALPA_DP_INF_I32 : (int32_t)(1 + rng() % 500);
        alpa_dp_t *h = nullptr;
        CK(alpa_dp_create(&h, tab.data(), c.K, c.N, c.M, c.B, sh.data(), S));
        int n = 0; CK(alpa_dp_count_candidates(h, &n));
        std::vector<int64_t> T(n > 0 ? n : 1);
        alpa_plan_t plan;
        CK(alpa_dp_solve(h, nullptr, 0, 0, T.data(), &plan));
        CK(alpa_dp_solve(h, nullptr, 0, ALPA_DP_PRUNE, T.data(), &plan));
        for (int key_value : {ALPA_DP_TUNE_CANDIDATES_PER_WG * 16 + 2, ALPA_DP_TUNE_CANDIDATES_PER_WG * 16 + 0,
                              ALPA_DP_TUNE_DISTINCT_BY_SORT * 16 + 1, ALPA_DP_TUNE_DISTINCT_BY_SORT * 16 + 0,
                              ALPA_DP_TUNE_LANE_GROUPS * 16 + 1, ALPA_DP_TUNE_LANE_GROUPS * 16 + 4,
                              ALPA_DP_TUNE_LANE_GROUPS * 16 + 0, ALPA_DP_TUNE_WG_PER_CU * 16 + 1,
                              ALPA_DP_TUNE_WG_PER_CU * 16 + 0, ALPA_DP_TUNE_WORKGROUPS * 16 + 3,
                              ALPA_DP_TUNE_WORKGROUPS * 16 + 0}) {
            CK(alpa_dp_set_tuning(h, key_value / 16, key_value % 16));
            CK(alpa_dp_solve(h, nullptr, 0, ALPA_DP_PRUNE, T.data(), &plan));
        }
        if (n >= 2) CK(alpa_dp_solve(h, nullptr, 2, ALPA_DP_GENERIC, T.data(), &plan));
        std::vector<int32_t> cand = {5, 500, 17, 17, 250, 0, 499};
        std::vector<int64_t> T2(cand.size());
        CK(alpa_dp_solve(h, cand.data(), (int)cand.size(), ALPA_DP_COUNT_WORK, T2.data(), &plan));
        CK(alpa_dp_solve(h, cand.data(), (int)cand.size(), ALPA_DP_GENERIC | ALPA_DP_PRUNE, T2.data(), nullptr));
        std::vector<int32_t> Bs = {1, 2, 64, 1000};
        std::vector<alpa_plan_t> plans(Bs.size());
        CK(alpa_dp_solve_sweep(h, nullptr, 0, 0, Bs.data(), (int)Bs.size(), plans.data()));
        CK(alpa_dp_solve_sweep(h, cand.data(), (int)cand.size(), ALPA_DP_PRUNE, Bs.data(), (int)Bs.size(), plans.data()));
        std::vector<int32_t> out(n + 4); int got = 0;
        CK(alpa_dp_candidates(h, out.data(), n + 4, &got));
        CK(alpa_dp_best(h, &plan));
        float a, b, d; CK(alpa_dp_last_timing(h, &a, &b, &d));
        int nc; int64_t wr; CK(alpa_dp_last_counters(h, &nc, &wr));
        CK(alpa_dp_set_B(h, 7));
        CK(alpa_dp_best(h, &plan));                 // no solve since the change of B: solves itself
        std::vector<int32_t> back(tab.size());
        CK(alpa_dp_get_table(h, back.data()));
        CK(alpa_dp_restrict_equal_layers(h));
        CK(alpa_dp_solve(h, nullptr, 0, 0, nullptr, &plan));
        if (plan.num_stages > 0) {
            std::vector<alpa_shape_t> st(plan.num_stages); std::vector<int32_t> r(plan.num_stages), cc(plan.num_stages);
            for (int p = 0; p < plan.num_stages; ++p) st[p] = sh[plan.shape_idx[p]];
            CK(alpa_place_submeshes(c.N, c.M, st.data(), plan.num_stages, r.data(), cc.data()));
        }
        alpa_dp_destroy(h);
        // profiles
        int O = 3; size_t np = (size_t)c.K * c.K * S * O;
        std::vector<int32_t> tl(np); std::vector<int64_t> ms(np), ma(np);
        for (size_t x = 0; x < np; ++x) { tl[x] = (rng() % 7 == 0) ? ALPA_DP_INF_I32 : (int32_t)(1 + rng() % 900); ms[x] = rng() % 1000; ma[x] = rng() % 50; }
        CK(alpa_dp_create_from_profiles(&h, tl.data(), ms.data(), ma.data(), O, 1500, c.K, c.N, c.M, c.B, sh.data(), S));
        CK(alpa_dp_solve(h, nullptr, 0, ALPA_DP_PRUNE, nullptr, &plan));
        alpa_dp_destroy(h);
    }
    // error paths
    alpa_dp_t *h = nullptr; alpa_shape_t bad = {3, 3};
    int32_t one = 5;
    printf("einval %d %d\n", alpa_dp_create(&h, &one, 1, 1, 1, 1, &bad, 1), alpa_dp_create(nullptr, nullptr, 0, 0, 0, 0, nullptr, 0)); fflush(stdout);
    // clustering
    for (int K : {1, 5, 100, 962}) {
        int E = 3 * K; std::vector<int32_t> flop(K), es, ed; std::vector<int64_t> eb;
        for (auto &f : flop) f = 1 + rng() % 9;
        for (int e = 0; e < E && K > 1; ++e) { int a = rng() % (K - 1); int b = a + 1 + rng() % (K - 1 - a); es.push_back(a); ed.push_back(b); eb.push_back(rng() % 1000); }
        for (int L : {1, 4, 64}) {
            if (L > K) continue;
            int64_t comm, sq; std::vector<int32_t> first(L + 1); float ms;
            CK(alpa_cluster_layers(flop.data(), K, es.data(), ed.data(), eb.data(), (int)es.size(), L, 500000, &comm, &sq, first.data(), &ms));
            CK(alpa_cluster_layers_exact(flop.data(), K, es.data(), ed.data(), eb.data(), (int)es.size(), L, 500000, &comm, &sq, first.data(), &ms));
        }
    }
    double pk; CK(alpa_dp_measure_valu_peak(&pk));
    printf("ALL OK peak %.3g\n", pk);
    fflush(stdout);
    _exit(0);   // the runtime's own teardown trips the sanitizer's allocator check
}
