// Drives the host planner with seeded random clusters under AddressSanitizer / UBSan (built and run by
// tests/test_planner_sanitize.py).  Checks the invariants that need no oracle: every replica placed, C per
// device, every token routed to a holder of its expert.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "moe_planner.h"

// the planner reports errors through the library's error buffer; this driver links the planner alone
namespace moe {
void set_error(const char*, ...) {}
}  // namespace moe

static uint64_t rng_state = 1;
static uint64_t rnd() {
    rng_state += 0x9E3779B97F4A7C15ull;
    uint64_t z = rng_state;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

#define CHECK(c)                                                         \
    if (!(c)) {                                                          \
        std::fprintf(stderr, "check failed: %s (line %d)\n", #c, __LINE__); \
        return 1;                                                        \
    }

int main() {
    const moe_plan_cost cost{8192.0, 300e9, 25e9, 3.5e8, 3e14, 0};
    for (int iter = 0; iter < 300; ++iter) {
        const int D = 1 << (rnd() % 4), N = D * (1 + (int)(rnd() % 5)), C = 1 + (int)(rnd() % 4);
        const int E = 1 + (int)(rnd() % (uint64_t)(N * C));
        const moe_plan_shape s{N, E, C, D};
        std::vector<int64_t> R((size_t)N * E);
        for (auto& v : R) v = (int64_t)(rnd() % 5000) * (rnd() % 4 == 0 ? 0 : 1);
        std::vector<int32_t> rep(E), A((size_t)N * E), cands((size_t)6 * E);
        CHECK(moe_plan_replica_allocation(&s, R.data(), rep.data()) == MOE_OK);
        int64_t total = 0;
        for (int j = 0; j < E; ++j) { CHECK(rep[j] >= 1); total += rep[j]; }
        CHECK(total == (int64_t)N * C);
        double T = 0;
        int32_t best = -1;
        CHECK(moe_plan_expert_layout(&s, &cost, R.data(), 1 + (int)(rnd() % 6), rnd(), A.data(), &T, &best, cands.data()) == MOE_OK);
        for (int i = 0; i < N; ++i) {
            int c = 0;
            for (int j = 0; j < E; ++j) c += A[(size_t)i * E + j];
            CHECK(c == C);
        }
        std::vector<int64_t> S((size_t)N * E * N);
        CHECK(moe_plan_lite_routing(&s, R.data(), A.data(), S.data()) == MOE_OK);
        for (int i = 0; i < N; ++i)
            for (int j = 0; j < E; ++j) {
                int64_t sum = 0;
                for (int k = 0; k < N; ++k) {
                    const int64_t v = S[((size_t)i * E + j) * N + k];
                    CHECK(v >= 0 && (v == 0 || A[(size_t)k * E + j] > 0));
                    sum += v;
                }
                CHECK(sum == R[(size_t)i * E + j]);
            }
        double t3[3];
        CHECK(moe_plan_time_cost(&s, &cost, S.data(), t3) == MOE_OK);
        CHECK(t3[0] == T);  // the streamed cost of the layout search equals the cost of the materialised S
        std::vector<int32_t> eog((size_t)N * C), dog((size_t)N * C), rb(E + 1), rg((size_t)N * C);
        int32_t G = 0, nrep = 0;
        CHECK(moe_plan_dispatch_table(&s, A.data(), (int32_t)(rnd() % (uint64_t)N), &G, &nrep, eog.data(), dog.data(), rb.data(), rg.data()) == MOE_OK);
        CHECK(G == N * C && nrep <= G && rb[E] == nrep);
    }
    std::puts("planner fuzz ok");
    return 0;
}
