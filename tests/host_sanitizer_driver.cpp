// Exercises the host-only parts of the library (planner, evaluator, exact optimum, cost model, table
// builder) on random and degenerate inputs.  Built by tests/test_host_sanitizers.py with
// -fsanitize=address,undefined; any finding aborts the run.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "mgwfbp.h"
#include "tables.h"

#define REQUIRE(cond) do { if (!(cond)) { std::fprintf(stderr, "REQUIRE failed: %s (line %d)\n", #cond, __LINE__); std::abort(); } } while (0)

int main() {
    std::mt19937_64 rng(1912);
    auto uni = [&](double lo, double hi) { return std::uniform_real_distribution<double>(lo, hi)(rng); };
    for (int trial = 0; trial < 400; ++trial) {
        const int32_t L = static_cast<int32_t>(rng() % 70);
        std::vector<uint64_t> n(static_cast<size_t>(L)), bytes(static_cast<size_t>(L));
        std::vector<double> tb(static_cast<size_t>(L));
        for (int32_t i = 0; i < L; ++i) {
            const int kind = static_cast<int>(rng() % 10);
            n[i] = kind == 0 ? 0 : (kind == 1 ? 1 : static_cast<uint64_t>(std::exp(uni(0, 11))));
            bytes[i] = n[i] * 4;
            tb[i] = kind == 2 ? 0.0 : uni(1e-6, 5e-4);
        }
        const double a = std::pow(10.0, uni(-6, -3)), b = std::pow(10.0, uni(-11, -8));
        std::vector<uint8_t> merged(static_cast<size_t>(L) + 1), opt(static_cast<size_t>(L) + 1);
        std::vector<int32_t> first(static_cast<size_t>(L) + 1);
        int32_t G = -1, G2 = -1;
        double t = -1, t_opt = -1, t_eval = -1;
        REQUIRE(mgwfbp_plan(bytes.data(), tb.data(), L, a, b, merged.data(), first.data(), &G) == MGWFBP_OK);
        REQUIRE(mgwfbp_eval(merged.data(), bytes.data(), tb.data(), L, a, b, &t) == MGWFBP_OK);
        REQUIRE(mgwfbp_plan_opt(bytes.data(), tb.data(), L, a, b, opt.data(), first.data(), &G2, &t_opt) == MGWFBP_OK);
        REQUIRE(mgwfbp_eval(opt.data(), bytes.data(), tb.data(), L, a, b, &t_eval) == MGWFBP_OK);
        REQUIRE(t_opt == t_eval && t_opt <= t);
        REQUIRE(L == 0 || (merged[0] == 0 && opt[0] == 0 && G >= 1 && G2 >= 1 && first[G2] == -1));

        HostTables tab;
        REQUIRE(mgwfbp_build_tables(n.data(), L, merged.data(), tab) == MGWFBP_OK);
        REQUIRE(tab.G == G && tab.group_tile.size() == static_cast<size_t>(G) + 1);
        uint64_t total = 0, sum_groups = 0;
        for (uint64_t x : n) total += x;
        for (uint64_t x : tab.group_elems) sum_groups += x;
        REQUIRE(total == sum_groups);                                   // buffers total the model size (Sec. 5.3)
        REQUIRE(tab.arena_elems == tab.tiles.size() * static_cast<uint64_t>(MGWFBP_TILE_ELEMS));
        for (const TileHdr& h : tab.tiles) {
            REQUIRE(h.nseg >= 1 && h.valid >= 1 && h.valid <= MGWFBP_TILE_ELEMS && h.first_start <= 0);
            REQUIRE(h.first_end >= 1 && h.first_end <= h.valid);
            REQUIRE(static_cast<size_t>(h.seg0 + h.nseg) <= tab.seg_layer.size());
        }

        int32_t counts[3] = {2, 16, 512};
        double tw[3], ts[3], tm[3];
        int32_t g[3];
        REQUIRE(mgwfbp_simulate(bytes.data(), tb.data(), L, 0.01, MGWFBP_AR_RING, 5e-5, 1e-9, 1e-11, counts, 3, tw, ts, tm, g) == MGWFBP_OK);
        if (L > 0) REQUIRE(tm[0] <= tw[0] * (1 + 1e-12));
    }
    // rejected inputs leave no trace
    uint8_t m2[2] = {1, 0};
    uint64_t n2[2] = {4, 4};
    double tb2[2] = {1.0, NAN};
    HostTables tab;
    double out;
    REQUIRE(mgwfbp_build_tables(n2, 2, m2, tab) == MGWFBP_EINVAL);
    REQUIRE(mgwfbp_plan(n2, tb2, 2, 1.0, 1.0, m2, nullptr, nullptr) == MGWFBP_EINVAL);
    REQUIRE(mgwfbp_eval(m2, n2, tb2, 2, 1.0, 1.0, &out) == MGWFBP_EINVAL);
    REQUIRE(mgwfbp_fit_ab(n2, tb2, 2, &out, &out) == MGWFBP_EINVAL);
    double a, b;
    for (int algo = 0; algo < 5; ++algo) REQUIRE(mgwfbp_allreduce_ab(algo, 64, 1e-5, 1e-9, 1e-10, &a, &b) == MGWFBP_OK && a > 0 && b > 0);
    std::puts("host sanitizer driver: ok");
    return 0;
}
