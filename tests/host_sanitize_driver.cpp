// Host-only entry points of the library under AddressSanitizer / UBSan: random and hostile
// arguments, with the invariants the header promises checked on every accepted call.
// Built and run by tests/test_host_sanitizers.py (g++ -fsanitize=address,undefined).
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "nezha_sim.h"

#define REQUIRE(c)                                                         \
    do {                                                                   \
        if (!(c)) {                                                        \
            std::fprintf(stderr, "line %d: %s\n", __LINE__, #c);           \
            return 1;                                                      \
        }                                                                  \
    } while (0)

int main()
{
    std::mt19937_64 rng(12345);
    auto pick = [&](uint64_t lo, uint64_t hi) { return lo + rng() % (hi - lo + 1); };

    for (int it = 0; it < 20000; ++it) {
        const uint32_t R = (uint32_t)pick(1, 8), N = (uint32_t)pick(1, 128);
        const uint32_t e = pick(0, 1) ? 2 : 4;
        std::vector<uint32_t> w(R);
        uint64_t W = 0;
        for (auto &x : w) {
            x = pick(0, 3) == 0 ? 0 : (uint32_t)pick(0, pick(0, 1) ? 200 : 0xffffffffu);
            W += x;
        }
        const uint64_t n = pick(0, 2) == 0 ? pick(0, 5000) : pick(0, (uint64_t)1 << pick(1, 60));
        std::vector<uint64_t> b(R + 1, 77);
        const nz_status s = nz_rail_partition(n, e, w.data(), R, b.data());
        if (W == 0) {
            REQUIRE(s == NZ_ERR_INVALID_ARG);
            continue;
        }
        REQUIRE(s == NZ_OK);
        REQUIRE(b[0] == 0 && b[R] == n);
        for (uint32_t k = 0; k < R; ++k) {
            REQUIRE(b[k] <= b[k + 1]);
            if (w[k] == 0) REQUIRE(b[k] == b[k + 1]);
            if (k > 0 && b[k] != n) REQUIRE(b[k] % (256 / e) == 0);
        }
        std::vector<uint64_t> seg((size_t)R * (N + 1), 99);
        REQUIRE(nz_segment_map(b.data(), R, N, seg.data()) == NZ_OK);
        for (uint32_t k = 0; k < R; ++k) {
            const uint64_t *row = &seg[(size_t)k * (N + 1)];
            REQUIRE(row[0] == b[k] && row[N] == b[k + 1]);
            uint64_t prev = UINT64_MAX;
            for (uint32_t j = 0; j < N; ++j) {
                const uint64_t len = row[j + 1] - row[j];
                REQUIRE(row[j] <= row[j + 1]);
                REQUIRE(prev == UINT64_MAX || len == prev || len + 1 == prev);
                prev = len;
            }
        }
        std::vector<uint8_t> alive(R);
        bool any = false;
        for (auto &a : alive) {
            a = (uint8_t)pick(0, 1);
            any = any || a;
        }
        uint32_t target = 1234;
        const nz_status f = nz_failover_target(b.data(), R, alive.data(), &target);
        REQUIRE(f == (any ? NZ_OK : NZ_ERR_INVALID_ARG));
        if (any) {
            REQUIRE(target < R && alive[target]);
            for (uint32_t k = 0; k < R; ++k)
                if (alive[k]) REQUIRE(b[k + 1] - b[k] <= b[target + 1] - b[target]);
        }

        std::vector<nz_rail_model> m(R);
        for (auto &r : m) {
            r.setup_s = (double)pick(1, 1000) * 1e-6;
            r.bytes_per_s = (double)pick(1, 20000) * 1e6;
        }
        std::vector<double> alpha(R);
        std::vector<uint32_t> ratios(R);
        double tc, th, thr;
        uint32_t best;
        int hot;
        const double S = (double)pick(0, (uint64_t)1 << pick(1, 36));
        REQUIRE(nz_balance(m.data(), R, S, alpha.data(), ratios.data(), &tc, &th, &best, &hot) == NZ_OK);
        double asum = 0;
        uint64_t rsum = 0;
        for (uint32_t k = 0; k < R; ++k) {
            REQUIRE(alpha[k] >= 0.0 && alpha[k] <= 1.0 + 1e-12);
            asum += alpha[k];
            rsum += ratios[k];
        }
        REQUIRE(std::fabs(asum - 1.0) < 1e-9 && rsum == NZ_RATIO_SCALE);
        REQUIRE(th <= tc * (1 + 1e-12) && best < R);
        REQUIRE(nz_balance_threshold(m.data(), R, &thr) == NZ_OK && thr >= 0.0);
        REQUIRE((hot != 0) == (S > thr));
        // Eq. 2 and Eq. 3 on the same model, with the balancer's own shares and with an even split
        double delta = -1.0, rho = -1.0;
        if (S > 0.0) {
            REQUIRE(nz_net_efficiency(&m[0], S, &delta) == NZ_OK && delta > 0.0 && delta <= 1.0);
            REQUIRE(nz_efficiency_ratio(m.data(), R, S, alpha.data(), &rho) == NZ_OK && rho >= 1.0);
            REQUIRE(nz_efficiency_ratio(m.data(), R, S, nullptr, &rho) == NZ_OK && rho >= 1.0);
        }
    }

    // hostile arguments: nothing may be written or read out of bounds, only statuses returned
    uint64_t out[4] = {0, 0, 0, 0};
    const uint32_t w1[2] = {1, 1};
    REQUIRE(nz_rail_partition(10, 4, nullptr, 2, out) == NZ_ERR_INVALID_ARG);
    REQUIRE(nz_rail_partition(10, 4, w1, 2, nullptr) == NZ_ERR_INVALID_ARG);
    REQUIRE(nz_rail_partition(10, 4, w1, 0, out) == NZ_ERR_INVALID_ARG);
    REQUIRE(nz_rail_partition(10, 3, w1, 2, out) == NZ_ERR_INVALID_ARG);
    REQUIRE(nz_rail_partition(UINT64_MAX, 4, w1, 2, out) == NZ_ERR_INVALID_ARG);
    REQUIRE(nz_rail_partition_ex(10, 4, 0, w1, 2, out) == NZ_ERR_INVALID_ARG);
    REQUIRE(nz_rail_partition_ex(10, 4, 6, w1, 2, out) == NZ_ERR_INVALID_ARG);
    REQUIRE(nz_segment_map(nullptr, 1, 1, out) == NZ_ERR_INVALID_ARG);
    REQUIRE(nz_segment_map(out, 1, 0, out) == NZ_ERR_INVALID_ARG);
    const uint64_t bad[3] = {0, 10, 5};
    REQUIRE(nz_segment_map(bad, 2, 3, out) == NZ_ERR_INVALID_ARG);
    REQUIRE(nz_failover_target(nullptr, 1, nullptr, nullptr) == NZ_ERR_INVALID_ARG);
    nz_rail_model one = {1e-3, 0.0};
    REQUIRE(nz_balance(&one, 1, 1.0, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == NZ_ERR_INVALID_ARG);
    one.bytes_per_s = 1e9;
    REQUIRE(nz_balance(&one, 1, -1.0, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == NZ_ERR_INVALID_ARG);
    REQUIRE(nz_balance(&one, 1, 1.0, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == NZ_OK);
    REQUIRE(nz_balance(nullptr, 1, 1.0, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == NZ_ERR_INVALID_ARG);
    REQUIRE(nz_balance(&one, 9, 1.0, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr) == NZ_ERR_UNSUPPORTED);
    double d = 0.0;
    const double zero_shares[1] = {0.0};
    REQUIRE(nz_net_efficiency(nullptr, 1.0, &d) == NZ_ERR_INVALID_ARG);
    REQUIRE(nz_net_efficiency(&one, 1.0, nullptr) == NZ_ERR_INVALID_ARG);
    REQUIRE(nz_net_efficiency(&one, 0.0, &d) == NZ_ERR_INVALID_ARG);
    REQUIRE(nz_efficiency_ratio(&one, 1, 1.0, zero_shares, &d) == NZ_ERR_INVALID_ARG);
    REQUIRE(nz_efficiency_ratio(&one, 9, 1.0, nullptr, &d) == NZ_ERR_UNSUPPORTED);
    REQUIRE(nz_efficiency_ratio(&one, 1, 1.0, nullptr, &d) == NZ_OK && d == 1.0);
    for (int st = 0; st < 8; ++st) REQUIRE(nz_status_str((nz_status)st) != nullptr);
    std::puts("host sanitizer run ok");
    return 0;
}
