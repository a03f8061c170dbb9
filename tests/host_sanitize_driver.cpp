// Host-only entry points of the library under AddressSanitizer / UBSan: random and hostile
// arguments, with the invariants the header promises checked on every accepted call.
// Built and run by tests/test_host_sanitizers.py (g++ -fsanitize=address,undefined).
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <utility>
#include <vector>

#include "nezha_sim.h"
#include "nz_internal.h"

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
        // the paper's iteration (Eq. 8 start, Eq. 7 steps) never does worse than its start and
        // never beats the closed-form minimum
        if (S > 0.0) {
            double th0 = 0.0, th100 = 0.0;
            uint32_t used = 0;
            REQUIRE(nz_balance_iterate(m.data(), R, S, 0, nullptr, nullptr, &th0, nullptr) == NZ_OK);
            REQUIRE(nz_balance_iterate(m.data(), R, S, 100, alpha.data(), ratios.data(), &th100, &used) == NZ_OK);
            REQUIRE(used <= 100 && th100 <= th0 * (1 + 1e-12));
            const double closed = hot ? th : tc;
            REQUIRE(th100 >= closed * (1 - 1e-9));
            uint64_t rs2 = 0;
            for (uint32_t k = 0; k < R; ++k) rs2 += ratios[k];
            REQUIRE(rs2 == NZ_RATIO_SCALE);
        }
        // Eq. 2 and Eq. 3 on the same model, with the balancer's own shares and with an even split
        double delta = -1.0, rho = -1.0;
        if (S > 0.0) {
            REQUIRE(nz_net_efficiency(&m[0], S, &delta) == NZ_OK && delta > 0.0 && delta <= 1.0);
            REQUIRE(nz_efficiency_ratio(m.data(), R, S, alpha.data(), &rho) == NZ_OK && rho >= 1.0);
            REQUIRE(nz_efficiency_ratio(m.data(), R, S, nullptr, &rho) == NZ_OK && rho >= 1.0);
        }
    }

    // The buffer-overlap rules (nz_validate.cpp) on made-up addresses, which are compared and
    // never dereferenced, against the rules applied pair by pair:
    //   a written buffer may not partly overlap any other buffer;
    //   where distinct outputs are needed, outputs are pairwise different and an output may be
    //   its own node's input only.
    for (int it = 0; it < 40000; ++it) {
        const uint32_t N = (uint32_t)pick(1, pick(0, 3) ? 6 : 128);
        const uint64_t bytes = pick(0, 9) == 0 ? 0 : 256 * pick(1, 8);
        const bool distinct = pick(0, 1) != 0;
        std::vector<const void *> in(N);
        std::vector<void *> out(N);
        const int layout = (int)pick(0, 5);
        const uintptr_t base = 0x100000, far = 0x40000000;
        for (uint32_t i = 0; i < N; ++i) {
            uintptr_t pi, po;
            switch (layout) {
            case 0:  // two runs handed out one after the other, ascending
                pi = base + i * (bytes + 256), po = far + i * (bytes + 256);
                break;
            case 1:  // descending, as allocators often do
                pi = far - i * (bytes + 512), po = base + (N - i) * (bytes + 512);
                break;
            case 2:  // in place
                pi = po = base + i * (bytes + 256);
                break;
            default:  // anything on a coarse grid: overlaps, repeats, cross-aliases
                pi = base + 256 * pick(0, 3 * N);
                po = pick(0, 2) == 0 ? pi : base + 256 * pick(0, 3 * N);
                break;
            }
            in[i] = reinterpret_cast<const void *>(pi);
            out[i] = reinterpret_cast<void *>(po);
        }
        if (layout == 5 && N > 1) out[pick(0, N - 1)] = out[pick(0, N - 1)];  // a repeated output
        bool bad = false;
        auto partly = [&](uintptr_t a, uintptr_t b) { return a != b && (a < b ? b - a : a - b) < bytes; };
        for (uint32_t i = 0; i < N && !bad; ++i)
            for (uint32_t j = 0; j < N && !bad; ++j) {
                const uintptr_t oi = (uintptr_t)out[i], oj = (uintptr_t)out[j], ij = (uintptr_t)in[j];
                if (partly(oi, oj) || partly(oi, ij)) bad = true;
                if (distinct && i != j && (oi == oj || oi == ij)) bad = true;
            }
        const nz_status got = nz::check_collective_buffers(in.data(), out.data(), N, bytes, distinct);
        REQUIRE(got == (bad ? NZ_ERR_UNSUPPORTED : NZ_OK));
        // pack / unpack: the written range of every buffer against every other range
        const uint64_t s_lo = 256 * pick(0, 2), s_hi = s_lo + 64 * pick(0, 8);
        const uint64_t d_lo = 256 * pick(0, 2), d_hi = d_lo + 64 * pick(0, 8);
        bool clash = false;
        auto meet = [](uintptr_t a0, uintptr_t a1, uintptr_t b0, uintptr_t b1) {
            return a0 < a1 && b0 < b1 && a0 < b1 && b0 < a1;
        };
        for (uint32_t i = 0; i < N && !clash; ++i)
            for (uint32_t j = 0; j < N && !clash; ++j) {
                const uintptr_t di = (uintptr_t)out[i], dj = (uintptr_t)out[j], sj = (uintptr_t)in[j];
                if (i != j && meet(di + d_lo, di + d_hi, dj + d_lo, dj + d_hi)) clash = true;
                if (meet(di + d_lo, di + d_hi, sj + s_lo, sj + s_hi)) clash = true;
            }
        REQUIRE(nz::check_copy_buffers(in.data(), out.data(), N, s_lo, s_hi, d_lo, d_hi) ==
                (clash ? NZ_ERR_UNSUPPORTED : NZ_OK));
    }

    // placement offsets: in range, aligned, disjoint, counters untouched on failure
    for (int it = 0; it < 2000; ++it) {
        const uint64_t arena = pick(0, 300) << 30;
        uint64_t used[NZ_HBM_REGIONS] = {0, 0, 0};
        std::vector<std::pair<uint64_t, uint64_t>> got;
        for (int call = 0; call < 6; ++call) {
            const uint32_t count = (uint32_t)pick(0, 40);
            const uint64_t each = pick(0, 3) == 0 ? pick(0, 100) : pick(1, (uint64_t)3 << 30);
            std::vector<uint64_t> off(count + 1, 12345);
            uint64_t before[NZ_HBM_REGIONS] = {used[0], used[1], used[2]};
            const nz_status s = nz_hbm_place(arena, used, count, each, (int)pick(0, 1), (uint32_t)pick(0, 2), off.data());
            REQUIRE(off[count] == 12345);
            if (s != NZ_OK) {
                REQUIRE(s == NZ_ERR_CAPACITY);
                REQUIRE(used[0] == before[0] && used[1] == before[1] && used[2] == before[2]);
                continue;
            }
            for (uint32_t i = 0; i < count; ++i) {
                REQUIRE(off[i] % (2u << 20) == 0 && off[i] + each <= arena);
                got.push_back({off[i], off[i] + (each ? each : 1)});
            }
        }
        std::sort(got.begin(), got.end());
        for (size_t i = 0; i + 1 < got.size(); ++i) REQUIRE(got[i].second <= got[i + 1].first);
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
