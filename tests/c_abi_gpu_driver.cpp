// The library used the way a C caller uses it: nezha_sim.h, hipMalloc'ed buffers, a stream of the
// caller's own, no Python and no torch.  Expected values are closed forms and plain host loops
// written here (they do not come from the oracle): index inputs whose sum is known per element,
// bit fingerprints, a two-node sum that is one IEEE add, and pack / unpack against memcpy.
// Built by paper_2405_17870_amd/build.py as a small shared object of its own; tests/test_gpu_c_abi.py
// loads it and calls nz_c_abi_checks() (in-process: a GPU test starts no other program).
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>

#include "nezha_sim.h"

#define REQUIRE(c)                                                          \
    do {                                                                    \
        if (!(c)) {                                                         \
            std::fprintf(stderr, "line %d: %s\n", __LINE__, #c);            \
            return 1;                                                       \
        }                                                                   \
    } while (0)
#define HIP_OK(x) REQUIRE((x) == hipSuccess)

namespace {

// N device buffers of `bytes` bytes each (256-byte aligned: hipMalloc gives more).
struct DeviceBuffers {
    std::vector<void *> p;
    ~DeviceBuffers()
    {
        for (void *q : p) (void)hipFree(q);
    }
    bool make(uint32_t n, size_t bytes)
    {
        for (uint32_t i = 0; i < n; ++i) {
            void *q = nullptr;
            if (hipMalloc(&q, bytes ? bytes : 1) != hipSuccess) return false;
            p.push_back(q);
        }
        return true;
    }
};

template <class T>
int allreduce_case(const char *what, hipStream_t st, uint32_t N, uint64_t n, const uint32_t *ratios,
                   uint32_t R, nz_dtype dtype, const std::vector<std::vector<T>> &in,
                   const std::vector<T> &expect)
{
    std::printf("%s: N=%u n=%llu\n", what, N, (unsigned long long)n);
    std::fflush(stdout);
    DeviceBuffers din, dout;
    REQUIRE(din.make(N, n * sizeof(T)) && dout.make(N, n * sizeof(T)));
    for (uint32_t i = 0; i < N; ++i)
        HIP_OK(hipMemcpy(din.p[i], in[i].data(), n * sizeof(T), hipMemcpyHostToDevice));
    std::vector<T> got(n);
    for (nz_mode mode : {NZ_FUSED, NZ_RING_STEPWISE}) {
        for (uint32_t i = 0; i < N; ++i) HIP_OK(hipMemsetAsync(dout.p[i], 0xCD, n * sizeof(T), st));
        const nz_status s = nz_allreduce_sim(din.p.data(), N, n, ratios, R, dtype, mode, dout.p.data(), st);
        if (s != NZ_OK) std::fprintf(stderr, "%s (%s)\n", nz_status_str(s), nz_last_hip_error());
        REQUIRE(s == NZ_OK);
        HIP_OK(hipStreamSynchronize(st));
        for (uint32_t i = 0; i < N; ++i) {
            HIP_OK(hipMemcpy(got.data(), dout.p[i], n * sizeof(T), hipMemcpyDeviceToHost));
            REQUIRE(std::memcmp(got.data(), expect.data(), n * sizeof(T)) == 0);
        }
    }
    return 0;
}

}  // namespace

extern "C" int nz_c_abi_checks(void)
{
    int n_dev = 0;
    HIP_OK(hipGetDeviceCount(&n_dev));
    REQUIRE(n_dev >= 1);
    HIP_OK(hipSetDevice(0));
    hipStream_t st;
    HIP_OK(hipStreamCreate(&st));

    // 1. index inputs: in[i][x] = (x mod 2^16) * (i + 1)  ->  (x mod 2^16) * N (N + 1) / 2
    {
        const uint32_t N = 8, ratios[2] = {100, 40};
        const uint64_t n = 1000003;
        std::vector<std::vector<int32_t>> in(N, std::vector<int32_t>(n));
        std::vector<int32_t> expect(n);
        for (uint64_t x = 0; x < n; ++x) {
            for (uint32_t i = 0; i < N; ++i) in[i][x] = (int32_t)((x & 0xffff) * (i + 1));
            expect[x] = (int32_t)((x & 0xffff) * (N * (N + 1) / 2));
        }
        if (allreduce_case("index inputs", st, N, n, ratios, 2, NZ_I32, in, expect)) return 1;
    }
    // 2. fingerprints: node i holds 2^i everywhere -> every element is 2^31 - 1
    {
        const uint32_t N = 31, ratios[3] = {100, 100, 40};
        const uint64_t n = 70001;
        std::vector<std::vector<int32_t>> in(N);
        for (uint32_t i = 0; i < N; ++i) in[i].assign(n, (int32_t)(1u << i));
        std::vector<int32_t> expect(n, 0x7fffffff);
        if (allreduce_case("fingerprints", st, N, n, ratios, 3, NZ_I32, in, expect)) return 1;
    }
    // 2b. the same fingerprints at a size whose fused form is the pipeline of launches
    //     (31 outputs x 4.5 MB > 128 MiB), checked through the launch count and bit by bit
    {
        const uint32_t N = 31, ratios[2] = {100, 25};
        const uint64_t n = 1123457;
        uint64_t launches = 0;
        REQUIRE(nz_allreduce_launches(N, n, ratios, 2, NZ_I32, NZ_FUSED, N, 0, &launches) == NZ_OK && launches > 1);
        REQUIRE(nz_allreduce_launches(N, n, ratios, 2, NZ_I32, NZ_FUSED, 1, 0, &launches) == NZ_OK && launches == 1);
        std::vector<std::vector<int32_t>> in(N);
        for (uint32_t i = 0; i < N; ++i) in[i].assign(n, (int32_t)(1u << i));
        std::vector<int32_t> expect(n, 0x7fffffff);
        if (allreduce_case("fingerprints, staged", st, N, n, ratios, 2, NZ_I32, in, expect)) return 1;
    }
    // 3. two nodes, fp32: the result is one IEEE addition, whatever the mode
    {
        const uint32_t N = 2, ratios[2] = {3, 1};
        const uint64_t n = 333337;
        std::mt19937 rng(99);
        std::normal_distribution<float> g(0.0f, 1.0f);
        std::vector<std::vector<float>> in(N, std::vector<float>(n));
        std::vector<float> expect(n);
        for (uint64_t x = 0; x < n; ++x) {
            in[0][x] = g(rng);
            in[1][x] = g(rng) * 1e-3f;
            volatile float s = in[0][x] + in[1][x];
            expect[x] = s;
        }
        if (allreduce_case("two-node fp32", st, N, n, ratios, 2, NZ_F32, in, expect)) return 1;
    }
    // 4. pack / unpack of rail 1 in the order node 2 sends its segments, against memcpy
    {
        const uint32_t N = 5, R = 2, ratios[2] = {100, 40}, e = 2, rail = 1;
        const uint64_t n = 200001;
        std::printf("pack / unpack: N=%u n=%llu\n", N, (unsigned long long)n);
        std::fflush(stdout);
        uint64_t rail_off[R + 1], seg[R * (N + 1)];
        REQUIRE(nz_rail_partition(n, e, ratios, R, rail_off) == NZ_OK);
        REQUIRE(nz_segment_map(rail_off, R, N, seg) == NZ_OK);
        REQUIRE(rail_off[0] == 0 && rail_off[R] == n && rail_off[1] % (NZ_RAIL_ALIGN_BYTES / e) == 0);
        uint32_t ids[N];
        for (uint32_t s = 0; s < N; ++s) ids[s] = (2 + N - s) % N;
        const uint64_t *row = seg + rail * (N + 1);
        const uint64_t total = (row[N] - row[0]) * e;
        std::mt19937 rng(5);
        std::vector<std::vector<uint16_t>> host(N, std::vector<uint16_t>(n));
        for (auto &h : host)
            for (auto &v : h) v = (uint16_t)rng();
        DeviceBuffers node, send, back;
        REQUIRE(node.make(N, n * e) && send.make(N, total) && back.make(N, n * e));
        for (uint32_t m = 0; m < N; ++m) {
            HIP_OK(hipMemcpy(node.p[m], host[m].data(), n * e, hipMemcpyHostToDevice));
            HIP_OK(hipMemset(back.p[m], 0xA5, n * e));
        }
        uint64_t packed = 0;
        REQUIRE(nz_pack(node.p.data(), N, seg, R, rail, ids, N, e, send.p.data(), total - e, &packed, st) ==
                NZ_ERR_CAPACITY);
        REQUIRE(nz_pack(node.p.data(), N, seg, R, rail, ids, N, e, send.p.data(), total, &packed, st) == NZ_OK);
        REQUIRE(packed == total);
        REQUIRE(nz_unpack(send.p.data(), N, seg, R, rail, ids, N, e, back.p.data(), st) == NZ_OK);
        HIP_OK(hipStreamSynchronize(st));
        std::vector<uint8_t> got(total), want(total);
        std::vector<uint16_t> got_back(n), want_back(n);
        for (uint32_t m = 0; m < N; ++m) {
            uint64_t pos = 0;
            want_back.assign(n, 0xA5A5);
            for (uint32_t s = 0; s < N; ++s) {
                const uint64_t off = row[ids[s]], len = row[ids[s] + 1] - row[ids[s]];
                std::memcpy(want.data() + pos, host[m].data() + off, len * e);
                std::memcpy(want_back.data() + off, host[m].data() + off, len * e);
                pos += len * e;
            }
            REQUIRE(pos == total);
            HIP_OK(hipMemcpy(got.data(), send.p[m], total, hipMemcpyDeviceToHost));
            REQUIRE(got == want);
            HIP_OK(hipMemcpy(got_back.data(), back.p[m], n * e, hipMemcpyDeviceToHost));
            REQUIRE(got_back == want_back);
        }
    }
    // 5. a base that is not 256-byte aligned is refused and nothing runs
    {
        const uint32_t N = 2, ratios[1] = {1};
        const uint64_t n = 1000;
        DeviceBuffers din, dout;
        REQUIRE(din.make(N, n * 4 + 64) && dout.make(N, n * 4));
        for (uint32_t i = 0; i < N; ++i) HIP_OK(hipMemset(dout.p[i], 0x11, n * 4));
        const void *bad[2] = {static_cast<char *>(din.p[0]) + 16, din.p[1]};
        REQUIRE(nz_allreduce_sim(bad, N, n, ratios, 1, NZ_F32, NZ_FUSED, dout.p.data(), st) == NZ_ERR_ALIGNMENT);
        HIP_OK(hipStreamSynchronize(st));
        std::vector<uint8_t> got(n * 4);
        HIP_OK(hipMemcpy(got.data(), dout.p[0], n * 4, hipMemcpyDeviceToHost));
        for (uint8_t b : got) REQUIRE(b == 0x11);
    }
    HIP_OK(hipStreamDestroy(st));
    std::printf("c abi gpu run ok\n");
    return 0;
}
