// Torch-free driver for hardware-counter runs of the library's kernels (rocprofv3 --pmc ... -- wk_profile_driver).
// It allocates the LingBot-shaped window (40 heads, 4,680 queries, 28,080 keys, d = 128, bf16) with the HIP
// runtime, fills Q/K/V with seeded N(0,1) values generated on the host, pushes the source of the calibration copy
// out of the caches, and then calls, through the C ABI only:
//     wk_calibration_copy   one plain copy of the K window (575 MB read, 575 MB written): the known quantity
//                           the FETCH_SIZE / WRITE_SIZE readings are scaled by
//     wk_attention          `reps` launches over the window (default 3)
// and prints the mean launch time from HIP events.  Usage: wk_profile_driver [reps] [H N_q N_kv]
#include <hip/hip_runtime_api.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "wk.h"

#define CHECK(x)                                                                    \
    do {                                                                            \
        hipError_t e_ = (x);                                                        \
        if (e_ != hipSuccess) {                                                     \
            std::fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));           \
            return 2;                                                               \
        }                                                                           \
    } while (0)

static uint16_t to_bf16(float f) {   // round to nearest even
    uint32_t u;
    std::memcpy(&u, &f, 4);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

static void fill_normal(std::vector<uint16_t> &dst, uint64_t seed) {
    uint64_t s = seed * 0x9E3779B97F4A7C15ull + 1;
    auto next = [&]() {   // xorshift64*
        s ^= s >> 12; s ^= s << 25; s ^= s >> 27;
        return (uint32_t)((s * 0x2545F4914F6CDD1Dull) >> 32);
    };
    for (size_t i = 0; i + 1 < dst.size(); i += 2) {   // Box-Muller, two values per pair of uniforms
        const float u1 = ((float)next() + 1.0f) * (1.0f / 4294967296.0f), u2 = (float)next() * (1.0f / 4294967296.0f);
        const float r = std::sqrt(-2.0f * std::log(u1)), a = 6.2831853f * u2;
        dst[i] = to_bf16(r * std::cos(a));
        dst[i + 1] = to_bf16(r * std::sin(a));
    }
}

int main(int argc, char **argv) {
    const int reps = argc > 1 ? std::atoi(argv[1]) : 3;
    const int H = argc > 4 ? std::atoi(argv[2]) : 40, N_q = argc > 4 ? std::atoi(argv[3]) : 4680,
              N_kv = argc > 4 ? std::atoi(argv[4]) : 28080;
    const size_t q_elems = (size_t)H * N_q * 128, kv_elems = (size_t)H * N_kv * 128;
    void *Q, *K, *V, *O, *copy_dst, *flush;
    CHECK(hipMalloc(&Q, q_elems * 2));
    CHECK(hipMalloc(&O, q_elems * 2));
    CHECK(hipMalloc(&K, kv_elems * 2));
    CHECK(hipMalloc(&V, kv_elems * 2));
    CHECK(hipMalloc(&copy_dst, kv_elems * 2));
    CHECK(hipMalloc(&flush, kv_elems * 2));
    {
        std::vector<uint16_t> h(kv_elems);
        fill_normal(h, 1);
        CHECK(hipMemcpy(K, h.data(), kv_elems * 2, hipMemcpyHostToDevice));
        fill_normal(h, 2);
        CHECK(hipMemcpy(V, h.data(), kv_elems * 2, hipMemcpyHostToDevice));
        h.resize(q_elems);
        fill_normal(h, 3);
        CHECK(hipMemcpy(Q, h.data(), q_elems * 2, hipMemcpyHostToDevice));
    }
    CHECK(hipMemset(flush, 0, kv_elems * 2));   // written after K: pushes K out of the Infinity Cache
    CHECK(hipDeviceSynchronize());
    if (wk_calibration_copy(copy_dst, K, kv_elems * 2, nullptr) != WK_OK) return 3;
    CHECK(hipDeviceSynchronize());
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    if (wk_attention(Q, K, V, O, nullptr, H, N_q, N_kv, 128, N_kv, WK_BF16, 0.f, nullptr, nullptr, 0, nullptr) != WK_OK) return 4;
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(e0, nullptr));
    for (int r = 0; r < reps; ++r)
        if (wk_attention(Q, K, V, O, nullptr, H, N_q, N_kv, 128, N_kv, WK_BF16, 0.f, nullptr, nullptr, 0, nullptr) != WK_OK) return 4;
    CHECK(hipEventRecord(e1, nullptr));
    CHECK(hipDeviceSynchronize());
    float ms = 0.f;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    const double flop = 4.0 * N_q * (double)N_kv * 128 * H;
    std::printf("wk_attention H=%d N_q=%d N_kv=%d: %.3f ms per launch, %.1f TFLOP/s (%d launches)\n", H, N_q, N_kv, ms / reps,
                flop / (ms / reps * 1e-3) / 1e12, reps);
    return 0;
}
