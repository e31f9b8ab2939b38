// Torch-free driver for hardware-counter runs of the library's kernels (rocprofv3 --pmc ... -- wk_profile_driver).
// It allocates the LingBot-shaped window (40 heads, 4,680 queries, 28,080 keys, d = 128, bf16) with the HIP
// runtime, fills Q/K/V with seeded N(0,1) values generated on the host, pushes the source of the calibration copy
// out of the caches, and then calls, through the C ABI only:
//     wk_calibration_copy   one plain copy of the K window (575 MB read, 575 MB written): the known quantity
//                           the FETCH_SIZE / WRITE_SIZE readings are scaled by
//     the call named by `mode`, one warm-up launch and then `reps` timed ones (HIP events):
//       attention   wk_attention over the assembled window
//       in_place    wk_attention_in_place over the same keys: 9,360 native rows + 8 stored chunks of 2,340 rows
//       chunk_lse   wk_chunk_lse of the queries against the anchor keys (1,560 per chunk) of a 120-chunk store
// Usage: wk_profile_driver [reps = 3] [mode = attention]
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
    const char *mode = argc > 2 ? argv[2] : "attention";
    const int H = 40, N_q = 4680, N_kv = 28080, n_native = 9360, R = 8, chunk_rows = 2340, M = 120, T = 1560;
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
    // A chunk store for the two store-reading modes: every chunk an array of its own, [H][rows][128], filled
    // from the window's rows (the values only have to look like keys and values).
    wk_store_desc store;
    std::memset(&store, 0, sizeof store);
    int32_t *ids = nullptr;
    float *lse = nullptr;
    double flop = 4.0 * N_q * (double)N_kv * 128 * H;
    const bool in_place = std::strcmp(mode, "in_place") == 0, chunk_lse = std::strcmp(mode, "chunk_lse") == 0;
    if (!in_place && !chunk_lse && std::strcmp(mode, "attention") != 0) {
        std::fprintf(stderr, "unknown mode %s (attention, in_place, chunk_lse)\n", mode);
        return 1;
    }
    if (in_place || chunk_lse) {
        const int n_chunks = in_place ? R : M, rows = in_place ? chunk_rows : T;
        std::vector<void *> kp(n_chunks), vp(n_chunks);
        std::vector<int32_t> nt(n_chunks, rows), id(n_chunks);
        const size_t chunk_bytes = (size_t)H * rows * 256;
        for (int c = 0; c < n_chunks; ++c) {
            CHECK(hipMalloc(&kp[c], chunk_bytes));
            CHECK(hipMalloc(&vp[c], chunk_bytes));
            const size_t src = ((size_t)c * chunk_bytes) % (kv_elems * 2 - chunk_bytes) / 256 * 256;
            CHECK(hipMemcpy(kp[c], (const char *)K + src, chunk_bytes, hipMemcpyDeviceToDevice));
            CHECK(hipMemcpy(vp[c], (const char *)V + src, chunk_bytes, hipMemcpyDeviceToDevice));
            id[c] = c;
        }
        void *d_kp, *d_vp, *d_nt;
        CHECK(hipMalloc(&d_kp, n_chunks * sizeof(void *)));
        CHECK(hipMalloc(&d_vp, n_chunks * sizeof(void *)));
        CHECK(hipMalloc(&d_nt, n_chunks * 4));
        CHECK(hipMalloc((void **)&ids, n_chunks * 4));
        CHECK(hipMemcpy(d_kp, kp.data(), n_chunks * sizeof(void *), hipMemcpyHostToDevice));
        CHECK(hipMemcpy(d_vp, vp.data(), n_chunks * sizeof(void *), hipMemcpyHostToDevice));
        CHECK(hipMemcpy(d_nt, nt.data(), n_chunks * 4, hipMemcpyHostToDevice));
        CHECK(hipMemcpy(ids, id.data(), n_chunks * 4, hipMemcpyHostToDevice));
        store.K_ptr = (const void *const *)d_kp;
        store.V_ptr = (const void *const *)d_vp;
        store.n_tok = (const int32_t *)d_nt;
        store.M = n_chunks;
        store.max_tok = rows;
        store.H = H;
        store.d = 128;
        store.dtype = WK_BF16;
        if (chunk_lse) {
            CHECK(hipMalloc((void **)&lse, (size_t)M * H * N_q * 4));
            flop = 2.0 * N_q * (double)M * T * 128 * H;   // the S^T products only
        }
    }
    CHECK(hipMemset(flush, 0, kv_elems * 2));   // written after K: pushes K out of the Infinity Cache
    CHECK(hipDeviceSynchronize());
    if (wk_calibration_copy(copy_dst, K, kv_elems * 2, nullptr) != WK_OK) return 3;
    CHECK(hipDeviceSynchronize());
    auto launch = [&]() -> wk_status {
        if (in_place)
            return wk_attention_in_place(Q, K, V, n_native, N_kv, &store, ids, nullptr, R, O, nullptr, N_q, 0.f, nullptr);
        if (chunk_lse) return wk_chunk_lse(&store, Q, N_q, 0.f, lse, nullptr);
        return wk_attention(Q, K, V, O, nullptr, H, N_q, N_kv, 128, N_kv, WK_BF16, 0.f, nullptr, nullptr, 0, nullptr);
    };
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    if (launch() != WK_OK) return 4;
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(e0, nullptr));
    for (int r = 0; r < reps; ++r)
        if (launch() != WK_OK) return 4;
    CHECK(hipEventRecord(e1, nullptr));
    CHECK(hipDeviceSynchronize());
    float ms = 0.f;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    std::printf("%s H=%d N_q=%d %s: %.3f ms per launch, %.1f TFLOP/s (%d launches)\n", mode, H, N_q,
                chunk_lse ? "120 x 1560 anchor keys" : "N_kv=28080", ms / reps, flop / (ms / reps * 1e-3) / 1e12, reps);
    return 0;
}
