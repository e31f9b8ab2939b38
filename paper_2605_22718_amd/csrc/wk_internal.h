// Internal helpers shared by the HIP translation units of libwk (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "wk.h"

#define WK_D 128  // head dimension every kernel is written for

#define WK_LAUNCH_CHECK()                                   \
    do {                                                    \
        if (hipGetLastError() != hipSuccess) return WK_ERR_HIP; \
    } while (0)

namespace wk {

__host__ __device__ inline size_t esize(int dtype) { return dtype == WK_BF16 ? 2 : 4; }

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Once per device and process: true if `flags` did not yet have the current device's bit (the caller then
// does its per-device set-up, e.g. raising a kernel's dynamic-LDS limit, and calls it done with mark_device).
// A lost race only repeats an idempotent set-up.  Devices beyond 63 always report "not yet".
inline bool device_needs_setup(const std::atomic<uint64_t> &flags, int &dev) {
    if (hipGetDevice(&dev) != hipSuccess) dev = -1;
    return dev < 0 || dev > 63 || !((flags.load(std::memory_order_acquire) >> dev) & 1u);
}
inline void mark_device(std::atomic<uint64_t> &flags, int dev) {
    if (dev >= 0 && dev <= 63) flags.fetch_or(uint64_t(1) << dev, std::memory_order_release);
}

// wk_gather_window with a cap on the number of workgroups (0 = one per 32 KB work unit)
wk_status gather_launch(const wk_store_desc *store, const int32_t *ids, const int32_t *n_ids, int32_t R_max,
                        const void *K_native, const void *V_native, int32_t n_native, void *K_win, void *V_win,
                        int32_t win_capacity, int32_t *n_win, int32_t max_workgroups, hipStream_t stream);

// 16 lanes share one 128-element row; each lane owns elements 8*sub .. 8*sub+7.
constexpr int kRowLanes = 16;

template <int DT>
__device__ inline void load_row8(const void *row_base, int sub, float (&v)[8]) {
    if constexpr (DT == WK_BF16) {
        const uint4 u = reinterpret_cast<const uint4 *>(row_base)[sub];
        const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(w[i] << 16);
            v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    } else {
        const float4 a = reinterpret_cast<const float4 *>(row_base)[2 * sub];
        const float4 b = reinterpret_cast<const float4 *>(row_base)[2 * sub + 1];
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
        v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    }
}

// sum over the 16 lanes of a row group (groups are aligned to 16 lanes)
__device__ inline double row_group_sum(double x) {
#pragma unroll
    for (int o = 8; o >= 1; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

}  // namespace wk
