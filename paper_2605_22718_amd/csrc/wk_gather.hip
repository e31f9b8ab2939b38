// Window assembly (paper Sec. 1: stored caches are reused as they are, not re-encoded; Sec. 4.2): the retrieved chunks' stored
// K/V rows are placed behind the native sliding-window rows, byte for byte.
//
// In the head-major layout every (head, chunk) pair is one contiguous byte range, so the gather
// is a set of H x (1 + R) straight copies.  One launch covers K and V.  A work unit is 32 KB of
// one head's K or V window; a workgroup walks units blockIdx.x, blockIdx.x + gridDim.x, ...: with
// the default grid that is one unit each, with a capped grid (a prefetch that runs beside other
// kernels and is bound by the host link anyway) a few workgroups stream the whole window.  The
// source of each 16-byte vector is found by binary search over the retrieved chunks' prefix
// offsets, built per workgroup in LDS from the device-resident ids (the ids never visit the
// host); 8 vectors per lane in flight cover the latency of HBM and of reads from a pinned-host
// store over the host link.  Loads and stores are nontemporal (the data is touched once here), rows
// are 16 or 32 vectors so all index arithmetic is shifts on 32-bit values, and a unit that lies in
// one segment -- the usual case -- looks its segment up once: together these bring the kernel from
// 3.2 TB/s to the rate of a plain device copy (5.5 TB/s read + written at the LingBot shape).
#include "wk_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kVecPerThread = 8;
constexpr int kVecPerBlock = kThreads * kVecPerThread;  // 16-byte vectors per work unit
constexpr int kMaxR = 1024;

typedef unsigned int uvec4 __attribute__((ext_vector_type(4)));   // a 16-byte vector the nontemporal builtins accept

struct GatherArgs {
    const void *const *K_ptr;
    const void *const *V_ptr;
    const int32_t *n_tok;
    int M, max_tok, H;
    const int32_t *ids;
    const int32_t *n_ids;
    int R_max;
    const char *K_native;
    const char *V_native;
    int n_native;
    char *K_win;
    char *V_win;
    int win_capacity;
    int32_t *n_win;
    int vec_per_row;  // 16 (bf16) or 32 (fp32)
    int units_per_head;  // work units covering win_capacity-bounded rows of one head
};

// dynamic LDS: per segment s (0 = native rows, 1.. = retrieved chunks in the order of ids) the
// base address of its K block and V block, its length and the first window row after it
__global__ __launch_bounds__(kThreads) void k_gather(GatherArgs a) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int cap = a.R_max + 1;
    const char **seg_k = reinterpret_cast<const char **>(lds);
    const char **seg_v = seg_k + cap;
    int *seg_end = reinterpret_cast<int *>(seg_v + cap);
    int *seg_len = seg_end + cap;
    const int tid = threadIdx.x;
    const size_t row_bytes = (size_t)a.vec_per_row * 16;

    int n = a.n_ids ? *a.n_ids : a.R_max;
    n = n < 0 ? 0 : (n > a.R_max ? a.R_max : n);
    for (int t = tid; t < n; t += kThreads) {
        const int id = a.ids[t];
        int len = 0;
        const char *k = nullptr, *v = nullptr;
        if (id >= 0 && id < a.M) {
            len = a.n_tok[id];
            // a chunk that claims more rows than the descriptor's bound is skipped, like an id outside the
            // store: its length is the stride between its heads, so it cannot be cut short, and the window
            // was sized by the host for max_tok rows per chunk
            if (len < 0 || len > a.max_tok) len = 0;
            k = reinterpret_cast<const char *>(a.K_ptr[id]);
            v = reinterpret_cast<const char *>(a.V_ptr[id]);
        }
        seg_len[t + 1] = len;
        seg_k[t + 1] = k;
        seg_v[t + 1] = v;
    }
    if (tid == 0) {
        seg_k[0] = a.K_native;   // NULL: the native rows are already in place
        seg_v[0] = a.V_native;
        seg_len[0] = a.n_native;
    }
    __syncthreads();
    if (tid == 0) {
        int acc = 0;
        for (int t = 0; t <= n; ++t) {
            acc += seg_len[t];
            seg_end[t] = acc;
        }
        if (a.n_win && blockIdx.x == 0) *a.n_win = acc;
    }
    __syncthreads();
    const int nseg = n + 1;
    int total_rows = seg_end[nseg - 1];
    if (total_rows > a.win_capacity) total_rows = a.win_capacity;  // cannot happen after the host check
    // rows are 16 or 32 vectors: shifts, and 32-bit indices inside a head (capacity * 32 < 2^31 is
    // checked on the host)
    const int row_shift = a.vec_per_row == 16 ? 4 : 5;
    const unsigned total_vec = (unsigned)total_rows << row_shift;
    const long long units = (long long)a.units_per_head * a.H * 2;
    // smallest s in [lo, hi] with row < seg_end[s]
    auto segment_of = [&](int row, int lo, int hi) {
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (row < seg_end[mid]) hi = mid; else lo = mid + 1;
        }
        return lo;
    };

    for (long long u = blockIdx.x; u < units; u += gridDim.x) {
        const unsigned unit = (unsigned)(u % a.units_per_head);
        const unsigned hz = (unsigned)(u / a.units_per_head);
        const unsigned v0 = unit * kVecPerBlock;
        if (v0 >= total_vec) continue;
        const int h = (int)(hz % (unsigned)a.H);
        const bool is_v = hz >= (unsigned)a.H;
        const char *const *seg_src = is_v ? seg_v : seg_k;
        uvec4 *win = reinterpret_cast<uvec4 *>((is_v ? a.V_win : a.K_win) + (size_t)h * a.win_capacity * row_bytes);
        // the unit's rows usually lie in one segment: look that up once
        const unsigned v_last = min(v0 + kVecPerBlock, total_vec) - 1;
        const int s_first = segment_of((int)(v0 >> row_shift), 0, nseg - 1);
        const int s_last = segment_of((int)(v_last >> row_shift), s_first, nseg - 1);
        uvec4 buf[kVecPerThread];
        bool have[kVecPerThread];
#pragma unroll
        for (int i = 0; i < kVecPerThread; ++i) {
            const unsigned v = v0 + tid + i * kThreads;
            have[i] = false;
            if (v < total_vec) {
                const int row = (int)(v >> row_shift);
                const int sg = s_first == s_last ? s_first : segment_of(row, s_first, s_last);
                const char *src = seg_src[sg];
                if (src) {
                    const int seg_begin = sg == 0 ? 0 : seg_end[sg - 1];
                    const size_t src_row = (size_t)h * seg_len[sg] + (size_t)(row - seg_begin);
                    const uvec4 *sp = reinterpret_cast<const uvec4 *>(src + src_row * row_bytes) + (v & (a.vec_per_row - 1));
                    buf[i] = __builtin_nontemporal_load(sp);   // streamed once: keep it out of the caches' way
                    have[i] = true;
                }
            }
        }
#pragma unroll
        for (int i = 0; i < kVecPerThread; ++i) {
            const unsigned v = v0 + tid + i * kThreads;
            if (have[i]) __builtin_nontemporal_store(buf[i], win + v);
        }
    }
}

}  // namespace

wk_status wk::gather_launch(const wk_store_desc *store, const int32_t *ids, const int32_t *n_ids, int32_t R_max,
                            const void *K_native, const void *V_native, int32_t n_native, void *K_win,
                            void *V_win, int32_t win_capacity, int32_t *n_win, int32_t max_workgroups,
                            hipStream_t stream) {
    if (!store || !K_win || !V_win) return WK_ERR_INVALID_ARG;
    if (R_max < 0 || n_native < 0 || win_capacity < 0 || store->M < 0 || store->max_tok < 0 || store->H < 1)
        return WK_ERR_INVALID_ARG;
    if (max_workgroups < 0) return WK_ERR_INVALID_ARG;
    if (store->dtype != WK_F32 && store->dtype != WK_BF16) return WK_ERR_INVALID_ARG;
    if (R_max > 0 && (!ids || !store->K_ptr || !store->V_ptr || !store->n_tok)) return WK_ERR_INVALID_ARG;
    if ((K_native == nullptr) != (V_native == nullptr)) return WK_ERR_INVALID_ARG;
    if (store->d != WK_D || R_max > kMaxR) return WK_ERR_UNSUPPORTED;
    if ((int64_t)n_native + (int64_t)R_max * store->max_tok > (int64_t)win_capacity) return WK_ERR_SHAPE;
    if ((int64_t)win_capacity * 32 > 0x7fffffffLL) return WK_ERR_UNSUPPORTED;   // 32-bit vector indices inside a head
    GatherArgs a;
    a.K_ptr = store->K_ptr; a.V_ptr = store->V_ptr; a.n_tok = store->n_tok;
    a.M = store->M; a.max_tok = store->max_tok; a.H = store->H;
    a.ids = ids; a.n_ids = n_ids; a.R_max = R_max;
    a.K_native = reinterpret_cast<const char *>(K_native);
    a.V_native = reinterpret_cast<const char *>(V_native);
    a.n_native = n_native;
    a.K_win = reinterpret_cast<char *>(K_win);
    a.V_win = reinterpret_cast<char *>(V_win);
    a.win_capacity = win_capacity;
    a.n_win = n_win;
    a.vec_per_row = (int)(WK_D * wk::esize(store->dtype) / 16);
    const long long cap_vec = (long long)(n_native + (int64_t)R_max * store->max_tok) * a.vec_per_row;
    long long per_head = (cap_vec + kVecPerBlock - 1) / kVecPerBlock;
    if (per_head == 0) per_head = 1;  // nothing to copy: one workgroup still reports the (zero) length
    a.units_per_head = (int)per_head;
    long long grid = per_head * store->H * 2;
    if (max_workgroups > 0 && grid > max_workgroups) grid = max_workgroups;
    if (grid > 0x7fffffffLL) return WK_ERR_UNSUPPORTED;
    const size_t lds_bytes = (size_t)(R_max + 1) * (2 * sizeof(char *) + 2 * sizeof(int));
    hipLaunchKernelGGL(k_gather, dim3((unsigned)grid), dim3(kThreads), lds_bytes, stream, a);
    WK_LAUNCH_CHECK();
    return WK_OK;
}

extern "C" wk_status wk_gather_window(const wk_store_desc *store, const int32_t *ids, const int32_t *n_ids,
                                      int32_t R_max, const void *K_native, const void *V_native,
                                      int32_t n_native, void *K_win, void *V_win, int32_t win_capacity,
                                      int32_t *n_win, void *hip_stream) {
    return wk::gather_launch(store, ids, n_ids, R_max, K_native, V_native, n_native, K_win, V_win, win_capacity,
                             n_win, 0, reinterpret_cast<hipStream_t>(hip_stream));
}

namespace {

// Straight copy with ordinary (cached) 16-byte loads and stores, one vector per lane and pass: the
// access pattern of the tile loads in the attention kernels, with a byte count known exactly.
__global__ __launch_bounds__(kThreads) void k_copy_plain(const uint4 *__restrict__ src, uint4 *__restrict__ dst,
                                                         long long n_vec) {
    const long long per_block = (long long)kThreads * kVecPerThread;
    for (long long base = (long long)blockIdx.x * per_block; base < n_vec; base += (long long)gridDim.x * per_block) {
        uint4 buf[kVecPerThread];
#pragma unroll
        for (int i = 0; i < kVecPerThread; ++i) {
            const long long v = base + threadIdx.x + (long long)i * kThreads;
            if (v < n_vec) buf[i] = src[v];
        }
#pragma unroll
        for (int i = 0; i < kVecPerThread; ++i) {
            const long long v = base + threadIdx.x + (long long)i * kThreads;
            if (v < n_vec) dst[v] = buf[i];
        }
    }
}

}  // namespace

extern "C" wk_status wk_calibration_copy(void *dst, const void *src, size_t bytes, void *hip_stream) {
    if (!dst || !src || bytes % 16 != 0) return WK_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(dst) % 16 != 0 || reinterpret_cast<uintptr_t>(src) % 16 != 0)
        return WK_ERR_INVALID_ARG;
    if (bytes == 0) return WK_OK;
    const long long n_vec = (long long)(bytes / 16);
    long long grid = (n_vec + kVecPerBlock - 1) / kVecPerBlock;
    if (grid > 0x7fffffffLL) grid = 0x7fffffffLL;
    hipLaunchKernelGGL(k_copy_plain, dim3((unsigned)grid), dim3(kThreads), 0,
                       reinterpret_cast<hipStream_t>(hip_stream), reinterpret_cast<const uint4 *>(src),
                       reinterpret_cast<uint4 *>(dst), n_vec);
    WK_LAUNCH_CHECK();
    return WK_OK;
}

extern "C" wk_status wk_host_device_pointer(void *host_ptr, void **device_ptr) {
    if (!host_ptr || !device_ptr) return WK_ERR_INVALID_ARG;
    void *dp = nullptr;
    if (hipHostGetDevicePointer(&dp, host_ptr, 0) != hipSuccess) {
        (void)hipGetLastError();
        return WK_ERR_HIP;
    }
    *device_ptr = dp;
    return WK_OK;
}
