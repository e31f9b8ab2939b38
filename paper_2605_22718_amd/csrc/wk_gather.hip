// Window assembly (paper Sec. 1 "without re-encoding", Sec. 4.2): the retrieved chunks' stored
// K/V rows are placed behind the native sliding-window rows, byte for byte.
//
// In the head-major layout every (head, chunk) pair is one contiguous byte range, so the gather
// is a set of H x (1 + R) straight copies.  One launch covers K and V; a workgroup owns 32 KB of
// one head's window, finds the source of each 16-byte vector by binary search over the retrieved
// chunks' prefix offsets (built per workgroup in LDS from the device-resident ids, so the ids
// never visit the host) and keeps 8 vectors per lane in flight, which is enough to cover the
// latency of HBM and of reads from a pinned-host store over the host link.
#include "wk_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kVecPerThread = 8;
constexpr int kVecPerBlock = kThreads * kVecPerThread;  // 16-byte vectors per workgroup
constexpr int kMaxR = 1024;

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
};

__global__ __launch_bounds__(kThreads) void k_gather(GatherArgs a) {
    __shared__ int seg_end[kMaxR + 1];          // seg_end[s] = first window row after segment s
    __shared__ const char *seg_src[kMaxR + 1];  // source of segment s for this head and tensor
    __shared__ int s_nseg;
    const int h = blockIdx.y;
    const bool is_v = blockIdx.z == 1;
    const int tid = threadIdx.x;
    const size_t row_bytes = (size_t)a.vec_per_row * 16;

    int n = a.n_ids ? *a.n_ids : a.R_max;
    n = n < 0 ? 0 : (n > a.R_max ? a.R_max : n);
    for (int t = tid; t < n; t += kThreads) {
        const int id = a.ids[t];
        int len = 0;
        const char *src = nullptr;
        if (id >= 0 && id < a.M) {
            len = a.n_tok[id];
            len = len < 0 ? 0 : (len > a.max_tok ? a.max_tok : len);
            const char *base = reinterpret_cast<const char *>(is_v ? a.V_ptr[id] : a.K_ptr[id]);
            src = base + (size_t)h * len * row_bytes;
        }
        seg_end[t + 1] = len;  // lengths first, prefix sum below
        seg_src[t + 1] = src;
    }
    if (tid == 0) {
        const char *nat = is_v ? a.V_native : a.K_native;
        seg_src[0] = nat ? nat + (size_t)h * a.n_native * row_bytes : nullptr;
        s_nseg = n + 1;
    }
    __syncthreads();
    if (tid == 0) {
        int acc = a.n_native;
        seg_end[0] = acc;
        for (int t = 1; t <= n; ++t) {
            acc += seg_end[t];
            seg_end[t] = acc;
        }
        if (a.n_win && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0) *a.n_win = acc;
    }
    __syncthreads();
    const int nseg = s_nseg;
    int total_rows = seg_end[nseg - 1];
    if (total_rows > a.win_capacity) total_rows = a.win_capacity;  // cannot happen after the host check
    const long long total_vec = (long long)total_rows * a.vec_per_row;
    const long long v0 = (long long)blockIdx.x * kVecPerBlock;
    if (v0 >= total_vec) return;

    char *win = (is_v ? a.V_win : a.K_win) + (size_t)h * a.win_capacity * row_bytes;
    uint4 buf[kVecPerThread];
    bool have[kVecPerThread];
#pragma unroll
    for (int i = 0; i < kVecPerThread; ++i) {
        const long long v = v0 + tid + (long long)i * kThreads;
        have[i] = false;
        if (v < total_vec) {
            const int row = (int)(v / a.vec_per_row);
            int lo = 0, hi = nseg - 1;  // smallest s with row < seg_end[s]
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (row < seg_end[mid]) hi = mid; else lo = mid + 1;
            }
            const char *src = seg_src[lo];
            if (src) {
                const int seg_begin = lo == 0 ? 0 : seg_end[lo - 1];
                const size_t off = (size_t)(row - seg_begin) * row_bytes + (size_t)(v % a.vec_per_row) * 16;
                buf[i] = *reinterpret_cast<const uint4 *>(src + off);
                have[i] = true;
            }
        }
    }
#pragma unroll
    for (int i = 0; i < kVecPerThread; ++i) {
        const long long v = v0 + tid + (long long)i * kThreads;
        if (have[i]) *reinterpret_cast<uint4 *>(win + (size_t)v * 16) = buf[i];
    }
}

}  // namespace

extern "C" wk_status wk_gather_window(const wk_store_desc *store, const int32_t *ids, const int32_t *n_ids,
                                      int32_t R_max, const void *K_native, const void *V_native,
                                      int32_t n_native, void *K_win, void *V_win, int32_t win_capacity,
                                      int32_t *n_win, void *hip_stream) {
    if (!store || !K_win || !V_win) return WK_ERR_INVALID_ARG;
    if (R_max < 0 || n_native < 0 || win_capacity < 0 || store->M < 0 || store->max_tok < 0 || store->H < 1)
        return WK_ERR_INVALID_ARG;
    if (store->dtype != WK_F32 && store->dtype != WK_BF16) return WK_ERR_INVALID_ARG;
    if (R_max > 0 && (!ids || !store->K_ptr || !store->V_ptr || !store->n_tok)) return WK_ERR_INVALID_ARG;
    if ((K_native == nullptr) != (V_native == nullptr)) return WK_ERR_INVALID_ARG;
    if (store->d != WK_D || R_max > kMaxR) return WK_ERR_UNSUPPORTED;
    if ((int64_t)n_native + (int64_t)R_max * store->max_tok > (int64_t)win_capacity) return WK_ERR_SHAPE;
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
    unsigned nbx = (unsigned)((cap_vec + kVecPerBlock - 1) / kVecPerBlock);
    if (nbx == 0) nbx = 1;  // nothing to copy: one workgroup still reports the (zero) length
    hipLaunchKernelGGL(k_gather, dim3(nbx, store->H, 2), dim3(kThreads), 0,
                       reinterpret_cast<hipStream_t>(hip_stream), a);
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
