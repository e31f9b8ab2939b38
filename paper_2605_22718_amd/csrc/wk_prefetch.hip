// Overlap of the CPU-offloaded store's traffic with attention (paper Sec. 7: with every KV chunk
// in CPU memory the host-to-device transfer at retrieval time is what stands in the way of real
// time).  Retrieval by camera/action distance gives the same chunk ids to every layer of a
// denoising step, so the window of layer l+1 can be assembled while layer l attends: a second
// HIP stream (default priority) runs wk_gather_window for the next layer into the other of two
// window buffers, and events order the two streams per buffer ("slot"):
//
//     copy stream:     wait released[s] -> gather into slot s -> record ready[s]
//     compute stream:  wait ready[s]    -> attention on slot s -> record released[s]
//
// A gather that reads pinned host memory is bound by the host link, not by the CUs, so it is
// launched with a small, capped grid: the few workgroups it keeps resident leave the rest of the
// chip to the attention kernel, whose workgroups need whole CUs (all VGPRs of their SIMDs).
// Host code only; the kernels are those of wk_gather.hip.
#include "wk_internal.h"

namespace {
constexpr int kMaxSlots = 8;
}

struct wk_prefetch {
    int device;
    int n_slots;
    hipStream_t copy;
    hipEvent_t fence;
    hipEvent_t ready[kMaxSlots];
    hipEvent_t released[kMaxSlots];
    bool has_ready[kMaxSlots];
    bool has_released[kMaxSlots];
};

extern "C" wk_status wk_prefetch_create(wk_prefetch **out, int32_t n_slots) {
    if (!out || n_slots < 1 || n_slots > kMaxSlots) return WK_ERR_INVALID_ARG;
    *out = nullptr;
    wk_prefetch *p = new (std::nothrow) wk_prefetch();
    if (!p) return WK_ERR_HIP;
    p->n_slots = 0;
    p->copy = nullptr;
    p->fence = nullptr;
    bool ok = hipGetDevice(&p->device) == hipSuccess &&
              hipStreamCreateWithFlags(&p->copy, hipStreamNonBlocking) == hipSuccess &&
              hipEventCreateWithFlags(&p->fence, hipEventDisableTiming) == hipSuccess;
    for (int s = 0; ok && s < n_slots; ++s) {
        p->ready[s] = p->released[s] = nullptr;
        p->has_ready[s] = p->has_released[s] = false;
        ok = hipEventCreateWithFlags(&p->ready[s], hipEventDisableTiming) == hipSuccess;
        if (ok) {
            ok = hipEventCreateWithFlags(&p->released[s], hipEventDisableTiming) == hipSuccess;
            if (!ok) (void)hipEventDestroy(p->ready[s]);
        }
        if (ok) p->n_slots = s + 1;
    }
    if (!ok) {
        (void)hipGetLastError();
        for (int s = 0; s < p->n_slots; ++s) {
            (void)hipEventDestroy(p->ready[s]);
            (void)hipEventDestroy(p->released[s]);
        }
        if (p->fence) (void)hipEventDestroy(p->fence);
        if (p->copy) (void)hipStreamDestroy(p->copy);
        delete p;
        return WK_ERR_HIP;
    }
    *out = p;
    return WK_OK;
}

extern "C" wk_status wk_prefetch_destroy(wk_prefetch *p) {
    if (!p) return WK_OK;
    bool ok = hipStreamSynchronize(p->copy) == hipSuccess;
    for (int s = 0; s < p->n_slots; ++s) {
        ok = (hipEventDestroy(p->ready[s]) == hipSuccess) && ok;
        ok = (hipEventDestroy(p->released[s]) == hipSuccess) && ok;
    }
    ok = (hipEventDestroy(p->fence) == hipSuccess) && ok;
    ok = (hipStreamDestroy(p->copy) == hipSuccess) && ok;
    delete p;
    if (!ok) (void)hipGetLastError();
    return ok ? WK_OK : WK_ERR_HIP;
}

extern "C" void *wk_prefetch_stream(wk_prefetch *p) { return p ? reinterpret_cast<void *>(p->copy) : nullptr; }

extern "C" wk_status wk_prefetch_after(wk_prefetch *p, void *hip_stream) {
    if (!p) return WK_ERR_INVALID_ARG;
    if (hipEventRecord(p->fence, reinterpret_cast<hipStream_t>(hip_stream)) != hipSuccess ||
        hipStreamWaitEvent(p->copy, p->fence, 0) != hipSuccess) {
        (void)hipGetLastError();
        return WK_ERR_HIP;
    }
    return WK_OK;
}

extern "C" wk_status wk_prefetch_gather(wk_prefetch *p, int32_t slot, const wk_store_desc *store,
                                        const int32_t *ids, const int32_t *n_ids, int32_t R_max,
                                        const void *K_native, const void *V_native, int32_t n_native,
                                        void *K_win, void *V_win, int32_t win_capacity, int32_t *n_win,
                                        int32_t max_workgroups) {
    if (!p || slot < 0 || slot >= p->n_slots) return WK_ERR_INVALID_ARG;
    if (p->has_released[slot] && hipStreamWaitEvent(p->copy, p->released[slot], 0) != hipSuccess) {
        (void)hipGetLastError();
        return WK_ERR_HIP;
    }
    const wk_status st = wk::gather_launch(store, ids, n_ids, R_max, K_native, V_native, n_native, K_win, V_win,
                                           win_capacity, n_win, max_workgroups, p->copy);
    if (st != WK_OK) return st;
    if (hipEventRecord(p->ready[slot], p->copy) != hipSuccess) {
        (void)hipGetLastError();
        return WK_ERR_HIP;
    }
    p->has_ready[slot] = true;
    return WK_OK;
}

extern "C" wk_status wk_prefetch_acquire(wk_prefetch *p, int32_t slot, void *hip_stream) {
    if (!p || slot < 0 || slot >= p->n_slots || !p->has_ready[slot]) return WK_ERR_INVALID_ARG;
    if (hipStreamWaitEvent(reinterpret_cast<hipStream_t>(hip_stream), p->ready[slot], 0) != hipSuccess) {
        (void)hipGetLastError();
        return WK_ERR_HIP;
    }
    return WK_OK;
}

extern "C" wk_status wk_prefetch_release(wk_prefetch *p, int32_t slot, void *hip_stream) {
    if (!p || slot < 0 || slot >= p->n_slots) return WK_ERR_INVALID_ARG;
    if (hipEventRecord(p->released[slot], reinterpret_cast<hipStream_t>(hip_stream)) != hipSuccess) {
        (void)hipGetLastError();
        return WK_ERR_HIP;
    }
    p->has_released[slot] = true;
    return WK_OK;
}
