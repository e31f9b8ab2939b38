// Window bookkeeping (paper Sec. 4.2: the sliding window has a sink, a retrieved, a recent and a
// denoising region; Sec. 5.1: 3 + 9 + 3 + 3 latent frames).
//
// Two parts.  wk_window_plan is host arithmetic: where the chunk being generated lives, which
// chunk leaves the ring and must go to the store first.  Physical layout per head, in rows:
//
//     [ sink chunks | ring of (recent_chunks + 1) chunk slots | R retrieved slots ]
//
// Attention is a sum over keys, so the order of regions inside the window is free; this order
// makes every valid prefix contiguous (ring slots fill in ascending order, and nothing is
// retrieved before the ring is full) and needs no copy when a denoised chunk becomes "recent":
// the roles rotate over the ring slots instead.
//
// wk_window_update refreshes the retrieved region in place on the device.  Consecutive steps of
// a smooth camera path want mostly the same chunks; only chunks that are not already resident
// are copied from the store (HBM or pinned host), into the slots of the chunks that left.  One
// small kernel turns (old slot table, wanted ids) into (new slot table, fetch list); a second
// copies the fetch list with the same 32 KB work units as the window gather.
#include "wk_internal.h"

namespace {

constexpr int kPlanThreads = 1024;
constexpr int kMaxSlots = 1024;
constexpr int kThreads = 256;
constexpr int kVecPerThread = 8;
constexpr int kVecPerBlock = kThreads * kVecPerThread;

typedef unsigned int uvec4 __attribute__((ext_vector_type(4)));   // a 16-byte vector the nontemporal builtins accept

struct PlanOut {   // head of the workspace
    int32_t n_fetch;
    int32_t n_used;
};

__global__ __launch_bounds__(kPlanThreads) void k_slot_plan(const int32_t *__restrict__ ids,
                                                            const int32_t *__restrict__ n_ids, int R, int M,
                                                            const int32_t *__restrict__ n_tok, int slot_tokens,
                                                            int32_t *__restrict__ slot_ids, int n_native,
                                                            int32_t *__restrict__ n_win, int32_t *__restrict__ n_fetched,
                                                            PlanOut *__restrict__ head, int32_t *__restrict__ fetch_slot,
                                                            int32_t *__restrict__ fetch_id) {
    __shared__ int raw[kMaxSlots], want[kMaxSlots], old[kMaxSlots], inc[kMaxSlots];
    __shared__ unsigned char ok[kMaxSlots], keep[kMaxSlots], res[kMaxSlots], fetch[kMaxSlots];
    __shared__ int s_n;
    const int s = threadIdx.x;   // one thread per slot / per wanted rank
    int n_in = n_ids ? *n_ids : R;
    n_in = n_in < 0 ? 0 : (n_in > R ? R : n_in);
    if (s < R) {
        old[s] = slot_ids[s];
        int id = s < n_in ? ids[s] : -1;
        if (id < 0 || id >= M || n_tok[id] != slot_tokens) id = -1;   // not placeable: dropped
        raw[s] = id;
    }
    if (s == 0) s_n = 0;
    __syncthreads();
    // drop repeats of an earlier rank; compact the rest in rank order
    if (s < R) {
        bool good = raw[s] >= 0;
        for (int t = 0; good && t < s; ++t) good = raw[t] != raw[s];
        ok[s] = good;
    }
    __syncthreads();
    if (s < R && ok[s]) {
        int pos = 0;
        for (int t = 0; t < s; ++t) pos += ok[t];
        want[pos] = raw[s];
        atomicAdd(&s_n, 1);
    }
    __syncthreads();
    const int n = s_n;
    // resident and wanted chunks keep their slot -- unless one sits at or beyond slot n
    // (a slot table that names one chunk twice keeps the first copy only)
    bool my_keep = false;
    if (s < R && old[s] >= 0) {
        for (int w = 0; w < n; ++w) my_keep |= want[w] == old[s];
        for (int t = 0; my_keep && t < s; ++t) my_keep = old[t] != old[s];
    }
    if (s < R) keep[s] = my_keep;
    const int rebuild = __syncthreads_or(my_keep && s >= n);
    if (s < n) {   // is the chunk of rank s already resident (in a kept slot)?
        bool r = false;
        for (int t = 0; t < R; ++t) r |= keep[t] && old[t] == want[s];
        res[s] = r;
    }
    __syncthreads();
    if (s < n && !res[s] && !rebuild) {   // newcomers in rank order
        int pos = 0;
        for (int w = 0; w < s; ++w) pos += !res[w];
        inc[pos] = want[s];
    }
    __syncthreads();
    int mine = -1;
    bool my_fetch = false;
    if (s < n) {
        if (rebuild) {
            mine = want[s];
            my_fetch = old[s] != mine;
        } else if (keep[s]) {
            mine = old[s];
        } else {
            int pos = 0;   // rank of this slot among the free ones below n
            for (int t = 0; t < s; ++t) pos += !keep[t];
            mine = inc[pos];
            my_fetch = true;
        }
    }
    if (s < R) {
        fetch[s] = my_fetch;
        slot_ids[s] = mine;
    }
    __syncthreads();
    if (my_fetch) {
        int pos = 0;
        for (int t = 0; t < s; ++t) pos += fetch[t];
        fetch_slot[pos] = s;
        fetch_id[pos] = mine;
    }
    if (s == 0) {
        int total = 0;
        for (int t = 0; t < n; ++t) total += fetch[t];
        head->n_fetch = total;
        head->n_used = n;
        if (n_win) *n_win = n_native + n * slot_tokens;
        if (n_fetched) *n_fetched = total;
    }
}

struct FetchArgs {
    const void *const *K_ptr;
    const void *const *V_ptr;
    const PlanOut *head;
    const int32_t *fetch_slot;
    const int32_t *fetch_id;
    char *K_win;
    char *V_win;
    int H, R, slot_tokens, n_native, win_capacity, vec_per_row, units_per_slot;
};

// work unit u = ((f*2 + kv)*H + h)*units_per_slot + b: 32 KB of head h's K (kv=0) or V (kv=1) rows
// of the f-th entry of the fetch list
__global__ __launch_bounds__(kThreads) void k_slot_fetch(FetchArgs a) {
    const int n_fetch = a.head->n_fetch;
    const long long per_entry = 2ll * a.H * a.units_per_slot;
    const long long units = per_entry * n_fetch;
    const size_t row_bytes = (size_t)a.vec_per_row * 16;
    const long long slot_vec = (long long)a.slot_tokens * a.vec_per_row;
    const int tid = threadIdx.x;
    for (long long u = blockIdx.x; u < units; u += gridDim.x) {
        const int f = (int)(u / per_entry);
        const long long r = u % per_entry;
        const bool is_v = r >= (long long)a.H * a.units_per_slot;
        const int h = (int)((r / a.units_per_slot) % a.H);
        const long long v0 = (r % a.units_per_slot) * kVecPerBlock;
        const int slot = a.fetch_slot[f], id = a.fetch_id[f];
        const char *src = reinterpret_cast<const char *>(is_v ? a.V_ptr[id] : a.K_ptr[id]) +
                          (size_t)h * a.slot_tokens * row_bytes;
        char *dst = (is_v ? a.V_win : a.K_win) +
                    ((size_t)h * a.win_capacity + a.n_native + (size_t)slot * a.slot_tokens) * row_bytes;
        uvec4 buf[kVecPerThread];
#pragma unroll
        for (int i = 0; i < kVecPerThread; ++i) {
            const long long v = v0 + tid + (long long)i * kThreads;
            if (v < slot_vec) buf[i] = __builtin_nontemporal_load(reinterpret_cast<const uvec4 *>(src) + v);
        }
#pragma unroll
        for (int i = 0; i < kVecPerThread; ++i) {
            const long long v = v0 + tid + (long long)i * kThreads;
            if (v < slot_vec) __builtin_nontemporal_store(buf[i], reinterpret_cast<uvec4 *>(dst) + v);
        }
    }
}

}  // namespace

extern "C" wk_status wk_window_plan(const wk_window_desc *w, int64_t chunk_index, wk_window_step *out) {
    if (!w || !out || chunk_index < 0) return WK_ERR_INVALID_ARG;
    if (w->T < 1 || w->chunk_frames < 1 || w->sink_chunks < 0 || w->recent_chunks < 0 || w->R < 0 ||
        w->slot_tokens < 0)
        return WK_ERR_INVALID_ARG;
    const int64_t chunk_rows = (int64_t)w->chunk_frames * w->T;
    const int64_t ring_slots = (int64_t)w->recent_chunks + 1;
    const int64_t native_cap = ((int64_t)w->sink_chunks + ring_slots) * chunk_rows;
    const int64_t cap = native_cap + (int64_t)w->R * w->slot_tokens;
    if (cap > 0x7fffffffLL) return WK_ERR_UNSUPPORTED;
    out->denoise_rows = (int32_t)chunk_rows;
    out->retrieved_row0 = (int32_t)native_cap;
    out->win_capacity = (int32_t)cap;
    out->evict = 0;
    out->evict_row0 = 0;
    out->evict_chunk = -1;
    out->store_id = -1;
    if (chunk_index < w->sink_chunks) {   // one of the initial chunks: it is (part of) the sink
        out->denoise_row0 = (int32_t)(chunk_index * chunk_rows);
        out->n_native = (int32_t)((chunk_index + 1) * chunk_rows);
        out->M = 0;
        return WK_OK;
    }
    const int64_t k = chunk_index - w->sink_chunks;   // chunks that entered the ring before this one
    const int64_t slot = k % ring_slots;
    out->denoise_row0 = (int32_t)((w->sink_chunks + slot) * chunk_rows);
    const int64_t in_ring = k + 1 < ring_slots ? k + 1 : ring_slots;
    out->n_native = (int32_t)((w->sink_chunks + in_ring) * chunk_rows);
    if (k >= ring_slots) {   // the slot still holds chunk (chunk_index - ring_slots): store it first
        out->evict = 1;
        out->evict_row0 = out->denoise_row0;
        out->evict_chunk = chunk_index - ring_slots;
        const int64_t sid = k - ring_slots;
        if (sid > 0x7fffffffLL) return WK_ERR_UNSUPPORTED;
        out->store_id = (int32_t)sid;
    }
    const int64_t stored = k >= ring_slots ? k - ring_slots + 1 : 0;
    out->M = (int32_t)(stored > 0x7fffffffLL ? 0x7fffffffLL : stored);
    return WK_OK;
}

extern "C" size_t wk_window_update_workspace_bytes(int32_t R) {
    if (R < 0 || R > kMaxSlots) return 0;
    return 256 + wk::align_up((size_t)(R > 0 ? R : 1) * 2 * sizeof(int32_t), 256);
}

extern "C" wk_status wk_window_update(const wk_store_desc *store, const int32_t *ids, const int32_t *n_ids,
                                      int32_t R, int32_t slot_tokens, int32_t *slot_ids, int32_t n_native,
                                      void *K_win, void *V_win, int32_t win_capacity, int32_t *n_win,
                                      int32_t *n_fetched, void *workspace, size_t workspace_bytes,
                                      int32_t max_workgroups, void *hip_stream) {
    if (!store || !K_win || !V_win) return WK_ERR_INVALID_ARG;
    if (R < 0 || slot_tokens < 1 || n_native < 0 || win_capacity < 0 || max_workgroups < 0 || store->M < 0 ||
        store->H < 1)
        return WK_ERR_INVALID_ARG;
    if (store->dtype != WK_F32 && store->dtype != WK_BF16) return WK_ERR_INVALID_ARG;
    if (R > 0 && (!ids || !slot_ids)) return WK_ERR_INVALID_ARG;
    if (R > 0 && store->M > 0 && (!store->K_ptr || !store->V_ptr || !store->n_tok)) return WK_ERR_INVALID_ARG;
    if (store->d != WK_D || R > kMaxSlots) return WK_ERR_UNSUPPORTED;
    if ((int64_t)n_native + (int64_t)R * slot_tokens > (int64_t)win_capacity) return WK_ERR_SHAPE;
    if (slot_tokens > store->max_tok && store->M > 0) return WK_ERR_SHAPE;   // no chunk within the store's bound fits the slots
    const size_t need = wk_window_update_workspace_bytes(R);
    if (!workspace || workspace_bytes < need || reinterpret_cast<uintptr_t>(workspace) % 256 != 0)
        return WK_ERR_WORKSPACE;
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    PlanOut *head = reinterpret_cast<PlanOut *>(workspace);
    int32_t *fetch_slot = reinterpret_cast<int32_t *>(reinterpret_cast<char *>(workspace) + 256);
    int32_t *fetch_id = fetch_slot + (R > 0 ? R : 1);
    hipLaunchKernelGGL(k_slot_plan, dim3(1), dim3(kPlanThreads), 0, st, ids, n_ids, (int)R, (int)store->M,
                       store->n_tok, (int)slot_tokens, slot_ids, (int)n_native, n_win, n_fetched, head, fetch_slot,
                       fetch_id);
    WK_LAUNCH_CHECK();
    if (R == 0 || store->M == 0) return WK_OK;
    FetchArgs a;
    a.K_ptr = store->K_ptr; a.V_ptr = store->V_ptr;
    a.head = head; a.fetch_slot = fetch_slot; a.fetch_id = fetch_id;
    a.K_win = reinterpret_cast<char *>(K_win);
    a.V_win = reinterpret_cast<char *>(V_win);
    a.H = store->H; a.R = R; a.slot_tokens = slot_tokens; a.n_native = n_native; a.win_capacity = win_capacity;
    a.vec_per_row = (int)(WK_D * wk::esize(store->dtype) / 16);
    const long long slot_vec = (long long)slot_tokens * a.vec_per_row;
    a.units_per_slot = (int)((slot_vec + kVecPerBlock - 1) / kVecPerBlock);
    long long grid = 2ll * store->H * a.units_per_slot * R;
    if (max_workgroups > 0 && grid > max_workgroups) grid = max_workgroups;
    if (grid > 0x7fffffffLL) grid = 0x7fffffffLL;
    hipLaunchKernelGGL(k_slot_fetch, dim3((unsigned)grid), dim3(kThreads), 0, st, a);
    WK_LAUNCH_CHECK();
    return WK_OK;
}
