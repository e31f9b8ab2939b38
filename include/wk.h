/*
 * wk.h -- C ABI of the WorldKV hot path for AMD MI355X (gfx950).
 *
 * One call = one transformer layer.  The paper's method (Sec. 4) keeps evicted
 * KV-cache chunks in a store, prunes each chunk by key-key similarity to its
 * anchor frame when it is stored (World Compression, Sec. 4.3), selects the
 * Top-k stored chunks by camera/action correspondence when a new chunk is
 * generated (World Retrieval, Sec. 4.2, Eq. 4), inserts them into the sliding
 * window without re-encoding, and runs ordinary softmax attention of the
 * denoising chunk's queries over that window.
 *
 * Conventions for every call
 *   - Tensors are head-major and dense: [H][N][d] with d = 128 contiguous.
 *     Element types: WK_F32 (IEEE binary32) or WK_BF16 (bfloat16).
 *   - "device" pointers must be readable/writable by kernels on the current
 *     HIP device (HBM, or host memory allocated pinned+mapped where stated).
 *     "host" pointers are ordinary host memory read during the call.
 *   - The caller owns every buffer.  The library allocates no memory, frees
 *     nothing and keeps no pointer after a call returns.  (wk_prefetch_create
 *     is the one call that creates runtime objects: a stream and events.)
 *   - Work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL =
 *     the default stream) and the call returns without waiting for it.
 *   - Argument errors are detected before anything is launched, leave all
 *     outputs untouched and are returned as a wk_status.  A failed launch
 *     returns WK_ERR_HIP.  Nothing throws across this boundary.
 *   - Inputs must be finite; NaN/Inf give unspecified selections.
 */
#ifndef WK_H
#define WK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    WK_OK = 0,
    WK_ERR_INVALID_ARG = 1, /* null pointer, negative size, unknown enum value */
    WK_ERR_SHAPE = 2,       /* sizes inconsistent with each other (e.g. window too small) */
    WK_ERR_RATIO = 3,       /* keep ratio outside what the chunk allows */
    WK_ERR_WORKSPACE = 4,   /* workspace missing or too small */
    WK_ERR_UNSUPPORTED = 5, /* valid request this build has no kernel for (d != 128, M too large) */
    WK_ERR_HIP = 6          /* the HIP runtime reported an error */
} wk_status;

typedef enum { WK_F32 = 0, WK_BF16 = 1 } wk_dtype;

/* Eq. 5 is written for the key vectors of a layer and never mentions heads.
 * SHARED: the key vector of a token is the concatenation of its H head slices and one
 *         index set serves the whole layer (the literal reading; default).
 * INDEPENDENT: Eq. 5 is applied per head (d = 128) and every head keeps its own,
 *         equally sized, index set. */
typedef enum { WK_HEADS_SHARED = 0, WK_HEADS_INDEPENDENT = 1 } wk_head_mode;

/* FIRST_FRAME: the anchor is the first of the chunk's F frames (Sec. 4.3) and is stored in full.
 * EXTERNAL: the anchor frame is passed separately and is not stored with the chunk; all F*T
 *         tokens are candidates (needed for one-frame chunks). */
typedef enum { WK_ANCHOR_FIRST_FRAME = 0, WK_ANCHOR_EXTERNAL = 1 } wk_anchor_mode;

/* CHUNK: rho is the kept fraction of the whole stored chunk (0.5 for "3 frames -> 1.5").
 * NONANCHOR: rho is the paper's P, the kept fraction of the pooled non-anchor tokens (0.25). */
typedef enum { WK_RATIO_CHUNK = 0, WK_RATIO_NONANCHOR = 1 } wk_ratio_kind;

/* Two ways to evaluate Eq. 5 (same result up to rounding).
 * FACTORED: mean cosine = dot product with the mean of the normalised anchor keys; one pass
 *         over K, bound by HBM bandwidth (default).
 * GEMM:   token-by-anchor similarity tiles on the matrix cores with the row mean taken in the
 *         tile epilogue; the T x (F-1)T matrix is never written.  bf16 only. */
typedef enum { WK_SCORE_FACTORED = 0, WK_SCORE_GEMM = 1 } wk_score_algo;

/* How each distance term is normalised over the set of retrieval candidates (Sec. 5.1). */
typedef enum { WK_NORM_MAX = 0, WK_NORM_MINMAX = 1, WK_NORM_MEAN = 2 } wk_norm_mode;

typedef struct wk_compress_desc {
    int32_t H;           /* heads */
    int32_t d;           /* head dimension, must be 128 */
    int32_t T;           /* tokens per latent frame */
    int32_t F;           /* frames per chunk */
    int32_t batch;       /* independent chunk-layers in this call (>= 1) */
    int32_t dtype;       /* wk_dtype */
    int32_t head_mode;   /* wk_head_mode */
    int32_t anchor_mode; /* wk_anchor_mode */
    int32_t ratio_kind;  /* wk_ratio_kind */
    int32_t score_algo;  /* wk_score_algo */
    float rho;           /* keep ratio in [0, 1] */
} wk_compress_desc;

/* Token counts of a compressed chunk (Sec. 4.3: anchor tokens plus the retained tokens; F = 3,
 * P = 25% gives 3T -> 1.5T).  Counts round half away from zero.  Pure host arithmetic.
 * Writes the stored tokens per chunk to *n_out and the retained non-anchor tokens to *n_keep
 * (either may be NULL).  WK_ERR_RATIO if rho is outside [0,1], asks for fewer tokens than the
 * anchor frame, or leaves the chunk empty. */
wk_status wk_keep_count(float rho, int32_t ratio_kind, int32_t anchor_mode, int32_t F, int32_t T,
                        int32_t *n_out, int32_t *n_keep);

/* Bytes of device workspace wk_compress_chunk needs for this descriptor (0 if it is invalid). */
size_t wk_compress_workspace_bytes(const wk_compress_desc *desc);

/* World Compression (Sec. 4.3): Eq. 5 redundancy score of every non-anchor key against the
 * anchor frame's keys, scores pooled over the non-anchor frames, the lowest-scoring n_keep
 * tokens retained (ties: lower token index first), and the chunk compacted to anchor tokens
 * followed by the retained tokens in their original order.  K and V are pruned with the same
 * indices and rows are copied bit for bit.
 *
 *   K, V       device, [batch][H][F*T][d]
 *   K_anchor   device, [batch][H][T][d]; WK_ANCHOR_EXTERNAL only, else must be NULL
 *   kept_idx   device out, [batch][G][n_out] int32, ascending token indices into the chunk's
 *              F*T tokens; G = 1 (SHARED) or H (INDEPENDENT).  May be NULL.
 *   K_out,V_out device out (HBM or pinned+mapped host), [batch][H][n_out][d]
 *   n_out      host out, stored tokens per chunk (same value wk_keep_count gives). May be NULL.
 *   workspace  device, at least wk_compress_workspace_bytes(desc) bytes, 256-byte aligned.
 *              After the call its first batch*G*N_c doubles hold the Eq. 5 scores
 *              ([batch][G][N_c], N_c = candidates per chunk), which callers may read.
 * Errors: INVALID_ARG (null/enum), UNSUPPORTED (d != 128; GEMM scoring with fp32),
 *         RATIO, WORKSPACE. */
wk_status wk_compress_chunk(const wk_compress_desc *desc, const void *K, const void *V,
                            const void *K_anchor, int32_t *kept_idx, void *K_out, void *V_out,
                            int32_t *n_out, void *workspace, size_t workspace_bytes,
                            void *hip_stream);

/* For callers that cannot allocate device memory or pass a workspace along (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): wk_compress_chunk with the same
 * arguments, results and errors, minus the workspace, which is a fixed array of
 * WK_COMPRESS_SCRATCH_BYTES built into the library (each GPU the library runs on holds one until the
 * process ends).  The call allocates and frees nothing.  One LingBot-sized chunk (H = 40, T = 1,560,
 * F = 3) fits in either head mode with factored scoring and in shared-head mode with GEMM scoring.
 *   - WK_ERR_WORKSPACE if wk_compress_workspace_bytes(desc) exceeds WK_COMPRESS_SCRATCH_BYTES (nothing
 *     is launched); WK_ERR_HIP if the array's address cannot be resolved.
 *   - Every call on a GPU uses that GPU's one array: calls that may overlap on one GPU (different
 *     streams, or different host threads) race; keep them in order on one stream.  The array keeps the
 *     last call's contents; no call depends on them.
 *   - The first call on a device resolves the array's device address (a runtime query, not a stream
 *     operation); make one call on the device before capturing a graph that holds this call.
 *   - The Eq. 5 scores are not readable by the caller here (the array is private to the library). */
#define WK_COMPRESS_SCRATCH_BYTES (4u << 20)
size_t wk_compress_scratch_bytes(void);
wk_status wk_compress_chunk_noalloc(const wk_compress_desc *desc, const void *K, const void *V,
                                    const void *K_anchor, int32_t *kept_idx, void *K_out, void *V_out,
                                    int32_t *n_out, void *hip_stream);

#define WK_SCORE_MAX_CHUNKS 4096

/* World Retrieval (Sec. 4.2, Eq. 4) with the camera/action distance of Sec. 5.1: for every
 * stored chunk the squared L2 distance between translations and the geodesic angle between
 * rotations (R = R_y(yaw) R_x(pitch), radians), each normalised over the M candidates
 * (norm_mode) and summed; the min(R, M) chunks of smallest distance are returned in order of
 * increasing distance (ties: lower chunk id first).  Arithmetic is fp64.
 *
 *   poses      device, [M][5] float = (x, y, z, yaw, pitch) of each stored chunk
 *   cur_pose   host, [5] float, the current camera/action state (read during the call)
 *   ids_out    device out, [R] int32; entries past n_found are -1
 *   dist_out   device out, [R] double; entries past n_found are +inf.  May be NULL.
 *   n_found    device out, int32 = min(R, M)
 * M = 0 is valid (nothing found).  Errors: INVALID_ARG, UNSUPPORTED (M > WK_SCORE_MAX_CHUNKS). */
wk_status wk_score_chunks(const float *poses, int32_t M, const float *cur_pose, int32_t norm_mode,
                          int32_t R, int32_t *ids_out, double *dist_out, int32_t *n_found,
                          void *hip_stream);

#define WK_QUERY_MAX_CHUNKS 1024

/* Query-based retrieval (Sec. 4.2: the relevance function may be a query-based importance score;
 * App. C: stored chunks ranked by their attention scores with respect to the current denoising
 * query).  The relevance of chunk c is the attention mass its keys receive from the current queries
 * in one softmax over the keys of all M candidate chunks, averaged over all (head, query) rows; the
 * min(R, M) chunks of largest mass are returned in order of decreasing mass (ties: lower id first).
 *
 *   lse        device, [M][n_rows] float: lse[c][r] = natural-log sum over the keys k of chunk c of
 *              exp(scale * q_r . k) for (head, query) row r -- what wk_chunk_lse writes (or the
 *              `lse` output of wk_attention run with chunk c's keys as the window, O = NULL)
 *   ids_out    device out, [R] int32; entries past n_found are -1
 *   mass_out   device out, [R] double; entries past n_found are -inf.  May be NULL.
 *   n_found    device out, int32 = min(R, M)
 *   workspace  device, wk_score_chunks_query_workspace_bytes(M, n_rows) bytes, 256-byte aligned.
 *              After the call its first M doubles hold the mass of every chunk.
 * Errors: INVALID_ARG, UNSUPPORTED (M > WK_QUERY_MAX_CHUNKS), WORKSPACE. */
wk_status wk_score_chunks_query(const float *lse, int32_t M, int64_t n_rows, int32_t R, int32_t *ids_out,
                                double *mass_out, int32_t *n_found, void *workspace,
                                size_t workspace_bytes, void *hip_stream);
size_t wk_score_chunks_query_workspace_bytes(int32_t M, int64_t n_rows);

/* Pseudo-poses for keyboard/mouse models (Sec. 5.1): accumulate discrete actions into a
 * translation and a rotation.  Labels: 0 W forward, 1 A left, 2 S back, 3 D right, 4 yaw-,
 * 5 yaw+, 6 pitch-, 7 pitch+.  Translation steps of length `step` are taken in the body frame
 * of the current yaw (forward = (sin yaw, 0, cos yaw), right = (cos yaw, 0, -sin yaw)); rotation
 * steps are `dangle` radians; pitch is clamped to +-pitch_limit.  poses_out[i] is the state
 * after label i.  Host function, host pointers.  (The paper gives no step sizes; callers
 * choose them.)  Errors: INVALID_ARG (null pointer, label outside 0..7). */
wk_status wk_accumulate_actions(const int32_t *labels, int32_t n, float step, float dangle,
                                float pitch_limit, float *poses_out /* [n][5] */);

typedef struct wk_store_desc {
    const void *const *K_ptr; /* device array [M]: address of chunk c's keys, [H][n_tok[c]][d] */
    const void *const *V_ptr; /* device array [M]: same for values */
    const int32_t *n_tok;     /* device array [M]: stored tokens of chunk c */
    int32_t M;                /* chunks in the store */
    int32_t max_tok;          /* host-known upper bound of n_tok[]: a hard bound.  Buffers and offsets are sized
                                 by it on the host; a chunk whose n_tok[c] exceeds it is treated as absent
                                 (skipped, like an id outside [0, M)) by every call that reads the store */
    int32_t H, d, dtype;
} wk_store_desc;

/* Window assembly (Sec. 1: retrieved caches are reused as stored, not re-encoded; Sec. 4.2): window = native rows followed by
 * the stored rows of each retrieved chunk in the order of ids, byte for byte, for K and V.
 * The addresses in K_ptr/V_ptr may point to HBM or to pinned+mapped host memory (CPU-offloaded
 * store, Sec. 7); ids and n_ids come from wk_score_chunks and are read on the device, so no
 * host synchronisation separates the two calls.
 *
 *   ids        device, [R_max] int32; entries < 0 or >= M, and chunks with n_tok > max_tok, are skipped
 *   n_ids      device, int32; only the first min(*n_ids, R_max) ids are used.  NULL = R_max.
 *   K_native,V_native device, [H][n_native][d]; NULL with n_native > 0 means the native rows
 *              are already in place in the window and are not copied
 *   K_win,V_win device out, [H][win_capacity][d]; rows past the assembled length are untouched
 *   n_win      device out, int32 = n_native + sum of retrieved chunk lengths.  May be NULL.
 * Errors: INVALID_ARG, UNSUPPORTED (d != 128, R_max > 1024, win_capacity >= 2^26 rows),
 *         SHAPE (win_capacity < n_native + R_max * max_tok). */
wk_status wk_gather_window(const wk_store_desc *store, const int32_t *ids, const int32_t *n_ids,
                           int32_t R_max, const void *K_native, const void *V_native,
                           int32_t n_native, void *K_win, void *V_win, int32_t win_capacity,
                           int32_t *n_win, void *hip_stream);

/* Attention of the denoising chunk's queries over the assembled window (Sec. 4.2, Sec. 4.3):
 * O = softmax(Q K^T * scale) V per head, every window key visible to every query.
 * bf16: matrix-core products with fp32 accumulation, probabilities rounded to bf16 before the
 * P*V product, one rounding of O to bf16 at the end.  fp32: fp32 throughout.
 *
 *   Q          device, [H][N_q][d]
 *   K_win,V_win device, [H][kv_row_stride][d]; the first N_kv rows of each head are attended
 *   O          device out, [H][N_q][d], same element type as the inputs.  May be NULL if lse is
 *              given: only the log-sum-exp is produced and the value product is skipped.
 *   lse        device out, [H][N_q] float: natural-log sum of exp of the scaled logits. May be NULL.
 *   scale      logit scale; 0 means 1/sqrt(d)
 *   n_kv_dev   device, int32 or NULL.  If given, min(N_kv, *n_kv_dev) keys are attended (the
 *              length wk_gather_window wrote), read on the device.  A length of 0 gives O = 0
 *              and lse = -inf.
 *   workspace  device, 256-byte aligned, or NULL.  When one workgroup per head and query tile would leave
 *              compute units idle (few heads, short query chunk, long window) the key range is split
 *              over several workgroups whose partial results are merged by a second kernel; that
 *              needs wk_attention_workspace_bytes(...) bytes.  Without (enough) workspace the call
 *              runs unsplit: same result up to fp32 rounding order, lower occupancy.
 * Errors: INVALID_ARG, UNSUPPORTED (d != 128; bf16 with N_kv > 2^24 - 512 rows), SHAPE (N_kv < 1 or
 *         N_kv > kv_row_stride). */
wk_status wk_attention(const void *Q, const void *K_win, const void *V_win, void *O, float *lse,
                       int32_t H, int32_t N_q, int32_t N_kv, int32_t d, int32_t kv_row_stride,
                       int32_t dtype, float scale, const int32_t *n_kv_dev, void *workspace,
                       size_t workspace_bytes, void *hip_stream);

/* Bytes of workspace with which wk_attention splits the key range for this shape (0: it would not). */
size_t wk_attention_workspace_bytes(int32_t H, int32_t N_q, int32_t N_kv, int32_t dtype);

/* wk_attention with a frame-level causal mask inside the chunk being denoised -- an option; the
 * paper's method itself states no mask (Sec. 4.2), frame-causal attention inside a chunk is a
 * property some of the autoregressive video backbones of Sec. 3 have.  The N_q queries are the
 * chunk's tokens, N_q / frame_T frames of frame_T tokens, and their own keys are window rows
 * [denoise_row0, denoise_row0 + N_q) in the same order (wk_window_step.denoise_row0).  Query i
 * sees every window row outside that range and, inside it, the rows of frames 0 .. i / frame_T.
 * Arguments as for wk_attention; O is required.
 *
 *   n_kv_dev   if given, *n_kv_dev must be >= denoise_row0 + N_q (the chunk lies inside the window)
 *   workspace  device, 256-byte aligned, wk_attention_block_causal_workspace_bytes(H, N_q) bytes:
 *              the two visible key ranges of a query are attended separately and merged
 * Errors: INVALID_ARG, UNSUPPORTED (d != 128; bf16 with N_kv > 2^24 - 512 rows), SHAPE (N_kv, or N_q not a
 * multiple of frame_T, or the chunk's rows run past N_kv), WORKSPACE. */
wk_status wk_attention_block_causal(const void *Q, const void *K_win, const void *V_win, void *O,
                                    float *lse, int32_t H, int32_t N_q, int32_t N_kv, int32_t d,
                                    int32_t kv_row_stride, int32_t dtype, float scale,
                                    const int32_t *n_kv_dev, int32_t denoise_row0, int32_t frame_T,
                                    void *workspace, size_t workspace_bytes, void *hip_stream);
size_t wk_attention_block_causal_workspace_bytes(int32_t H, int32_t N_q);

/* wk_gather_window and wk_attention in one: attention over the window of Sec. 4.2 without building it.
 * The window is the native rows followed by the stored rows of chunks ids[0 .. min(*n_ids, R_max)),
 * exactly what wk_gather_window would assemble (the stored caches are used as they are, Sec. 1), but
 * the kernel reads each retrieved chunk where the store keeps it.  Meant for a store that lives in
 * HBM, where copying 2 x R chunks per layer and step costs more than the indirection; a store in pinned
 * host memory is better served by wk_gather_window / wk_prefetch_gather, which cross the host link once.
 * bf16 only.  The result equals wk_attention over the assembled window up to the order of fp32 sums
 * (key tiles are cut per segment here).
 *
 *   Q          device, [H][N_q][d]; H, d and the element type are the store's
 *   K_native,V_native device, [H][native_row_stride][d]; the first n_native rows of each head are
 *              attended.  May be NULL when n_native is 0.
 *   ids,n_ids  device; as for wk_gather_window (ids outside [0, M) and empty chunks are skipped,
 *              n_ids NULL means R_max)
 *   O          device out, [H][N_q][d] bf16; all zero when the window is empty
 *   lse        device out, [H][N_q] float or NULL; -inf when the window is empty
 *   scale      logit scale; 0 means 1/sqrt(d)
 * Errors: INVALID_ARG, UNSUPPORTED (d != 128, fp32 store, R_max > 32, 2^23 or more rows in the
 *         native part or in a chunk), SHAPE (n_native > native_row_stride). */
wk_status wk_attention_in_place(const void *Q, const void *K_native, const void *V_native,
                                int32_t n_native, int32_t native_row_stride, const wk_store_desc *store,
                                const int32_t *ids, const int32_t *n_ids, int32_t R_max, void *O,
                                float *lse, int32_t N_q, float scale, void *hip_stream);

/* First half of query-based retrieval (Sec. 4.2, App. C): the log-sum-exp of the current queries'
 * scaled logits against the stored keys of every chunk of the store, all chunks in one launch.
 * The result is the `lse` input of wk_score_chunks_query.  Only K_ptr, n_tok, M, H, d and dtype
 * of the store are used; the key tables may describe whole compacted chunks or, for a cheaper
 * index, the anchor-frame keys of each chunk alone.
 *
 *   Q          device, [H][N_q][d], element type store->dtype
 *   scale      logit scale; 0 means 1/sqrt(d)
 *   lse_out    device out, [M][H][N_q] float; -inf where a chunk holds no token
 * Errors: INVALID_ARG, UNSUPPORTED (d != 128, more than 2^31 workgroups, bf16 with max_tok > 2^24 - 512). */
wk_status wk_chunk_lse(const wk_store_desc *store, const void *Q, int32_t N_q, float scale,
                       float *lse_out, void *hip_stream);

/* ---- Window bookkeeping (Sec. 4.2: sink, retrieved, recent and denoising regions of the sliding
 * window; Sec. 5.1: 3 + 9 + 3 + 3 latent frames).  Physical rows of a window buffer, per head:
 *
 *     [ sink_chunks chunks | ring of recent_chunks + 1 chunk slots | R retrieved slots ]
 *
 * each chunk chunk_frames * T rows, each retrieved slot slot_tokens rows.  The chunk being generated
 * and the recent chunks rotate over the ring slots (no copy when a chunk turns from "denoising"
 * into "recent"); the order of regions is free because attention sums over all window keys. */
typedef struct wk_window_desc {
    int32_t T;             /* tokens per latent frame */
    int32_t chunk_frames;  /* latent frames per generated chunk (3) */
    int32_t sink_chunks;   /* initial chunks kept for ever (1 = 3 sink frames) */
    int32_t recent_chunks; /* chunks kept behind the one being generated (1 = 3 recent frames) */
    int32_t R;             /* retrieved slots (6 compressed chunks = 9 frames at 3 -> 1.5) */
    int32_t slot_tokens;   /* rows per retrieved slot = stored tokens of a compressed chunk */
} wk_window_desc;

typedef struct wk_window_step {
    int32_t denoise_row0;   /* the K/V of the chunk being generated live at rows [denoise_row0, +denoise_rows) */
    int32_t denoise_rows;
    int32_t n_native;       /* rows [0, n_native) are the valid sink + recent + denoising rows at this step */
    int32_t evict;          /* 1: rows [evict_row0, +denoise_rows) still hold chunk evict_chunk, which must be
                               compressed into the store as chunk store_id BEFORE the new chunk's K/V are
                               written there (same rows) */
    int32_t evict_row0;
    int32_t store_id;       /* -1 when evict == 0 */
    int64_t evict_chunk;    /* generation index of the chunk leaving the window; -1 when evict == 0 */
    int32_t M;              /* stored chunks available to retrieval at this step (eviction included) */
    int32_t retrieved_row0; /* first row of the retrieved slots (= n_native once the ring is full) */
    int32_t win_capacity;   /* rows per head of the window buffer */
} wk_window_step;

/* Host arithmetic: the placement for generated chunk chunk_index (0, 1, 2, ...).
 * Errors: INVALID_ARG, UNSUPPORTED (a count does not fit in 31 bits). */
wk_status wk_window_plan(const wk_window_desc *w, int64_t chunk_index, wk_window_step *out);

/* In-place refresh of the retrieved region (Sec. 4.2: the top-k chunks are what this region holds).  slot_ids
 * says which stored chunk each of the R slots holds (-1: none); ids are the chunks wanted now (from
 * wk_score_chunks or wk_score_chunks_query).  Ids that are out of range, repeat an earlier one, or
 * name a chunk whose n_tok differs from slot_tokens are dropped; n are left.  Afterwards exactly slots
 * 0..n-1 are in use: a wanted chunk that is already resident keeps its slot and is not copied; the
 * others are copied from the store (HBM or pinned host) into the remaining slots below n, ascending,
 * in the order of ids.  If a resident wanted chunk sits at or beyond slot n the region is rebuilt
 * (slot j = j-th wanted chunk), copying only slots whose content changes.
 *
 *   ids, n_ids device, as for wk_gather_window (NULL n_ids = R)
 *   slot_ids   device in/out, [R] int32
 *   n_native   first row of slot 0 (wk_window_step.retrieved_row0)
 *   n_win      device out, int32 = n_native + n * slot_tokens.  May be NULL.
 *   n_fetched  device out, int32 = chunks copied by this call.  May be NULL.
 *   workspace  device, wk_window_update_workspace_bytes(R) bytes, 256-byte aligned
 *   max_workgroups  > 0 caps the copy grid (see wk_prefetch_gather); 0 = one per 32 KB
 * Errors: INVALID_ARG, UNSUPPORTED (d != 128, R > 1024), SHAPE (slots exceed win_capacity, or slot_tokens
 *         exceeds the store's max_tok), WORKSPACE. */
wk_status wk_window_update(const wk_store_desc *store, const int32_t *ids, const int32_t *n_ids, int32_t R,
                           int32_t slot_tokens, int32_t *slot_ids, int32_t n_native, void *K_win,
                           void *V_win, int32_t win_capacity, int32_t *n_win, int32_t *n_fetched,
                           void *workspace, size_t workspace_bytes, int32_t max_workgroups,
                           void *hip_stream);
size_t wk_window_update_workspace_bytes(int32_t R);

/* ---- Overlap of a CPU-offloaded store with attention (Sec. 7: the host-to-device transfer at
 * retrieval time is the stated obstacle to real time with all KV chunks in CPU memory).
 *
 * A wk_prefetch owns one extra HIP stream of default priority (the "copy stream") and, per window
 * buffer ("slot", at most 8), two events.  The intended loop over the layers l of a denoising step,
 * with two window buffers and the ids of wk_score_chunks (the same for every layer):
 *
 *     wk_prefetch_after(p, compute)                         ids/n_found are ready before any gather
 *     wk_prefetch_gather(p, 0, store[0], ..., win[0], ...)
 *     for l = 0 .. L-1:
 *         if l+1 < L: wk_prefetch_gather(p, (l+1)%2, store[l+1], ..., win[(l+1)%2], ...)
 *         wk_prefetch_acquire(p, l%2, compute)
 *         wk_attention(Q[l], win[l%2], ..., compute)
 *         wk_prefetch_release(p, l%2, compute)
 *
 * so that the assembly of layer l+1's window (host-link-bound when the store is in pinned host
 * memory) runs while layer l attends.  The same stream serves the other direction: after
 * wk_prefetch_after(p, compute), wk_compress_chunk(..., wk_prefetch_stream(p)) with K_out/V_out in
 * mapped host memory writes an evicted chunk to the CPU-side store without stalling the compute
 * stream.  Calls on one wk_prefetch must come from one host thread at a time.  Nothing here
 * synchronises the host except wk_prefetch_destroy. */
typedef struct wk_prefetch wk_prefetch;

/* Creates the copy stream and 2*n_slots events on the current device.  Errors: INVALID_ARG
 * (n_slots outside 1..8), HIP. */
wk_status wk_prefetch_create(wk_prefetch **out, int32_t n_slots);
/* Waits for the copy stream to drain, then frees stream and events.  NULL is allowed. */
wk_status wk_prefetch_destroy(wk_prefetch *p);
/* The copy stream (a hipStream_t), for enqueueing other transfers in order with the gathers. */
void *wk_prefetch_stream(wk_prefetch *p);
/* Work enqueued on the copy stream from now on starts only after everything enqueued so far on
 * hip_stream has finished. */
wk_status wk_prefetch_after(wk_prefetch *p, void *hip_stream);
/* wk_gather_window (same arguments, same errors) on the copy stream into the window buffers of
 * `slot`: first waits until the consumers recorded by the last wk_prefetch_release of that slot
 * have finished, afterwards marks the slot ready.  max_workgroups > 0 caps the grid (a host-link
 * bound gather needs only a few workgroups in flight; 0 = one workgroup per 32 KB). */
wk_status wk_prefetch_gather(wk_prefetch *p, int32_t slot, const wk_store_desc *store, const int32_t *ids,
                             const int32_t *n_ids, int32_t R_max, const void *K_native,
                             const void *V_native, int32_t n_native, void *K_win, void *V_win,
                             int32_t win_capacity, int32_t *n_win, int32_t max_workgroups);
/* Work enqueued on hip_stream from now on starts only after the slot's last gather has finished.
 * Errors: INVALID_ARG (no gather was enqueued for this slot yet), HIP. */
wk_status wk_prefetch_acquire(wk_prefetch *p, int32_t slot, void *hip_stream);
/* Declares that every reader of the slot's window has been enqueued on hip_stream: the next gather
 * into the slot waits for them. */
wk_status wk_prefetch_release(wk_prefetch *p, int32_t slot, void *hip_stream);

/* ---- Measurement aid -------------------------------------------------------------------------
 * Not a step of the method and not needed by any caller of the path: a straight device copy of `bytes` bytes (a multiple of
 * 16, both pointers 16-byte aligned, ranges must not overlap) with ordinary cached 16-byte loads and
 * stores.  Profilers' HBM byte counters are calibrated against it: it moves a known number of bytes
 * with the access pattern of the attention kernels' tile loads.  Errors: INVALID_ARG. */
wk_status wk_calibration_copy(void *dst, const void *src, size_t bytes, void *hip_stream);

/* Device-visible address of a pinned+mapped host allocation (for K_ptr/V_ptr tables and for
 * K_out/V_out of wk_compress_chunk).  Errors: INVALID_ARG, HIP (memory is not pinned). */
wk_status wk_host_device_pointer(void *host_ptr, void **device_ptr);

const char *wk_status_string(wk_status s);

#ifdef __cplusplus
}
#endif
#endif /* WK_H */
