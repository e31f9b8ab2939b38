// World Compression (paper Sec. 4.3, Eq. 5): redundancy scores, pooled bottom-P% selection,
// chunk compaction.  Kernels for gfx950; every pass is a coalesced stream over K (or K and V),
// 16 lanes x 16 bytes per bf16 row, bound by HBM bandwidth.
//
// Factored evaluation of Eq. 5: cos is bilinear in the normalised vectors, so
//   s_j = (1/T) sum_i khat_j . khat_i = khat_j . m,   m = (1/T) sum_i khat_i.
// The pass structure is: squared norms of the anchor tokens -> m -> one pass over the
// candidates that accumulates both k_j . m and |k_j|^2.  Partial sums over a lane's 8 elements
// are fp32 (bf16 products are exact in fp32), everything across lanes and heads is fp64, so the
// scores agree with an fp64 evaluation of the double sum to ~1e-9 absolute.
#include <cmath>
#include <type_traits>

#include "wk_internal.h"

namespace {

using wk::kRowLanes;
using wk::load_row8;

constexpr int kRowsPerBlock = 16;  // 256 threads

struct CompressDims {
    int H, T, n_tok;    // heads, anchors per chunk, rows per head in K
    int first_cand;     // first candidate row in K (T, or 0 with an external anchor)
    int n_cand;         // candidate rows
    int G, hg;          // score lists per chunk, heads per list
    int a_rows;         // rows per head in the anchor buffer
    int n_keep, n_out;
};

// Rows kernels (norms, factored scores): 16 lanes share a 256- or 512-byte row.  With HS > 1 the heads of
// a list are dealt round-robin to HS such lane groups (a whole wave per token at HS = 4), so that a token
// whose vector spans many heads has its rows in flight from several groups at once; kHeadBatch rows
// per group are requested before any is consumed.  Partial sums meet in a fixed order.
constexpr int kHeadBatch = 5;

template <int HS>
__device__ inline double head_split_sum(double x) {
    x = wk::row_group_sum(x);
    if constexpr (HS >= 2) x += __shfl_xor(x, 16);
    if constexpr (HS >= 4) x += __shfl_xor(x, 32);
    return x;
}

// out[(b*G+g)*n_rows + i] = |key first_row + i|^2 over the heads of group g; src is [batch][H][rows_per_head][128]
template <int DT, int HS>
__global__ __launch_bounds__(256) void k_rows_normsq(const char *__restrict__ src, CompressDims p, int rows_per_head,
                                                     int first_row, int n_rows, double *__restrict__ out) {
    const int i = blockIdx.x * (kRowsPerBlock / HS) + threadIdx.x / (kRowLanes * HS);
    const int hq = (threadIdx.x / kRowLanes) % HS;
    const int sub = threadIdx.x % kRowLanes;
    const int g = blockIdx.y, b = blockIdx.z;
    if (i >= n_rows) return;
    const size_t row_bytes = WK_D * wk::esize(DT);
    const size_t head_bytes = (size_t)rows_per_head * row_bytes;
    const char *base = src + ((size_t)b * p.H * rows_per_head + first_row + i) * row_bytes;
    double acc = 0.0;
    for (int hh0 = hq; hh0 < p.hg; hh0 += HS * kHeadBatch) {
        float v[kHeadBatch][8];
#pragma unroll
        for (int u = 0; u < kHeadBatch; ++u) {
            const int hh = hh0 + u * HS;
            if (hh < p.hg) {
                load_row8<DT>(base + (size_t)(p.G == 1 ? hh : g) * head_bytes, sub, v[u]);
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) v[u][e] = 0.f;
            }
        }
#pragma unroll
        for (int u = 0; u < kHeadBatch; ++u) {
            float s = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) s = fmaf(v[u][e], v[u][e], s);
            acc += (double)s;
        }
    }
    acc = head_split_sum<HS>(acc);
    if (sub == 0 && hq == 0) out[((size_t)b * p.G + g) * n_rows + i] = acc;
}

// m[(b*H+h)*128 + c] = (1/T) sum_i A[b][h][i][c] / |anchor key i|   (fp32 result of an fp64 sum).
// The T rows of a head are split over kMeanSplits workgroups (one head alone would keep only H CUs
// busy); partial sums meet in a fixed order in k_anchor_mean_finish, so the result is deterministic.
constexpr int kMeanSplits = 16;

template <int DT>
__global__ __launch_bounds__(256) void k_anchor_mean_partial(const char *__restrict__ A, CompressDims p,
                                                             const double *__restrict__ nsq,
                                                             double *__restrict__ partial) {
    __shared__ double red[kRowsPerBlock][WK_D];
    const int h = blockIdx.x, sp = blockIdx.y, b = blockIdx.z;
    const int g = p.G == 1 ? 0 : h;
    const int slot = threadIdx.x / kRowLanes, sub = threadIdx.x % kRowLanes;
    const size_t row_bytes = WK_D * wk::esize(DT);
    const char *base = A + ((size_t)b * p.H + h) * p.a_rows * row_bytes;
    const double *nq = nsq + ((size_t)b * p.G + g) * p.T;
    const int per = (p.T + kMeanSplits - 1) / kMeanSplits;
    const int i_end = min(p.T, (sp + 1) * per);
    double acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int i = sp * per + slot; i < i_end; i += kRowsPerBlock) {
        float v[8];
        load_row8<DT>(base + (size_t)i * row_bytes, sub, v);
        const double n2 = nq[i];
        const double rn = n2 < 1e-60 ? 0.0 : 1.0 / sqrt(n2);  // zero-norm key: its cosines are 0
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += (double)v[e] * rn;
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) red[slot][sub * 8 + e] = acc[e];
    __syncthreads();
    if (threadIdx.x < WK_D) {
        double s = 0.0;
#pragma unroll
        for (int r = 0; r < kRowsPerBlock; ++r) s += red[r][threadIdx.x];
        partial[(((size_t)b * p.H + h) * kMeanSplits + sp) * WK_D + threadIdx.x] = s;
    }
}

__global__ __launch_bounds__(WK_D) void k_anchor_mean_finish(const double *__restrict__ partial, CompressDims p,
                                                            float *__restrict__ m) {
    const size_t bh = (size_t)blockIdx.y * p.H + blockIdx.x;
    double s = 0.0;
#pragma unroll
    for (int sp = 0; sp < kMeanSplits; ++sp) s += partial[(bh * kMeanSplits + sp) * WK_D + threadIdx.x];
    m[bh * WK_D + threadIdx.x] = (float)(s / (double)p.T);
}

// Anchor norms and the normalised anchor mean in ONE pass over the anchor rows, for head-shared lists (a token's
// norm runs over all heads, so a wave takes whole tokens): each of the workgroup's four waves walks
// tok_per_wave anchor tokens; per token it requests the token's rows of all heads at once (head h goes to
// 16-lane group h & 3, IT >= ceil(H / 4) rows per group), sums their squares across the wave in fp64 and adds
// row / |k_i| to per-lane fp32 sums (at most 32 terms of magnitude <= 1: the rounding stays below 1e-10 of the
// scores).  The four waves' sums meet through LDS in a fixed order, and one workgroup writes one partial sum per
// (head, feature); k_anchor_mean_fold adds the partials in fp64.  The separate norm pass and its buffer are gone.
constexpr int kFuseWaves = 4;

template <int DT, int IT>
__global__ __launch_bounds__(kFuseWaves * 64) void k_anchor_norm_mean(const char *__restrict__ A, CompressDims p,
                                                                      int tok_per_wave, int n_splits,
                                                                      float *__restrict__ partial) {
    extern __shared__ __attribute__((aligned(16))) float fuse_red[];   // [kFuseWaves][H][128]
    const int split = blockIdx.x, b = blockIdx.z;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int q = lane >> 4, sub = lane & 15;
    const size_t row_bytes = WK_D * wk::esize(DT);
    const size_t head_bytes = (size_t)p.a_rows * row_bytes;
    const char *base = A + (size_t)b * p.H * head_bytes;
    float acc[IT][8];
#pragma unroll
    for (int it = 0; it < IT; ++it)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[it][e] = 0.f;
    const int i0 = (split * kFuseWaves + wave) * tok_per_wave;
    const int i1 = min(p.T, i0 + tok_per_wave);
    // rows stay as loaded (16 bytes per lane and row, bf16; 32 bytes, fp32) until they are used, and the next
    // token's rows are requested before the current token's are reduced
    constexpr int kVec = DT == WK_BF16 ? 1 : 2;
    uint4 cur[IT][kVec], nxt[IT][kVec];
    auto request = [&](int i, uint4 (&dst)[IT][kVec]) __attribute__((always_inline)) {
#pragma unroll
        for (int it = 0; it < IT; ++it) {
            const int h = 4 * it + q;
            const uint4 *row = reinterpret_cast<const uint4 *>(base + (size_t)(h < p.H ? h : 0) * head_bytes + (size_t)i * row_bytes);
#pragma unroll
            for (int u = 0; u < kVec; ++u) dst[it][u] = h < p.H ? row[kVec * sub + u] : uint4{0, 0, 0, 0};
        }
    };
    auto unpack = [&](const uint4 (&src)[kVec], float (&v)[8]) __attribute__((always_inline)) {
        if constexpr (DT == WK_BF16) {
            const uint32_t w[4] = {src[0].x, src[0].y, src[0].z, src[0].w};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                v[2 * k] = __uint_as_float(w[k] << 16);
                v[2 * k + 1] = __uint_as_float(w[k] & 0xffff0000u);
            }
        } else {
            const uint32_t w[8] = {src[0].x, src[0].y, src[0].z, src[0].w, src[kVec - 1].x, src[kVec - 1].y, src[kVec - 1].z, src[kVec - 1].w};
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] = __uint_as_float(w[k]);
        }
    };
    if (i0 < i1) request(i0, cur);
    for (int i = i0; i < i1; ++i) {
        if (i + 1 < i1) request(i + 1, nxt);
        double n2 = 0.0;
#pragma unroll
        for (int it = 0; it < IT; ++it) {
            float v[8];
            unpack(cur[it], v);
            float sq = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) sq = fmaf(v[e], v[e], sq);
            n2 += (double)sq;
        }
        n2 = wk::row_group_sum(n2);
        n2 += __shfl_xor(n2, 16);
        n2 += __shfl_xor(n2, 32);
        const float rn = n2 < 1e-60 ? 0.f : (float)(1.0 / sqrt(n2));   // zero-norm key: its cosines are 0
#pragma unroll
        for (int it = 0; it < IT; ++it) {
            float v[8];
            unpack(cur[it], v);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[it][e] = fmaf(v[e], rn, acc[it][e]);
        }
#pragma unroll
        for (int it = 0; it < IT; ++it)
#pragma unroll
            for (int u = 0; u < kVec; ++u) cur[it][u] = nxt[it][u];
    }
#pragma unroll
    for (int it = 0; it < IT; ++it) {
        const int h = 4 * it + q;
        if (h < p.H) {
            float *dst = fuse_red + ((size_t)wave * p.H + h) * WK_D + 8 * sub;
            *reinterpret_cast<float4 *>(dst) = float4{acc[it][0], acc[it][1], acc[it][2], acc[it][3]};
            *reinterpret_cast<float4 *>(dst + 4) = float4{acc[it][4], acc[it][5], acc[it][6], acc[it][7]};
        }
    }
    __syncthreads();
    const int n = p.H * WK_D;
    for (int idx = threadIdx.x; idx < n; idx += kFuseWaves * 64) {
        double t = 0.0;
#pragma unroll
        for (int w = 0; w < kFuseWaves; ++w) t += (double)fuse_red[(size_t)w * n + idx];
        const int h = idx / WK_D, c = idx % WK_D;
        partial[(((size_t)b * p.H + h) * n_splits + split) * WK_D + c] = (float)t;
    }
}

// m[(b*H+h)*128 + c] = (1/T) sum over the n_splits partial sums of k_anchor_norm_mean, in fp64 and in a fixed order
__global__ __launch_bounds__(WK_D) void k_anchor_mean_fold(const float *__restrict__ partial, CompressDims p, int n_splits,
                                                          float *__restrict__ m) {
    const size_t bh = (size_t)blockIdx.y * p.H + blockIdx.x;
    const float *src = partial + bh * n_splits * WK_D + threadIdx.x;
    double s = 0.0;
    int sp = 0;
    for (; sp + 8 <= n_splits; sp += 8) {
        float t[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) t[u] = src[(size_t)(sp + u) * WK_D];
#pragma unroll
        for (int u = 0; u < 8; ++u) s += (double)t[u];
    }
    for (; sp < n_splits; ++sp) s += (double)src[(size_t)sp * WK_D];
    m[bh * WK_D + threadIdx.x] = (float)(s / (double)p.T);
}

// scores[(b*G+g)*n_cand + j] = (k_j . m) / |k_j|
template <int DT, int HS>
__global__ __launch_bounds__(256) void k_score_factored(const char *__restrict__ K, CompressDims p,
                                                        const float *__restrict__ m,
                                                        double *__restrict__ scores) {
    const int j = blockIdx.x * (kRowsPerBlock / HS) + threadIdx.x / (kRowLanes * HS);
    const int hq = (threadIdx.x / kRowLanes) % HS;
    const int sub = threadIdx.x % kRowLanes;
    const int g = blockIdx.y, b = blockIdx.z;
    if (j >= p.n_cand) return;
    const size_t row_bytes = WK_D * wk::esize(DT);
    const size_t head_bytes = (size_t)p.n_tok * row_bytes;
    const char *base = K + ((size_t)b * p.H * p.n_tok + p.first_cand + j) * row_bytes;
    const float *mb = m + (size_t)b * p.H * WK_D + 8 * sub;
    double dacc = 0.0, nacc = 0.0;
    for (int hh0 = hq; hh0 < p.hg; hh0 += HS * kHeadBatch) {
        float v[kHeadBatch][8];
#pragma unroll
        for (int u = 0; u < kHeadBatch; ++u) {
            const int hh = hh0 + u * HS;
            if (hh < p.hg) {
                load_row8<DT>(base + (size_t)(p.G == 1 ? hh : g) * head_bytes, sub, v[u]);
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) v[u][e] = 0.f;
            }
        }
#pragma unroll
        for (int u = 0; u < kHeadBatch; ++u) {
            const int hh = hh0 + u * HS;
            if (hh < p.hg) {
                const float4 *mp = reinterpret_cast<const float4 *>(mb + (size_t)(p.G == 1 ? hh : g) * WK_D);
                const float4 m0 = mp[0], m1 = mp[1];
                const float mm[8] = {m0.x, m0.y, m0.z, m0.w, m1.x, m1.y, m1.z, m1.w};
                float dp = 0.f, ns = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    dp = fmaf(v[u][e], mm[e], dp);
                    ns = fmaf(v[u][e], v[u][e], ns);
                }
                dacc += (double)dp;
                nacc += (double)ns;
            }
        }
    }
    dacc = head_split_sum<HS>(dacc);
    nacc = head_split_sum<HS>(nacc);
    if (sub == 0 && hq == 0) {
        double s = nacc < 1e-60 ? 0.0 : dacc / sqrt(nacc);
        scores[((size_t)b * p.G + g) * p.n_cand + j] = s + 0.0;  // -0.0 -> +0.0
    }
}

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
// ---- Eq. 5 as the similarity GEMM on the matrix cores (WK_SCORE_GEMM) ------------------------
//
// C[i][j] = sum over the group's heads and the 128 features of (anchor key i) . (candidate key j),
// then partial[j] = sum_i C[i][j] / |k_i|.  A workgroup of 8 waves owns a 256 (anchors) x 256
// (candidates) block of C: wave (wa, wc) holds 128 x 64 of it in eight 32x32 accumulators, so a
// 16-feature step costs 4 + 2 operand reads from LDS for 8 MFMAs.  The contraction runs over
// heads x 128 features in steps of 64 features; both operand tiles of a step (256 rows x 128 bytes
// each) go from global memory straight into one of two LDS stages (global_load_lds), the next step's
// loads being in flight while the current one is multiplied.  Rows are 128 bytes, their eight
// 16-byte chunks stored at chunk ^ ((row >> 1) & 7), which makes the 16 lanes of an operand read
// hit 16 different bank groups.  The block of C never leaves registers: it is folded with the
// column weights 1/|k_i| and summed over the anchors in the epilogue.
constexpr int kGemmTile = 256;        // anchors and candidates per workgroup block
constexpr int kGemmMaxSplits = 32;    // partial sums per candidate: (anchor blocks) x (head ranges), one workgroup each
constexpr int kGemmStage = 2 * kGemmTile * 128;   // bytes: anchor tile + candidate tile of one 64-feature step
constexpr int kGemmLds = 2 * kGemmStage + kGemmTile * 4 + 2 * kGemmTile * 4;

#define WK_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))
#define WK_GLB_PTR(p) ((const __attribute__((address_space(1))) void *)(p))

// partial[((b*G+g)*splits + sp)*n_cand + j], splits = asplits*hsplits, sp = sh*asplits + sa: the sum over the
// anchors of blocks sa, sa+asplits, ... and over the heads of range sh of (k_j . k_i)_heads / |k_i|.  (The sum
// over heads commutes with the weighting, so head ranges are just more partial sums for the finish kernel;
// they fill the chip when one chunk alone gives too few blocks.)
__global__ __launch_bounds__(512, 2) void k_score_gemm(const char *__restrict__ K, const char *__restrict__ A,
                                                       CompressDims p, const double *__restrict__ nsq_a,
                                                       int asplits, int hsplits, float *__restrict__ partial) {
    extern __shared__ __attribute__((aligned(256))) char smem[];
    float *w_lds = reinterpret_cast<float *>(smem + 2 * kGemmStage);   // [256] column weights of the anchor block
    float *red = w_lds + kGemmTile;                                    // [2][256] partial sums of the two anchor halves
    const int splits = asplits * hsplits;
    const int g = blockIdx.y / splits, sp = blockIdx.y % splits, b = blockIdx.z;
    const int sa = sp % asplits, sh = sp / asplits;
    const int j0 = blockIdx.x * kGemmTile;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, gh = lane >> 5;
    const int wa = wave & 1, wc = wave >> 1;
    const double *na = nsq_a + ((size_t)b * p.G + g) * p.T;
    const int n_ablocks = (p.T + kGemmTile - 1) / kGemmTile;
    const int h_per = (p.hg + hsplits - 1) / hsplits;
    const int h_lo = sh * h_per, h_hi = min(p.hg, h_lo + h_per);
    const int n_steps = max(h_hi - h_lo, 0) * 2;   // 64-feature steps of the contraction

    // operand reads: chunk 2*st + gh of row (128*wa + 32*mb + col) resp. (64*wc + 32*nb + col)
    const char *a_rd[4], *b_rd[4];
#pragma unroll
    for (int st = 0; st < 4; ++st) {
        const int slot = ((2 * st + gh) ^ ((col >> 1) & 7)) << 4;
        a_rd[st] = smem + (128 * wa + col) * 128 + slot;
        b_rd[st] = smem + kGemmTile * 128 + (64 * wc + col) * 128 + slot;
    }
    // tile loads: thread t fills 16-byte slot (t & 7) of rows 64*i + (t >> 3), i = 0..3, of both tiles
    const int ld_row = tid >> 3;
    const unsigned ld_chunk = (unsigned)(((tid & 7) ^ ((tid >> 4) & 7)) << 4);
    unsigned cand_off[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)   // rows past the last candidate are clamped; their sums are never written
        cand_off[i] = (unsigned)(p.first_cand + min(j0 + 64 * i + ld_row, p.n_cand - 1)) * 256u + ld_chunk;
    char *const dma_dst = smem + wave * 1024;

    float psum[2] = {0.f, 0.f};
    for (int ab = sa; ab < n_ablocks; ab += asplits) {
        unsigned anc_off[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)   // anchors past T are clamped and get weight 0
            anc_off[i] = (unsigned)min(ab * kGemmTile + 64 * i + ld_row, p.T - 1) * 256u + ld_chunk;
        auto issue = [&](int step, int stage) {
            const int hh = h_lo + (step >> 1);
            const int h = p.G == 1 ? hh : g;
            const char *Ah = A + ((size_t)b * p.H + h) * p.a_rows * 256 + (step & 1) * 128;
            const char *Kh = K + ((size_t)b * p.H + h) * p.n_tok * 256 + (step & 1) * 128;
            char *dst = dma_dst + stage * kGemmStage;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                __builtin_amdgcn_global_load_lds(WK_GLB_PTR(Ah + anc_off[i]), WK_LDS_PTR(dst + i * 8192), 16, 0, 0);
                __builtin_amdgcn_global_load_lds(WK_GLB_PTR(Kh + cand_off[i]), WK_LDS_PTR(dst + kGemmTile * 128 + i * 8192),
                                                 16, 0, 0);
            }
        };
        __syncthreads();   // the previous block's weights and stages are no longer read
        if (tid < kGemmTile) {
            const int i = ab * kGemmTile + tid;
            float rn = 0.f;   // anchors past T (clamped duplicates) and zero-norm anchors contribute nothing
            if (i < p.T) {
                const double n2 = na[i];
                rn = n2 < 1e-60 ? 0.f : (float)(1.0 / sqrt(n2));
            }
            w_lds[tid] = rn;
        }
        f32x16 acc[4][2];
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[mb][nb][r] = 0.f;
        // 32-row groups of this wave's 128 anchors that hold at least one anchor below T: all 4 except in
        // the last anchor block, where the groups of pure padding are skipped (their weights are 0 anyway)
        const int rows_left = p.T - (ab * kGemmTile + 128 * wa);
        const int mb_valid = rows_left >= 128 ? 4 : (rows_left <= 0 ? 0 : (rows_left + 31) / 32);
        // likewise the wave's two 32-candidate blocks: past the last candidate (last candidate tile) nothing
        // is multiplied
        const int cols_left = p.n_cand - (j0 + 64 * wc);
        const int nb_valid = cols_left >= 64 ? 2 : (cols_left <= 0 ? 0 : (cols_left + 31) / 32);
        auto contract = [&](auto mv_tag, auto nv_tag) {
            constexpr int MV = decltype(mv_tag)::value, NV = decltype(nv_tag)::value;
            for (int step = 0; step < n_steps; ++step) {
                __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's part of the step's tiles has landed
                __syncthreads();                      // everyone's has, and the other stage is free again
                if (step + 1 < n_steps) issue(step + 1, (step + 1) & 1);
                const int off = (step & 1) * kGemmStage;
                if constexpr (MV > 0) {
#pragma unroll
                    for (int st = 0; st < 4; ++st) {
                        bf16x8 fa[MV], fb[NV];
#pragma unroll
                        for (int mb = 0; mb < MV; ++mb)
                            fa[mb] = *reinterpret_cast<const bf16x8 *>(a_rd[st] + off + mb * 4096);
#pragma unroll
                        for (int nb = 0; nb < NV; ++nb)
                            fb[nb] = *reinterpret_cast<const bf16x8 *>(b_rd[st] + off + nb * 4096);
#pragma unroll
                        for (int mb = 0; mb < MV; ++mb)
#pragma unroll
                            for (int nb = 0; nb < NV; ++nb)
                                acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[mb], fb[nb], acc[mb][nb], 0, 0, 0);
                    }
                }
            }
        };
        if (n_steps > 0) issue(0, 0);
        using I0 = std::integral_constant<int, 0>;
        using I1 = std::integral_constant<int, 1>;
        using I2 = std::integral_constant<int, 2>;
        using I3 = std::integral_constant<int, 3>;
        using I4 = std::integral_constant<int, 4>;
        switch (nb_valid == 0 ? 0 : 2 * mb_valid + nb_valid - 1) {   // wave-uniform; every variant passes the same barriers
        case 9: contract(I4{}, I2{}); break;
        case 8: contract(I4{}, I1{}); break;
        case 7: contract(I3{}, I2{}); break;
        case 6: contract(I3{}, I1{}); break;
        case 5: contract(I2{}, I2{}); break;
        case 4: contract(I2{}, I1{}); break;
        case 3: contract(I1{}, I2{}); break;
        case 2: contract(I1{}, I1{}); break;
        default: contract(I0{}, I0{}); break;
        }
        // fold the block in: accumulator register r of block mb is anchor 128*wa + 32*mb + 8*(r/4) + 4*gh + r%4
        // (an empty head range has passed no barrier since the weights were written, and has nothing to add)
        if (n_steps > 0)
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float w = w_lds[128 * wa + 32 * mb + 8 * (r >> 2) + 4 * gh + (r & 3)];
                psum[0] = fmaf(acc[mb][0][r], w, psum[0]);
                psum[1] = fmaf(acc[mb][1][r], w, psum[1]);
            }
    }
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
        const float v = psum[nb] + __shfl_xor(psum[nb], 32);
        if (gh == 0) red[wa * kGemmTile + 64 * wc + 32 * nb + col] = v;
    }
    __syncthreads();
    if (tid < kGemmTile && j0 + tid < p.n_cand)
        partial[(((size_t)b * p.G + g) * splits + sp) * p.n_cand + j0 + tid] = red[tid] + red[kGemmTile + tid];
}

// scores[(b*G+g)*n_cand + j] = (sum of the splits' partial sums) / (|k_j| T)
__global__ __launch_bounds__(256) void k_score_gemm_finish(const float *__restrict__ partial, CompressDims p,
                                                           int splits, const double *__restrict__ nsq_c,
                                                           double *__restrict__ scores) {
    const int j = blockIdx.x * 256 + threadIdx.x;
    const size_t list = blockIdx.y;
    if (j >= p.n_cand) return;
    double tot = 0.0;
    for (int sp = 0; sp < splits; ++sp) tot += (double)partial[(list * splits + sp) * p.n_cand + j];
    const double n2 = nsq_c[list * p.n_cand + j];
    const double s = n2 < 1e-60 ? 0.0 : tot / (sqrt(n2) * (double)p.T);
    scores[list * p.n_cand + j] = s + 0.0;
}

// ---- selection: n_keep lowest scores of one list, ties to the lower index -------------------

__device__ inline uint64_t order_key(double s) {
    const uint64_t u = (uint64_t)__double_as_longlong(s);
    return (u >> 63) ? ~u : (u | 0x8000000000000000ull);  // unsigned order == numeric order
}

constexpr int kSelThreads = 1024;

// exclusive scan of one int per thread over the block; total = sum over the block
__device__ inline int block_excl_scan(int v, int *wsum /*[kSelThreads/64]*/, int &total) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int x = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int y = __shfl_up(x, o);
        if (lane >= o) x += y;
    }
    __syncthreads();  // wsum may still be read from the previous scan
    if (lane == 63) wsum[w] = x;
    __syncthreads();
    int off = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < kSelThreads / 64; ++i) {
        const int t = wsum[i];
        if (i < w) off += t;
        tot += t;
    }
    total = tot;
    return off + x - v;
}

// One block per list.  Radix-select (up to 8 passes of 8 bits, from the top, over order-preserving
// 64-bit keys) finds the n_keep-th smallest score tau; then tokens with score < tau, plus the first
// few (by index) with score == tau, are written in ascending index order via block scans.  The passes
// stop as soon as every key that shares tau's leading digits is kept anyway (for fp64 scores usually
// after three or four digits); comparisons then look at those leading digits only.  Lists of up to
// kSelLds keys are held in LDS for all passes; longer lists are re-read from global memory.
constexpr int kSelLds = 6144;   // 48 KB of keys

__global__ __launch_bounds__(kSelThreads) void k_select(const double *__restrict__ scores,
                                                        CompressDims p, int32_t *__restrict__ kept_idx) {
    __shared__ uint64_t keys[kSelLds];
    __shared__ unsigned hist[256];
    __shared__ uint64_t s_prefix;
    __shared__ int s_k, s_cnt;
    __shared__ int wsum[kSelThreads / 64];
    const int list = blockIdx.x;  // b*G + g
    const double *s = scores + (size_t)list * p.n_cand;
    int32_t *out = kept_idx + (size_t)list * p.n_out;
    const int n = p.n_cand, tid = threadIdx.x;
    const bool in_lds = n <= kSelLds;

    for (int i = tid; i < p.first_cand; i += kSelThreads) out[i] = i;  // anchor tokens, kept in full
    if (p.n_keep == 0) return;
    if (in_lds) {
        for (int j = tid; j < n; j += kSelThreads) keys[j] = order_key(s[j]);
        __syncthreads();
    }
    auto key_at = [&](int j) { return in_lds ? keys[j] : order_key(s[j]); };

    uint64_t prefix = 0;
    int k = p.n_keep;  // rank (1-based) still to locate among keys matching the prefix
    int low = 0;       // digits below this bit were not needed to separate kept from dropped
    if (p.n_keep < n) {
        for (int pass = 7; pass >= 0; --pass) {
            const int shift = pass * 8;
            const uint64_t himask = pass == 7 ? 0ull : (~0ull << (shift + 8));
            if (tid < 256) hist[tid] = 0;
            __syncthreads();
            for (int j = tid; j < n; j += kSelThreads) {
                const uint64_t key = key_at(j);
                if ((key & himask) == prefix) atomicAdd(&hist[(key >> shift) & 255], 1u);
            }
            __syncthreads();
            // bucket holding rank k: inclusive prefix sums of the 256 counts (4 waves), first one >= k
            int incl = 0, cnt = 0;
            if (tid < 256) {
                cnt = (int)hist[tid];
                incl = cnt;
#pragma unroll
                for (int o = 1; o < 64; o <<= 1) {
                    const int y = __shfl_up(incl, o);
                    if ((tid & 63) >= o) incl += y;
                }
                if ((tid & 63) == 63) wsum[tid >> 6] = incl;
            }
            __syncthreads();
            if (tid < 256) {
                for (int w = 0; w < (tid >> 6); ++w) incl += wsum[w];
                if (incl >= k && incl - cnt < k) {   // exactly one bucket satisfies this
                    s_k = k - (incl - cnt);
                    s_cnt = cnt;
                    s_prefix = prefix | ((uint64_t)tid << shift);
                }
            }
            __syncthreads();
            k = s_k;
            prefix = s_prefix;
            if (s_cnt == k) {   // the whole bucket is kept: nothing below this digit matters
                low = shift;
                break;
            }
        }
    } else {
        prefix = ~0ull;  // keep everything: every key is below (or equal to) the largest key
        k = n;
    }
    // prefix = tau (its digits from bit `low` up), k = how many of the keys equal to it there are kept
    // (lowest indices first)
    int eq_base = 0, out_base = 0;
    for (int j0 = 0; j0 < n; j0 += kSelThreads) {
        const int j = j0 + tid;
        bool less = false, eq = false;
        if (j < n) {
            const uint64_t key = key_at(j);
            less = (key >> low) < (prefix >> low);
            eq = (key >> low) == (prefix >> low);
        }
        int eq_tot, keep_tot;
        const int eq_rank = eq_base + block_excl_scan(eq ? 1 : 0, wsum, eq_tot);
        const bool keep = less || (eq && eq_rank < k);
        const int pos = out_base + block_excl_scan(keep ? 1 : 0, wsum, keep_tot);
        if (keep && pos < p.n_keep) out[p.first_cand + pos] = p.first_cand + j;
        eq_base += eq_tot;
        out_base += keep_tot;
    }
}

// K_out/V_out[b][h][r] = K/V[b][h][kept_idx[b][g(h)][r]], rows copied verbatim
template <int DT>
__global__ __launch_bounds__(256) void k_compact(const char *__restrict__ K, const char *__restrict__ V,
                                                 CompressDims p, const int32_t *__restrict__ kept_idx,
                                                 char *__restrict__ K_out, char *__restrict__ V_out) {
    const int r = blockIdx.x * kRowsPerBlock + threadIdx.x / kRowLanes;
    const int sub = threadIdx.x % kRowLanes;
    const int h = blockIdx.y, b = blockIdx.z;
    if (r >= p.n_out) return;
    const int g = p.G == 1 ? 0 : h;
    int src = kept_idx[((size_t)b * p.G + g) * p.n_out + r];
    src = src < 0 ? 0 : (src >= p.n_tok ? p.n_tok - 1 : src);  // never read outside the chunk
    constexpr size_t row_bytes = WK_D * (DT == WK_BF16 ? 2 : 4);
    constexpr int vec_per_lane = row_bytes / (kRowLanes * 16);  // 1 (bf16) or 2 (fp32)
    const size_t in_off = (((size_t)b * p.H + h) * p.n_tok + src) * row_bytes;
    const size_t out_off = (((size_t)b * p.H + h) * p.n_out + r) * row_bytes;
#pragma unroll
    for (int t = 0; t < vec_per_lane; ++t) {
        const int c = sub + t * kRowLanes;
        const uint4 kv = reinterpret_cast<const uint4 *>(K + in_off)[c];
        const uint4 vv = reinterpret_cast<const uint4 *>(V + in_off)[c];
        reinterpret_cast<uint4 *>(K_out + out_off)[c] = kv;
        reinterpret_cast<uint4 *>(V_out + out_off)[c] = vv;
    }
}

struct WsLayout {
    size_t scores, nsq, nsq_cand, gemm_partial, mean, mean_partial, kept, total;
};

// The one-pass anchor kernel serves factored scoring with head-shared lists of up to 64 heads in batches large
// enough that a wave walks 8 to 32 tokens (a single LingBot-sized chunk would have to give each wave 4 tokens to
// spread over the chip at all, and that dependent chain is slower than the two separate passes: 65 against 52 us
// for the whole call).
struct FusePlan { bool use; int tok_per_wave, n_splits, it; };

FusePlan fuse_plan(const wk_compress_desc *d, const CompressDims &p) {
    FusePlan f{false, 0, 0, 0};
    if (d->score_algo != WK_SCORE_FACTORED || p.G != 1 || p.H > 64) return f;
    const long long tpw = ((long long)p.T * d->batch + 4095) / 4096;
    if (tpw < 8) return f;   // too few tokens to keep every wave on a long run of them: the two short passes win
    f.use = true;
    f.tok_per_wave = (int)(tpw > 32 ? 32 : tpw);
    f.n_splits = (p.T + kFuseWaves * f.tok_per_wave - 1) / (kFuseWaves * f.tok_per_wave);
    f.it = p.H <= 12 ? 3 : (p.H <= 40 ? 10 : 16);
    return f;
}

bool make_dims(const wk_compress_desc *d, CompressDims &p, WsLayout &ws) {
    if (!d || d->H < 1 || d->T < 1 || d->F < 1 || d->batch < 1) return false;
    int32_t n_out = 0, n_keep = 0;
    if (wk_keep_count(d->rho, d->ratio_kind, d->anchor_mode, d->F, d->T, &n_out, &n_keep) != WK_OK)
        return false;
    const bool ext = d->anchor_mode == WK_ANCHOR_EXTERNAL;
    p.H = d->H;
    p.T = d->T;
    p.n_tok = d->F * d->T;
    p.first_cand = ext ? 0 : d->T;
    p.n_cand = p.n_tok - p.first_cand;
    p.G = d->head_mode == WK_HEADS_INDEPENDENT ? d->H : 1;
    p.hg = d->head_mode == WK_HEADS_INDEPENDENT ? 1 : d->H;
    p.a_rows = ext ? d->T : p.n_tok;
    p.n_keep = n_keep;
    p.n_out = n_out;
    const size_t lists = (size_t)d->batch * p.G;
    size_t off = 0;
    ws.scores = off; off = wk::align_up(off + lists * (size_t)(p.n_cand > 0 ? p.n_cand : 1) * sizeof(double), 256);
    ws.nsq = off;    off = wk::align_up(off + lists * (size_t)p.T * sizeof(double), 256);
    ws.nsq_cand = off;
    ws.gemm_partial = off;
    if (d->score_algo == WK_SCORE_GEMM) {
        const size_t nc = (size_t)(p.n_cand > 0 ? p.n_cand : 1);
        off = wk::align_up(off + lists * nc * sizeof(double), 256);
        ws.gemm_partial = off;
        off = wk::align_up(off + lists * kGemmMaxSplits * nc * sizeof(float), 256);
    }
    ws.mean = off;   off = wk::align_up(off + (size_t)d->batch * d->H * WK_D * sizeof(float), 256);
    ws.mean_partial = off;
    {
        const size_t two_pass = (size_t)d->batch * d->H * kMeanSplits * WK_D * sizeof(double);
        const FusePlan fp = fuse_plan(d, p);
        const size_t fused = fp.use ? (size_t)d->batch * d->H * fp.n_splits * WK_D * sizeof(float) : 0;
        off = wk::align_up(off + (two_pass > fused ? two_pass : fused), 256);
    }
    ws.kept = off;   off = wk::align_up(off + lists * (size_t)n_out * sizeof(int32_t), 256);
    ws.total = off;
    return true;
}

wk_status check_desc(const wk_compress_desc *d) {
    if (!d) return WK_ERR_INVALID_ARG;
    if (d->H < 1 || d->T < 1 || d->F < 1 || d->batch < 1 || d->d < 1) return WK_ERR_INVALID_ARG;
    if (d->dtype != WK_F32 && d->dtype != WK_BF16) return WK_ERR_INVALID_ARG;
    if (d->head_mode != WK_HEADS_SHARED && d->head_mode != WK_HEADS_INDEPENDENT) return WK_ERR_INVALID_ARG;
    if (d->anchor_mode != WK_ANCHOR_FIRST_FRAME && d->anchor_mode != WK_ANCHOR_EXTERNAL) return WK_ERR_INVALID_ARG;
    if (d->ratio_kind != WK_RATIO_CHUNK && d->ratio_kind != WK_RATIO_NONANCHOR) return WK_ERR_INVALID_ARG;
    if (d->score_algo != WK_SCORE_FACTORED && d->score_algo != WK_SCORE_GEMM) return WK_ERR_INVALID_ARG;
    if (d->d != WK_D) return WK_ERR_UNSUPPORTED;
    if (d->score_algo == WK_SCORE_GEMM && d->dtype != WK_BF16) return WK_ERR_UNSUPPORTED;
    if ((int64_t)d->F * d->T > (1 << 24)) return WK_ERR_UNSUPPORTED;
    return WK_OK;
}

// k_anchor_norm_mean for the plan's rows-per-group count; its LDS (four waves' sums of H x 128 floats) can exceed
// the default 64 KB of dynamic LDS, so the limit is raised once per device and instantiation.
template <int DT, int IT>
wk_status launch_norm_mean_it(const FusePlan &f, const char *A, const CompressDims &p, int batch, float *partial,
                              hipStream_t st) {
    const size_t lds = (size_t)kFuseWaves * p.H * WK_D * sizeof(float);
    static std::atomic<uint64_t> lds_limit_set{0};
    int dev;
    if (wk::device_needs_setup(lds_limit_set, dev)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&k_anchor_norm_mean<DT, IT>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kFuseWaves * 64 * WK_D * (int)sizeof(float)) !=
            hipSuccess)
            return WK_ERR_HIP;
        wk::mark_device(lds_limit_set, dev);
    }
    hipLaunchKernelGGL((k_anchor_norm_mean<DT, IT>), dim3(f.n_splits, 1, batch), dim3(kFuseWaves * 64), lds, st, A, p,
                       f.tok_per_wave, f.n_splits, partial);
    WK_LAUNCH_CHECK();
    return WK_OK;
}

template <int DT>
wk_status launch_norm_mean(const FusePlan &f, const char *A, const CompressDims &p, int batch, float *partial,
                           hipStream_t st) {
    switch (f.it) {
    case 3: return launch_norm_mean_it<DT, 3>(f, A, p, batch, partial, st);
    case 10: return launch_norm_mean_it<DT, 10>(f, A, p, batch, partial, st);
    default: return launch_norm_mean_it<DT, 16>(f, A, p, batch, partial, st);
    }
}

template <int DT>
wk_status launch_all(const wk_compress_desc *d, const CompressDims &p, const WsLayout &ws, const void *K,
                     const void *V, const void *K_anchor, int32_t *kept_idx, void *K_out, void *V_out,
                     char *wsp, hipStream_t st) {
    double *scores = reinterpret_cast<double *>(wsp + ws.scores);
    double *nsq = reinterpret_cast<double *>(wsp + ws.nsq);
    float *mean = reinterpret_cast<float *>(wsp + ws.mean);
    int32_t *kept = kept_idx ? kept_idx : reinterpret_cast<int32_t *>(wsp + ws.kept);
    const char *A = reinterpret_cast<const char *>(d->anchor_mode == WK_ANCHOR_EXTERNAL ? K_anchor : K);
    const char *Kc = reinterpret_cast<const char *>(K);
    if (p.n_cand > 0) {  // scores are always produced: callers may read them from the workspace
        // a token's vector spans hg heads: with four or more, a wave per token (heads dealt to its four
        // 16-lane groups), otherwise 16 lanes per token
        const bool split = p.hg >= 4;
        const int rows_pb = split ? kRowsPerBlock / 4 : kRowsPerBlock;
        const FusePlan fuse = fuse_plan(d, p);
        if (!fuse.use) {   // squared norms of the anchor tokens, a pass of their own
            dim3 g1((p.T + rows_pb - 1) / rows_pb, p.G, d->batch);
            if (split) hipLaunchKernelGGL((k_rows_normsq<DT, 4>), g1, dim3(256), 0, st, A, p, p.a_rows, 0, p.T, nsq);
            else hipLaunchKernelGGL((k_rows_normsq<DT, 1>), g1, dim3(256), 0, st, A, p, p.a_rows, 0, p.T, nsq);
            WK_LAUNCH_CHECK();
        }
        if (d->score_algo == WK_SCORE_GEMM) {
            if constexpr (DT == WK_BF16) {
                double *nsq_cand = reinterpret_cast<double *>(wsp + ws.nsq_cand);
                dim3 g2((p.n_cand + rows_pb - 1) / rows_pb, p.G, d->batch);
                if (split)
                    hipLaunchKernelGGL((k_rows_normsq<DT, 4>), g2, dim3(256), 0, st, Kc, p, p.n_tok, p.first_cand,
                                       p.n_cand, nsq_cand);
                else
                    hipLaunchKernelGGL((k_rows_normsq<DT, 1>), g2, dim3(256), 0, st, Kc, p, p.n_tok, p.first_cand,
                                       p.n_cand, nsq_cand);
                WK_LAUNCH_CHECK();
                // one workgroup per (candidate block, anchor block); beyond 8 anchor blocks a workgroup
                // walks several
                const int cand_tiles = (p.n_cand + kGemmTile - 1) / kGemmTile;
                const int n_ablocks = (p.T + kGemmTile - 1) / kGemmTile;
                const int asplits = n_ablocks < 8 ? n_ablocks : 8;
                // head ranges: as many as keep the grid within one round of 256 workgroups
                const long long blocks = (long long)cand_tiles * p.G * asplits * d->batch;
                int hsplits = (int)(256 / (blocks > 0 ? blocks : 1));
                hsplits = hsplits < 1 ? 1 : hsplits;
                hsplits = hsplits > p.hg ? p.hg : hsplits;
                hsplits = hsplits > kGemmMaxSplits / asplits ? kGemmMaxSplits / asplits : hsplits;
                const int splits = asplits * hsplits;
                float *partial = reinterpret_cast<float *>(wsp + ws.gemm_partial);
                static std::atomic<uint64_t> lds_limit_set{0};   // more than the default 64 KB of dynamic LDS
                int dev;
                if (wk::device_needs_setup(lds_limit_set, dev)) {
                    if (hipFuncSetAttribute(reinterpret_cast<const void *>(&k_score_gemm),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, kGemmLds) != hipSuccess)
                        return WK_ERR_HIP;
                    wk::mark_device(lds_limit_set, dev);
                }
                hipLaunchKernelGGL(k_score_gemm, dim3(cand_tiles, p.G * splits, d->batch), dim3(512), kGemmLds, st, Kc,
                                   A, p, nsq, asplits, hsplits, partial);
                WK_LAUNCH_CHECK();
                hipLaunchKernelGGL(k_score_gemm_finish, dim3((p.n_cand + 255) / 256, d->batch * p.G), dim3(256), 0, st,
                                   partial, p, splits, nsq_cand, scores);
                WK_LAUNCH_CHECK();
            } else {
                return WK_ERR_UNSUPPORTED;
            }
        } else {
            if (fuse.use) {
                float *fpartial = reinterpret_cast<float *>(wsp + ws.mean_partial);
                const wk_status rc = launch_norm_mean<DT>(fuse, A, p, d->batch, fpartial, st);
                if (rc != WK_OK) return rc;
                hipLaunchKernelGGL(k_anchor_mean_fold, dim3(p.H, d->batch), dim3(WK_D), 0, st, fpartial, p, fuse.n_splits,
                                   mean);
                WK_LAUNCH_CHECK();
            } else {
                double *mean_partial = reinterpret_cast<double *>(wsp + ws.mean_partial);
                hipLaunchKernelGGL(k_anchor_mean_partial<DT>, dim3(p.H, kMeanSplits, d->batch), dim3(256), 0, st, A, p,
                                   nsq, mean_partial);
                WK_LAUNCH_CHECK();
                hipLaunchKernelGGL(k_anchor_mean_finish, dim3(p.H, d->batch), dim3(WK_D), 0, st, mean_partial, p, mean);
                WK_LAUNCH_CHECK();
            }
            dim3 g3((p.n_cand + rows_pb - 1) / rows_pb, p.G, d->batch);
            if (split) hipLaunchKernelGGL((k_score_factored<DT, 4>), g3, dim3(256), 0, st, Kc, p, mean, scores);
            else hipLaunchKernelGGL((k_score_factored<DT, 1>), g3, dim3(256), 0, st, Kc, p, mean, scores);
            WK_LAUNCH_CHECK();
        }
    }
    hipLaunchKernelGGL(k_select, dim3(d->batch * p.G), dim3(kSelThreads), 0, st, scores, p, kept);
    WK_LAUNCH_CHECK();
    dim3 g5((p.n_out + kRowsPerBlock - 1) / kRowsPerBlock, p.H, d->batch);
    hipLaunchKernelGGL(k_compact<DT>, g5, dim3(256), 0, st, Kc, reinterpret_cast<const char *>(V), p, kept,
                       reinterpret_cast<char *>(K_out), reinterpret_cast<char *>(V_out));
    WK_LAUNCH_CHECK();
    return WK_OK;
}

}  // namespace

extern "C" wk_status wk_keep_count(float rho, int32_t ratio_kind, int32_t anchor_mode, int32_t F, int32_t T,
                                   int32_t *n_out, int32_t *n_keep) {
    if (F < 1 || T < 1) return WK_ERR_INVALID_ARG;
    if (ratio_kind != WK_RATIO_CHUNK && ratio_kind != WK_RATIO_NONANCHOR) return WK_ERR_INVALID_ARG;
    if (anchor_mode != WK_ANCHOR_FIRST_FRAME && anchor_mode != WK_ANCHOR_EXTERNAL) return WK_ERR_INVALID_ARG;
    if (!(rho >= 0.f) || !(rho <= 1.f)) return WK_ERR_RATIO;
    const int64_t n_anchor = anchor_mode == WK_ANCHOR_EXTERNAL ? 0 : T;
    const int64_t n_tok = (int64_t)F * T, n_cand = n_tok - n_anchor;
    // half away from zero, in double (a float rho is exactly representable in double)
    auto round_half_away = [](double x) { return (int64_t)llround(x); };
    int64_t keep, out;
    if (ratio_kind == WK_RATIO_CHUNK) {
        out = round_half_away((double)rho * (double)n_tok);
        keep = out - n_anchor;
    } else {
        keep = round_half_away((double)rho * (double)n_cand);
        out = keep + n_anchor;
    }
    if (keep < 0 || keep > n_cand || out < 1 || out > INT32_MAX) return WK_ERR_RATIO;
    if (n_out) *n_out = (int32_t)out;
    if (n_keep) *n_keep = (int32_t)keep;
    return WK_OK;
}

extern "C" size_t wk_compress_workspace_bytes(const wk_compress_desc *desc) {
    CompressDims p;
    WsLayout ws;
    if (check_desc(desc) != WK_OK || !make_dims(desc, p, ws)) return 0;
    return ws.total;
}

extern "C" wk_status wk_compress_chunk(const wk_compress_desc *desc, const void *K, const void *V,
                                       const void *K_anchor, int32_t *kept_idx, void *K_out, void *V_out,
                                       int32_t *n_out, void *workspace, size_t workspace_bytes,
                                       void *hip_stream) {
    wk_status st = check_desc(desc);
    if (st != WK_OK) return st;
    if (!K || !V || !K_out || !V_out) return WK_ERR_INVALID_ARG;
    const bool ext = desc->anchor_mode == WK_ANCHOR_EXTERNAL;
    if (ext != (K_anchor != nullptr)) return WK_ERR_INVALID_ARG;
    int32_t no = 0, nk = 0;
    st = wk_keep_count(desc->rho, desc->ratio_kind, desc->anchor_mode, desc->F, desc->T, &no, &nk);
    if (st != WK_OK) return st;
    CompressDims p;
    WsLayout ws;
    if (!make_dims(desc, p, ws)) return WK_ERR_INVALID_ARG;
    if (!workspace || workspace_bytes < ws.total) return WK_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0) return WK_ERR_WORKSPACE;
    hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
    char *wsp = reinterpret_cast<char *>(workspace);
    if (desc->dtype == WK_BF16)
        st = launch_all<WK_BF16>(desc, p, ws, K, V, K_anchor, kept_idx, K_out, V_out, wsp, stream);
    else
        st = launch_all<WK_F32>(desc, p, ws, K, V, K_anchor, kept_idx, K_out, V_out, wsp, stream);
    if (st == WK_OK && n_out) *n_out = no;
    return st;
}

// ---- wk_compress_chunk for callers that cannot allocate ----------------------------------------
// The workspace of wk_compress_chunk (scores, squared norms, the anchor mean and its partial sums,
// the index list when the caller wants none) lives in this array instead of a caller's buffer.  Every
// device the library runs on holds its own copy at its own address; in host code the array's name
// is only a handle for hipGetSymbolAddress, never an address a kernel may be given.
static __device__ __align__(256) unsigned char scratch[WK_COMPRESS_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::atomic<void *> scratch_addr[kMaxDevices];   // device address of `scratch`, per device (null: not asked yet)

// The current device's copy of `scratch`; resolved once per device, with that device current.
wk_status scratch_of_current_device(char **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0) return WK_ERR_HIP;
    void *ptr = dev < kMaxDevices ? scratch_addr[dev].load(std::memory_order_acquire) : nullptr;
    if (!ptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return WK_ERR_HIP;
        if (dev < kMaxDevices) scratch_addr[dev].store(ptr, std::memory_order_release);
    }
    *out = reinterpret_cast<char *>(ptr);
    return WK_OK;
}

}  // namespace

extern "C" size_t wk_compress_scratch_bytes(void) { return WK_COMPRESS_SCRATCH_BYTES; }

extern "C" wk_status wk_compress_chunk_noalloc(const wk_compress_desc *desc, const void *K, const void *V,
                                               const void *K_anchor, int32_t *kept_idx, void *K_out,
                                               void *V_out, int32_t *n_out, void *hip_stream) {
    wk_status st = check_desc(desc);
    if (st != WK_OK) return st;
    if (!K || !V || !K_out || !V_out) return WK_ERR_INVALID_ARG;
    const bool ext = desc->anchor_mode == WK_ANCHOR_EXTERNAL;
    if (ext != (K_anchor != nullptr)) return WK_ERR_INVALID_ARG;
    int32_t no = 0, nk = 0;
    st = wk_keep_count(desc->rho, desc->ratio_kind, desc->anchor_mode, desc->F, desc->T, &no, &nk);
    if (st != WK_OK) return st;
    CompressDims p;
    WsLayout ws;
    if (!make_dims(desc, p, ws)) return WK_ERR_INVALID_ARG;
    if (ws.total > WK_COMPRESS_SCRATCH_BYTES) return WK_ERR_WORKSPACE;   // larger than the built-in scratch
    char *wsp = nullptr;
    st = scratch_of_current_device(&wsp);
    if (st != WK_OK) return st;
    // Nothing in the workspace has to start at zero: every kernel of the call writes each element it
    // or a later kernel reads (scores, norms, mean partials, similarity partials, the index list).
    hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
    if (desc->dtype == WK_BF16)
        st = launch_all<WK_BF16>(desc, p, ws, K, V, K_anchor, kept_idx, K_out, V_out, wsp, stream);
    else
        st = launch_all<WK_F32>(desc, p, ws, K, V, K_anchor, kept_idx, K_out, V_out, wsp, stream);
    if (st == WK_OK && n_out) *n_out = no;
    return st;
}
