// Attention of the denoising chunk's queries over the assembled KV window (paper Sec. 4.2,
// Sec. 4.3): O = softmax(Q K^T * scale) V per head, every window key visible.
//
// Both kernels (bf16 and fp32) use the same transposed formulation, chosen for the CDNA
// 32x32 MFMA register layout (lane l of a wave owns column l%32 of the 32x32 result and
// rows 8*(r/4) + 4*(l/32) + r%4 for accumulator register r):
//
//     S^T = K  Q^T     A operand = K rows (from LDS),     B operand = Q^T (registers, loaded once)
//     O^T = V^T P^T    A operand = V^T    (from LDS),     B operand = P^T (registers)
//
// In S^T a lane's column is one query, so the online-softmax row statistics are per-lane scalars:
// the row max needs one exchange between lane l and lane l+32, the row sum none until the end,
// and the rescale factor of O^T is again a per-lane scalar.  The S^T accumulator registers are,
// after exp2 and rounding, exactly the B operand of the second product: which key an MFMA
// "k slot" means is a free choice, as long as the V^T operand uses the same choice.
#include <cmath>
#include <type_traits>

#include "wk_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short i16x8 __attribute__((ext_vector_type(8)));

struct AttnArgs {
    const char *Q;
    const char *K;
    const char *V;
    char *O;
    float *lse;
    int H, N_q, N_kv, kv_row_stride;
    float scale_log2;  // scale * log2(e): softmax is evaluated with exp2
    const int32_t *n_kv_dev;
    int n_qtiles;
    int per_xcd;       // work items per XCD in the launch order
    int splits;        // key-range splits per (head, query tile); 1 = none
    float *part_o;     // splits > 1: [splits][H][N_q][128] unnormalised fp32 partial outputs
    float *part_ml;    //             [splits][H][N_q][2] running max (log2 units) and row sum
    // batch over stored chunks (log-sum-exp only): chunk c has keys k_table[c] = [H][n_tok[c]][128]
    // and writes lse + c*H*N_q.  n_chunks = 0: one window, K above.
    const void *const *k_table;
    const int32_t *n_tok;
    int n_chunks;
    // a launch may cover queries [q_off, q_off + N_q) of arrays that hold q_rows rows per head
    // (Q, O, lse and the partial results), and a key range that starts kv_start rows into the
    // window (only used to convert *n_kv_dev); part_slot >= 0 makes it write its (O, max, sum)
    // as split `part_slot` for k_attn_merge instead of a final result.
    int q_rows, q_off, kv_start, part_slot;
    // attention in place over the store (k_attn_bf16<.., IN_PLACE>): the window is K/V above (N_kv native
    // rows, may be 0) followed by the stored chunks ids[0 .. min(*n_ids, R_max)), read where they are
    // stored: chunk c has keys k_table[c] and values v_table[c], both [H][n_tok[c]][128].
    const void *const *v_table;
    const int32_t *ids;
    const int32_t *n_ids;
    int R_max, store_M;
    // host-known upper bound of n_tok[] (store descriptors): a chunk that claims more rows is treated as
    // absent, so no length the host has not seen can reach the 32-bit byte offsets of the tile loads
    int max_tok;
};

// bf16 tile loads form 32-bit byte offsets of rows (256 B each), up to four tiles past the last one
constexpr int kMaxRowsBf16 = (1 << 24) - 512;

constexpr int kXcds = 8;

// Workgroups are handed to the 8 XCDs round-robin by their linear id.  Work items are numbered
// head-major (all query tiles of head 0, then head 1, ...); giving XCD x the contiguous range
// [x*per_xcd, (x+1)*per_xcd) keeps the query tiles that stream the same head's K/V on one XCD,
// so that head's window is fetched from HBM once into that XCD's L2 instead of once per tile.
// With a split key range the items of one head are ordered split-major, so the query tiles that
// stream the same slice of K/V stay neighbours.  A batch over stored chunks (one key range each)
// is ordered head, chunk, query tile: a head's queries stay in the XCD's L2 while the chunks' keys
// stream through once.
__device__ inline bool work_item(const AttnArgs &a, int &c, int &h, int &qt, int &sp) {
    const int lin = blockIdx.x;
    const int w = (lin % kXcds) * a.per_xcd + lin / kXcds;
    if (lin / kXcds >= a.per_xcd) return false;
    if (a.n_chunks > 0) {
        const int per_head = a.n_chunks * a.n_qtiles;
        if (w >= a.H * per_head) return false;
        h = w / per_head;
        c = (w % per_head) / a.n_qtiles;
        qt = w % a.n_qtiles;
        sp = 0;
        return true;
    }
    if (w >= a.H * a.n_qtiles * a.splits) return false;
    c = 0;
    h = w / (a.n_qtiles * a.splits);
    const int rem = w % (a.n_qtiles * a.splits);
    sp = rem / a.n_qtiles;
    qt = rem % a.n_qtiles;
    return true;
}

// Several launches folded into one grid (used by the frame-causal entry point): each entry is what
// one plain launch would have been told -- which queries, which key range, which partial slot.
// Work items are numbered head-major over all entries, so a head's entries share an XCD.
struct SubLaunch { int q_off, N_q, n_qtiles, kv_off, N_kv, kv_start, part_slot; };
constexpr int kMaxSub = 8;
struct SubTable { int n, per_head; SubLaunch s[kMaxSub]; };

// MULTI: pick this workgroup's entry and make the (by-value) arguments look like that launch.
template <bool MULTI>
__device__ inline bool select_work(AttnArgs &a, const SubTable &t, size_t row_bytes, int &c, int &h, int &qt,
                                   int &sp);

// The window this workgroup reads: its keys, row stride between heads and length; where lse goes.
struct Window {
    const char *K;
    float *lse;
    int stride, n_kv;
};

__device__ inline Window window_of(const AttnArgs &a, int c) {
    Window w;
    if (a.n_chunks > 0) {
        w.K = reinterpret_cast<const char *>(a.k_table[c]);
        w.n_kv = w.stride = a.n_tok[c];
        if (w.n_kv > a.max_tok) w.n_kv = 0;   // violates the descriptor's bound: holds no token
        w.lse = a.lse + (size_t)c * a.H * a.q_rows;
    } else {
        w.K = a.K;
        w.stride = a.kv_row_stride;
        w.lse = a.lse;
        w.n_kv = a.N_kv;
        if (a.n_kv_dev) {
            const int m = *a.n_kv_dev - a.kv_start;
            w.n_kv = m < w.n_kv ? m : w.n_kv;
        }
    }
    if (w.n_kv < 0) w.n_kv = 0;
    return w;
}

template <bool MULTI>
__device__ inline bool select_work(AttnArgs &a, const SubTable &t, size_t row_bytes, int &c, int &h, int &qt,
                                   int &sp) {
    if constexpr (!MULTI) {
        return work_item(a, c, h, qt, sp);
    } else {
        const int lin = blockIdx.x;
        const int w = (lin % kXcds) * a.per_xcd + lin / kXcds;
        if (lin / kXcds >= a.per_xcd || w >= a.H * t.per_head) return false;
        h = w / t.per_head;
        int r = w % t.per_head, e = 0;
        while (e + 1 < t.n && r >= t.s[e].n_qtiles) {
            r -= t.s[e].n_qtiles;
            ++e;
        }
        qt = r;
        c = 0;
        sp = 0;
        const SubLaunch u = t.s[e];
        a.q_off = u.q_off; a.N_q = u.N_q; a.n_qtiles = u.n_qtiles;
        a.N_kv = u.N_kv; a.kv_start = u.kv_start; a.part_slot = u.part_slot;
        a.K += (size_t)u.kv_off * row_bytes;
        a.V += (size_t)u.kv_off * row_bytes;
        return true;
    }
}

// ------------------------------------------------------------------------------------------
// fp32: v_mfma_f32_32x32x2_f32, 4 waves x 32 queries per workgroup, 32-key tiles.
// ------------------------------------------------------------------------------------------
constexpr int kF32Waves = 4;
constexpr int kF32Keys = 32;
constexpr int kF32KPitch = WK_D + 4;  // floats; 16 lanes x 16 B then cover all 64 banks
constexpr int kF32VPitch = WK_D + 8;  // rows 4 apart land 32 banks apart

template <bool MULTI>
__global__ __launch_bounds__(kF32Waves * 64) void k_attn_f32(AttnArgs a, SubTable sub) {
    __shared__ float Ks[kF32Keys * kF32KPitch];
    __shared__ float Vs[kF32Keys * kF32VPitch];
    int c, h, qt, sp;
    if (!select_work<MULTI>(a, sub, 512, c, h, qt, sp)) return;
    const Window win = window_of(a, c);
    const int n_kv = win.n_kv;
    float *const lse = win.lse;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, g = lane >> 5;
    const int q = qt * (kF32Waves * 32) + wave * 32 + col;
    const bool q_ok = q < a.N_q;
    const int q_ld = q_ok ? q : a.N_q - 1;
    const size_t qrow = (size_t)h * a.q_rows + a.q_off + q_ld;   // row of this lane's query in Q / O / lse
    const float *Qrow = reinterpret_cast<const float *>(a.Q) + qrow * WK_D;
    float *Orow = reinterpret_cast<float *>(a.O) + qrow * WK_D;
    const bool with_o = a.O != nullptr;   // false: log-sum-exp only, V is not read (zeros stand in)
    const bool partial_out = a.part_slot >= 0 || a.splits > 1;
    const size_t prow = ((size_t)(a.part_slot >= 0 ? a.part_slot : sp) * a.H + h) * a.q_rows + a.q_off + q_ld;
    // this workgroup's keys [kt0, kt1): the whole window, or split sp of a.splits (whole tiles each)
    const int n_tiles = (n_kv + kF32Keys - 1) / kF32Keys;
    const int tiles_per_split = (n_tiles + a.splits - 1) / a.splits;
    const int kt0 = sp * tiles_per_split * kF32Keys;
    const int kt1 = min(n_kv, (sp + 1) * tiles_per_split * kF32Keys);

    if (kt0 >= kt1) {   // empty window, or a split past its end: contributes nothing
        if (q_ok && partial_out) {
            for (int c = g * 64; c < g * 64 + 64; c += 4)
                *reinterpret_cast<float4 *>(a.part_o + prow * WK_D + c) = float4{0, 0, 0, 0};
            if (g == 0) { a.part_ml[prow * 2] = -INFINITY; a.part_ml[prow * 2 + 1] = 0.f; }
        } else if (q_ok) {
            if (with_o)
                for (int c = g * 64; c < g * 64 + 64; c += 4) *reinterpret_cast<float4 *>(Orow + c) = float4{0, 0, 0, 0};
            if (lse && g == 0) lse[qrow] = -INFINITY;
        }
        return;
    }

    // B operand of S^T = K Q^T: k slot (g, step 4c+e) means feature 8c + 4g + e
    float4 qr[16];
#pragma unroll
    for (int c = 0; c < 16; ++c) qr[c] = *reinterpret_cast<const float4 *>(Qrow + 8 * c + 4 * g);

    f32x16 o[4];
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[b][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    const float *Kh = reinterpret_cast<const float *>(win.K) + (size_t)h * win.stride * WK_D;
    const float *Vh = reinterpret_cast<const float *>(a.V) + (size_t)h * win.stride * WK_D;

    for (int kt = kt0; kt < kt1; kt += kF32Keys) {
        __syncthreads();  // previous tile fully consumed
#pragma unroll
        for (int i = 0; i < (kF32Keys * WK_D / 4) / (kF32Waves * 64); ++i) {
            const int x = tid + i * (kF32Waves * 64);
            const int row = x / (WK_D / 4), c4 = x % (WK_D / 4);
            float4 kv = float4{0, 0, 0, 0}, vv = float4{0, 0, 0, 0};
            if (kt + row < kt1) {
                kv = *reinterpret_cast<const float4 *>(Kh + (size_t)(kt + row) * WK_D + 4 * c4);
                if (with_o) vv = *reinterpret_cast<const float4 *>(Vh + (size_t)(kt + row) * WK_D + 4 * c4);
            }
            *reinterpret_cast<float4 *>(&Ks[row * kF32KPitch + 4 * c4]) = kv;
            *reinterpret_cast<float4 *>(&Vs[row * kF32VPitch + 4 * c4]) = vv;
        }
        __syncthreads();

        f32x16 s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int c = 0; c < 16; ++c) {
            const float4 ka = *reinterpret_cast<const float4 *>(&Ks[col * kF32KPitch + 8 * c + 4 * g]);
            s = __builtin_amdgcn_mfma_f32_32x32x2f32(ka.x, qr[c].x, s, 0, 0, 0);
            s = __builtin_amdgcn_mfma_f32_32x32x2f32(ka.y, qr[c].y, s, 0, 0, 0);
            s = __builtin_amdgcn_mfma_f32_32x32x2f32(ka.z, qr[c].z, s, 0, 0, 0);
            s = __builtin_amdgcn_mfma_f32_32x32x2f32(ka.w, qr[c].w, s, 0, 0, 0);
        }
        // accumulator register r of this lane is key kt + 8*(r/4) + 4*g + r%4
        float m_tile = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int key = kt + 8 * (r >> 2) + 4 * g + (r & 3);
            s[r] = key < kt1 ? s[r] * a.scale_log2 : -INFINITY;
            m_tile = fmaxf(m_tile, s[r]);
        }
        m_tile = fmaxf(m_tile, __shfl_xor(m_tile, 32));
        const float m_new = fmaxf(m_run, m_tile);  // finite: every tile holds at least one valid key
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        float l_tile = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            s[r] = __builtin_amdgcn_exp2f(s[r] - m_new);
            l_tile += s[r];
        }
        l_run = l_run * alpha + l_tile;
        m_run = m_new;
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[b][r] *= alpha;
        // O^T += V^T P^T: k slot g of step r means key 8*(r/4) + 4*g + r%4
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int krow = 8 * (r >> 2) + 4 * g + (r & 3);
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const float va = Vs[krow * kF32VPitch + 32 * b + col];
                o[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(va, s[r], o[b], 0, 0, 0);
            }
        }
    }
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (q_ok && partial_out) {   // (O, max, sum) of this key range, merged by k_attn_merge
        float *Po = a.part_o + prow * WK_D;
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int t = 0; t < 4; ++t)
                *reinterpret_cast<float4 *>(Po + 32 * b + 8 * t + 4 * g) =
                    float4{o[b][4 * t], o[b][4 * t + 1], o[b][4 * t + 2], o[b][4 * t + 3]};
        if (g == 0) { a.part_ml[prow * 2] = m_run; a.part_ml[prow * 2 + 1] = l_tot; }
    } else if (q_ok) {
        const float inv = 1.f / l_tot;
        if (with_o)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int dv = 32 * b + 8 * t + 4 * g;
                *reinterpret_cast<float4 *>(Orow + dv) =
                    float4{o[b][4 * t] * inv, o[b][4 * t + 1] * inv, o[b][4 * t + 2] * inv, o[b][4 * t + 3] * inv};
            }
        if (lse && g == 0) lse[qrow] = (m_run + log2f(l_tot)) * 0.6931471805599453f;
    }
}

// ------------------------------------------------------------------------------------------
// bf16: v_mfma_f32_32x32x16_bf16, 8 waves x 32 queries per workgroup (4 waves x 32 for small grids),
// 64-key tiles.
//
// K and V tiles go from global memory straight into a 4-deep LDS ring (global_load_lds, no
// register staging), K tiles four and V tiles three ahead of the step that loads them, which
// gives each three steps to land (S^T is formed one step early, so K leads V by one tile).  Both tiles are row-major with their
// 16-byte chunks permuted inside a row; the permutation is applied on the source side (each
// lane fetches the chunk that belongs in its linear LDS slot).  K^ operands are plain 16-byte
// reads; V^T operands are LDS transpose reads (ds_read_b64_tr_b16) of the row-major V tile.
// While a wave turns S^T of tile j into probabilities and multiplies them into O^T it already
// computes S^T of tile j+1, so the softmax arithmetic has independent matrix work to hide under.
// ------------------------------------------------------------------------------------------
constexpr int kKeys = 64;               // keys per tile
constexpr int kTileBytes = kKeys * 256; // one K or V tile
constexpr int kStages = 4;
constexpr int kVRing = kStages * kTileBytes;          // K ring at 0, V ring behind it
constexpr int kSmemBytes = 2 * kStages * kTileBytes;  // 128 KB

typedef short i16x4 __attribute__((ext_vector_type(4)));

__device__ inline float max3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }

// max over lanes l and l^32
__device__ inline float max_across_halves(float x) {
    const unsigned u = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// registers the hand-scheduled loop uses beyond its operands: the odd-position S^T tile, P, the K and V^T
// fragment buffers and three temporaries
#define WK_ATTN_LOOP_CLOBBERS \
    "v96", "v97", "v98", "v99", "v100", "v101", "v102", "v103", "v104", "v105", "v106", "v107", \
    "v108", "v109", "v110", "v111", "v112", "v113", "v114", "v115", "v116", "v117", "v118", "v119", \
    "v120", "v121", "v122", "v123", "v124", "v125", "v126", "v127", "v160", "v161", "v162", "v163", \
    "v164", "v165", "v166", "v167", "v168", "v169", "v170", "v171", "v172", "v173", "v174", "v175", \
    "v176", "v177", "v178", "v179", "v180", "v181", "v182", "v183", "v184", "v185", "v186", "v187", \
    "v188", "v189", "v190", "v191", "v192", "v193", "v194", "v195", "v196", "v197", "v198", "v199", \
    "v200", "v201", "v202", "v203", "v204", "v205", "v206", "v207", "v208", "v209", "v210", "v211", \
    "v212", "v213", "v214", "v215", "v216", "v217", "v218", "v219", "v220", "v221", "v222", "v223", \
    "v244", "v245", "v246"

#define WK_LDS(p) ((__attribute__((address_space(3))) void *)(p))
// typed LDS pointer from a 32-bit LDS byte address
#define WK_LDS_AT(T, addr) ((__attribute__((address_space(3))) T *)(size_t)(addr))
#define WK_GLB(p) ((const __attribute__((address_space(1))) void *)(p))

// IN_PLACE: the window is a list of segments (the native rows, then each retrieved chunk where the store
// keeps it) instead of one array.  Tiles never straddle segments: a segment's last tile may be partial and
// is masked like the window's last tile; a wave-uniform cursor walks the list.
constexpr int kMaxSegments = 33;   // native rows + up to 32 retrieved chunks
struct Segment { const char *K; const char *V; int len; int pad; };

__device__ inline const char *uniform_ptr(const char *p) {
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const char *>(((uint64_t)hi << 32) | lo);
}

template <int WAVES, bool MULTI, bool IN_PLACE>
__global__ __launch_bounds__(WAVES * 64, 2) void k_attn_bf16(AttnArgs a, SubTable sub) {
    static_assert(WAVES == 8 || WAVES == 4, "8 or 4 waves of 32 queries");
    constexpr int NB = 16 / WAVES;     // 1 KB blocks of a tile that a wave loads
    // s_waitcnt vmcnt(4 * NB), everything else unconstrained: all but the last four tile shares have landed
    constexpr int kWaitTwoSteps = NB == 2 ? 0x0F78 : 0x4F70;
    static_assert(!(MULTI && IN_PLACE), "a table of launches over one window array only");
    extern __shared__ __attribute__((aligned(256))) char smem[];
    int c, h, qt, sp;
    if (!select_work<MULTI>(a, sub, 256, c, h, qt, sp)) return;
    const Window win = window_of(a, c);
    float *const lse = win.lse;
    const int tid = threadIdx.x, lane = tid & 63;
    // segment list of this head and its number of tiles
    int n_seg = 0, seg_tiles = 0;
    const Segment *seg_list = nullptr;
    if constexpr (IN_PLACE) {
        __shared__ Segment segs[kMaxSegments];
        __shared__ Segment raw[kMaxSegments];
        __shared__ int seg_meta[2];
        // entry 0 = native rows, entry 1 + r = retrieved chunk r; one thread each fetches its entry (the
        // id, then the chunk's length and addresses), thread 0 then drops the empty ones
        if (tid <= a.R_max) {
            Segment e{nullptr, nullptr, 0, 0};
            if (tid == 0) {
                if (a.N_kv > 0)
                    e = Segment{a.K + (size_t)h * a.kv_row_stride * 256, a.V + (size_t)h * a.kv_row_stride * 256, a.N_kv, 0};
            } else {
                int nf = a.n_ids ? *a.n_ids : a.R_max;
                nf = nf < a.R_max ? nf : a.R_max;
                const int id = tid - 1 < nf ? a.ids[tid - 1] : -1;
                if (id >= 0 && id < a.store_M) {
                    const int len = a.n_tok[id];
                    if (len > 0 && len <= a.max_tok)   // a chunk beyond the descriptor's bound is skipped
                        e = Segment{reinterpret_cast<const char *>(a.k_table[id]) + (size_t)h * len * 256,
                                    reinterpret_cast<const char *>(a.v_table[id]) + (size_t)h * len * 256, len, 0};
                }
            }
            raw[tid] = e;
        }
        __syncthreads();
        if (tid == 0) {
            int n = 0, tiles = 0;
            for (int r = 0; r <= a.R_max; ++r) {
                const Segment e = raw[r];
                if (e.len > 0) {
                    segs[n++] = e;
                    tiles += (e.len + 63) / 64;
                }
            }
            seg_meta[0] = n;
            seg_meta[1] = tiles;
        }
        __syncthreads();
        n_seg = __builtin_amdgcn_readfirstlane(seg_meta[0]);
        seg_tiles = __builtin_amdgcn_readfirstlane(seg_meta[1]);
        seg_list = segs;
    }
    const int n_kv = IN_PLACE ? seg_tiles * 64 : win.n_kv;   // IN_PLACE: only its tile count is used
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, g = lane >> 5;
    const int q = qt * (WAVES * 32) + wave * 32 + col;
    const bool q_ok = q < a.N_q;
    const int q_ld = q_ok ? q : a.N_q - 1;
    const char *Qrow = a.Q + ((size_t)h * a.q_rows + a.q_off + q_ld) * 256;
    const bool partial_out = a.splits > 1 || a.part_slot >= 0;  // (O, max, sum) for k_attn_merge
    // rows of this lane's query in O / lse and in the partial arrays (formed where they are used:
    // two 64-bit values per lane are not worth carrying through the loop)
    auto out_row = [&]() { return (size_t)h * a.q_rows + a.q_off + q; };
    auto part_row = [&]() { return ((size_t)(a.part_slot >= 0 ? a.part_slot : sp) * a.H + h) * a.q_rows + a.q_off + q; };

    // this workgroup's tiles [t0, t1) of the window
    const int n_tiles = (n_kv + kKeys - 1) / kKeys;
    const int tiles_per_split = (n_tiles + a.splits - 1) / a.splits;
    const int t0 = sp * tiles_per_split;
    const int t1 = min(n_tiles, t0 + tiles_per_split);
    if (t0 >= t1) {   // empty window, or a split past its end: contributes nothing
        if (q_ok) {
            if (!partial_out) {
                const size_t qrow = out_row();
                char *Orow = a.O + qrow * 256;
                for (int c = g * 8; c < g * 8 + 8; ++c) reinterpret_cast<uint4 *>(Orow)[c] = uint4{0, 0, 0, 0};
                if (lse && g == 0) lse[qrow] = -INFINITY;
            } else {
                const size_t prow = part_row();
                for (int c = g * 16; c < g * 16 + 16; ++c) reinterpret_cast<float4 *>(a.part_o + prow * WK_D)[c] = float4{0, 0, 0, 0};
                if (g == 0) { a.part_ml[prow * 2] = -INFINITY; a.part_ml[prow * 2 + 1] = 0.f; }
            }
        }
        return;
    }

    // B operand of S^T = K Q^T, step st: features 16*st + 8*g .. +7 of this lane's query
    bf16x8 qb[8];
#pragma unroll
    for (int st = 0; st < 8; ++st) qb[st] = *reinterpret_cast<const bf16x8 *>(Qrow + (2 * st + g) * 16);

    // K tile: row-major, chunk c of key k at slot c ^ (k & 15).  A operand of S^T block b, step st:
    // key 32*b + col, chunk 2*st + g.   address = k_rd[st] + stage*16384 + b*8192
    // (operand read addresses are kept as 32-bit LDS addresses: the hand-scheduled loop takes them as they are)
    const unsigned lds0 = (unsigned)(size_t)WK_LDS(smem);
    unsigned k_rd[8];
#pragma unroll
    for (int st = 0; st < 8; ++st) k_rd[st] = lds0 + col * 256 + (((2 * st + g) ^ (col & 15)) << 4);
    // V tile: row-major, chunk c of key k at slot c ^ ((k & 3) << 2).  The transpose read hands lane
    // i of a 16-lane group element (i & 3) of source lane 4*j + (i >> 2), j = 0..3.  Source lane p of
    // group u points at key 16*ks + 8*tt + 4*g + (p >> 2), features 32*blk + 16*(u&1) + 4*(p&3) .. +3,
    // so lane i receives feature 32*blk + 16*(u&1) + i of keys 16*ks + 8*tt + 4*g + 0..3: the four
    // k slots that registers 4*tt .. 4*tt+3 of the P^T operand of step ks stand for.
    //   address = v_rd[blk] + stage*16384 + ks*4096 + tt*2048
    unsigned v_rd[4];
    {
        const int u = lane >> 4, p = lane & 15;
#pragma unroll
        for (int blk = 0; blk < 4; ++blk)
            v_rd[blk] = lds0 + kVRing + (4 * g + (p >> 2)) * 256 +
                        ((4 * (blk ^ (p >> 2)) + 2 * (u & 1) + ((p & 3) >> 1)) << 4) + 8 * (p & 1);
    }
    // tile loads: wave w fills 1 KB blocks NB*w .. NB*w + NB-1 of the K tile and of the V tile; lane l
    // of a block lands in 16-byte slot l = (row r = l >> 4 of the block, slot p = l & 15)
    unsigned k_src[NB], v_src[NB];
    {
        const int r = lane >> 4, p = lane & 15;
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int R = 4 * (NB * wave + i) + r;
            k_src[i] = R * 256 + ((p ^ (R & 15)) << 4);
            v_src[i] = R * 256 + ((p ^ (r << 2)) << 4);
        }
    }
    const char *Kh = win.K + (size_t)h * win.stride * 256;
    const char *Vh = a.V + (size_t)h * win.stride * 256;
    const unsigned last_off = (unsigned)(n_kv - 1) * 256u;
    char *const dma_dst = smem + wave * (NB * 1024);   // + slot*16384 (+ kVRing) + i*1024

    // Loads: NB per wave for a K tile, NB for a V tile (rel = tile index relative to t0).  Rows past the
    // window clamp to the last key; those keys are masked (weight exactly 0) before they can contribute.
    // IN_PLACE: one cursor walks the segment list in steps of a tile, at the K loads, which lead
    // everything else.  What later stages need of a tile is kept from the moment its K tile was requested:
    // the V tile is requested one K request later (two-deep line of its address and bounds) and S^T of
    // the tile is formed three K requests later (four-deep line of its number of valid keys).  Moving past
    // the list's last tile leaves the cursor on it (the look-ahead fetches it again and nobody reads it).
    // All of this is wave-uniform scalar state.
    struct TileRef { const char *base; int row, len; };
    const char *cur_k = nullptr, *cur_v = nullptr;
    int cur_len = 0, cur_row = 0, cur_seg = 0;
    TileRef v_line[2] = {{nullptr, 0, 0}, {nullptr, 0, 0}};
    unsigned valid_line = 0;   // four entries of 8 bits, newest lowest: valid keys of a tile, capped at 64 (scalar registers are scarce here)
    if constexpr (IN_PLACE) {
        if (n_seg > 0) {
            cur_len = __builtin_amdgcn_readfirstlane(seg_list[0].len);
            cur_k = uniform_ptr(seg_list[0].K);
            cur_v = uniform_ptr(seg_list[0].V);
        }
    }
    // one tile: rows past the segment's end clamp to its last row (those keys are masked when consumed)
    auto issue_at = [&](const char *base, int row, int len, const unsigned (&src)[NB], char *dst) {
        const unsigned t_off = (unsigned)row * 256u;
        if (row + kKeys <= len) {
#pragma unroll
            for (int i = 0; i < NB; ++i)
                __builtin_amdgcn_global_load_lds(WK_GLB(base + (t_off + src[i])), WK_LDS(dst + i * 1024), 16, 0, 0);
        } else {
            const unsigned seg_last = (unsigned)(len - 1) * 256u;
#pragma unroll
            for (int i = 0; i < NB; ++i) {
                const unsigned o = min(t_off + src[i], seg_last + (src[i] & 255u));
                __builtin_amdgcn_global_load_lds(WK_GLB(base + o), WK_LDS(dst + i * 1024), 16, 0, 0);
            }
        }
    };
    auto issue_k_in_place = [&](char *dst) {
        issue_at(cur_k, cur_row, cur_len, k_src, dst);
        v_line[1] = v_line[0];
        v_line[0] = TileRef{cur_v, cur_row, cur_len};
        valid_line = (valid_line << 8) | (unsigned)min(cur_len - cur_row, kKeys);   // 64: a full tile
        if (cur_row + kKeys < cur_len) {
            cur_row += kKeys;
        } else if (cur_seg + 1 < n_seg) {
            ++cur_seg;
            cur_row = 0;
            cur_len = __builtin_amdgcn_readfirstlane(seg_list[cur_seg].len);
            cur_k = uniform_ptr(seg_list[cur_seg].K);
            cur_v = uniform_ptr(seg_list[cur_seg].V);
        }
    };
    auto issue_k = [&](int rel, int slot) {
        const unsigned t_off = (unsigned)(t0 + rel) * (kKeys * 256u);
        char *dst = dma_dst + slot * kTileBytes;
        if constexpr (IN_PLACE) {
            issue_k_in_place(dst);
            return;
        }
        if ((t0 + rel + 1) * kKeys <= n_kv) {
#pragma unroll
            for (int i = 0; i < NB; ++i)
                __builtin_amdgcn_global_load_lds(WK_GLB(Kh + (t_off + k_src[i])), WK_LDS(dst + i * 1024), 16, 0, 0);
        } else {
#pragma unroll
            for (int i = 0; i < NB; ++i) {
                const unsigned ko = min(t_off + k_src[i], last_off + (k_src[i] & 255u));
                __builtin_amdgcn_global_load_lds(WK_GLB(Kh + ko), WK_LDS(dst + i * 1024), 16, 0, 0);
            }
        }
    };
    auto issue_v = [&](int rel, int slot) {
        const unsigned t_off = (unsigned)(t0 + rel) * (kKeys * 256u);
        char *dst = dma_dst + slot * kTileBytes + kVRing;
        if constexpr (IN_PLACE) {
            issue_at(v_line[1].base, v_line[1].row, v_line[1].len, v_src, dst);
            return;
        }
        if ((t0 + rel + 1) * kKeys <= n_kv) {
#pragma unroll
            for (int i = 0; i < NB; ++i)
                __builtin_amdgcn_global_load_lds(WK_GLB(Vh + (t_off + v_src[i])), WK_LDS(dst + i * 1024), 16, 0, 0);
        } else {
#pragma unroll
            for (int i = 0; i < NB; ++i) {
                const unsigned vo = min(t_off + v_src[i], last_off + (v_src[i] & 255u));
                __builtin_amdgcn_global_load_lds(WK_GLB(Vh + vo), WK_LDS(dst + i * 1024), 16, 0, 0);
            }
        }
    };

    f32x16 o[4];
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[b][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;   // m_run in scaled (log2) units
    const float c_log2 = a.scale_log2;

    auto compute_s = [&](int byte_off, f32x16 (&s)[2]) __attribute__((always_inline)) {
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[b][r] = 0.f;
        // the two 32-key blocks are independent accumulation chains: alternate them
#pragma unroll
        for (int st = 0; st < 8; ++st)
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                const bf16x8 ka = *WK_LDS_AT(const bf16x8, k_rd[st] + byte_off + b * 8192);
                s[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qb[st], s[b], 0, 0, 0);
            }
    };
    // IN_PLACE: the tile whose S^T has just been formed had its K tile requested three requests ago; keys
    // past its segment's end get -inf (weight exactly 0).
    auto mask_segment_tail = [&](f32x16 (&s)[2]) __attribute__((always_inline)) {
        const int valid = (int)(valid_line >> 24);
        if (valid < kKeys) {
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (32 * b + 8 * (r >> 2) + 4 * g + (r & 3) >= valid) s[b][r] = -INFINITY;
        }
    };
    // scaled row max of a tile's raw logits (both lane halves combined)
    auto tile_max = [&](const f32x16 (&s)[2]) __attribute__((always_inline)) {
        float mx[10];
#pragma unroll
        for (int i = 0; i < 10; ++i) {
            const int e = 3 * i;
            mx[i] = max3(s[e >> 4][e & 15], s[(e + 1) >> 4][(e + 1) & 15], s[(e + 2) >> 4][(e + 2) & 15]);
        }
        float m = max3(max3(mx[0], mx[1], mx[2]), max3(mx[3], mx[4], mx[5]), max3(mx[6], mx[7], mx[8]));
        m = max3(m, mx[9], fmaxf(s[1][14], s[1][15]));
        return max_across_halves(m) * c_log2;
    };
    // lazy rescale: the running max only moves when some row's max grew by more than 2^8
    auto maybe_rescale = [&](float m_tile) __attribute__((always_inline)) {
        if (__any(m_tile > m_run + 8.0f)) {
            const float m_new = fmaxf(m_run, m_tile);
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
            m_run = m_new;
            l_run *= alpha;
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[b][r] *= alpha;
        }
    };
    // p = exp2(s*c - m) rounded to bf16; registers 8*t2 .. 8*t2+7 of block b -> k step 2*b + t2.
    // The row sum uses the rounded probabilities, the ones the P V product sees.
    auto probabilities = [&](const f32x16 (&s)[2], bf16x8 (&pb)[4]) __attribute__((always_inline)) {
        const float neg_m = -m_run;
        const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
                for (int e = 0; e < 8; e += 2) {
                    const float p0 = __builtin_amdgcn_exp2f(fmaf(s[b][8 * t2 + e], c_log2, neg_m));
                    const float p1 = __builtin_amdgcn_exp2f(fmaf(s[b][8 * t2 + e + 1], c_log2, neg_m));
                    const bf16x2 pk = __builtin_convertvector(f32x2{p0, p1}, bf16x2);
                    pb[2 * b + t2][e] = pk[0];
                    pb[2 * b + t2][e + 1] = pk[1];
                    l_run = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, l_run, false);
                }
    };
    auto accumulate_pv = [&](int byte_off, const bf16x8 (&pb)[4]) __attribute__((always_inline)) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const unsigned p = v_rd[b] + byte_off + ks * 4096;
                const i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(WK_LDS_AT(i16x4, p));
                const i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(WK_LDS_AT(i16x4, p + 2048));
                const i16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                o[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), pb[ks], o[b], 0, 0, 0);
            }
    };

    // The ring slot of tile j is j & 3.  Whole groups of four steps come first (the steady state), then the
    // n_steps & 3 left-over steps, then the last tile at whatever ring position that leaves it.
    const int n_steps = t1 - t0 - 1;
    // Step j multiplies K tile j+1 (S^T one step early) and V tile j, so K runs one tile ahead of V:
    // step j loads K tile j+4 into the slot of K tile j (read in step j-1) and V tile j+3 into the slot
    // of V tile j-1.  Both then have three steps to land before the step that needs them.
    issue_k(0, 0);
    issue_k(1, 1);
    issue_v(0, 0);
    issue_k(2, 2);
    issue_v(1, 1);
    issue_k(3, 3);
    issue_v(2, 2);
    __builtin_amdgcn_s_waitcnt(kWaitTwoSteps);   // K tiles 0, 1 and V tile 0 of this wave have landed
    __syncthreads();
    if (qt * (WAVES * 32) + wave * 32 >= a.N_q) {
        // A wave whose 32 queries all lie past N_q (last query tile of a head): it keeps loading its
        // share of every tile and meets every barrier, but leaves the matrix and vector pipes of its
        // SIMD to the wave that has work.
        __syncthreads();   // the others' first S^T has been formed from K tile 0
        for (int j = 0; j < n_steps; ++j) {
            issue_k(j + 4, j & 3);
            issue_v(j + 3, (j + 3) & 3);
            __builtin_amdgcn_s_waitcnt(kWaitTwoSteps);
            __syncthreads();
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);
        return;
    }
    f32x16 s_a[2], s_b[2];   // S^T of tiles at even / odd ring positions
    float mt;
    compute_s(0, s_a);
    if constexpr (IN_PLACE) mask_segment_tail(s_a);
    mt = tile_max(s_a);
    __syncthreads();   // K tile 0 has been read by every wave: step 0 may load K tile 4 into its slot

    // one pipeline step: tile j (ring position POS) is consumed, S^T of tile j+1 produced
    auto step = [&](int j, const int POS, f32x16 (&s_cur)[2], f32x16 (&s_next)[2]) __attribute__((always_inline)) {
        issue_k(j + 4, POS);
        issue_v(j + 3, (POS + 3) & 3);
        maybe_rescale(mt);
        compute_s(((POS + 1) & 3) * kTileBytes, s_next);
        bf16x8 pb[4];
        probabilities(s_cur, pb);
        // (the rare branch sits between the two matrix products, so that the row max below can still be
        // interleaved with the second one)
        if constexpr (IN_PLACE) mask_segment_tail(s_next);
        accumulate_pv(POS * kTileBytes, pb);
        mt = tile_max(s_next);
        __builtin_amdgcn_s_waitcnt(kWaitTwoSteps);   // all but the loads of this step and the one before have landed
        __syncthreads();
    };
    int j = 0;
    if constexpr (WAVES == 8 && !IN_PLACE) {
        // Steady state: whole groups of four steps whose look-ahead loads all lie inside the window run in the
        // hand-scheduled loop of wk_attn_loop_gfx950.inc (written by gen_attn_loop.py, which documents its schedule
        // and register map).  It is the four `step`s below instruction for instruction in what it computes -- same
        // ring protocol, same arithmetic in the same order, bit-identical results -- so the steps behind it
        // stay in C++: the last whole groups, whose loads are clamped to the window, the left-over steps and the
        // last, possibly partial tile.  Its operands are pinned to the registers its text names.
        int G = (n_kv / kKeys - 4 - t0 - j) / 4;
        const int G_steps = (n_steps - j) / 4;
        G = G < G_steps ? G : G_steps;
        if (G > 0) {
            const unsigned koff = (unsigned)(t0 + j + 4) * (kKeys * 256u), voff = (unsigned)(t0 + j + 3) * (kKeys * 256u);
            const unsigned dst = (unsigned)(size_t)WK_LDS(dma_dst);
            int g_left = G;
            const bf16x8 q0 = qb[0], q1 = qb[1], q2 = qb[2], q3 = qb[3], q4 = qb[4], q5 = qb[5], q6 = qb[6], q7 = qb[7];
            f32x16 o0 = o[0], o1 = o[1], o2 = o[2], o3 = o[3], sa0 = s_a[0], sa1 = s_a[1];
            const unsigned ks0 = k_src[0], ks1 = k_src[NB - 1], vs0 = v_src[0], vs1 = v_src[NB - 1];
            asm volatile(
#include "wk_attn_loop_gfx950.inc"
                : "+{v[0:15]}"(o0), "+{v[16:31]}"(o1), "+{v[32:47]}"(o2), "+{v[48:63]}"(o3), "+{v[64:79]}"(sa0),
                  "+{v[80:95]}"(sa1), "+{v240}"(m_run), "+{v241}"(l_run), "+{v243}"(mt), "+{s44}"(g_left)
                : "{v[128:131]}"(q0), "{v[132:135]}"(q1), "{v[136:139]}"(q2), "{v[140:143]}"(q3), "{v[144:147]}"(q4),
                  "{v[148:151]}"(q5), "{v[152:155]}"(q6), "{v[156:159]}"(q7), "{v224}"(k_rd[0]), "{v225}"(k_rd[1]),
                  "{v226}"(k_rd[2]), "{v227}"(k_rd[3]), "{v228}"(k_rd[4]), "{v229}"(k_rd[5]), "{v230}"(k_rd[6]), "{v231}"(k_rd[7]),
                  "{v232}"(v_rd[0]), "{v233}"(v_rd[1]), "{v234}"(v_rd[2]), "{v235}"(v_rd[3]), "{v236}"(ks0), "{v237}"(ks1),
                  "{v238}"(vs0), "{v239}"(vs1), "{s[36:37]}"(Kh), "{s[38:39]}"(Vh), "{s40}"(koff), "{s41}"(voff),
                  "{s42}"(dst), "{s43}"(c_log2)
                : WK_ATTN_LOOP_CLOBBERS, "s45", "vcc", "memory");
            o[0] = o0; o[1] = o1; o[2] = o2; o[3] = o3; s_a[0] = sa0; s_a[1] = sa1;
            j += 4 * G;
        }
    }
    for (; j + 4 <= n_steps; j += 4) {
        step(j, 0, s_a, s_b);
        step(j + 1, 1, s_b, s_a);
        step(j + 2, 2, s_a, s_b);
        step(j + 3, 3, s_b, s_a);
    }
    // last tile (ring position POS): the only one that can be partial.  Mask the keys past the window and
    // redo its max.
    auto last_tile = [&](const int POS, f32x16 (&s_cur)[2]) __attribute__((always_inline)) {
        const int kt = (t1 - 1) * kKeys;
        if (!IN_PLACE && kt + kKeys > n_kv) {
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = kt + 32 * b + 8 * (r >> 2) + 4 * g + (r & 3);
                    if (key >= n_kv) s_cur[b][r] = -INFINITY;
                }
            mt = tile_max(s_cur);
        }
        maybe_rescale(mt);
        bf16x8 pb[4];
        probabilities(s_cur, pb);
        accumulate_pv(POS * kTileBytes, pb);
    };
    // the n_steps & 3 left-over steps and the last tile: one copy of the code, ring position at run time,
    // S^T handed back to s_a after each step
    for (; j < n_steps; ++j) {
        step(j, j & 3, s_a, s_b);
#pragma unroll
        for (int b = 0; b < 2; ++b) s_a[b] = s_b[b];
    }
    last_tile(n_steps & 3, s_a);
    __builtin_amdgcn_s_waitcnt(0x0F70);   // drain the clamped look-ahead loads before the LDS is released

    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (q_ok && !partial_out) {
        const size_t qrow = out_row();
        char *Orow = a.O + qrow * 256;
        const float inv = 1.f / l_tot;
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int dv = 32 * b + 8 * t + 4 * g;
                const bf16x2 lo = __builtin_convertvector(f32x2{o[b][4 * t] * inv, o[b][4 * t + 1] * inv}, bf16x2);
                const bf16x2 hi = __builtin_convertvector(f32x2{o[b][4 * t + 2] * inv, o[b][4 * t + 3] * inv}, bf16x2);
                uint2 w;
                w.x = __builtin_bit_cast(uint32_t, lo);
                w.y = __builtin_bit_cast(uint32_t, hi);
                *reinterpret_cast<uint2 *>(Orow + dv * 2) = w;
            }
        if (lse && g == 0) lse[qrow] = (m_run + log2f(l_tot)) * 0.6931471805599453f;
    } else if (q_ok) {   // partial result of this key range, merged by k_attn_merge
        const size_t prow = part_row();
        float *Po = a.part_o + prow * WK_D;
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int t = 0; t < 4; ++t)
                *reinterpret_cast<float4 *>(Po + 32 * b + 8 * t + 4 * g) =
                    float4{o[b][4 * t], o[b][4 * t + 1], o[b][4 * t + 2], o[b][4 * t + 3]};
        if (g == 0) { a.part_ml[prow * 2] = m_run; a.part_ml[prow * 2 + 1] = l_tot; }
    }
}

// ------------------------------------------------------------------------------------------
// Log-sum-exp only (a.O == NULL; query-based retrieval, paper Sec. 4.2 / App. C).  Without the
// P V product the matrix work halves while the exp2 work per key stays, so the kernel is bound
// by the VALU, not by the matrix cores.  It therefore drops the in-wave software pipeline of
// k_attn_bf16 (two S^T tiles in registers) for occupancy: under 128 VGPRs and with a 64 KB K
// ring, two workgroups = four waves per SIMD share a CU, and one wave's MFMAs run under the
// others' exp2; the workgroup's waves meet at a barrier only every second tile.  Same tile layout,
// loads and arithmetic (bf16-rounded probabilities summed by
// dot2) as the full kernel: the lse values are bit-identical to those wk_attention returns
// beside O.
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(512, 4) void k_lse_bf16(AttnArgs a) {
    extern __shared__ __attribute__((aligned(256))) char smem[];
    int c, h, qt, sp;
    if (!work_item(a, c, h, qt, sp)) return;
    const Window win = window_of(a, c);
    const int n_kv = win.n_kv;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, g = lane >> 5;
    const int q = qt * 256 + wave * 32 + col;
    const bool q_ok = q < a.N_q;
    const int q_ld = q_ok ? q : a.N_q - 1;
    const char *Qrow = a.Q + ((size_t)h * a.q_rows + a.q_off + q_ld) * 256;
    float *const out = win.lse + (size_t)h * a.q_rows + a.q_off + q;
    if (n_kv == 0) {
        if (q_ok && g == 0) *out = -INFINITY;
        return;
    }
    bf16x8 qb[8];
#pragma unroll
    for (int st = 0; st < 8; ++st) qb[st] = *reinterpret_cast<const bf16x8 *>(Qrow + (2 * st + g) * 16);
    const char *k_rd[8];   // as in k_attn_bf16: chunk 2*st + g of key col, slot c ^ (key & 15)
#pragma unroll
    for (int st = 0; st < 8; ++st) k_rd[st] = smem + col * 256 + (((2 * st + g) ^ (col & 15)) << 4);
    unsigned k_src[2];
    {
        const int r = lane >> 4, p = lane & 15;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int R = 4 * (2 * wave + i) + r;
            k_src[i] = R * 256 + ((p ^ (R & 15)) << 4);
        }
    }
    const char *Kh = win.K + (size_t)h * win.stride * 256;
    const unsigned last_off = (unsigned)(n_kv - 1) * 256u;
    char *const dma_dst = smem + wave * 2048;
    // 2 loads per wave and tile; tiles that end past the window (also the look-ahead past the last
    // tile) clamp their rows to the last key
    auto issue_tile = [&](int t, int slot) {
        const unsigned t_off = (unsigned)t * (kKeys * 256u);
        char *dst = dma_dst + slot * kTileBytes;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const unsigned ko = min(t_off + k_src[i], last_off + (k_src[i] & 255u));
            __builtin_amdgcn_global_load_lds(WK_GLB(Kh + ko), WK_LDS(dst + i * 1024), 16, 0, 0);
        }
    };
    float m_run = -INFINITY, l_run = 0.f;
    const float c_log2 = a.scale_log2;
    auto tile = [&](int byte_off, int kt, bool partial) {
        f32x16 s[2];
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[b][r] = 0.f;
#pragma unroll
        for (int st = 0; st < 8; ++st)
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                const bf16x8 ka = *reinterpret_cast<const bf16x8 *>(k_rd[st] + byte_off + b * 8192);
                s[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qb[st], s[b], 0, 0, 0);
            }
        if (partial) {
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = kt + 32 * b + 8 * (r >> 2) + 4 * g + (r & 3);
                    if (key >= n_kv) s[b][r] = -INFINITY;
                }
        }
        float mx[10];
#pragma unroll
        for (int i = 0; i < 10; ++i) {
            const int e = 3 * i;
            mx[i] = max3(s[e >> 4][e & 15], s[(e + 1) >> 4][(e + 1) & 15], s[(e + 2) >> 4][(e + 2) & 15]);
        }
        float m = max3(max3(mx[0], mx[1], mx[2]), max3(mx[3], mx[4], mx[5]), max3(mx[6], mx[7], mx[8]));
        m = max3(m, mx[9], fmaxf(s[1][14], s[1][15]));
        const float mt = max_across_halves(m) * c_log2;
        if (__any(mt > m_run + 8.0f)) {   // lazy rescale, as in k_attn_bf16
            const float m_new = fmaxf(m_run, mt);
            l_run *= __builtin_amdgcn_exp2f(m_run - m_new);
            m_run = m_new;
        }
        const float neg_m = -m_run;
        const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int e = 0; e < 16; e += 2) {
                const float p0 = __builtin_amdgcn_exp2f(fmaf(s[b][e], c_log2, neg_m));
                const float p1 = __builtin_amdgcn_exp2f(fmaf(s[b][e + 1], c_log2, neg_m));
                l_run = __builtin_amdgcn_fdot2_f32_bf16(__builtin_convertvector(f32x2{p0, p1}, bf16x2), ones, l_run,
                                                        false);
            }
    };
    const int n_full = n_kv / kKeys;   // full tiles; one partial tile may follow
    const bool tail = n_full * kKeys < n_kv;
    issue_tile(0, 0);
    issue_tile(1, 1);
    // One barrier per two tiles.  Before it, this wave's loads of tiles j and j+1 have landed
    // (vmcnt(0): nothing newer is in flight yet); behind it every wave is done with tiles j-2 and
    // j-1, whose slots tiles j+2 and j+3 may overwrite.
    auto open_pair = [&](int j, auto pos_tag) {
        constexpr int POS = decltype(pos_tag)::value;
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
        issue_tile(j + 2, (POS + 2) & 3);
        issue_tile(j + 3, (POS + 3) & 3);
    };
    using P0 = std::integral_constant<int, 0>;
    using P2 = std::integral_constant<int, 2>;
    const bool idle = qt * 256 + wave * 32 >= a.N_q;   // no valid query in this wave: loads and barriers only
    auto full_pair = [&](int j, auto pos_tag) {
        constexpr int POS = decltype(pos_tag)::value;
        open_pair(j, pos_tag);
        if (idle) return;
        tile(POS * kTileBytes, j * kKeys, false);
        tile((POS + 1) * kTileBytes, (j + 1) * kKeys, false);
    };
    // what is left after the full pairs: at most one full tile and the partial one
    auto last_pair = [&](int j, auto pos_tag, int full) {
        constexpr int POS = decltype(pos_tag)::value;
        open_pair(j, pos_tag);
        if (idle) return;
        if (full) {
            tile(POS * kTileBytes, j * kKeys, false);
            if (tail) tile((POS + 1) * kTileBytes, (j + 1) * kKeys, true);
        } else {
            tile(POS * kTileBytes, j * kKeys, true);
        }
    };
    int j = 0;
    for (; j + 4 <= n_full; j += 4) {
        full_pair(j, P0{});
        full_pair(j + 2, P2{});
    }
    int rest = n_full - j;   // 0..3 full tiles, then perhaps the partial one
    if (rest >= 2) {
        full_pair(j, P0{});
        j += 2;
        rest -= 2;
        if (rest || tail) last_pair(j, P2{}, rest);
    } else if (rest || tail) {
        last_pair(j, P0{}, rest);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);   // drain the clamped look-ahead loads before the LDS is released
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (q_ok && g == 0) *out = (m_run + log2f(l_tot)) * 0.6931471805599453f;
}

// Merge of the key-range splits: O = sum_s 2^(m_s - m) O_s / sum_s 2^(m_s - m) l_s, m = max_s m_s.
// 16 lanes per query row, 8 features each; fixed summation order.
template <int DT>
__global__ __launch_bounds__(256) void k_attn_merge(AttnArgs a) {
    const size_t row = (size_t)blockIdx.x * 16 + threadIdx.x / 16;   // h * q_rows + q
    const int sub = threadIdx.x % 16;
    const size_t rows = (size_t)a.H * a.q_rows;
    if (row >= rows) return;
    float m = -INFINITY;
    for (int s = 0; s < a.splits; ++s) m = fmaxf(m, a.part_ml[((size_t)s * rows + row) * 2]);
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    float l = 0.f;
    for (int s = 0; s < a.splits; ++s) {
        const float ms = a.part_ml[((size_t)s * rows + row) * 2];
        if (ms == -INFINITY) continue;   // empty split
        const float w = __builtin_amdgcn_exp2f(ms - m);
        l = fmaf(w, a.part_ml[((size_t)s * rows + row) * 2 + 1], l);
        const float4 *po = reinterpret_cast<const float4 *>(a.part_o + ((size_t)s * rows + row) * WK_D) + 2 * sub;
        const float4 x = po[0], y = po[1];
        acc[0] = fmaf(w, x.x, acc[0]); acc[1] = fmaf(w, x.y, acc[1]); acc[2] = fmaf(w, x.z, acc[2]); acc[3] = fmaf(w, x.w, acc[3]);
        acc[4] = fmaf(w, y.x, acc[4]); acc[5] = fmaf(w, y.y, acc[5]); acc[6] = fmaf(w, y.z, acc[6]); acc[7] = fmaf(w, y.w, acc[7]);
    }
    const float inv = l > 0.f ? 1.f / l : 0.f;
    if constexpr (DT == WK_BF16) {
        uint4 out;
        uint32_t *ow = reinterpret_cast<uint32_t *>(&out);
#pragma unroll
        for (int e = 0; e < 4; ++e)
            ow[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{acc[2 * e] * inv, acc[2 * e + 1] * inv}, bf16x2));
        reinterpret_cast<uint4 *>(a.O + row * 256)[sub] = out;
    } else {
        float4 *po = reinterpret_cast<float4 *>(a.O + row * 512) + 2 * sub;
        po[0] = float4{acc[0] * inv, acc[1] * inv, acc[2] * inv, acc[3] * inv};
        po[1] = float4{acc[4] * inv, acc[5] * inv, acc[6] * inv, acc[7] * inv};
    }
    if (a.lse && sub == 0) a.lse[row] = l > 0.f ? (m + log2f(l)) * 0.6931471805599453f : -INFINITY;
}

// Key-range splits for grids that would leave compute units idle: the count that fills the 256 CUs best
// over whole rounds of workgroups; ties go to fewer.  Up to 8 splits of at least 8 tiles each; windows
// long enough to leave 128 tiles per split may use up to 16.  (Query tiles that walk the same slice of a
// head's keys run side by side and share it through the L2, which cutting the work into equal runs
// regardless of item boundaries would give up: that was measured 5 to 14 % slower.)
constexpr int kMaxSplits = 16;

int choose_splits(int items, int n_tiles) {
    int best = 1;
    double best_util = 0.0;
    for (int s = 1; s <= kMaxSplits && (s == 1 || n_tiles / s >= (s <= 8 ? 8 : 128)); ++s) {
        const int wgs = items * s;
        const double util = (double)wgs / (double)(((wgs + 255) / 256) * 256);
        if (util > best_util + 0.02) { best_util = util; best = s; }
    }
    return best;
}

// How a bf16 launch is laid out, chosen by a cost model in units of one 64-key step of a 256-query
// workgroup (measured: a 128-query workgroup, one wave per SIMD, takes 0.69 of that per step; a workgroup's
// fill and drain cost about 4 steps; the merge of s partial results costs about 6 steps plus its traffic):
//   waves = 8, splits = 1   one workgroup per (head, 256 queries): large grids
//   waves = 8, splits > 1   the key range split over workgroups and merged: small grids, long windows
//   waves = 4               one workgroup per (head, 128 queries), twice as many of them: small grids, short
//                           windows, or no workspace for partial results
struct LaunchPlan { int waves, splits; };

LaunchPlan plan_bf16(int H, int N_q, int N_kv, bool workspace_ok) {
    const int n_tiles = (N_kv + 63) / 64;
    const long long items8 = (long long)H * ((N_q + 255) / 256), items4 = (long long)H * ((N_q + 127) / 128);
    auto rounds = [](long long wgs) { return (double)((wgs + 255) / 256); };
    const double plain8 = rounds(items8) * (n_tiles + 4);
    const double plain4 = rounds(items4) * (n_tiles + 4) * 0.69;
    LaunchPlan best{8, 1};
    double best_cost = plain8;
    if (plain4 < 0.97 * best_cost) { best = LaunchPlan{4, 1}; best_cost = plain4; }
    if (workspace_ok && items8 <= 0x7fffffff / kMaxSplits) {
        const int s = choose_splits((int)items8, n_tiles);
        if (s > 1) {
            const double merge = 6.0 + 2.0 * s * H * (double)N_q * 516.0 / 5e12 / 1.76e-6;
            const double split8 = rounds(items8 * s) * ((double)n_tiles / s + 4) + merge;
            if (split8 < 0.97 * best_cost) best = LaunchPlan{8, s};
        }
    }
    return best;
}

// fp32 kernel: four of its workgroups fit a compute unit, so up to 1024 are resident; the smallest split
// count that reaches that, at most 16 and leaving at least 4 tiles of 32 keys per split.
int choose_splits_f32(long long items, int n_tiles) {
    int s = 1;
    while (s < kMaxSplits && items * s < 1024 && n_tiles / (s + 1) >= 4) ++s;
    return s;
}

size_t split_workspace_bytes(int H, int N_q, int splits) {
    const size_t rows = (size_t)splits * H * N_q;
    return wk::align_up(rows * WK_D * sizeof(float), 256) + wk::align_up(rows * 2 * sizeof(float), 256);
}

// k_attn_bf16 uses more than the default 64 KB of dynamic LDS: raise its limit once per device and
// process (not a stream operation, so a first call under graph capture is fine too).
wk_status allow_large_lds() {
    static std::atomic<uint64_t> done{0};
    int dev;
    if (wk::device_needs_setup(done, dev)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&k_attn_bf16<8, false, false>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kSmemBytes) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void *>(&k_attn_bf16<4, false, false>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kSmemBytes) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void *>(&k_attn_bf16<8, true, false>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kSmemBytes) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void *>(&k_attn_bf16<8, false, true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kSmemBytes) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void *>(&k_attn_bf16<4, false, true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kSmemBytes) != hipSuccess)
            return WK_ERR_HIP;
        wk::mark_device(done, dev);
    }
    return WK_OK;
}

template <int WAVES>
wk_status launch_bf16(AttnArgs a, int splits, void *workspace, hipStream_t st) {
    const int q_per_wg = WAVES * 32;
    a.n_qtiles = (a.N_q + q_per_wg - 1) / q_per_wg;
    a.splits = splits;
    a.part_o = reinterpret_cast<float *>(workspace);
    a.part_ml = reinterpret_cast<float *>(reinterpret_cast<char *>(workspace) +
                                          wk::align_up((size_t)a.splits * a.H * a.N_q * WK_D * sizeof(float), 256));
    const long long items = (long long)a.H * a.n_qtiles * a.splits * (a.n_chunks > 0 ? a.n_chunks : 1);
    if (items + kXcds > 0x7fffffffLL) return WK_ERR_UNSUPPORTED;
    a.per_xcd = (int)((items + kXcds - 1) / kXcds);
    const wk_status lds_rc = allow_large_lds();
    if (lds_rc != WK_OK) return lds_rc;
    if (a.O) {
        hipLaunchKernelGGL((k_attn_bf16<WAVES, false, false>), dim3(a.per_xcd * kXcds), dim3(WAVES * 64), kSmemBytes, st, a,
                           SubTable{});
    } else {
        if (WAVES != 8) return WK_ERR_UNSUPPORTED;   // the log-sum-exp kernel is laid out for 256-query workgroups
        hipLaunchKernelGGL(k_lse_bf16, dim3(a.per_xcd * kXcds), dim3(512), kVRing, st, a);
    }
    WK_LAUNCH_CHECK();
    if (a.splits > 1) {
        const size_t rows = (size_t)a.H * a.N_q;
        hipLaunchKernelGGL(k_attn_merge<WK_BF16>, dim3((unsigned)((rows + 15) / 16)), dim3(256), 0, st, a);
        WK_LAUNCH_CHECK();
    }
    return WK_OK;
}

}  // namespace

extern "C" wk_status wk_attention(const void *Q, const void *K_win, const void *V_win, void *O, float *lse,
                                  int32_t H, int32_t N_q, int32_t N_kv, int32_t d, int32_t kv_row_stride,
                                  int32_t dtype, float scale, const int32_t *n_kv_dev, void *workspace,
                                  size_t workspace_bytes, void *hip_stream) {
    if (!Q || !K_win) return WK_ERR_INVALID_ARG;
    if (O ? !V_win : !lse) return WK_ERR_INVALID_ARG;   // O == NULL: log-sum-exp only, V is not read
    if (H < 1 || N_q < 0 || d < 1) return WK_ERR_INVALID_ARG;
    if (dtype != WK_F32 && dtype != WK_BF16) return WK_ERR_INVALID_ARG;
    if (!(scale >= 0.f) || std::isinf(scale)) return WK_ERR_INVALID_ARG;
    if (d != WK_D) return WK_ERR_UNSUPPORTED;
    if (N_kv < 1 || N_kv > kv_row_stride) return WK_ERR_SHAPE;
    if (dtype == WK_BF16 && N_kv > kMaxRowsBf16) return WK_ERR_UNSUPPORTED;   // 32-bit byte offsets inside a head
    if (N_q == 0) return WK_OK;
    if ((long long)H * ((N_q + 31) / 32) > 0x7fffffffLL / kMaxSplits) return WK_ERR_UNSUPPORTED;   // grid size
    AttnArgs a;
    a.Q = reinterpret_cast<const char *>(Q);
    a.K = reinterpret_cast<const char *>(K_win);
    a.V = reinterpret_cast<const char *>(V_win);
    a.O = reinterpret_cast<char *>(O);
    a.lse = lse;
    a.H = H; a.N_q = N_q; a.N_kv = N_kv; a.kv_row_stride = kv_row_stride;
    const float sc = scale == 0.f ? 1.f / std::sqrt((float)d) : scale;
    a.scale_log2 = sc * 1.4426950408889634f;
    a.n_kv_dev = n_kv_dev;
    a.splits = 1;
    a.part_o = nullptr;
    a.part_ml = nullptr;
    a.k_table = nullptr;
    a.n_tok = nullptr;
    a.n_chunks = 0;
    a.q_rows = N_q; a.q_off = 0; a.kv_start = 0; a.part_slot = -1;
    a.v_table = nullptr; a.ids = nullptr; a.n_ids = nullptr; a.R_max = 0; a.store_M = 0; a.max_tok = 0;
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    if (dtype == WK_F32) {
        const int q_per_wg = kF32Waves * 32;
        a.n_qtiles = (N_q + q_per_wg - 1) / q_per_wg;
        const long long items1 = (long long)H * a.n_qtiles;
        a.splits = O ? choose_splits_f32(items1, (N_kv + kF32Keys - 1) / kF32Keys) : 1;
        if (a.splits > 1 && (!workspace || workspace_bytes < split_workspace_bytes(H, N_q, a.splits) ||
                             reinterpret_cast<uintptr_t>(workspace) % 256 != 0))
            a.splits = 1;
        a.part_o = reinterpret_cast<float *>(workspace);
        a.part_ml = reinterpret_cast<float *>(reinterpret_cast<char *>(workspace) +
                                              wk::align_up((size_t)a.splits * H * N_q * WK_D * sizeof(float), 256));
        const long long items = items1 * a.splits;
        if (items + kXcds > 0x7fffffffLL) return WK_ERR_UNSUPPORTED;
        a.per_xcd = (int)((items + kXcds - 1) / kXcds);
        hipLaunchKernelGGL(k_attn_f32<false>, dim3(a.per_xcd * kXcds), dim3(kF32Waves * 64), 0, st, a, SubTable{});
        WK_LAUNCH_CHECK();
        if (a.splits > 1) {
            const size_t rows = (size_t)H * N_q;
            hipLaunchKernelGGL(k_attn_merge<WK_F32>, dim3((unsigned)((rows + 15) / 16)), dim3(256), 0, st, a);
            WK_LAUNCH_CHECK();
        }
        return WK_OK;
    }
    if (!O) return launch_bf16<8>(a, 1, nullptr, st);   // log-sum-exp only
    const bool ws_aligned = workspace && reinterpret_cast<uintptr_t>(workspace) % 256 == 0;
    // the plan with a workspace, if the one given is big enough for it; otherwise the best plan without
    LaunchPlan plan = plan_bf16(H, N_q, N_kv, ws_aligned);
    if (plan.splits > 1 && workspace_bytes < split_workspace_bytes(H, N_q, plan.splits))
        plan = plan_bf16(H, N_q, N_kv, false);
    return plan.waves == 8 ? launch_bf16<8>(a, plan.splits, workspace, st) : launch_bf16<4>(a, 1, nullptr, st);
}

namespace {

// One launch of the attention kernel for the dtype, exactly as the arguments say: no choice of
// key-range splits, no merge.
wk_status launch_plain(AttnArgs a, int dtype, hipStream_t st) {
    a.splits = 1;
    if (dtype == WK_F32) {
        a.n_qtiles = (a.N_q + kF32Waves * 32 - 1) / (kF32Waves * 32);
        a.per_xcd = (a.H * a.n_qtiles + kXcds - 1) / kXcds;
        hipLaunchKernelGGL(k_attn_f32<false>, dim3(a.per_xcd * kXcds), dim3(kF32Waves * 64), 0, st, a, SubTable{});
    } else {
        a.n_qtiles = (a.N_q + 255) / 256;
        a.per_xcd = (a.H * a.n_qtiles + kXcds - 1) / kXcds;
        const wk_status rc = allow_large_lds();
        if (rc != WK_OK) return rc;
        hipLaunchKernelGGL((k_attn_bf16<8, false, false>), dim3(a.per_xcd * kXcds), dim3(512), kSmemBytes, st, a,
                           SubTable{});
    }
    WK_LAUNCH_CHECK();
    return WK_OK;
}

}  // namespace

extern "C" size_t wk_attention_block_causal_workspace_bytes(int32_t H, int32_t N_q) {
    if (H < 1 || N_q < 1) return 0;
    return split_workspace_bytes(H, N_q, 2);
}

// Frame-level causal mask inside the chunk being denoised, as two key ranges per query frame
// whose partial (O, max, sum) results k_attn_merge combines: range A = window rows up to and
// including the query's own frame of the chunk (all queries of a frame share it), range B = the
// rows behind the chunk (shared by all queries).  The attention loop runs unchanged; a workgroup is
// only told which queries, which rows and which partial slot are its own -- through a table of up
// to 8 such (queries, rows, slot) entries served by one grid, or, for more frames than that, by
// one launch per entry.
extern "C" wk_status wk_attention_block_causal(const void *Q, const void *K_win, const void *V_win, void *O,
                                               float *lse, int32_t H, int32_t N_q, int32_t N_kv, int32_t d,
                                               int32_t kv_row_stride, int32_t dtype, float scale,
                                               const int32_t *n_kv_dev, int32_t denoise_row0, int32_t frame_T,
                                               void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (!Q || !K_win || !V_win || !O) return WK_ERR_INVALID_ARG;
    if (H < 1 || N_q < 0 || d < 1 || frame_T < 1 || denoise_row0 < 0) return WK_ERR_INVALID_ARG;
    if (dtype != WK_F32 && dtype != WK_BF16) return WK_ERR_INVALID_ARG;
    if (!(scale >= 0.f) || std::isinf(scale)) return WK_ERR_INVALID_ARG;
    if (d != WK_D) return WK_ERR_UNSUPPORTED;
    if (N_kv < 1 || N_kv > kv_row_stride) return WK_ERR_SHAPE;
    if (N_q % frame_T != 0 || (int64_t)denoise_row0 + N_q > (int64_t)N_kv) return WK_ERR_SHAPE;
    if (dtype == WK_BF16 && N_kv > kMaxRowsBf16) return WK_ERR_UNSUPPORTED;   // 32-bit byte offsets inside a head
    if (N_q == 0) return WK_OK;
    if (!workspace || workspace_bytes < split_workspace_bytes(H, N_q, 2) ||
        reinterpret_cast<uintptr_t>(workspace) % 256 != 0)
        return WK_ERR_WORKSPACE;
    const size_t row_bytes = WK_D * wk::esize(dtype);
    AttnArgs a;
    a.Q = reinterpret_cast<const char *>(Q);
    a.K = reinterpret_cast<const char *>(K_win);
    a.V = reinterpret_cast<const char *>(V_win);
    a.O = reinterpret_cast<char *>(O);
    a.lse = lse;
    a.H = H; a.N_q = N_q; a.N_kv = N_kv; a.kv_row_stride = kv_row_stride;
    const float sc = scale == 0.f ? 1.f / std::sqrt((float)d) : scale;
    a.scale_log2 = sc * 1.4426950408889634f;
    a.n_kv_dev = n_kv_dev;
    a.splits = 1;
    a.part_o = reinterpret_cast<float *>(workspace);
    a.part_ml = reinterpret_cast<float *>(reinterpret_cast<char *>(workspace) +
                                          wk::align_up((size_t)2 * H * N_q * WK_D * sizeof(float), 256));
    a.k_table = nullptr; a.n_tok = nullptr; a.n_chunks = 0;
    a.q_rows = N_q; a.q_off = 0; a.kv_start = 0; a.part_slot = -1;
    a.v_table = nullptr; a.ids = nullptr; a.n_ids = nullptr; a.R_max = 0; a.store_M = 0; a.max_tok = 0;
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);

    const int frames = N_q / frame_T;
    const int start = denoise_row0 + N_q;
    if (frames + 1 <= kMaxSub) {
        // all ranges in one grid: entry 0 = the rows behind the chunk for every query (the long
        // items first), entries 1.. = the prefix up to frame f for that frame's queries
        const int q_per_wg = dtype == WK_F32 ? kF32Waves * 32 : 256;
        SubTable t;
        t.n = frames + 1;
        t.s[0] = SubLaunch{0, N_q, (N_q + q_per_wg - 1) / q_per_wg, start, N_kv - start, start, 1};
        t.per_head = t.s[0].n_qtiles;
        for (int f = 0; f < frames; ++f) {
            t.s[f + 1] = SubLaunch{f * frame_T, frame_T, (frame_T + q_per_wg - 1) / q_per_wg, 0,
                                   denoise_row0 + (f + 1) * frame_T, 0, 0};
            t.per_head += t.s[f + 1].n_qtiles;
        }
        for (int e = t.n; e < kMaxSub; ++e) t.s[e] = SubLaunch{0, 0, 0, 0, 0, 0, 0};
        AttnArgs g = a;
        if ((long long)H * t.per_head + kXcds > 0x7fffffffLL) return WK_ERR_UNSUPPORTED;
        g.per_xcd = (H * t.per_head + kXcds - 1) / kXcds;
        g.n_qtiles = 0;
        if (dtype == WK_F32) {
            hipLaunchKernelGGL(k_attn_f32<true>, dim3(g.per_xcd * kXcds), dim3(kF32Waves * 64), 0, st, g, t);
        } else {
            const wk_status lrc = allow_large_lds();
            if (lrc != WK_OK) return lrc;
            hipLaunchKernelGGL((k_attn_bf16<8, true, false>), dim3(g.per_xcd * kXcds), dim3(512), kSmemBytes, st, g, t);
        }
        WK_LAUNCH_CHECK();
    } else {
        // more frames than the table holds: the same ranges as separate launches
        AttnArgs b = a;   // the rows behind the chunk, every query
        b.K += (size_t)start * row_bytes;
        b.V += (size_t)start * row_bytes;
        b.N_kv = N_kv - start;
        b.kv_start = start;
        b.part_slot = 1;
        wk_status rc = launch_plain(b, dtype, st);
        if (rc != WK_OK) return rc;
        for (int f = 0; f < frames; ++f) {   // rows up to the end of frame f of the chunk, that frame's queries
            AttnArgs p = a;
            p.N_q = frame_T;
            p.q_off = f * frame_T;
            p.N_kv = denoise_row0 + (f + 1) * frame_T;
            p.part_slot = 0;
            rc = launch_plain(p, dtype, st);
            if (rc != WK_OK) return rc;
        }
    }
    AttnArgs m = a;
    m.splits = 2;
    const size_t rows = (size_t)H * N_q;
    if (dtype == WK_F32)
        hipLaunchKernelGGL(k_attn_merge<WK_F32>, dim3((unsigned)((rows + 15) / 16)), dim3(256), 0, st, m);
    else
        hipLaunchKernelGGL(k_attn_merge<WK_BF16>, dim3((unsigned)((rows + 15) / 16)), dim3(256), 0, st, m);
    WK_LAUNCH_CHECK();
    return WK_OK;
}

extern "C" wk_status wk_chunk_lse(const wk_store_desc *store, const void *Q, int32_t N_q, float scale,
                                  float *lse_out, void *hip_stream) {
    if (!store || !Q || !lse_out) return WK_ERR_INVALID_ARG;
    if (store->M < 0 || store->H < 1 || N_q < 0 || store->max_tok < 0) return WK_ERR_INVALID_ARG;
    if (store->dtype != WK_F32 && store->dtype != WK_BF16) return WK_ERR_INVALID_ARG;
    if (!(scale >= 0.f) || std::isinf(scale)) return WK_ERR_INVALID_ARG;
    if (store->d != WK_D) return WK_ERR_UNSUPPORTED;
    if (store->dtype == WK_BF16 && store->max_tok > kMaxRowsBf16) return WK_ERR_UNSUPPORTED;   // 32-bit byte offsets
    if (store->M == 0 || N_q == 0) return WK_OK;
    if (!store->K_ptr || !store->n_tok) return WK_ERR_INVALID_ARG;
    AttnArgs a;
    a.Q = reinterpret_cast<const char *>(Q);
    a.K = a.V = nullptr;
    a.O = nullptr;
    a.lse = lse_out;
    a.H = store->H; a.N_q = N_q; a.N_kv = 0; a.kv_row_stride = 0;
    const float sc = scale == 0.f ? 1.f / std::sqrt((float)WK_D) : scale;
    a.scale_log2 = sc * 1.4426950408889634f;
    a.n_kv_dev = nullptr;
    a.splits = 1;
    a.part_o = nullptr;
    a.part_ml = nullptr;
    a.k_table = store->K_ptr;
    a.n_tok = store->n_tok;
    a.n_chunks = store->M;
    a.q_rows = N_q; a.q_off = 0; a.kv_start = 0; a.part_slot = -1;
    a.v_table = nullptr; a.ids = nullptr; a.n_ids = nullptr; a.R_max = 0; a.store_M = 0; a.max_tok = store->max_tok;
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    const int q_per_wg = (store->dtype == WK_F32 ? kF32Waves : 8) * 32;
    const long long items = (long long)store->M * store->H * ((N_q + q_per_wg - 1) / q_per_wg);
    if (items + kXcds > 0x7fffffffLL) return WK_ERR_UNSUPPORTED;
    if (store->dtype == WK_F32) {
        a.n_qtiles = (N_q + q_per_wg - 1) / q_per_wg;
        a.per_xcd = (int)((items + kXcds - 1) / kXcds);
        hipLaunchKernelGGL(k_attn_f32<false>, dim3(a.per_xcd * kXcds), dim3(kF32Waves * 64), 0, st, a, SubTable{});
        WK_LAUNCH_CHECK();
        return WK_OK;
    }
    return launch_bf16<8>(a, 1, nullptr, st);
}

extern "C" wk_status wk_attention_in_place(const void *Q, const void *K_native, const void *V_native,
                                           int32_t n_native, int32_t native_row_stride,
                                           const wk_store_desc *store, const int32_t *ids, const int32_t *n_ids,
                                           int32_t R_max, void *O, float *lse, int32_t N_q, float scale,
                                           void *hip_stream) {
    if (!store || !Q || !O) return WK_ERR_INVALID_ARG;
    if (store->M < 0 || store->H < 1 || store->max_tok < 0 || N_q < 0 || R_max < 0 || n_native < 0)
        return WK_ERR_INVALID_ARG;
    if (store->dtype != WK_F32 && store->dtype != WK_BF16) return WK_ERR_INVALID_ARG;
    if (!(scale >= 0.f) || std::isinf(scale)) return WK_ERR_INVALID_ARG;
    if (n_native > 0 && (!K_native || !V_native)) return WK_ERR_INVALID_ARG;
    if (R_max > 0 && store->M > 0 && (!ids || !store->K_ptr || !store->V_ptr || !store->n_tok))
        return WK_ERR_INVALID_ARG;
    if (store->d != WK_D || store->dtype != WK_BF16) return WK_ERR_UNSUPPORTED;
    if (R_max > kMaxSegments - 1) return WK_ERR_UNSUPPORTED;
    if (n_native >= (1 << 23) || store->max_tok >= (1 << 23)) return WK_ERR_UNSUPPORTED;   // 32-bit byte offsets
    if (n_native > native_row_stride) return WK_ERR_SHAPE;
    if (N_q == 0) return WK_OK;
    if ((long long)store->H * ((N_q + 255) / 256) + kXcds > 0x7fffffffLL) return WK_ERR_UNSUPPORTED;
    AttnArgs a;
    a.Q = reinterpret_cast<const char *>(Q);
    a.K = reinterpret_cast<const char *>(K_native);
    a.V = reinterpret_cast<const char *>(V_native);
    a.O = reinterpret_cast<char *>(O);
    a.lse = lse;
    a.H = store->H; a.N_q = N_q; a.N_kv = n_native; a.kv_row_stride = native_row_stride;
    const float sc = scale == 0.f ? 1.f / std::sqrt((float)WK_D) : scale;
    a.scale_log2 = sc * 1.4426950408889634f;
    a.n_kv_dev = nullptr;
    a.splits = 1;
    a.part_o = nullptr;
    a.part_ml = nullptr;
    a.k_table = store->K_ptr;
    a.n_tok = store->n_tok;
    a.n_chunks = 0;
    a.q_rows = N_q; a.q_off = 0; a.kv_start = 0; a.part_slot = -1;
    a.v_table = store->V_ptr; a.ids = ids; a.n_ids = n_ids; a.R_max = store->M > 0 ? R_max : 0; a.store_M = store->M;
    a.max_tok = store->max_tok;
    // 256- or 128-query workgroups, by the cost model of wk_attention for the longest window the ids can give
    const long long longest = (long long)n_native + (long long)a.R_max * store->max_tok;
    const LaunchPlan plan = plan_bf16(a.H, N_q, (int)(longest < 64 ? 64 : (longest > 0x7fffffff ? 0x7fffffff : longest)), false);
    const int q_per_wg = plan.waves * 32;
    a.n_qtiles = (N_q + q_per_wg - 1) / q_per_wg;
    if ((long long)a.H * a.n_qtiles + kXcds > 0x7fffffffLL) return WK_ERR_UNSUPPORTED;
    a.per_xcd = (a.H * a.n_qtiles + kXcds - 1) / kXcds;
    const wk_status rc = allow_large_lds();
    if (rc != WK_OK) return rc;
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    if (plan.waves == 8)
        hipLaunchKernelGGL((k_attn_bf16<8, false, true>), dim3(a.per_xcd * kXcds), dim3(512), kSmemBytes, st, a, SubTable{});
    else
        hipLaunchKernelGGL((k_attn_bf16<4, false, true>), dim3(a.per_xcd * kXcds), dim3(256), kSmemBytes, st, a, SubTable{});
    WK_LAUNCH_CHECK();
    return WK_OK;
}

extern "C" size_t wk_attention_workspace_bytes(int32_t H, int32_t N_q, int32_t N_kv, int32_t dtype) {
    if (H < 1 || N_q < 1 || N_kv < 1 || (dtype != WK_BF16 && dtype != WK_F32)) return 0;
    if ((long long)H * ((N_q + 31) / 32) > 0x7fffffffLL / kMaxSplits) return 0;
    if (dtype == WK_F32) {
        const int s = choose_splits_f32((long long)H * ((N_q + kF32Waves * 32 - 1) / (kF32Waves * 32)),
                                        (N_kv + kF32Keys - 1) / kF32Keys);
        return s > 1 ? split_workspace_bytes(H, N_q, s) : 0;
    }
    const LaunchPlan plan = plan_bf16(H, N_q, N_kv, true);
    return plan.splits > 1 ? split_workspace_bytes(H, N_q, plan.splits) : 0;
}

extern "C" const char *wk_status_string(wk_status s) {
    switch (s) {
    case WK_OK: return "ok";
    case WK_ERR_INVALID_ARG: return "invalid argument";
    case WK_ERR_SHAPE: return "inconsistent shape";
    case WK_ERR_RATIO: return "keep ratio out of range";
    case WK_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case WK_ERR_UNSUPPORTED: return "unsupported configuration";
    case WK_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}
