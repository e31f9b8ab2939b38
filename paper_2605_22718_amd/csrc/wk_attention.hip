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

#include "wk_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

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
};

constexpr int kXcds = 8;

// Workgroups are handed to the 8 XCDs round-robin by their linear id.  Work items are numbered
// head-major (all query tiles of head 0, then head 1, ...); giving XCD x the contiguous range
// [x*per_xcd, (x+1)*per_xcd) keeps the query tiles that stream the same head's K/V on one XCD,
// so that head's window is fetched from HBM once into that XCD's L2 instead of once per tile.
__device__ inline bool work_item(const AttnArgs &a, int &h, int &qt) {
    const int lin = blockIdx.x;
    const int w = (lin % kXcds) * a.per_xcd + lin / kXcds;
    if (lin / kXcds >= a.per_xcd || w >= a.H * a.n_qtiles) return false;
    h = w / a.n_qtiles;
    qt = w % a.n_qtiles;
    return true;
}

__device__ inline int window_length(const AttnArgs &a) {
    int n = a.N_kv;
    if (a.n_kv_dev) {
        const int m = *a.n_kv_dev;
        n = m < n ? m : n;
    }
    return n < 0 ? 0 : n;
}

// ------------------------------------------------------------------------------------------
// fp32: v_mfma_f32_32x32x2_f32, 4 waves x 32 queries per workgroup, 32-key tiles.
// ------------------------------------------------------------------------------------------
constexpr int kF32Waves = 4;
constexpr int kF32Keys = 32;
constexpr int kF32KPitch = WK_D + 4;  // floats; 16 lanes x 16 B then cover all 64 banks
constexpr int kF32VPitch = WK_D + 8;  // rows 4 apart land 32 banks apart

__global__ __launch_bounds__(kF32Waves * 64) void k_attn_f32(AttnArgs a) {
    __shared__ float Ks[kF32Keys * kF32KPitch];
    __shared__ float Vs[kF32Keys * kF32VPitch];
    int h, qt;
    if (!work_item(a, h, qt)) return;
    const int n_kv = window_length(a);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, g = lane >> 5;
    const int q = qt * (kF32Waves * 32) + wave * 32 + col;
    const bool q_ok = q < a.N_q;
    const int q_ld = q_ok ? q : a.N_q - 1;
    const float *Qrow = reinterpret_cast<const float *>(a.Q) + ((size_t)h * a.N_q + q_ld) * WK_D;
    float *Orow = reinterpret_cast<float *>(a.O) + ((size_t)h * a.N_q + q_ld) * WK_D;

    if (n_kv == 0) {
        if (q_ok) {
            for (int c = g * 64; c < g * 64 + 64; c += 4) *reinterpret_cast<float4 *>(Orow + c) = float4{0, 0, 0, 0};
            if (a.lse && g == 0) a.lse[(size_t)h * a.N_q + q] = -INFINITY;
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

    const float *Kh = reinterpret_cast<const float *>(a.K) + (size_t)h * a.kv_row_stride * WK_D;
    const float *Vh = reinterpret_cast<const float *>(a.V) + (size_t)h * a.kv_row_stride * WK_D;

    for (int kt = 0; kt < n_kv; kt += kF32Keys) {
        __syncthreads();  // previous tile fully consumed
#pragma unroll
        for (int i = 0; i < (kF32Keys * WK_D / 4) / (kF32Waves * 64); ++i) {
            const int x = tid + i * (kF32Waves * 64);
            const int row = x / (WK_D / 4), c4 = x % (WK_D / 4);
            float4 kv = float4{0, 0, 0, 0}, vv = float4{0, 0, 0, 0};
            if (kt + row < n_kv) {
                kv = *reinterpret_cast<const float4 *>(Kh + (size_t)(kt + row) * WK_D + 4 * c4);
                vv = *reinterpret_cast<const float4 *>(Vh + (size_t)(kt + row) * WK_D + 4 * c4);
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
            s[r] = key < n_kv ? s[r] * a.scale_log2 : -INFINITY;
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
    if (q_ok) {
        const float inv = 1.f / l_tot;
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int dv = 32 * b + 8 * t + 4 * g;
                *reinterpret_cast<float4 *>(Orow + dv) =
                    float4{o[b][4 * t] * inv, o[b][4 * t + 1] * inv, o[b][4 * t + 2] * inv, o[b][4 * t + 3] * inv};
            }
        if (a.lse && g == 0) a.lse[(size_t)h * a.N_q + q] = (m_run + log2f(l_tot)) * 0.6931471805599453f;
    }
}

// ------------------------------------------------------------------------------------------
// bf16: v_mfma_f32_32x32x16_bf16, WAVES waves x 32 queries per workgroup, 64-key tiles,
// K and V^T tiles double-buffered in LDS.
// ------------------------------------------------------------------------------------------
constexpr int kKeys = 64;                    // keys per tile
constexpr int kKTileBytes = kKeys * 256;     // K tile: [64 keys][16 chunks of 16 B], chunk c of key k at c ^ (k & 15)
constexpr int kVTileBytes = WK_D * kKeys * 2;  // V^T tile: [128 features][64 key slots]
constexpr int kStageBytes = kKTileBytes + kVTileBytes;

// Byte offset of 16-byte chunk c (0..7) of feature row dv in the V^T tile.  Rows are 128 B, two
// rows per 256-byte bank sweep; XOR-ing the chunk with (dv >> 1) & 7 spreads 16 consecutive rows
// over all 16 chunk slots.
__device__ inline int vt_chunk_off(int dv, int c) { return dv * 128 + ((c ^ ((dv >> 1) & 7)) << 4); }

// Slot of key kk (0..63 within the tile) in a V^T row.  Key 32*b + 8*(2*t2 + tt) + 4*g + j sits at
// slot 32*b + 16*t2 + 8*g + 4*tt + j, so that the 8 accumulator registers 8*t2 .. 8*t2+7 of
// S^T block b held by lane half g are 8 consecutive slots: one 16-byte read per MFMA operand.
__device__ inline int vt_slot(int kk) {
    const int b = kk >> 5, t2 = (kk >> 4) & 1, tt = (kk >> 3) & 1, g = (kk >> 2) & 1, j = kk & 3;
    return 32 * b + 16 * t2 + 8 * g + 4 * tt + j;
}

template <int WAVES>
struct TileRegs {
    static constexpr int kThreads = WAVES * 64;
    static constexpr int kKVec = (kKeys * 16) / kThreads;      // 16-byte K chunks per thread
    static constexpr int kVTask = (kKeys / 4) * 32 / kThreads;  // 4x4 V blocks per thread
    uint4 k[kKVec];
    uint2 v[kVTask][4];
};

template <int WAVES>
__device__ inline void load_tile(TileRegs<WAVES> &t, const char *Kh, const char *Vh, int kt, int n_kv, int tid) {
#pragma unroll
    for (int i = 0; i < TileRegs<WAVES>::kKVec; ++i) {
        const int x = tid + i * TileRegs<WAVES>::kThreads;
        const int key = x >> 4, c = x & 15;
        t.k[i] = uint4{0, 0, 0, 0};
        if (kt + key < n_kv) t.k[i] = *reinterpret_cast<const uint4 *>(Kh + (size_t)(kt + key) * 256 + c * 16);
    }
#pragma unroll
    for (int i = 0; i < TileRegs<WAVES>::kVTask; ++i) {
        const int x = tid + i * TileRegs<WAVES>::kThreads;
        const int kg = x >> 5, dg = x & 31;  // keys 4*kg .. 4*kg+3, features 4*dg .. 4*dg+3
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int key = kt + 4 * kg + j;
            t.v[i][j] = uint2{0, 0};  // rows past the window must be zero: their weight is 0, not their value
            if (key < n_kv) t.v[i][j] = *reinterpret_cast<const uint2 *>(Vh + (size_t)key * 256 + dg * 8);
        }
    }
}

template <int WAVES>
__device__ inline void store_tile(const TileRegs<WAVES> &t, char *stage, int tid) {
#pragma unroll
    for (int i = 0; i < TileRegs<WAVES>::kKVec; ++i) {
        const int x = tid + i * TileRegs<WAVES>::kThreads;
        const int key = x >> 4, c = x & 15;
        *reinterpret_cast<uint4 *>(stage + key * 256 + ((c ^ (key & 15)) << 4)) = t.k[i];
    }
    char *vt = stage + kKTileBytes;
#pragma unroll
    for (int i = 0; i < TileRegs<WAVES>::kVTask; ++i) {
        const int x = tid + i * TileRegs<WAVES>::kThreads;
        const int kg = x >> 5, dg = x & 31;
        const int slot = vt_slot(4 * kg);  // multiple of 4
        // 4x4 transpose of 16-bit elements: row j = key, column i = feature
        const uint32_t r0x = t.v[i][0].x, r1x = t.v[i][1].x, r2x = t.v[i][2].x, r3x = t.v[i][3].x;
        const uint32_t r0y = t.v[i][0].y, r1y = t.v[i][1].y, r2y = t.v[i][2].y, r3y = t.v[i][3].y;
        uint2 c0, c1, c2, c3;  // feature 4*dg + 0..3, keys j = 0..3
        c0.x = __builtin_amdgcn_perm(r1x, r0x, 0x05040100u); c0.y = __builtin_amdgcn_perm(r3x, r2x, 0x05040100u);
        c1.x = __builtin_amdgcn_perm(r1x, r0x, 0x07060302u); c1.y = __builtin_amdgcn_perm(r3x, r2x, 0x07060302u);
        c2.x = __builtin_amdgcn_perm(r1y, r0y, 0x05040100u); c2.y = __builtin_amdgcn_perm(r3y, r2y, 0x05040100u);
        c3.x = __builtin_amdgcn_perm(r1y, r0y, 0x07060302u); c3.y = __builtin_amdgcn_perm(r3y, r2y, 0x07060302u);
        const int c = slot >> 3, half = (slot >> 2) & 1;
        const int dv = 4 * dg;
        *reinterpret_cast<uint2 *>(vt + vt_chunk_off(dv + 0, c) + 8 * half) = c0;
        *reinterpret_cast<uint2 *>(vt + vt_chunk_off(dv + 1, c) + 8 * half) = c1;
        *reinterpret_cast<uint2 *>(vt + vt_chunk_off(dv + 2, c) + 8 * half) = c2;
        *reinterpret_cast<uint2 *>(vt + vt_chunk_off(dv + 3, c) + 8 * half) = c3;
    }
}

// Two waves per SIMD in both shapes (one 8-wave workgroup, or two 4-wave workgroups per CU), so
// that one wave's softmax (VALU) overlaps the other's MFMAs: at most 256 VGPRs per lane.
template <int WAVES>
__global__ __launch_bounds__(WAVES * 64, 2) void k_attn_bf16(AttnArgs a) {
    extern __shared__ __attribute__((aligned(256))) char smem[];  // 2 stages of (K tile, V^T tile)
    int h, qt;
    if (!work_item(a, h, qt)) return;
    const int n_kv = window_length(a);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, g = lane >> 5;
    const int q = qt * (WAVES * 32) + wave * 32 + col;
    const bool q_ok = q < a.N_q;
    const int q_ld = q_ok ? q : a.N_q - 1;
    const char *Qrow = a.Q + ((size_t)h * a.N_q + q_ld) * 256;
    char *Orow = a.O + ((size_t)h * a.N_q + q_ld) * 256;

    if (n_kv == 0) {
        if (q_ok) {
            for (int c = g * 8; c < g * 8 + 8; ++c) reinterpret_cast<uint4 *>(Orow)[c] = uint4{0, 0, 0, 0};
            if (a.lse && g == 0) a.lse[(size_t)h * a.N_q + q] = -INFINITY;
        }
        return;
    }

    // B operand of S^T = K Q^T, step s: features 16*s + 8*g .. +7 of this lane's query
    bf16x8 qb[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) qb[s] = *reinterpret_cast<const bf16x8 *>(Qrow + (2 * s + g) * 16);

    f32x16 o[4];
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[b][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    const char *Kh = a.K + (size_t)h * a.kv_row_stride * 256;
    const char *Vh = a.V + (size_t)h * a.kv_row_stride * 256;
    const int n_tiles = (n_kv + kKeys - 1) / kKeys;

    TileRegs<WAVES> regs;
    load_tile<WAVES>(regs, Kh, Vh, 0, n_kv, tid);
    store_tile<WAVES>(regs, smem, tid);
    __syncthreads();

    for (int it = 0; it < n_tiles; ++it) {
        const int kt = it * kKeys;
        const char *stage = smem + (it & 1) * kStageBytes;
        const bool more = it + 1 < n_tiles;
        if (more) load_tile<WAVES>(regs, Kh, Vh, kt + kKeys, n_kv, tid);

        // S^T blocks: 2 x (32 keys x 32 queries)
        f32x16 s[2];
#pragma unroll
        for (int b = 0; b < 2; ++b) {
#pragma unroll
            for (int r = 0; r < 16; ++r) s[b][r] = 0.f;
            const int key = 32 * b + col;
#pragma unroll
            for (int st = 0; st < 8; ++st) {
                const bf16x8 ka =
                    *reinterpret_cast<const bf16x8 *>(stage + key * 256 + (((2 * st + g) ^ (key & 15)) << 4));
                s[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qb[st], s[b], 0, 0, 0);
            }
        }
        // online softmax in base 2; register r of block b is key kt + 32*b + 8*(r/4) + 4*g + r%4
        float m_tile = -INFINITY;
        if (kt + kKeys <= n_kv) {
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    s[b][r] *= a.scale_log2;
                    m_tile = fmaxf(m_tile, s[b][r]);
                }
        } else {
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = kt + 32 * b + 8 * (r >> 2) + 4 * g + (r & 3);
                    s[b][r] = key < n_kv ? s[b][r] * a.scale_log2 : -INFINITY;
                    m_tile = fmaxf(m_tile, s[b][r]);
                }
        }
        m_tile = fmaxf(m_tile, __shfl_xor(m_tile, 32));
        const float m_new = fmaxf(m_run, m_tile);  // finite: every tile holds at least one valid key
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        m_run = m_new;
        // P^T operands: registers 8*t2 .. 8*t2+7 of block b -> k step 2*b + t2
        bf16x8 pb[4];
        float l_tile = 0.f;
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int t2 = 0; t2 < 2; ++t2) {
#pragma unroll
                for (int e = 0; e < 8; e += 2) {
                    const float p0 = __builtin_amdgcn_exp2f(s[b][8 * t2 + e] - m_new);
                    const float p1 = __builtin_amdgcn_exp2f(s[b][8 * t2 + e + 1] - m_new);
                    const bf16x2 pk = __builtin_convertvector(f32x2{p0, p1}, bf16x2);
                    pb[2 * b + t2][e] = pk[0];
                    pb[2 * b + t2][e + 1] = pk[1];
                    // the row sum uses the rounded probabilities, the ones the P V product sees
                    l_tile += (float)pk[0] + (float)pk[1];
                }
            }
        l_run = l_run * alpha + l_tile;
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[b][r] *= alpha;
        // O^T += V^T P^T
        const char *vt = stage + kKTileBytes;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const bf16x8 va = *reinterpret_cast<const bf16x8 *>(vt + vt_chunk_off(32 * b + col, 2 * ks + g));
                o[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[ks], o[b], 0, 0, 0);
            }

        if (more) store_tile<WAVES>(regs, smem + ((it + 1) & 1) * kStageBytes, tid);
        __syncthreads();
    }

    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (q_ok) {
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
        if (a.lse && g == 0) a.lse[(size_t)h * a.N_q + q] = (m_run + log2f(l_tot)) * 0.6931471805599453f;
    }
}

template <int WAVES>
wk_status launch_bf16(AttnArgs a, hipStream_t st) {
    const int q_per_wg = WAVES * 32;
    a.n_qtiles = (a.N_q + q_per_wg - 1) / q_per_wg;
    const int items = a.H * a.n_qtiles;
    a.per_xcd = (items + kXcds - 1) / kXcds;
    hipLaunchKernelGGL(k_attn_bf16<WAVES>, dim3(a.per_xcd * kXcds), dim3(WAVES * 64), 2 * kStageBytes, st, a);
    WK_LAUNCH_CHECK();
    return WK_OK;
}

}  // namespace

extern "C" wk_status wk_attention(const void *Q, const void *K_win, const void *V_win, void *O, float *lse,
                                  int32_t H, int32_t N_q, int32_t N_kv, int32_t d, int32_t kv_row_stride,
                                  int32_t dtype, float scale, const int32_t *n_kv_dev, void *hip_stream) {
    if (!Q || !K_win || !V_win || !O) return WK_ERR_INVALID_ARG;
    if (H < 1 || N_q < 0 || d < 1) return WK_ERR_INVALID_ARG;
    if (dtype != WK_F32 && dtype != WK_BF16) return WK_ERR_INVALID_ARG;
    if (!(scale >= 0.f) || std::isinf(scale)) return WK_ERR_INVALID_ARG;
    if (d != WK_D) return WK_ERR_UNSUPPORTED;
    if (N_kv < 1 || N_kv > kv_row_stride) return WK_ERR_SHAPE;
    if (N_q == 0) return WK_OK;
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
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    if (dtype == WK_F32) {
        const int q_per_wg = kF32Waves * 32;
        a.n_qtiles = (N_q + q_per_wg - 1) / q_per_wg;
        const int items = H * a.n_qtiles;
        a.per_xcd = (items + kXcds - 1) / kXcds;
        hipLaunchKernelGGL(k_attn_f32, dim3(a.per_xcd * kXcds), dim3(kF32Waves * 64), 0, st, a);
        WK_LAUNCH_CHECK();
        return WK_OK;
    }
    // 256-query workgroups (8 waves, two per SIMD) when that still gives every CU work, else 128.
    const int items8 = H * ((N_q + 255) / 256);
    return items8 >= 256 ? launch_bf16<8>(a, st) : launch_bf16<4>(a, st);
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
