// World Retrieval (paper Sec. 4.2, Eq. 4) with the camera/action distance of Sec. 5.1.
//
// One workgroup, fp64 throughout.  M is a few hundred at most for minute-long rollouts, so the
// step is latency-bound: distances -> two block reductions for the normalisers -> every thread
// ranks its own candidates by counting how many (D, id) pairs precede them (all-pairs from LDS,
// broadcast reads), and the candidates of rank < R write themselves to slot `rank`.  That gives
// the Top-k already ordered, with ties to the lower chunk id, and no sort.
#include <cmath>

#include "wk_internal.h"

namespace {

constexpr int kThreads = 1024;
constexpr int kPerThread = WK_SCORE_MAX_CHUNKS / kThreads;  // 4

struct Pose5 { float v[5]; };

// Rotation angle of R_a^T R_b for R = R_y(yaw) R_x(pitch).  The relative rotation depends only on
// the yaw difference D and the pitch difference e:  cos(phi/2) = |cos(D/2) cos(e/2)|.  Evaluated
// as phi = 2 atan2(sin(phi/2), cos(phi/2)) with sin^2(phi/2) = sin^2(D/2) + cos^2(D/2) sin^2(e/2),
// which stays accurate for small and for near-pi angles.
__device__ inline double geodesic(double yaw_a, double pitch_a, double yaw_b, double pitch_b) {
    const double hD = 0.5 * (yaw_b - yaw_a), he = 0.5 * (pitch_b - pitch_a);
    const double sD = sin(hD), cD = cos(hD), se = sin(he), ce = cos(he);
    const double s2 = sD * sD + cD * cD * se * se;
    return 2.0 * atan2(sqrt(s2), fabs(cD * ce));
}

enum { RED_MAX = 0, RED_MIN = 1, RED_SUM = 2 };

template <int OP>
__device__ inline double combine(double a, double b) {
    if constexpr (OP == RED_MAX) return fmax(a, b);
    else if constexpr (OP == RED_MIN) return fmin(a, b);
    else return a + b;
}

template <int OP>
__device__ inline double block_reduce(double x, double *scratch /*[kThreads/64]*/) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) x = combine<OP>(x, __shfl_xor(x, o));
    __syncthreads();
    if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = x;
    __syncthreads();
    double r = scratch[0];
#pragma unroll
    for (int i = 1; i < kThreads / 64; ++i) r = combine<OP>(r, scratch[i]);
    return r;
}

__device__ inline double normalise(double v, int mode, double mx, double mn, double sum, int M) {
    if (mode == WK_NORM_MAX) return mx > 0.0 ? v / mx : 0.0;
    if (mode == WK_NORM_MINMAX) return mx > mn ? (v - mn) / (mx - mn) : 0.0;
    return sum > 0.0 ? v / (sum / (double)M) : 0.0;
}

__global__ __launch_bounds__(kThreads) void k_score_chunks(const float *__restrict__ poses, int M, Pose5 cur,
                                                           int norm_mode, int R, int32_t *__restrict__ ids_out,
                                                           double *__restrict__ dist_out,
                                                           int32_t *__restrict__ n_found) {
    __shared__ double D[WK_SCORE_MAX_CHUNKS];
    __shared__ double scratch[kThreads / 64];
    const int tid = threadIdx.x;
    const int found = R < M ? R : M;
    if (tid == 0) *n_found = found;
    for (int r = found + tid; r < R; r += kThreads) {
        ids_out[r] = -1;
        if (dist_out) dist_out[r] = INFINITY;
    }
    if (M == 0) return;

    double dt[kPerThread], dr[kPerThread];
    double t_max = 0.0, t_min = INFINITY, t_sum = 0.0, r_max = 0.0, r_min = INFINITY, r_sum = 0.0;
#pragma unroll
    for (int e = 0; e < kPerThread; ++e) {
        const int i = tid + e * kThreads;
        dt[e] = dr[e] = 0.0;
        if (i < M) {
            const float *a = poses + (size_t)i * 5;
            double s = 0.0;
#pragma unroll
            for (int c = 0; c < 3; ++c) {
                const double df = (double)cur.v[c] - (double)a[c];
                s += df * df;
            }
            dt[e] = s;
            dr[e] = geodesic((double)cur.v[3], (double)cur.v[4], (double)a[3], (double)a[4]);
            t_max = fmax(t_max, dt[e]); t_min = fmin(t_min, dt[e]); t_sum += dt[e];
            r_max = fmax(r_max, dr[e]); r_min = fmin(r_min, dr[e]); r_sum += dr[e];
        }
    }
    t_max = block_reduce<RED_MAX>(t_max, scratch);
    r_max = block_reduce<RED_MAX>(r_max, scratch);
    if (norm_mode == WK_NORM_MINMAX) {
        t_min = block_reduce<RED_MIN>(t_min, scratch);
        r_min = block_reduce<RED_MIN>(r_min, scratch);
    } else if (norm_mode == WK_NORM_MEAN) {
        t_sum = block_reduce<RED_SUM>(t_sum, scratch);
        r_sum = block_reduce<RED_SUM>(r_sum, scratch);
    }
    double mine[kPerThread];
#pragma unroll
    for (int e = 0; e < kPerThread; ++e) {
        const int i = tid + e * kThreads;
        mine[e] = normalise(dt[e], norm_mode, t_max, t_min, t_sum, M) +
                  normalise(dr[e], norm_mode, r_max, r_min, r_sum, M);
        if (i < M) D[i] = mine[e];
    }
    __syncthreads();
    if (R == 0) return;
#pragma unroll
    for (int e = 0; e < kPerThread; ++e) {
        const int i = tid + e * kThreads;
        if (i >= M) continue;
        const double di = mine[e];
        int rank = 0;
        for (int j = 0; j < M; ++j) {
            const double dj = D[j];
            rank += (dj < di || (dj == di && j < i)) ? 1 : 0;
        }
        if (rank < found) {
            ids_out[rank] = i;
            if (dist_out) dist_out[rank] = di;
        }
    }
}

}  // namespace

extern "C" wk_status wk_score_chunks(const float *poses, int32_t M, const float *cur_pose, int32_t norm_mode,
                                     int32_t R, int32_t *ids_out, double *dist_out, int32_t *n_found,
                                     void *hip_stream) {
    if (M < 0 || R < 0 || !cur_pose || !n_found) return WK_ERR_INVALID_ARG;
    if (M > 0 && !poses) return WK_ERR_INVALID_ARG;
    if (R > 0 && !ids_out) return WK_ERR_INVALID_ARG;
    if (norm_mode != WK_NORM_MAX && norm_mode != WK_NORM_MINMAX && norm_mode != WK_NORM_MEAN)
        return WK_ERR_INVALID_ARG;
    if (M > WK_SCORE_MAX_CHUNKS) return WK_ERR_UNSUPPORTED;
    Pose5 cur;
    for (int c = 0; c < 5; ++c) cur.v[c] = cur_pose[c];
    hipLaunchKernelGGL(k_score_chunks, dim3(1), dim3(kThreads), 0, reinterpret_cast<hipStream_t>(hip_stream),
                       poses, (int)M, cur, (int)norm_mode, (int)R, ids_out, dist_out, n_found);
    WK_LAUNCH_CHECK();
    return WK_OK;
}

// ---- query-based retrieval (paper Sec. 4.2, App. C) -------------------------------------------------
//
// Input: lse[c][r] = log sum_k exp(q_r . k / sqrt(d)) over the keys k of stored chunk c, for every
// (head, query) row r -- what wk_attention writes as `lse` when run over one chunk.  In a softmax
// over the keys of all M chunks, chunk c receives mass exp(lse[c][r] - logsumexp_c' lse[c'][r]) from
// row r; the relevance of a chunk is the mean of that mass over the rows.  fp64 throughout.
namespace {

constexpr int kQThreads = 256;

__global__ __launch_bounds__(kQThreads) void k_query_mass_partial(const float *__restrict__ lse, int M,
                                                                  long long n_rows, double *__restrict__ partial) {
    __shared__ double acc[kQThreads / 64][WK_QUERY_MAX_CHUNKS];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int c = lane; c < M; c += 64) acc[wave][c] = 0.0;
    // (each wave only touches its own row of acc: no barrier needed until the end)
    for (long long r0 = (long long)blockIdx.x * kQThreads; r0 < n_rows; r0 += (long long)gridDim.x * kQThreads) {
        const long long r = r0 + tid;
        const bool ok = r < n_rows;
        double mx = -INFINITY;
        if (ok)
            for (int c = 0; c < M; ++c) mx = fmax(mx, (double)lse[(size_t)c * n_rows + r]);
        double sum = 0.0;
        if (ok && mx > -INFINITY)
            for (int c = 0; c < M; ++c) sum += exp((double)lse[(size_t)c * n_rows + r] - mx);
        const double L = mx + log(sum);   // -inf or NaN for rows that see no key at all: they are skipped
        for (int c = 0; c < M; ++c) {
            double w = 0.0;
            if (ok && sum > 0.0) w = exp((double)lse[(size_t)c * n_rows + r] - L);
#pragma unroll
            for (int o = 32; o >= 1; o >>= 1) w += __shfl_xor(w, o);
            if (lane == 0) acc[wave][c] += w;
        }
    }
    __syncthreads();
    for (int c = tid; c < M; c += kQThreads) {
        double s = 0.0;
#pragma unroll
        for (int w = 0; w < kQThreads / 64; ++w) s += acc[w][c];
        partial[(size_t)blockIdx.x * M + c] = s;
    }
}

// mass[c] = sum of the blocks' partial sums / n_rows; the min(R, M) largest, ties to the lower id
__global__ __launch_bounds__(kThreads) void k_query_topk(const double *__restrict__ partial, int n_blocks, int M,
                                                         long long n_rows, int R, double *__restrict__ mass_all,
                                                         int32_t *__restrict__ ids_out,
                                                         double *__restrict__ mass_out,
                                                         int32_t *__restrict__ n_found) {
    __shared__ double mass[WK_QUERY_MAX_CHUNKS];
    const int tid = threadIdx.x;
    const int found = R < M ? R : M;
    if (tid == 0) *n_found = found;
    for (int r = found + tid; r < R; r += kThreads) {
        ids_out[r] = -1;
        if (mass_out) mass_out[r] = -INFINITY;
    }
    if (M == 0) return;
    // one wave per chunk: lanes sum interleaved blocks, then a fixed-shape tree over the lanes
    for (int c = tid >> 6; c < M; c += kThreads / 64) {
        double s = 0.0;
        for (int b = tid & 63; b < n_blocks; b += 64) s += partial[(size_t)b * M + c];
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) s += __shfl_xor(s, o);
        s /= (double)n_rows;
        if ((tid & 63) == 0) {
            mass[c] = s;
            mass_all[c] = s;
        }
    }
    __syncthreads();
    for (int c = tid; c < M; c += kThreads) {
        const double mc = mass[c];
        int rank = 0;
        for (int j = 0; j < M; ++j) {
            const double mj = mass[j];
            rank += (mj > mc || (mj == mc && j < c)) ? 1 : 0;
        }
        if (rank < found) {
            ids_out[rank] = c;
            if (mass_out) mass_out[rank] = mc;
        }
    }
}

int query_blocks(long long n_rows) {
    const long long b = (n_rows + kQThreads - 1) / kQThreads;
    return (int)(b < 1 ? 1 : (b > 1024 ? 1024 : b));
}

}  // namespace

extern "C" size_t wk_score_chunks_query_workspace_bytes(int32_t M, int64_t n_rows) {
    if (M < 0 || M > WK_QUERY_MAX_CHUNKS || n_rows < 1) return 0;
    const size_t m = (size_t)(M > 0 ? M : 1);
    return wk::align_up(m * sizeof(double), 256) + wk::align_up((size_t)query_blocks(n_rows) * m * sizeof(double), 256);
}

extern "C" wk_status wk_score_chunks_query(const float *lse, int32_t M, int64_t n_rows, int32_t R, int32_t *ids_out,
                                           double *mass_out, int32_t *n_found, void *workspace,
                                           size_t workspace_bytes, void *hip_stream) {
    if (M < 0 || R < 0 || n_rows < 1 || !n_found) return WK_ERR_INVALID_ARG;
    if (M > 0 && !lse) return WK_ERR_INVALID_ARG;
    if (R > 0 && !ids_out) return WK_ERR_INVALID_ARG;
    if (M > WK_QUERY_MAX_CHUNKS) return WK_ERR_UNSUPPORTED;
    const size_t need = wk_score_chunks_query_workspace_bytes(M, n_rows);
    if (!workspace || workspace_bytes < need || reinterpret_cast<uintptr_t>(workspace) % 256 != 0)
        return WK_ERR_WORKSPACE;
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    double *mass_all = reinterpret_cast<double *>(workspace);
    double *partial = reinterpret_cast<double *>(reinterpret_cast<char *>(workspace) +
                                                 wk::align_up((size_t)(M > 0 ? M : 1) * sizeof(double), 256));
    const int nb = query_blocks(n_rows);
    if (M > 0) {
        hipLaunchKernelGGL(k_query_mass_partial, dim3(nb), dim3(kQThreads), 0, st, lse, (int)M, (long long)n_rows,
                           partial);
        WK_LAUNCH_CHECK();
    }
    hipLaunchKernelGGL(k_query_topk, dim3(1), dim3(kThreads), 0, st, partial, nb, (int)M, (long long)n_rows, (int)R,
                       mass_all, ids_out, mass_out, n_found);
    WK_LAUNCH_CHECK();
    return WK_OK;
}

extern "C" wk_status wk_accumulate_actions(const int32_t *labels, int32_t n, float step, float dangle,
                                           float pitch_limit, float *poses_out) {
    if (n < 0 || (n > 0 && (!labels || !poses_out))) return WK_ERR_INVALID_ARG;
    for (int i = 0; i < n; ++i)
        if (labels[i] < 0 || labels[i] > 7) return WK_ERR_INVALID_ARG;
    // state in double; the table of per-label increments keeps the loop branch-free
    double pos[3] = {0, 0, 0}, yaw = 0, pitch = 0;
    const double st = step, da = dangle, lim = pitch_limit;
    static const double fwd_c[8] = {1, 0, -1, 0, 0, 0, 0, 0};    // along the heading
    static const double right_c[8] = {0, -1, 0, 1, 0, 0, 0, 0};  // along the right vector
    static const double yaw_c[8] = {0, 0, 0, 0, -1, 1, 0, 0};
    static const double pitch_c[8] = {0, 0, 0, 0, 0, 0, -1, 1};
    for (int i = 0; i < n; ++i) {
        const int a = labels[i];
        const double sy = std::sin(yaw), cy = std::cos(yaw);
        pos[0] += st * (fwd_c[a] * sy + right_c[a] * cy);
        pos[2] += st * (fwd_c[a] * cy - right_c[a] * sy);
        yaw += da * yaw_c[a];
        pitch = std::fmin(lim, std::fmax(-lim, pitch + da * pitch_c[a]));
        float *o = poses_out + (size_t)i * 5;
        o[0] = (float)pos[0]; o[1] = (float)pos[1]; o[2] = (float)pos[2];
        o[3] = (float)yaw; o[4] = (float)pitch;
    }
    return WK_OK;
}
