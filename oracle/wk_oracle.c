/*
 * CPU oracle for the WorldKV hot path -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Plain C, fp64, written from the paper; deliberately slow and literal so it
 * can be checked against the paper by eye.  It shares no code with the HIP
 * library and must never be called by it.  Only the test-suite, the smoke
 * check and the benchmark's cpu_baseline leg may load this file.
 *
 * Inputs are the same dtype-rounded arrays the GPU receives (fp32 or bf16 bit
 * patterns); every value is widened to double before any arithmetic.
 *
 *   wko_compress_scores / wko_select_lowest / wko_compress
 *        World Compression, Sec. 4.3, Eq. 5 and the rule that the lowest-scoring P% are kept.
 *   wko_keep_count
 *        token counts of a compressed chunk (Sec. 4.3, Sec. 5.1, Sec. 5.4).
 *   wko_score_chunks
 *        camera/action retrieval distance (Sec. 5.1, implementation details)
 *        and Top-k of Eq. 4 (Sec. 4.2).
 *   wko_score_chunks_query
 *        query-based retrieval (Sec. 4.2, App. C): chunks ranked by the attention mass
 *        of the current queries.  The paper does not define the score further; the
 *        reading here (joint softmax over all candidates, mean over heads and
 *        queries) is pinned by invariants only: parity unpinned.
 *   wko_accumulate_actions
 *        discrete actions -> pseudo-pose (Sec. 5.1).  The step constants are
 *        this build's own choice (the paper gives none): parity unpinned
 *        against the authors' constants, pinned only by invariants.
 *   wko_gather
 *        insertion of retrieved chunks into the window, verbatim (Sec. 1,
 *        Sec. 4.2).
 *   wko_attention
 *        softmax attention over the assembled window (Sec. 4.2, Sec. 4.3).
 *   wko_attention_block_causal
 *        the same with a frame-level causal mask inside the chunk being denoised: an option
 *        (the paper states no mask; frame-causal attention inside a chunk is a property some
 *        autoregressive video backbones of Sec. 3 have).  Parity unpinned against any model;
 *        pinned against a library masked softmax and against wko_attention on reduced windows.
 *
 * Readings of silent points (each repeated where it is used):
 *   - zero-norm key: its cosine terms are 0;
 *   - ties in Eq. 5 scores / retrieval distances: lower index first;
 *   - normalisation of a distance term over the candidate set (Sec. 5.1): divide by the maximum
 *     over candidates (variants: min-max, mean).  Parity with the authors'
 *     normalisation is unpinned;
 *   - rotation = R_y(yaw) * R_x(pitch), no roll; geodesic = rotation angle of
 *     R_cur^T R_i;
 *   - Eq. 5 does not mention heads: by default a token's key is the concatenation of its
 *     head slices (one index set per layer); per-head scoring is the variant.  Parity with
 *     the authors' choice is unpinned (the two modes are pinned to each other by a
 *     reshaped-input equivalence).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { WKO_F32 = 0, WKO_BF16 = 1 };
enum { WKO_HEADS_SHARED = 0, WKO_HEADS_INDEPENDENT = 1 };
enum { WKO_ANCHOR_FIRST_FRAME = 0, WKO_ANCHOR_EXTERNAL = 1 };
enum { WKO_RATIO_CHUNK = 0, WKO_RATIO_NONANCHOR = 1 };
enum { WKO_NORM_MAX = 0, WKO_NORM_MINMAX = 1, WKO_NORM_MEAN = 2 };

static size_t esize_of(int dtype) { return dtype == WKO_BF16 ? 2 : 4; }

static double load_elem(const void *base, int dtype, size_t i)
{
    if (dtype == WKO_BF16) {
        uint32_t bits = ((uint32_t)((const uint16_t *)base)[i]) << 16;
        float f;
        memcpy(&f, &bits, 4);
        return (double)f;
    }
    return (double)((const float *)base)[i];
}

/* ------------------------------------------------------------------------ */
/* token counts                                                              */
/* ------------------------------------------------------------------------ */

/* Sec. 4.3: a chunk keeps all anchor tokens plus n_keep of the N_c pooled
 * non-anchor tokens.  ratio_kind CHUNK: rho is the kept fraction of the whole
 * stored chunk; NONANCHOR: rho is P, the kept fraction of non-anchor tokens
 * (P = 25% gives 3T -> 1.5T).  Counts round half away from zero.
 * With an external anchor the anchor is not stored and all F*T tokens are
 * candidates.  Returns 0 and writes n_out (stored tokens) and n_keep, or -1
 * if the ratio asks for fewer tokens than the anchor or more than the chunk. */
int wko_keep_count(double rho, int ratio_kind, int anchor_mode, int F, int T,
                   int64_t *n_out, int64_t *n_keep)
{
    if (F < 1 || T < 1 || !(rho >= 0.0) || !(rho <= 1.0)) return -1;
    int64_t n_anchor = anchor_mode == WKO_ANCHOR_EXTERNAL ? 0 : T;
    int64_t n_cand = (int64_t)F * T - n_anchor;
    int64_t keep, out;
    if (ratio_kind == WKO_RATIO_CHUNK) {
        out = llround(rho * (double)((int64_t)F * T));
        keep = out - n_anchor;
    } else {
        keep = llround(rho * (double)n_cand);
        out = keep + n_anchor;
    }
    if (keep < 0 || keep > n_cand || out < 1) return -1;
    *n_out = out;
    *n_keep = keep;
    return 0;
}

/* ------------------------------------------------------------------------ */
/* World Compression                                                         */
/* ------------------------------------------------------------------------ */

/* Eq. 5 as the literal double sum.  K is [H][n_tok][d] with n_tok = F*T.
 * FIRST_FRAME: anchors are tokens 0..T-1 of K, candidates tokens T..F*T-1.
 * EXTERNAL:    anchors are K_anchor [H][T][d], candidates all tokens of K.
 * HEADS_SHARED: one score list, the key vector of a token is the
 * concatenation of its H head slices; HEADS_INDEPENDENT: H lists, Eq. 5 per
 * head.  scores is [G][N_c].  cand_sel (may be NULL) restricts the evaluation to n_sel
 * candidate indices; the other entries of scores are left untouched. */
int wko_compress_scores(const void *K, const void *K_anchor, int dtype, int H, int d, int T, int F,
                        int head_mode, int anchor_mode, const int32_t *cand_sel, int64_t n_sel,
                        double *scores)
{
    if (!K || !scores || H < 1 || d < 1 || T < 1 || F < 1) return -1;
    if (anchor_mode == WKO_ANCHOR_EXTERNAL && !K_anchor) return -1;
    const int64_t n_tok = (int64_t)F * T;
    const int64_t first_cand = anchor_mode == WKO_ANCHOR_EXTERNAL ? 0 : T;
    const int64_t n_cand = n_tok - first_cand;
    const int G = head_mode == WKO_HEADS_INDEPENDENT ? H : 1;
    const int hg = head_mode == WKO_HEADS_INDEPENDENT ? 1 : H; /* heads per group */
    const int64_t D = (int64_t)hg * d;                         /* length of a key vector */
    const void *A = anchor_mode == WKO_ANCHOR_EXTERNAL ? K_anchor : K;
    const int64_t a_tok = anchor_mode == WKO_ANCHOR_EXTERNAL ? T : n_tok; /* rows per head in A */

    double *anc = (double *)malloc(sizeof(double) * (size_t)T * D);
    double *cand = (double *)malloc(sizeof(double) * (size_t)(n_cand > 0 ? n_cand : 1) * D);
    double *anc_norm = (double *)malloc(sizeof(double) * (size_t)T);
    if (!anc || !cand || !anc_norm) { free(anc); free(cand); free(anc_norm); return -2; }

    for (int g = 0; g < G; ++g) {
        /* widen this group's anchor and candidate key vectors to double */
        for (int64_t i = 0; i < T; ++i)
            for (int hh = 0; hh < hg; ++hh) {
                int h = head_mode == WKO_HEADS_INDEPENDENT ? g : hh;
                for (int c = 0; c < d; ++c)
                    anc[i * D + (int64_t)hh * d + c] = load_elem(A, dtype, ((size_t)h * a_tok + i) * d + c);
            }
        for (int64_t j = 0; j < n_cand; ++j)
            for (int hh = 0; hh < hg; ++hh) {
                int h = head_mode == WKO_HEADS_INDEPENDENT ? g : hh;
                for (int c = 0; c < d; ++c)
                    cand[j * D + (int64_t)hh * d + c] =
                        load_elem(K, dtype, ((size_t)h * n_tok + first_cand + j) * d + c);
            }
        for (int64_t i = 0; i < T; ++i) {
            double s = 0.0;
            for (int64_t c = 0; c < D; ++c) s += anc[i * D + c] * anc[i * D + c];
            anc_norm[i] = sqrt(s);
        }
        const int64_t n_eval = cand_sel ? n_sel : n_cand;
#pragma omp parallel for schedule(static)
        for (int64_t e = 0; e < n_eval; ++e) {
            const int64_t j = cand_sel ? cand_sel[e] : e;
            if (j < 0 || j >= n_cand) continue;
            const double *kj = cand + j * D;
            double nj = 0.0;
            for (int64_t c = 0; c < D; ++c) nj += kj[c] * kj[c];
            nj = sqrt(nj);
            double acc = 0.0;
            for (int64_t i = 0; i < T; ++i) {
                const double *ki = anc + i * D;
                double dot = 0.0;
                for (int64_t c = 0; c < D; ++c) dot += kj[c] * ki[c];
                double cosv = (nj < 1e-30 || anc_norm[i] < 1e-30) ? 0.0 : dot / (nj * anc_norm[i]);
                acc += cosv;
            }
            scores[(size_t)g * n_cand + j] = acc / (double)T;
        }
    }
    free(anc); free(cand); free(anc_norm);
    return 0;
}

typedef struct { double s; int32_t idx; } wko_pair;

static int cmp_pair(const void *a, const void *b)
{
    const wko_pair *x = (const wko_pair *)a, *y = (const wko_pair *)b;
    if (x->s < y->s) return -1;
    if (x->s > y->s) return 1;
    return (x->idx > y->idx) - (x->idx < y->idx);
}

static int cmp_i32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/* The lowest-scoring P% are the ones retained (Sec. 4.3): the n_keep lowest scores, ties to the lower index;
 * the kept indices are returned in ascending order. */
int wko_select_lowest(const double *s, int64_t n, int64_t n_keep, int32_t *idx_out)
{
    if (n_keep < 0 || n_keep > n) return -1;
    wko_pair *p = (wko_pair *)malloc(sizeof(wko_pair) * (size_t)(n > 0 ? n : 1));
    if (!p) return -2;
    for (int64_t i = 0; i < n; ++i) { p[i].s = s[i]; p[i].idx = (int32_t)i; }
    qsort(p, (size_t)n, sizeof(wko_pair), cmp_pair);
    for (int64_t i = 0; i < n_keep; ++i) idx_out[i] = p[i].idx;
    qsort(idx_out, (size_t)n_keep, sizeof(int32_t), cmp_i32);
    free(p);
    return 0;
}

/* Whole compression of one chunk-layer: scores, selection, and the compacted
 * chunk = anchor tokens followed by the retained tokens in their original
 * order, K and V pruned with the same indices, rows copied bit for bit.
 * kept_idx is [G][n_out] (indices into the chunk's F*T tokens), K_out/V_out
 * are [H][n_out][d].  scores_out ([G][N_c]) may be NULL. */
int wko_compress(const void *K, const void *V, const void *K_anchor, int dtype, int H, int d, int T, int F,
                 int head_mode, int anchor_mode, double rho, int ratio_kind,
                 int32_t *kept_idx, void *K_out, void *V_out, double *scores_out)
{
    int64_t n_out, n_keep;
    if (wko_keep_count(rho, ratio_kind, anchor_mode, F, T, &n_out, &n_keep) != 0) return -3;
    const int64_t n_tok = (int64_t)F * T;
    const int64_t first_cand = anchor_mode == WKO_ANCHOR_EXTERNAL ? 0 : T;
    const int64_t n_cand = n_tok - first_cand;
    const int G = head_mode == WKO_HEADS_INDEPENDENT ? H : 1;
    double *sc = scores_out ? scores_out : (double *)malloc(sizeof(double) * (size_t)G * (n_cand > 0 ? n_cand : 1));
    if (!sc) return -2;
    int rc = wko_compress_scores(K, K_anchor, dtype, H, d, T, F, head_mode, anchor_mode, NULL, 0, sc);
    if (rc == 0) {
        for (int g = 0; g < G && rc == 0; ++g) {
            int32_t *idx = kept_idx + (size_t)g * n_out;
            for (int64_t i = 0; i < first_cand; ++i) idx[i] = (int32_t)i;
            rc = wko_select_lowest(sc + (size_t)g * n_cand, n_cand, n_keep, idx + first_cand);
            for (int64_t i = 0; i < n_keep; ++i) idx[first_cand + i] += (int32_t)first_cand;
        }
    }
    if (rc == 0 && K_out && V_out) {
        const size_t row = (size_t)d * esize_of(dtype);
        for (int h = 0; h < H; ++h) {
            const int32_t *idx = kept_idx + (size_t)(head_mode == WKO_HEADS_INDEPENDENT ? h : 0) * n_out;
            for (int64_t r = 0; r < n_out; ++r) {
                memcpy((char *)K_out + ((size_t)h * n_out + r) * row,
                       (const char *)K + ((size_t)h * n_tok + idx[r]) * row, row);
                memcpy((char *)V_out + ((size_t)h * n_out + r) * row,
                       (const char *)V + ((size_t)h * n_tok + idx[r]) * row, row);
            }
        }
    }
    if (!scores_out) free(sc);
    return rc;
}

/* ------------------------------------------------------------------------ */
/* World Retrieval                                                           */
/* ------------------------------------------------------------------------ */

static void rot_yaw_pitch(double yaw, double pitch, double R[3][3])
{
    /* R = R_y(yaw) * R_x(pitch): yaw about the up (y) axis, pitch about the right (x) axis */
    double cy = cos(yaw), sy = sin(yaw), cp = cos(pitch), sp = sin(pitch);
    double Ry[3][3] = {{cy, 0, sy}, {0, 1, 0}, {-sy, 0, cy}};
    double Rx[3][3] = {{1, 0, 0}, {0, cp, -sp}, {0, sp, cp}};
    for (int i = 0; i < 3; ++i)
        for (int j = 0; j < 3; ++j) {
            double s = 0.0;
            for (int k = 0; k < 3; ++k) s += Ry[i][k] * Rx[k][j];
            R[i][j] = s;
        }
}

/* Geodesic distance on SO(3): the rotation angle of Ra^T Rb, in [0, pi]. */
double wko_geodesic(double yaw_a, double pitch_a, double yaw_b, double pitch_b)
{
    double Ra[3][3], Rb[3][3];
    rot_yaw_pitch(yaw_a, pitch_a, Ra);
    rot_yaw_pitch(yaw_b, pitch_b, Rb);
    double tr = 0.0;
    for (int i = 0; i < 3; ++i)          /* trace(Ra^T Rb) = sum_ik Ra[k][i] Rb[k][i] */
        for (int k = 0; k < 3; ++k) tr += Ra[k][i] * Rb[k][i];
    double c = (tr - 1.0) / 2.0;
    if (c > 1.0) c = 1.0;
    if (c < -1.0) c = -1.0;
    return acos(c);
}

/* Retrieval distance of Sec. 5.1 and Top-k of Eq. 4 with sim = -D.
 * poses [M][5] = (x, y, z, yaw, pitch) per stored chunk, cur [5].
 * D_i = d_t/norm(d_t) + d_r/norm(d_r), d_t squared L2 of translations, d_r the
 * geodesic angle; the min(R, M) smallest D, ties to the lower chunk id.
 * ids_out [R], D_sel [R] (may be NULL), D_all [M] (may be NULL). */
int wko_score_chunks(const float *poses, int M, const float *cur, int norm_mode, int R,
                     int32_t *ids_out, double *D_sel, double *D_all, int32_t *n_found)
{
    if (M < 0 || R < 0 || (M > 0 && !poses) || !cur || !n_found) return -1;
    int n = R < M ? R : M;
    *n_found = n;
    if (M == 0) return 0;
    double *dt = (double *)malloc(sizeof(double) * M), *dr = (double *)malloc(sizeof(double) * M);
    wko_pair *p = (wko_pair *)malloc(sizeof(wko_pair) * M);
    if (!dt || !dr || !p) { free(dt); free(dr); free(p); return -2; }
    for (int i = 0; i < M; ++i) {
        const float *a = poses + (size_t)i * 5;
        double s = 0.0;
        for (int c = 0; c < 3; ++c) {
            double df = (double)cur[c] - (double)a[c];
            s += df * df;
        }
        dt[i] = s;
        dr[i] = wko_geodesic((double)cur[3], (double)cur[4], (double)a[3], (double)a[4]);
    }
    double *term[2] = {dt, dr};
    for (int t = 0; t < 2; ++t) {
        double mx = term[t][0], mn = term[t][0], sum = 0.0;
        for (int i = 0; i < M; ++i) {
            if (term[t][i] > mx) mx = term[t][i];
            if (term[t][i] < mn) mn = term[t][i];
            sum += term[t][i];
        }
        for (int i = 0; i < M; ++i) {
            double v = term[t][i];
            if (norm_mode == WKO_NORM_MAX) v = mx > 0.0 ? v / mx : 0.0;
            else if (norm_mode == WKO_NORM_MINMAX) v = mx > mn ? (v - mn) / (mx - mn) : 0.0;
            else v = sum > 0.0 ? v / (sum / M) : 0.0;
            term[t][i] = v;
        }
    }
    for (int i = 0; i < M; ++i) {
        p[i].s = dt[i] + dr[i];
        p[i].idx = i;
        if (D_all) D_all[i] = p[i].s;
    }
    qsort(p, (size_t)M, sizeof(wko_pair), cmp_pair);
    for (int i = 0; i < n; ++i) {
        ids_out[i] = p[i].idx;
        if (D_sel) D_sel[i] = p[i].s;
    }
    free(dt); free(dr); free(p);
    return 0;
}

/* Query-based retrieval (Sec. 4.2 allows an importance score computed from the queries as the
 * relevance function; App. C ranks the stored chunks by how strongly the queries of the chunk being
 * denoised attend to them, without a formula).  Reading: the relevance of chunk c is the attention mass its keys receive from
 * the current queries in one softmax over the keys of all M candidate chunks, averaged over heads
 * and query rows; the min(R, M) chunks of largest mass are returned, ties to the lower chunk id.
 * Parity with the authors' exact score (which layers, heads or queries they average) is unpinned.
 * Q [H][N_q][d]; chunk c has keys K_ptrs[c] = [H][n_tok[c]][d].  mass_all [M] (may be NULL). */
int wko_score_chunks_query(const void *Q, const void *const *K_ptrs, const int32_t *n_tok, int M, int dtype,
                           int H, int64_t N_q, int d, double scale, int R, int32_t *ids_out, double *mass_sel,
                           double *mass_all, int32_t *n_found)
{
    if (M < 0 || R < 0 || !Q || !n_found || H < 1 || N_q < 1) return -1;
    int n = R < M ? R : M;
    *n_found = n;
    if (M == 0) return 0;
    double *mass = (double *)calloc((size_t)M, sizeof(double));
    wko_pair *p = (wko_pair *)malloc(sizeof(wko_pair) * M);
    if (!mass || !p) { free(mass); free(p); return -2; }
    int fail = 0;
#pragma omp parallel
    {
        double *local = (double *)calloc((size_t)M, sizeof(double));
        double *q = (double *)malloc(sizeof(double) * (size_t)d);
        int64_t max_tok = 0;
        for (int c = 0; c < M; ++c) if (n_tok[c] > max_tok) max_tok = n_tok[c];
        double **z = (double **)malloc(sizeof(double *) * (size_t)M);   /* logits per chunk */
        int ok = local && q && z;
        if (ok) for (int c = 0; c < M; ++c) { z[c] = (double *)malloc(sizeof(double) * (size_t)(n_tok[c] > 0 ? n_tok[c] : 1)); ok = ok && z[c]; }
        if (!ok) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for collapse(2) schedule(dynamic, 4)
            for (int h = 0; h < H; ++h)
                for (int64_t r = 0; r < N_q; ++r) {
                    for (int e = 0; e < d; ++e) q[e] = load_elem(Q, dtype, ((size_t)h * N_q + r) * d + e);
                    double zmax = -INFINITY;
                    for (int c = 0; c < M; ++c)
                        for (int64_t k = 0; k < n_tok[c]; ++k) {
                            size_t base = ((size_t)h * n_tok[c] + k) * d;
                            double dot = 0.0;
                            for (int e = 0; e < d; ++e) dot += q[e] * load_elem(K_ptrs[c], dtype, base + e);
                            z[c][k] = dot * scale;
                            if (z[c][k] > zmax) zmax = z[c][k];
                        }
                    double denom = 0.0;
                    for (int c = 0; c < M; ++c)
                        for (int64_t k = 0; k < n_tok[c]; ++k) { z[c][k] = exp(z[c][k] - zmax); denom += z[c][k]; }
                    for (int c = 0; c < M; ++c) {
                        double sum = 0.0;
                        for (int64_t k = 0; k < n_tok[c]; ++k) sum += z[c][k];
                        local[c] += sum / denom;
                    }
                }
#pragma omp critical
            for (int c = 0; c < M; ++c) mass[c] += local[c];
        }
        if (z) for (int c = 0; c < M; ++c) free(z[c]);
        free(z); free(local); free(q);
    }
    if (!fail) {
        for (int c = 0; c < M; ++c) {
            mass[c] /= (double)H * (double)N_q;
            if (mass_all) mass_all[c] = mass[c];
            p[c].s = -mass[c];   /* largest mass first, ties to the lower id */
            p[c].idx = c;
        }
        qsort(p, (size_t)M, sizeof(wko_pair), cmp_pair);
        for (int i = 0; i < n; ++i) {
            ids_out[i] = p[i].idx;
            if (mass_sel) mass_sel[i] = mass[p[i].idx];
        }
    }
    free(mass); free(p);
    return fail ? -2 : 0;
}

/* Accumulate discrete actions into pseudo-poses (Sec. 5.1).  Labels:
 * 0 W (forward), 1 A (left), 2 S (back), 3 D (right), 4 yaw-, 5 yaw+,
 * 6 pitch-, 7 pitch+.  Translation steps are taken in the body frame of the
 * current yaw (forward = (sin yaw, 0, cos yaw), right = (cos yaw, 0, -sin yaw));
 * pitch is clamped to +-pitch_limit.  poses_out[i] is the state after label i. */
int wko_accumulate_actions(const int32_t *labels, int n, double step, double dangle, double pitch_limit,
                           float *poses_out)
{
    double x = 0, y = 0, z = 0, yaw = 0, pitch = 0;
    for (int i = 0; i < n; ++i) {
        double fx = sin(yaw), fz = cos(yaw), rx = cos(yaw), rz = -sin(yaw);
        switch (labels[i]) {
        case 0: x += step * fx; z += step * fz; break;
        case 1: x -= step * rx; z -= step * rz; break;
        case 2: x -= step * fx; z -= step * fz; break;
        case 3: x += step * rx; z += step * rz; break;
        case 4: yaw -= dangle; break;
        case 5: yaw += dangle; break;
        case 6: pitch -= dangle; if (pitch < -pitch_limit) pitch = -pitch_limit; break;
        case 7: pitch += dangle; if (pitch > pitch_limit) pitch = pitch_limit; break;
        default: return -1;
        }
        float *o = poses_out + (size_t)i * 5;
        o[0] = (float)x; o[1] = (float)y; o[2] = (float)z; o[3] = (float)yaw; o[4] = (float)pitch;
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* window assembly                                                           */
/* ------------------------------------------------------------------------ */

/* Window = native rows, then each retrieved chunk's stored rows in the order
 * of ids, copied byte for byte.  Store chunk c holds K at K_ptrs[c] and V at
 * V_ptrs[c], each [H][n_tok[c]][d]; windows are [H][win_capacity][d].
 * Returns -4 if the window would overflow. */
int wko_gather(const void *const *K_ptrs, const void *const *V_ptrs, const int32_t *n_tok,
               const int32_t *ids, int n_ids, const void *K_native, const void *V_native, int n_native,
               int H, int d, int dtype, void *K_win, void *V_win, int win_capacity, int32_t *n_win)
{
    const size_t row = (size_t)d * esize_of(dtype);
    int64_t total = n_native;
    for (int r = 0; r < n_ids; ++r) total += n_tok[ids[r]];
    if (total > win_capacity) return -4;
    for (int h = 0; h < H; ++h) {
        char *kw = (char *)K_win + (size_t)h * win_capacity * row;
        char *vw = (char *)V_win + (size_t)h * win_capacity * row;
        if (n_native > 0) {
            memcpy(kw, (const char *)K_native + (size_t)h * n_native * row, (size_t)n_native * row);
            memcpy(vw, (const char *)V_native + (size_t)h * n_native * row, (size_t)n_native * row);
        }
        size_t off = (size_t)n_native;
        for (int r = 0; r < n_ids; ++r) {
            int c = ids[r];
            size_t nt = (size_t)n_tok[c];
            memcpy(kw + off * row, (const char *)K_ptrs[c] + (size_t)h * nt * row, nt * row);
            memcpy(vw + off * row, (const char *)V_ptrs[c] + (size_t)h * nt * row, nt * row);
            off += nt;
        }
    }
    *n_win = (int32_t)total;
    return 0;
}

/* ------------------------------------------------------------------------ */
/* attention                                                                 */
/* ------------------------------------------------------------------------ */

/* O = softmax(Q K^T * scale) V per head, every window key visible (no mask).
 * Q [H][N_q][d]; K, V [H][kv_row_stride][d] of which the first N_kv rows are
 * the window.  rows (may be NULL = all) selects n_rows query rows per head;
 * O is [H][n_rows][d] double, lse [H][n_rows] = log sum exp of the scaled
 * logits (may be NULL). */
int wko_attention(const void *Q, const void *K, const void *V, int dtype, int H, int64_t N_q, int64_t N_kv,
                  int d, int64_t kv_row_stride, double scale, const int32_t *rows, int64_t n_rows,
                  double *O, double *lse)
{
    if (!Q || !K || !V || !O || H < 1 || d < 1 || N_kv < 1 || kv_row_stride < N_kv) return -1;
    if (!rows) n_rows = N_q;
    int fail = 0;
#pragma omp parallel
    {
        double *z = (double *)malloc(sizeof(double) * (size_t)N_kv);
        double *q = (double *)malloc(sizeof(double) * (size_t)d);
        if (!z || !q) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for collapse(2) schedule(dynamic, 4)
            for (int h = 0; h < H; ++h)
                for (int64_t r = 0; r < n_rows; ++r) {
                    int64_t qi = rows ? rows[r] : r;
                    for (int c = 0; c < d; ++c) q[c] = load_elem(Q, dtype, ((size_t)h * N_q + qi) * d + c);
                    double zmax = -INFINITY;
                    for (int64_t n = 0; n < N_kv; ++n) {
                        size_t base = ((size_t)h * kv_row_stride + n) * d;
                        double dot = 0.0;
                        for (int c = 0; c < d; ++c) dot += q[c] * load_elem(K, dtype, base + c);
                        z[n] = dot * scale;
                        if (z[n] > zmax) zmax = z[n];
                    }
                    double denom = 0.0;
                    for (int64_t n = 0; n < N_kv; ++n) {
                        z[n] = exp(z[n] - zmax);
                        denom += z[n];
                    }
                    double *o = O + ((size_t)h * n_rows + r) * d;
                    for (int c = 0; c < d; ++c) o[c] = 0.0;
                    for (int64_t n = 0; n < N_kv; ++n) {
                        size_t base = ((size_t)h * kv_row_stride + n) * d;
                        double p = z[n] / denom;
                        for (int c = 0; c < d; ++c) o[c] += p * load_elem(V, dtype, base + c);
                    }
                    if (lse) lse[(size_t)h * n_rows + r] = zmax + log(denom);
                }
        }
        free(z); free(q);
    }
    return fail ? -2 : 0;
}

/* Attention with a frame-level causal mask inside the chunk being denoised.  The N_q queries are
 * the chunk's tokens, N_q / frame_T frames of frame_T tokens; their own keys occupy window rows
 * [denoise_row0, denoise_row0 + N_q) in the same order.  Query i sees every window row outside
 * that range, and inside it the rows of frames 0 .. i / frame_T (its own frame included).
 * Everything else as wko_attention. */
int wko_attention_block_causal(const void *Q, const void *K, const void *V, int dtype, int H, int64_t N_q,
                               int64_t N_kv, int d, int64_t kv_row_stride, double scale, int64_t denoise_row0,
                               int64_t frame_T, const int32_t *rows, int64_t n_rows, double *O, double *lse)
{
    if (!Q || !K || !V || !O || H < 1 || d < 1 || N_kv < 1 || kv_row_stride < N_kv) return -1;
    if (frame_T < 1 || N_q % frame_T != 0 || denoise_row0 < 0 || denoise_row0 + N_q > N_kv) return -1;
    if (!rows) n_rows = N_q;
    int fail = 0;
#pragma omp parallel
    {
        double *z = (double *)malloc(sizeof(double) * (size_t)N_kv);
        double *q = (double *)malloc(sizeof(double) * (size_t)d);
        if (!z || !q) {
#pragma omp atomic write
            fail = 1;
        } else {
#pragma omp for collapse(2) schedule(dynamic, 4)
            for (int h = 0; h < H; ++h)
                for (int64_t r = 0; r < n_rows; ++r) {
                    int64_t qi = rows ? rows[r] : r;
                    int64_t q_frame = qi / frame_T;
                    for (int c = 0; c < d; ++c) q[c] = load_elem(Q, dtype, ((size_t)h * N_q + qi) * d + c);
                    double zmax = -INFINITY;
                    for (int64_t n = 0; n < N_kv; ++n) {
                        int inside = n >= denoise_row0 && n < denoise_row0 + N_q;
                        if (inside && (n - denoise_row0) / frame_T > q_frame) {
                            z[n] = -INFINITY;   /* a later frame of the same chunk: not visible */
                            continue;
                        }
                        size_t base = ((size_t)h * kv_row_stride + n) * d;
                        double dot = 0.0;
                        for (int c = 0; c < d; ++c) dot += q[c] * load_elem(K, dtype, base + c);
                        z[n] = dot * scale;
                        if (z[n] > zmax) zmax = z[n];
                    }
                    double denom = 0.0;
                    for (int64_t n = 0; n < N_kv; ++n) {
                        z[n] = z[n] == -INFINITY ? 0.0 : exp(z[n] - zmax);
                        denom += z[n];
                    }
                    double *o = O + ((size_t)h * n_rows + r) * d;
                    for (int c = 0; c < d; ++c) o[c] = 0.0;
                    for (int64_t n = 0; n < N_kv; ++n) {
                        if (z[n] == 0.0) continue;
                        size_t base = ((size_t)h * kv_row_stride + n) * d;
                        double p = z[n] / denom;
                        for (int c = 0; c < d; ++c) o[c] += p * load_elem(V, dtype, base + c);
                    }
                    if (lse) lse[(size_t)h * n_rows + r] = zmax + log(denom);
                }
        }
        free(z); free(q);
    }
    return fail ? -2 : 0;
}
