/*
 * CPU oracle for Dual-scope temporal attention (Video-Infinity, arXiv 2406.16260).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, obviously-correct
 * statement of what the GPU library must compute.  It is compiled with gcc,
 * shares no code, header, table or helper with the HIP path, and is called only
 * from tests, from the smoke check and from the benchmark's cpu_baseline leg.
 *
 * What it computes (Section 4.2, "DualScope attention"; Section 4.1 for the
 * clip split and the per-clip context c^i = {c_pre, c_post, c_global}):
 *
 *   The video has F = N * F_clip frames split into N non-overlapping clips
 *   (Section 4, clip split).  Tensors Q, K, V are [F][P][h][D]: frame, spatial
 *   position, head, head channel.  A temporal module sees, per spatial position,
 *   a strip over frames (Section 3); heads are independent as in ordinary
 *   multi-head attention.
 *
 *   For clip i the key/value frame list is  Concat(local, global):
 *     local  = the clip's own frames plus `w` frames from the preceding clip
 *              side and `w` frames from the following side, i.e. the frame
 *              range [i*F_clip - w, (i+1)*F_clip + w) intersected with [0, F)
 *              (c_pre / c_post of Section 4.1; sizes of Section 4.2), ascending;
 *     global = the caller's global frame indices G, in the caller's order
 *              (Section 4.2, global context).
 *   Concat keeps duplicates: a frame in both parts is listed, and counted in
 *   the softmax, twice (Section 4.2 writes K = Concat(K_local, K_global)).
 *
 *   Every query frame a of clip i, at every position p and head g, then does
 *   ordinary softmax attention over that list:
 *     s_j = scale * sum_d Q[a][p][g][d] * K[ctx_j][p][g][d] + b_j
 *     A_j = exp(s_j - max_j s_j) / sum_j exp(s_j - max_j s_j)
 *     O[a][p][g][d] = sum_j A_j * V[ctx_j][p][g][d]
 *   b_j is the scope weight of Section 5.1 (there the two scopes are weighted
 *   differently from one denoising timestep to the next), taken as an additive
 *   logit bias: bias_local for the
 *   keys of the local part, bias_global for the keys of the global part; both 0
 *   unless the caller sets them (raising a scope's logits by b multiplies its
 *   unnormalised softmax weights by e^b).
 *   Optional sliding window (Section 4.2 describes the local context as the
 *   neighbouring frames of the query frame a and names window attention as the
 *   usual way to get it): with window = r >= 0 a LOCAL key frame f is visible to the
 *   query of frame a only if |f - a| <= r; hidden keys get weight exactly 0.
 *   Global keys are always visible.  window < 0 switches this off (every query
 *   of the clip sees the clip's whole local list).
 *   Optional set union (Section 4.2 first writes the key set of a query as the
 *   union of its local neighbours and the global frames, before turning to the
 *   concatenation used in practice): with dedup a global entry whose frame the
 *   query already sees (as a visible local key, or as an earlier global entry)
 *   is dropped, so that no frame counts twice.
 *   No other mask, no positional term.  Outputs of the clips are concatenated along
 *   frames (Section 4.1, v_out = Concat), i.e. O has the layout of Q.
 *
 * All arithmetic is IEEE double, in the loop order written.  Inputs are
 * doubles that hold the exact values of the fp32 or bf16 inputs.
 *
 * Parity pins (tests/test_oracle_pins.py): reduction to full attention,
 * per-clip check against a library attention routine, hand-derived index
 * lists, closed forms (Q = 0, constant V, frame-valued V), weight sums,
 * permutation invariance of G, key-translation invariance, linearity in V,
 * locality, duplicate = ln 2 bias, and a separate pure-Python brute force.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* Length of clip i's local frame range after truncation to [0, F). */
static int64_t local_range(int64_t clip_len, int64_t n_clips, int64_t w, int64_t i,
                           int64_t *lo_out)
{
    int64_t F = clip_len * n_clips;
    int64_t lo = i * clip_len - w;
    int64_t hi = (i + 1) * clip_len + w;
    if (lo < 0) lo = 0;
    if (hi > F) hi = F;
    *lo_out = lo;
    return hi - lo;
}

/* Largest context length over all clips: max_i (local_len(i) + n_global). */
int64_t oracle_ctx_max(int64_t clip_len, int64_t n_clips, int64_t w, int64_t n_global)
{
    int64_t best = 0;
    for (int64_t i = 0; i < n_clips; ++i) {
        int64_t lo;
        int64_t len = local_range(clip_len, n_clips, w, i, &lo) + n_global;
        if (len > best) best = len;
    }
    return best;
}

/*
 * Context frame lists.  ctx_idx is [n_clips][lk_max] int32, filled with the
 * list of clip i followed by -1 padding; ctx_len is [n_clips].
 * Returns 0, or -1 when an argument is out of range.
 */
int oracle_ctx_indices(int64_t clip_len, int64_t n_clips, int64_t w,
                       const int32_t *global_idx, int64_t n_global,
                       int64_t lk_max, int32_t *ctx_idx, int32_t *ctx_len)
{
    if (clip_len < 1 || n_clips < 1 || w < 0 || n_global < 0) return -1;
    int64_t F = clip_len * n_clips;
    for (int64_t j = 0; j < n_global; ++j)
        if (global_idx[j] < 0 || global_idx[j] >= F) return -1;
    if (lk_max < oracle_ctx_max(clip_len, n_clips, w, n_global)) return -1;

    for (int64_t i = 0; i < n_clips; ++i) {
        int64_t lo;
        int64_t nloc = local_range(clip_len, n_clips, w, i, &lo);
        int32_t *row = ctx_idx + i * lk_max;
        int64_t n = 0;
        for (int64_t f = lo; f < lo + nloc; ++f) row[n++] = (int32_t)f;
        for (int64_t j = 0; j < n_global; ++j) row[n++] = global_idx[j];
        ctx_len[i] = (int32_t)n;
        for (; n < lk_max; ++n) row[n] = -1;
    }
    return 0;
}

/*
 * Forward pass.  Q, K, V, O: [F][P][h][D] doubles, contiguous.
 * scale <= 0 selects 1/sqrt(D).  bias_local / bias_global: scope logit biases.
 * window: sliding-window radius for the local keys, or < 0 for none.
 * weights: NULL, or [F][P][h][lk_max] receiving the softmax weights A_j
 *          (zero padded past the clip's list length).
 * Returns 0 on success, -1 on bad arguments, -2 on allocation failure.
 * Parallel over spatial positions when built with OpenMP; every (a, p, g)
 * output is computed by one thread, alone, in the order written.
 */
int oracle_forward(int64_t clip_len, int64_t n_clips, int64_t w,
                   int64_t P, int64_t h, int64_t D,
                   const int32_t *global_idx, int64_t n_global, double scale,
                   double bias_local, double bias_global, int64_t window, int dedup,
                   const double *Q, const double *K, const double *V,
                   double *O, double *weights)
{
    if (clip_len < 1 || n_clips < 1 || w < 0 || P < 1 || h < 1 || D < 1 || n_global < 0)
        return -1;
    int64_t F = clip_len * n_clips;
    for (int64_t j = 0; j < n_global; ++j)
        if (global_idx[j] < 0 || global_idx[j] >= F) return -1;
    if (scale <= 0.0) scale = 1.0 / sqrt((double)D);

    int64_t lk_max = oracle_ctx_max(clip_len, n_clips, w, n_global);
    int32_t *ctx_idx = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_clips * lk_max));
    int32_t *ctx_len = (int32_t *)malloc(sizeof(int32_t) * (size_t)n_clips);
    if (!ctx_idx || !ctx_len) { free(ctx_idx); free(ctx_len); return -2; }
    oracle_ctx_indices(clip_len, n_clips, w, global_idx, n_global, lk_max, ctx_idx, ctx_len);

    int64_t C = h * D;           /* channels of one position */
    int64_t frame_stride = P * C;
    int failed = 0;

#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)(lk_max > 0 ? lk_max : 1));
        if (!s) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(static)
        for (int64_t p = 0; p < P; ++p) {
            if (!s) continue;
            for (int64_t i = 0; i < n_clips; ++i) {
                const int32_t *ctx = ctx_idx + i * lk_max;
                int64_t L = ctx_len[i];
                for (int64_t a = i * clip_len; a < (i + 1) * clip_len; ++a) {
                    for (int64_t g = 0; g < h; ++g) {
                        const double *q = Q + a * frame_stride + p * C + g * D;
                        /* scores */
                        double m = -INFINITY;
                        for (int64_t j = 0; j < L; ++j) {
                            const double *k = K + (int64_t)ctx[j] * frame_stride + p * C + g * D;
                            double dot = 0.0;
                            for (int64_t d = 0; d < D; ++d) dot += q[d] * k[d];
                            s[j] = scale * dot + (j < L - n_global ? bias_local : bias_global);
                            if (window >= 0 && j < L - n_global) {
                                int64_t dist = (int64_t)ctx[j] - a;
                                if (dist < 0) dist = -dist;
                                if (dist > window) s[j] = -INFINITY; /* hidden: exp gives 0 */
                            }
                            if (dedup && j >= L - n_global) {
                                /* set union: a global entry is dropped if its frame is already
                                   among the keys this query sees, i.e. among the visible local
                                   keys or among the global entries before it */
                                int seen = 0;
                                for (int64_t jj = 0; jj < j && !seen; ++jj)
                                    if (ctx[jj] == ctx[j] && s[jj] != -INFINITY) seen = 1;
                                if (seen) s[j] = -INFINITY;
                            }
                            if (s[j] > m) m = s[j];
                        }
                        /* softmax */
                        double Z = 0.0;
                        for (int64_t j = 0; j < L; ++j) {
                            s[j] = exp(s[j] - m);
                            Z += s[j];
                        }
                        for (int64_t j = 0; j < L; ++j) s[j] /= Z;
                        if (weights) {
                            double *wrow = weights + ((a * P + p) * h + g) * lk_max;
                            for (int64_t j = 0; j < lk_max; ++j) wrow[j] = j < L ? s[j] : 0.0;
                        }
                        /* output */
                        double *o = O + a * frame_stride + p * C + g * D;
                        for (int64_t d = 0; d < D; ++d) {
                            double acc = 0.0;
                            for (int64_t j = 0; j < L; ++j)
                                acc += s[j] *
                                       V[(int64_t)ctx[j] * frame_stride + p * C + g * D + d];
                            o[d] = acc;
                        }
                    }
                }
            }
        }
        free(s);
    }
    free(ctx_idx);
    free(ctx_len);
    return failed ? -2 : 0;
}

/*
 * Context gather by definition: Kctx[i][j][p][c] = K[ctx_idx[i][j]][p][c], zero
 * where j >= ctx_len[i] (the single-buffer image of the context exchange of
 * Section 4.1).  Element size is given in bytes so that any dtype can be used;
 * the copy is bitwise.
 */
int oracle_gather_context(int64_t clip_len, int64_t n_clips, int64_t w,
                          const int32_t *global_idx, int64_t n_global,
                          int64_t row_bytes /* bytes of one frame: P*C*elem */,
                          const unsigned char *X, unsigned char *Xctx)
{
    int64_t lk_max = oracle_ctx_max(clip_len, n_clips, w, n_global);
    int32_t *ctx_idx = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_clips * lk_max));
    int32_t *ctx_len = (int32_t *)malloc(sizeof(int32_t) * (size_t)n_clips);
    if (!ctx_idx || !ctx_len) { free(ctx_idx); free(ctx_len); return -2; }
    if (oracle_ctx_indices(clip_len, n_clips, w, global_idx, n_global, lk_max, ctx_idx,
                           ctx_len) != 0) {
        free(ctx_idx); free(ctx_len);
        return -1;
    }
    for (int64_t i = 0; i < n_clips; ++i)
        for (int64_t j = 0; j < lk_max; ++j) {
            unsigned char *dst = Xctx + (i * lk_max + j) * row_bytes;
            int32_t f = ctx_idx[i * lk_max + j];
            for (int64_t b = 0; b < row_bytes; ++b)
                dst[b] = f >= 0 ? X[(int64_t)f * row_bytes + b] : 0;
        }
    free(ctx_idx);
    free(ctx_len);
    return 0;
}

/* Threads the parallel region of oracle_forward will use. */
int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
