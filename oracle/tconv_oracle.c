/*
 * CPU oracle for the clip-parallel temporal convolution of Video-Infinity
 * (arXiv 2406.16260, Section 4.2, "Convolution module").
 *
 * TEST INFRASTRUCTURE ONLY; shares nothing with the HIP path.
 *
 * X is [F][P][C_in] with F = N * F_clip frames and P spatial positions; the module convolves
 * along the frame axis only, separately at every position, mixing channels densely.
 * Following the paper, clip i is processed on its own, with a context padded to it:
 *   c_pre(i)  = the last  n frames of clip i-1,
 *   c_post(i) = the first n frames of clip i+1,
 * where n is the reach of the kernel on each side (kernel size 2n + 1 taps).  The paper does
 * not say what the first clip's c_pre and the last clip's c_post are: they are zero frames
 * here (the zero padding a temporal convolution of the base model applies at the ends of its
 * input).  The padded clip [c_pre | clip | c_post] has F_clip + 2n frames; the output frame a
 * of the clip is
 *   Y[a][p][co] = bias[co] + sum_{t=0..2n} sum_{ci} W[t][co][ci] * padded[a + t][p][ci],
 * i.e. tap t looks at frame (a + t - n) of the clip: cross-correlation, the deep-learning
 * convention (the paper does not say; a flipped kernel is the same module with W reversed).
 * n <= F_clip is required, because the paper's context reaches one clip to each side only.
 * All arithmetic is IEEE double.
 */
#include <stdint.h>
#include <stdlib.h>

/*
 * X: [F][P][c_in]; W: [2n+1][c_out][c_in]; bias: [c_out] or NULL; Y: [F][P][c_out].
 * Returns 0, -1 on bad arguments, -2 on allocation failure.
 */
int oracle_temporal_conv(int64_t clip_len, int64_t n_clips, int64_t P, int64_t c_in, int64_t c_out,
                         int64_t n, const double *X, const double *W, const double *bias, double *Y)
{
    if (clip_len < 1 || n_clips < 1 || P < 1 || c_in < 1 || c_out < 1 || n < 0 || n > clip_len)
        return -1;
    const int64_t taps = 2 * n + 1;
    const int64_t padded_len = clip_len + 2 * n;
    const int64_t frame = P * c_in; /* doubles per input frame */
    double *padded = (double *)malloc((size_t)(padded_len * frame) * sizeof(double));
    if (!padded) return -2;

    for (int64_t i = 0; i < n_clips; ++i) {
        /* context of clip i, padded to the clip */
        for (int64_t j = 0; j < padded_len; ++j) {
            double *dst = padded + j * frame;
            int64_t src = -1; /* frame of the video, -1 = a zero frame */
            if (j < n) {                       /* c_pre: last n frames of clip i-1 */
                if (i > 0) src = (i - 1) * clip_len + (clip_len - n) + j;
            } else if (j < n + clip_len) {     /* the clip itself */
                src = i * clip_len + (j - n);
            } else {                           /* c_post: first n frames of clip i+1 */
                if (i + 1 < n_clips) src = (i + 1) * clip_len + (j - n - clip_len);
            }
            for (int64_t e = 0; e < frame; ++e) dst[e] = src >= 0 ? X[src * frame + e] : 0.0;
        }
        /* the convolution over the padded clip keeps exactly the clip's frames
           (output elements are independent: the loop nest is shared among threads) */
#pragma omp parallel for collapse(2) schedule(static)
        for (int64_t a = 0; a < clip_len; ++a)
            for (int64_t p = 0; p < P; ++p)
                for (int64_t co = 0; co < c_out; ++co) {
                    double acc = bias ? bias[co] : 0.0;
                    for (int64_t t = 0; t < taps; ++t) {
                        const double *x = padded + (a + t) * frame + p * c_in;
                        const double *w = W + (t * c_out + co) * c_in;
                        for (int64_t ci = 0; ci < c_in; ++ci) acc += w[ci] * x[ci];
                    }
                    Y[((i * clip_len + a) * P + p) * c_out + co] = acc;
                }
    }
    free(padded);
    return 0;
}
