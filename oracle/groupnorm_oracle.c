/*
 * CPU oracle for the clip-parallel group normalisation of Video-Infinity
 * (arXiv 2406.16260, Section 4.2, "Group normalization").
 *
 * TEST INFRASTRUCTURE ONLY; shares nothing with the HIP path.
 *
 * X is [F][P][C] with F = N * F_clip frames, P spatial positions, C channels in
 * `groups` contiguous groups of C / groups channels.  The statistics are taken
 * over the whole video (all clips, all positions, the channels of the group),
 * in the order the paper gives for clips held on different devices:
 *   1. every clip i computes its group mean            mu_i[g];
 *   2. the global mean is the mean of the clip means   mu[g]  = sum_i mu_i[g] / N;
 *   3. every clip computes its mean squared deviation ABOUT THE GLOBAL MEAN
 *                                                      v_i[g] = mean (x - mu[g])^2;
 *   4. the global variance is the mean of those        var[g] = sum_i v_i[g] / N
 *      (averaging per-clip standard deviations taken about per-clip means would
 *      not give the global one: the paper's footnote);
 *   5. y = (x - mu[g]) / sqrt(var[g] + eps) * gamma[c] + beta[c].
 * Clips are equally long, so steps 2 and 4 give exactly the mean and the
 * (biased) variance of the whole video.  All arithmetic is IEEE double.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

/*
 * X, Y: [F][P][C] doubles; gamma, beta: [C] (NULL = 1 and 0); mean_out, var_out:
 * [groups] or NULL.  Returns 0, -1 on bad arguments, -2 on allocation failure.
 */
int oracle_groupnorm(int64_t clip_len, int64_t n_clips, int64_t P, int64_t C, int64_t groups,
                     double eps, const double *X, const double *gamma, const double *beta,
                     double *Y, double *mean_out, double *var_out)
{
    if (clip_len < 1 || n_clips < 1 || P < 1 || C < 1 || groups < 1 || C % groups != 0 || eps < 0)
        return -1;
    const int64_t cg = C / groups;       /* channels per group */
    const int64_t F = clip_len * n_clips;
    const double n_clip = (double)(clip_len * P * cg); /* elements of one clip in one group */
    double *mu = (double *)calloc((size_t)groups, sizeof(double));
    double *var = (double *)calloc((size_t)groups, sizeof(double));
    if (!mu || !var) { free(mu); free(var); return -2; }

    for (int64_t g = 0; g < groups; ++g) {
        /* steps 1 and 2 */
        double mu_sum = 0.0;
        for (int64_t i = 0; i < n_clips; ++i) {
            double s = 0.0;
            for (int64_t f = i * clip_len; f < (i + 1) * clip_len; ++f)
                for (int64_t p = 0; p < P; ++p)
                    for (int64_t c = g * cg; c < (g + 1) * cg; ++c) s += X[(f * P + p) * C + c];
            mu_sum += s / n_clip;
        }
        mu[g] = mu_sum / (double)n_clips;
        /* steps 3 and 4 */
        double v_sum = 0.0;
        for (int64_t i = 0; i < n_clips; ++i) {
            double s = 0.0;
            for (int64_t f = i * clip_len; f < (i + 1) * clip_len; ++f)
                for (int64_t p = 0; p < P; ++p)
                    for (int64_t c = g * cg; c < (g + 1) * cg; ++c) {
                        double d = X[(f * P + p) * C + c] - mu[g];
                        s += d * d;
                    }
            v_sum += s / n_clip;
        }
        var[g] = v_sum / (double)n_clips;
    }
    /* step 5 */
    for (int64_t f = 0; f < F; ++f)
        for (int64_t p = 0; p < P; ++p)
            for (int64_t c = 0; c < C; ++c) {
                int64_t g = c / cg;
                double y = (X[(f * P + p) * C + c] - mu[g]) / sqrt(var[g] + eps);
                Y[(f * P + p) * C + c] = y * (gamma ? gamma[c] : 1.0) + (beta ? beta[c] : 0.0);
            }
    for (int64_t g = 0; g < groups; ++g) {
        if (mean_out) mean_out[g] = mu[g];
        if (var_out) var_out[g] = var[g];
    }
    free(mu);
    free(var);
    return 0;
}
