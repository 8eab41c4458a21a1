/*
 * CPU oracle for the token-wise linear projections around the temporal attention of
 * Video-Infinity (arXiv 2406.16260, Section 4.2: queries, keys and values are computed from the
 * tokens; the paper gives no formula beyond that, this is the usual affine map).
 *
 * TEST INFRASTRUCTURE ONLY; shares nothing with the HIP path.
 *
 *   Y[m][co] = bias[co] + sum_ci W[co][ci] * X[m][ci]        for every token m
 *
 * All arithmetic is IEEE double.
 */
#include <stdint.h>

/* X: [rows][c_in]; W: [c_out][c_in]; bias: [c_out] or NULL; Y: [rows][c_out].
 * Returns 0, -1 on bad arguments. */
int oracle_linear(int64_t rows, int64_t c_in, int64_t c_out, const double *X, const double *W,
                  const double *bias, double *Y)
{
    if (rows < 1 || c_in < 1 || c_out < 1) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < rows; ++m)
        for (int64_t co = 0; co < c_out; ++co) {
            double acc = bias ? bias[co] : 0.0;
            for (int64_t ci = 0; ci < c_in; ++ci) acc += W[co * c_in + ci] * X[m * c_in + ci];
            Y[m * c_out + co] = acc;
        }
    return 0;
}
