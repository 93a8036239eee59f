/*
 * CPU oracle for the FP16 batch-norm layer forward pass.  TEST INFRASTRUCTURE: only
 * tests, the smoke check and the benchmark's cpu_baseline leg may use it.  It shares no
 * code, header, table or helper with the HIP library.
 *
 * The paper describes how its FP16 engine keeps the batch-norm layer's accumulations in
 * range (Section 3.1): the mean of a long vector is taken as the mean of the means of
 * its parts, and values are multiplied by a power of two before they are squared and
 * scaled back afterwards.  Both devices change the rounding only: what they arrive at
 * is the layer's plain definition, the batch-norm layer of BVLC Caffe that the paper
 * keeps (Sections 2 and 5), followed by Caffe's per-channel scale layer when one is
 * attached.  This file is that definition, in FP64, over FP16 inputs:
 *
 *   L       = N * H * W                                  values of one channel
 *   mean[c] = (1/L) sum_{n,h,w} x[n][c][h][w]
 *   var[c]  = (1/L) sum_{n,h,w} (x[n][c][h][w] - mean[c])^2      (the biased variance)
 *   pre[n][c][h][w] = gamma[c] * (x[n][c][h][w] - mean[c]) / sqrt(var[c] + eps) + beta[c]
 *
 * With stored statistics (Caffe's use_global_stats) the first two lines are replaced by
 * mean[c] = stat_scale * mean_in[c], var[c] = stat_scale * var_in[c].  gamma = 1 and
 * beta = 0 when no scale layer is attached.  Per-channel parameters are FP32 (the paper
 * keeps scalars in float, Section 3.2); x is FP16 bit patterns.  Beside `pre` it returns
 *   mag = |gamma| * (|x| + |mean|) / sqrt(var + eps) + |beta|,
 * the size of the terms that cancel in `pre`, from which callers form the tolerance.
 * ReLU is left to the caller.
 *
 * Loops: channel, then (n, h, w) twice for the statistics and once for the output, as the
 * three lines above read; OpenMP only splits the channels.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

/* IEEE 754 binary16 bit pattern -> double, from the format's definition. */
static double bn_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1F;
    int f = h & 0x3FF;
    double v;
    if (e == 0)
        v = ldexp((double)f, -24);
    else if (e == 31)
        v = f ? NAN : INFINITY;
    else
        v = ldexp((double)(1024 + f), e - 25);
    return sign ? -v : v;
}

/*
 * desc = {N, C, H, W, use_global_stats, scale_bias, relu}.  x: N*C*H*W FP16 bit patterns.
 * stats_in: with use_global_stats, 2*C floats (C means, then C variances), else ignored.
 * gamma_beta: with scale_bias, 2*C floats (C gammas, then C betas), else ignored.
 * pre, mag: N*C*H*W doubles; mean, var: C doubles each (the statistics used).
 * Returns 0, or -1 for a bad descriptor or a missing array.
 */
int hgo_batch_norm_forward(const int32_t *desc, double eps, double stat_scale, const uint16_t *x,
                           const float *stats_in, const float *gamma_beta,
                           double *pre, double *mag, double *mean, double *var)
{
    const int N = desc[0], C = desc[1], H = desc[2], W = desc[3];
    const int global = desc[4], affine = desc[5];
    if (N < 1 || C < 1 || H < 1 || W < 1) return -1;
    if ((global != 0 && global != 1) || (affine != 0 && affine != 1) || (desc[6] != 0 && desc[6] != 1)) return -1;
    if (!(eps > 0.0) || !x || !pre || !mag || !mean || !var) return -1;
    if ((global && !stats_in) || (affine && !gamma_beta)) return -1;
    const size_t HW = (size_t)H * W;
    const double L = (double)N * (double)HW;
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        double mu, v;
        if (global) {
            mu = stat_scale * (double)stats_in[c];
            v = stat_scale * (double)stats_in[C + c];
        } else {
            double s = 0.0;
            for (int n = 0; n < N; ++n)
                for (size_t i = 0; i < HW; ++i)
                    s += bn_half_to_double(x[((size_t)n * C + c) * HW + i]);
            mu = s / L;
            double q = 0.0;
            for (int n = 0; n < N; ++n)
                for (size_t i = 0; i < HW; ++i) {
                    const double d = bn_half_to_double(x[((size_t)n * C + c) * HW + i]) - mu;
                    q += d * d;
                }
            v = q / L;
        }
        mean[c] = mu;
        var[c] = v;
        const double g = affine ? (double)gamma_beta[c] : 1.0;
        const double b = affine ? (double)gamma_beta[C + c] : 0.0;
        const double sd = sqrt(v + eps);
        for (int n = 0; n < N; ++n)
            for (size_t i = 0; i < HW; ++i) {
                const size_t o = ((size_t)n * C + c) * HW + i;
                const double xv = bn_half_to_double(x[o]);
                pre[o] = g * (xv - mu) / sd + b;
                mag[o] = fabs(g) * (fabs(xv) + fabs(mu)) / sd + fabs(b);
            }
    }
    return 0;
}

/*
 * Folding stored batch-norm statistics (and the scale layer) into the convolution that feeds it,
 * once, before inference -- the pattern of Section 3.3 (conversion work is paid offline, none is
 * left on the path): with a[m] = gamma[m] / sqrt(stat_scale * var[m] + eps),
 *
 *   w'[m][c][r][q] = a[m] * w[m][c][r][q]
 *   b'[m]          = a[m] * (b[m] - stat_scale * mean[m]) + beta[m]
 *
 * so that conv(x, w', b') = batchnorm(conv(x, w, b)) in exact arithmetic.  w: M*per FP16 bit
 * patterns (per = C/group * k * k), b: M FP16 bit patterns or NULL (zero); stats = M means then
 * M variances, gamma_beta = M gammas then M betas or NULL (1 and 0), all FP32.  Outputs are FP64
 * and unrounded: w_out M*per, b_out M.  Returns 0 or -1.
 */
int hgo_batch_norm_fold(int M, int per, double eps, double stat_scale, const uint16_t *w, const uint16_t *b,
                        const float *stats, const float *gamma_beta, double *w_out, double *b_out)
{
    if (M < 1 || per < 1 || !(eps > 0.0) || !w || !stats || !w_out || !b_out) return -1;
    for (int m = 0; m < M; ++m) {
        const double g = gamma_beta ? (double)gamma_beta[m] : 1.0;
        const double bt = gamma_beta ? (double)gamma_beta[M + m] : 0.0;
        const double a = g / sqrt(stat_scale * (double)stats[M + m] + eps);
        for (int i = 0; i < per; ++i) w_out[(size_t)m * per + i] = a * bn_half_to_double(w[(size_t)m * per + i]);
        b_out[m] = a * ((b ? bn_half_to_double(b[m]) : 0.0) - stat_scale * (double)stats[m]) + bt;
    }
    return 0;
}
