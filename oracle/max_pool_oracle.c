/*
 * CPU oracle for the max-pooling layer forward pass.  TEST INFRASTRUCTURE: only tests,
 * the smoke check and the benchmark's cpu_baseline leg may use it.  It shares no code,
 * header, table or helper with the HIP library.
 *
 * The paper keeps BVLC Caffe's layers (Sections 2 and 5); the networks it runs (LeNet,
 * AlexNet, ResNet: Section 4) put Caffe's MAX pooling between their convolutions.  The
 * layer, over NCHW tensors, square window k, stride s, symmetric padding p < k:
 *
 *   Ho = ceil((H + 2p - k) / s) + 1, and one less if p > 0 and the last window would start
 *        at or beyond H + p (entirely in the padding on the far side); Wo likewise
 *   y[n][c][oh][ow] = max over the window rows  max(oh*s - p, 0) .. min(oh*s - p + k, H) - 1
 *                     and columns               max(ow*s - p, 0) .. min(ow*s - p + k, W) - 1
 *                     of x[n][c][.][.]
 *
 * Padding never takes part in the maximum (a window is clipped to the image), and the
 * rounding up of the output size lets the last window hang over the edge.  The result is
 * one of the inputs, so it is returned as an FP16 bit pattern and compared exactly; values
 * are compared as reals (decoded to double), the first of equal values wins, inputs are finite.
 * Four plain loops over the output and two over the window.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

static double mp_half_to_double(uint16_t h)
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

static int mp_out(int size, int k, int s, int p)
{
    int span = size + 2 * p - k;
    int o = (span + s - 1) / s + 1;              /* ceil(span / s) + 1, span >= 0 */
    if (p > 0 && (o - 1) * s >= size + p) --o;
    return o;
}

/* desc = {N, C, H, W, kernel, stride, pad}; out_hw receives {Ho, Wo}.  Returns 0 or -1. */
int hgo_max_pool_shape(const int32_t *desc, int32_t *out_hw)
{
    const int N = desc[0], C = desc[1], H = desc[2], W = desc[3], k = desc[4], s = desc[5], p = desc[6];
    if (N < 1 || C < 1 || H < 1 || W < 1 || k < 1 || s < 1 || p < 0 || p >= k) return -1;
    if (H + 2 * p < k || W + 2 * p < k) return -1;
    out_hw[0] = mp_out(H, k, s, p);
    out_hw[1] = mp_out(W, k, s, p);
    return 0;
}

/* x: N*C*H*W FP16 bit patterns; y: N*C*Ho*Wo FP16 bit patterns.  Returns 0 or -1. */
int hgo_max_pool_forward(const int32_t *desc, const uint16_t *x, uint16_t *y)
{
    int32_t o[2];
    if (hgo_max_pool_shape(desc, o)) return -1;
    const int N = desc[0], C = desc[1], H = desc[2], W = desc[3], k = desc[4], s = desc[5], p = desc[6];
    const int Ho = o[0], Wo = o[1];
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c) {
            const uint16_t *plane = x + ((size_t)n * C + c) * H * W;
            uint16_t *out = y + ((size_t)n * C + c) * Ho * Wo;
            for (int oh = 0; oh < Ho; ++oh)
                for (int ow = 0; ow < Wo; ++ow) {
                    int h0 = oh * s - p, w0 = ow * s - p;
                    int h1 = h0 + k < H ? h0 + k : H, w1 = w0 + k < W ? w0 + k : W;
                    if (h0 < 0) h0 = 0;
                    if (w0 < 0) w0 = 0;
                    uint16_t best = plane[(size_t)h0 * W + w0];
                    double bv = mp_half_to_double(best);
                    for (int ih = h0; ih < h1; ++ih)
                        for (int iw = w0; iw < w1; ++iw) {
                            const uint16_t cand = plane[(size_t)ih * W + iw];
                            const double cv = mp_half_to_double(cand);
                            if (cv > bv) { bv = cv; best = cand; }
                        }
                    out[(size_t)oh * Wo + ow] = best;
                }
        }
    return 0;
}
