/*
 * CPU oracle for the FP16 inner-product (fully connected) layer forward pass.
 * TEST INFRASTRUCTURE: only tests, the smoke check and the benchmark's cpu_baseline
 * leg may use it.  It shares no code, header, table or helper with the HIP library.
 *
 * The paper names the inner-product layer, beside batch norm, as a place where FP16
 * overflows and underflows arise because many values are accumulated (Section 3.1);
 * the layer itself is the one of BVLC Caffe, which the paper keeps together with its
 * weight format (Sections 2 and 5):
 *
 *   pre[n][m] = b[m] + sum_{k<K} w[m][k] * x[n][k]
 *
 * x is [N][K] (an image's C*H*W values in their memory order), w is [M][K], b is [M].
 * Inputs are FP16 bit patterns; products and sums are FP64 (a product of two FP16
 * values is exact in FP64), so the reference carries no accumulation error.  Beside
 * `pre` it returns mag = sum |w * x|, from which callers form the tolerance.  ReLU is
 * left to the caller.  Three plain loops (n, m, k); OpenMP only splits the (n, m) pairs.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>

/* IEEE 754 binary16 bit pattern -> double, from the format's definition. */
static double half_bits_to_double(uint16_t h)
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

/* desc = {N, K, M, bias, relu}; returns 0, or -1 for a bad descriptor. */
int hgo_inner_product_forward(const int32_t *desc, const uint16_t *x, const uint16_t *w, const uint16_t *b,
                              double *pre, double *mag)
{
    const int N = desc[0], K = desc[1], M = desc[2], bias = desc[3];
    if (N < 1 || K < 1 || M < 1 || (bias != 0 && bias != 1) || (desc[4] != 0 && desc[4] != 1)) return -1;
    if (bias && !b) return -1;
    const long long total = (long long)N * M;
#pragma omp parallel for schedule(static)
    for (long long i = 0; i < total; ++i) {
        const int n = (int)(i / M), m = (int)(i % M);
        double acc = bias ? half_bits_to_double(b[m]) : 0.0;
        double a = 0.0;
        for (int k = 0; k < K; ++k) {
            const double t = half_bits_to_double(w[(size_t)m * K + k]) * half_bits_to_double(x[(size_t)n * K + k]);
            acc += t;
            a += fabs(t);
        }
        pre[i] = acc;
        mag[i] = a;
    }
    return 0;
}
