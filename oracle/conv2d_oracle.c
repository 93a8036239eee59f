/*
 * CPU oracle for the FP16 convolution-layer forward pass.  TEST INFRASTRUCTURE:
 * only tests, the smoke check and the benchmark's cpu_baseline leg may use it.
 * It shares no code, header, table or helper with the HIP library.
 *
 * What it computes is the plain definition of the layer the paper inherits from
 * BVLC Caffe (Section 2, "Modified from Caffe"; Section 5 states that Caffe's
 * layers and weight format are kept): a cross-correlation over NCHW tensors with
 * zero padding, stride, channel groups and a per-channel bias,
 *
 *   pre[n][m][oh][ow] = b[m] + sum_{c<Cg, r<k, q<k}
 *        w[m][c][r][q] * x[n][g*Cg + c][oh*s - p + r][ow*s - p + q],   g = m / Mg,
 *
 * taps outside the image contributing zero, Ho = floor((H + 2p - k)/s) + 1.
 * Inputs are FP16 bit patterns; every product and sum is taken in FP64 (the
 * product of two FP16 values is exact in FP64), which follows the paper's remark
 * that FP16 trouble arises during accumulation (Section 3.1): the reference
 * result carries no accumulation error at all.  Beside `pre` it returns
 * mag = sum |w * x| over the same taps, from which callers form the tolerance.
 * ReLU is left to the caller (max(pre, 0)).
 *
 * The loops are the seven of the definition (n, m, oh, ow, c, r, q), in that
 * order, with no blocking or reordering; OpenMP only splits the (n, m) pairs.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* IEEE 754 binary16 bit pattern -> double, from the format's definition. */
double hgo_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1F;
    int f = h & 0x3FF;
    double v;
    if (e == 0)
        v = ldexp((double)f, -24);                 /* zero and subnormals: f * 2^-24 */
    else if (e == 31)
        v = f ? NAN : INFINITY;
    else
        v = ldexp((double)(1024 + f), e - 25);     /* (1 + f/1024) * 2^(e-15) */
    return sign ? -v : v;
}

typedef struct {
    int N, C, H, W, M, k, s, p, G, bias, relu;
} geom_t;

static int read_desc(const int32_t *d, geom_t *g, int *Ho, int *Wo)
{
    g->N = d[0]; g->C = d[1]; g->H = d[2]; g->W = d[3]; g->M = d[4];
    g->k = d[5]; g->s = d[6]; g->p = d[7]; g->G = d[8]; g->bias = d[9]; g->relu = d[10];
    if (g->N < 1 || g->C < 1 || g->H < 1 || g->W < 1 || g->M < 1 || g->k < 1 ||
        g->s < 1 || g->p < 0 || g->G < 1)
        return -1;
    if (g->C % g->G || g->M % g->G)
        return -1;
    if (g->H + 2 * g->p < g->k || g->W + 2 * g->p < g->k)
        return -1;
    *Ho = (g->H + 2 * g->p - g->k) / g->s + 1;
    *Wo = (g->W + 2 * g->p - g->k) / g->s + 1;
    return 0;
}

static double *decode(const uint16_t *src, size_t n)
{
    double *d = (double *)malloc(n * sizeof(double) + 8);
    if (!d) return NULL;
    for (size_t i = 0; i < n; ++i) d[i] = hgo_half_to_double(src[i]);
    return d;
}

/* One output element: the three innermost loops of the definition. */
static void one_output(const geom_t *g, const double *x, const double *w, const double *b,
                       int n, int m, int oh, int ow, double *pre, double *mag)
{
    const int Cg = g->C / g->G, Mg = g->M / g->G;
    const int grp = m / Mg;
    double acc = (g->bias && b) ? b[m] : 0.0;
    double a = 0.0;
    for (int c = 0; c < Cg; ++c)
        for (int r = 0; r < g->k; ++r)
            for (int q = 0; q < g->k; ++q) {
                int ih = oh * g->s - g->p + r;
                int iw = ow * g->s - g->p + q;
                if (ih < 0 || ih >= g->H || iw < 0 || iw >= g->W) continue;
                double wv = w[(((size_t)m * Cg + c) * g->k + r) * g->k + q];
                double xv = x[(((size_t)n * g->C + (size_t)grp * Cg + c) * g->H + ih) * g->W + iw];
                double t = wv * xv;
                acc += t;
                a += fabs(t);
            }
    *pre = acc;
    *mag = a;
}

/*
 * Full tensor.  desc = {N,C,H,W,num_output,kernel,stride,pad,group,bias,relu};
 * x, w, b: FP16 bit patterns (b may be NULL when bias == 0); pre, mag: N*M*Ho*Wo doubles.
 * Returns 0, -1 for a bad descriptor, -2 for out of memory.
 */
int hgo_conv2d_forward(const int32_t *desc, const uint16_t *x, const uint16_t *w,
                       const uint16_t *b, double *pre, double *mag)
{
    geom_t g; int Ho, Wo;
    if (read_desc(desc, &g, &Ho, &Wo)) return -1;
    const int Cg = g.C / g.G;
    double *xd = decode(x, (size_t)g.N * g.C * g.H * g.W);
    double *wd = decode(w, (size_t)g.M * Cg * g.k * g.k);
    double *bd = (g.bias && b) ? decode(b, (size_t)g.M) : NULL;
    if (!xd || !wd || (g.bias && b && !bd)) { free(xd); free(wd); free(bd); return -2; }
    const long long NM = (long long)g.N * g.M;
#pragma omp parallel for schedule(dynamic, 1)
    for (long long nm = 0; nm < NM; ++nm) {
        int n = (int)(nm / g.M), m = (int)(nm % g.M);
        for (int oh = 0; oh < Ho; ++oh)
            for (int ow = 0; ow < Wo; ++ow) {
                size_t o = (((size_t)n * g.M + m) * Ho + oh) * Wo + ow;
                one_output(&g, xd, wd, bd, n, m, oh, ow, &pre[o], &mag[o]);
            }
    }
    free(xd); free(wd); free(bd);
    return 0;
}

/*
 * Selected outputs only (for tensors too large to evaluate in full):
 * idx holds npts quadruples (n, m, oh, ow); pre, mag: npts doubles.
 * Inputs are decoded element by element, so the cost is npts * Kg.
 * Returns 0, -1 for a bad descriptor, -3 for a coordinate out of range.
 */
int hgo_conv2d_points(const int32_t *desc, const uint16_t *x, const uint16_t *w,
                      const uint16_t *b, long long npts, const int32_t *idx,
                      double *pre, double *mag)
{
    geom_t g; int Ho, Wo;
    if (read_desc(desc, &g, &Ho, &Wo)) return -1;
    const int Cg = g.C / g.G, Mg = g.M / g.G;
    for (long long i = 0; i < npts; ++i) {
        const int32_t *q = idx + 4 * i;
        if (q[0] < 0 || q[0] >= g.N || q[1] < 0 || q[1] >= g.M ||
            q[2] < 0 || q[2] >= Ho || q[3] < 0 || q[3] >= Wo)
            return -3;
    }
#pragma omp parallel for schedule(static)
    for (long long i = 0; i < npts; ++i) {
        int n = idx[4 * i], m = idx[4 * i + 1], oh = idx[4 * i + 2], ow = idx[4 * i + 3];
        int grp = m / Mg;
        double acc = (g.bias && b) ? hgo_half_to_double(b[m]) : 0.0, a = 0.0;
        for (int c = 0; c < Cg; ++c)
            for (int r = 0; r < g.k; ++r)
                for (int qq = 0; qq < g.k; ++qq) {
                    int ih = oh * g.s - g.p + r, iw = ow * g.s - g.p + qq;
                    if (ih < 0 || ih >= g.H || iw < 0 || iw >= g.W) continue;
                    double wv = hgo_half_to_double(
                        w[(((size_t)m * Cg + c) * g.k + r) * g.k + qq]);
                    double xv = hgo_half_to_double(
                        x[(((size_t)n * g.C + (size_t)grp * Cg + c) * g.H + ih) * g.W + iw]);
                    double t = wv * xv;
                    acc += t;
                    a += fabs(t);
                }
        pre[i] = acc;
        mag[i] = a;
    }
    return 0;
}

/* Threads the parallel loops use (1 when built without OpenMP). */
int hgo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void hgo_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}
