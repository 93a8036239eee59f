// Max-pooling layer forward in FP16 for gfx950: BVLC Caffe's MAX pooling (the paper keeps Caffe's
// layers, Sections 2 and 5; the networks of its Section 4 pool between their convolutions), the
// step that sits between the convolutions of a chained forward pass.
//   Ho = ceil((H + 2p - k) / s) + 1, one less if p > 0 and the last window would start at or
//   beyond H + p; y = maximum of the window clipped to the image (padding never takes part).
// The result is one of the inputs: there is no rounding, FP16 values are compared as they are.
// The layer is pure data movement (2 bytes read per input value, 2 written per output): the
// 2x2 / stride 2 / no padding window of VGG-shaped nets on rows whose length is a multiple of 8
// takes a vector form (a thread reads 8 values of each of the two rows with 16-byte loads,
// v_pk_max_f16 down the rows, then across the pairs, and stores 4 outputs); every other window
// takes a thread per output.
#include "hgc_internal.h"

namespace hgc {

typedef _Float16 mp_h2 __attribute__((ext_vector_type(2)));
typedef uint32_t mp_u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t mp_u32x4 __attribute__((ext_vector_type(4)));

struct PoolArgs {
    const uint16_t *x;
    uint16_t *y;
    int H, W, Ho, Wo, k, s, p;
    uint32_t total;          // outputs (generic) or 4-output vectors (2x2 form)
    FastDiv fd_Wo, fd_Ho, fd_wv;
};

static int pool_out(int size, int k, int s, int p)
{
    const int span = size + 2 * p - k;
    int o = (span + s - 1) / s + 1;
    if (p > 0 && (o - 1) * s >= size + p) --o;
    return o;
}

__global__ __launch_bounds__(256) void max_pool_kernel(const PoolArgs a)
{
    const uint32_t o = blockIdx.x * 256u + threadIdx.x;
    if (o >= a.total) return;
    const uint32_t t = fast_div(o, a.fd_Wo);
    const int ow = (int)(o - t * (uint32_t)a.Wo);
    const uint32_t plane = fast_div(t, a.fd_Ho);
    const int oh = (int)(t - plane * (uint32_t)a.Ho);
    const int h0 = max(oh * a.s - a.p, 0), h1 = min(oh * a.s - a.p + a.k, a.H);
    const int w0 = max(ow * a.s - a.p, 0), w1 = min(ow * a.s - a.p + a.k, a.W);
    const uint16_t *src = a.x + (size_t)plane * a.H * a.W;
    _Float16 best = __builtin_bit_cast(_Float16, src[(size_t)h0 * a.W + w0]);
    for (int ih = h0; ih < h1; ++ih)
        for (int iw = w0; iw < w1; ++iw) {
            const _Float16 v = __builtin_bit_cast(_Float16, src[(size_t)ih * a.W + iw]);
            best = v > best ? v : best;
        }
    a.y[o] = __builtin_bit_cast(uint16_t, best);
}

__device__ __forceinline__ uint32_t mp_max2(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(mp_h2, a), __builtin_bit_cast(mp_h2, b)));
}
// maxima of the two pairs (a.lo, a.hi) and (b.lo, b.hi), packed
__device__ __forceinline__ uint32_t mp_pairs(uint32_t a, uint32_t b)
{
    const uint32_t lo = (a & 0xFFFFu) | (b << 16);          // a.lo, b.lo
    const uint32_t hi = (a >> 16) | (b & 0xFFFF0000u);      // a.hi, b.hi
    return mp_max2(lo, hi);
}

// k = 2, s = 2, p = 0, W % 8 == 0, 16-byte aligned x, 8-byte aligned y: a thread makes 4 outputs.
__global__ __launch_bounds__(256) void max_pool_2x2_kernel(const PoolArgs a)
{
    const uint32_t v = blockIdx.x * 256u + threadIdx.x;
    if (v >= a.total) return;
    const uint32_t row = fast_div(v, a.fd_wv);               // plane * Ho + oh
    const uint32_t wv = v - row * a.fd_wv.d;
    const uint32_t plane = fast_div(row, a.fd_Ho);
    const int oh = (int)(row - plane * (uint32_t)a.Ho);
    const size_t in0 = ((size_t)plane * a.H + 2 * oh) * a.W + 8 * wv;
    const mp_u32x4 r0 = *reinterpret_cast<const mp_u32x4 *>(a.x + in0);
    // an odd H leaves a last window of one row
    const mp_u32x4 r1 = (2 * oh + 1 < a.H) ? *reinterpret_cast<const mp_u32x4 *>(a.x + in0 + a.W) : r0;
    mp_u32x2 out;
    out.x = mp_pairs(mp_max2(r0.x, r1.x), mp_max2(r0.y, r1.y));
    out.y = mp_pairs(mp_max2(r0.z, r1.z), mp_max2(r0.w, r1.w));
    *reinterpret_cast<mp_u32x2 *>(a.y + (size_t)row * a.Wo + 4 * wv) = out;
}

static hgc_status pool_check(const hgc_max_pool_desc *d)
{
    if (d->N < 1 || d->C < 1 || d->H < 1 || d->W < 1 || d->kernel < 1 || d->stride < 1 || d->pad < 0 ||
        d->pad >= d->kernel)
        return HGC_ERR_BAD_DESC;
    if (d->H + 2 * d->pad < d->kernel || d->W + 2 * d->pad < d->kernel) return HGC_ERR_BAD_DESC;
    if ((long long)d->N * d->C * d->H * d->W > 0x7FFFFFFFLL) return HGC_ERR_TOO_LARGE;
    const long long out = (long long)d->N * d->C * pool_out(d->H, d->kernel, d->stride, d->pad) *
                          pool_out(d->W, d->kernel, d->stride, d->pad);
    if (out > 0x7FFFFFFFLL) return HGC_ERR_TOO_LARGE;
    return HGC_OK;
}

}  // namespace hgc

using namespace hgc;

extern "C" hgc_status hgc_max_pool_output_size(const hgc_max_pool_desc *desc, int32_t *Ho, int32_t *Wo)
{
    if (!desc || !Ho || !Wo) return HGC_ERR_NULL;
    const hgc_status st = pool_check(desc);
    if (st != HGC_OK) return st;
    *Ho = pool_out(desc->H, desc->kernel, desc->stride, desc->pad);
    *Wo = pool_out(desc->W, desc->kernel, desc->stride, desc->pad);
    return HGC_OK;
}

extern "C" hgc_status hgc_max_pool_forward(const hgc_max_pool_desc *desc, const void *x, void *y, void *stream)
{
    if (!desc || !x || !y) return HGC_ERR_NULL;
    const hgc_status st = pool_check(desc);
    if (st != HGC_OK) return st;
    PoolArgs a;
    a.x = static_cast<const uint16_t *>(x);
    a.y = static_cast<uint16_t *>(y);
    a.H = desc->H; a.W = desc->W; a.k = desc->kernel; a.s = desc->stride; a.p = desc->pad;
    a.Ho = pool_out(a.H, a.k, a.s, a.p);
    a.Wo = pool_out(a.W, a.k, a.s, a.p);
    const long long planes = (long long)desc->N * desc->C;
    a.fd_Wo = make_fastdiv((uint32_t)a.Wo);
    a.fd_Ho = make_fastdiv((uint32_t)a.Ho);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool vec = a.k == 2 && a.s == 2 && a.p == 0 && a.W % 8 == 0 && ((uintptr_t)x & 15) == 0 && ((uintptr_t)y & 7) == 0;
    if (vec) {
        a.fd_wv = make_fastdiv((uint32_t)(a.W / 8));
        a.total = (uint32_t)(planes * a.Ho * (a.W / 8));
        max_pool_2x2_kernel<<<dim3((a.total + 255) / 256), dim3(256), 0, s>>>(a);
    } else {
        a.fd_wv = make_fastdiv(1);
        a.total = (uint32_t)(planes * a.Ho * a.Wo);
        max_pool_kernel<<<dim3((a.total + 255) / 256), dim3(256), 0, s>>>(a);
    }
    const hipError_t e = hipGetLastError();
    set_last_hip_error(e);
    return e == hipSuccess ? HGC_OK : HGC_ERR_LAUNCH;
}
