// Implicit-GEMM convolution forward on FP16 MFMA for gfx950.
//
// Per group the layer is the contraction  Y[Mg x P] = W[Mg x Kg] * B[Kg x P],
// where B is the im2col matrix of the input (Caffe's formulation, which the paper
// keeps: Section 2).  B is never built.  A workgroup owns BM output channels and
// a TH x TW window of output pixels of one image.  For each block of CB = 8*NPL
// input channels it stages into LDS
//   - the input halo patch of that window, PH x PW pixels, ONCE for all k*k taps,
//     stored channel-innermost: one 16-byte unit = 8 channels of one pixel;
//   - the weight slab BM x CB x k*k, regrouped so that one 16-byte unit = 8
//     channels of one (row, tap).
// With that layout both MFMA operands of v_mfma_f32_32x32x16_f16 are single
// ds_read_b128 per lane: lanes 0..31 take channels 0..7 of a 16-channel pair of
// planes, lanes 32..63 channels 8..15; a tap (r,q) only shifts the patch address.
// The order in which the reduction index (c, r, q) is walked differs from the
// weight layout's; the sum does not depend on it beyond FP32 rounding.
// Accumulation is FP32 in the MFMA accumulators (paper Section 3.1: overflow and
// underflow arise during accumulation); bias, ReLU and the single FP32->FP16
// rounding happen in registers before the store (no conversion pass, Section 3.3).
#include <atomic>

#include "hgc_internal.h"

namespace hgc {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t pack_lo(uint32_t a, uint32_t b)   // a.lo | b.lo << 16
{
    return __builtin_amdgcn_perm(b, a, 0x05040100u);
}
__device__ __forceinline__ uint32_t pack_hi(uint32_t a, uint32_t b)   // a.hi | b.hi << 16
{
    return __builtin_amdgcn_perm(b, a, 0x07060302u);
}

// Decoded staging item of the input patch: XVEC pixels x 8 channels.
struct PatchItem {
    int goff;    // element offset of (channel 0 of the plane, pixel) from the channel-block base
    int unit;    // LDS unit index of the first pixel
    int pl8;     // first channel of the plane within the block (plane * 8)
    int flags;   // bit0: item exists, bit1: pixel(s) inside the image
};

template <int XVEC>
__device__ __forceinline__ PatchItem decode_patch_item(int id, int total, int ipr, int PH, int PWU,
                                                       int ih0, int iwa, int H, int W, int HW)
{
    PatchItem it;
    int pd = id % ipr;
    int t = id / ipr;
    int ph = t % PH;
    int pl = t / PH;
    int ih = ih0 + ph;
    int iw = iwa + pd * XVEC;
    bool active = id < total;
    bool inside = active && ih >= 0 && ih < H && iw >= 0 && iw < W;
    it.goff = pl * 8 * HW + ih * W + iw;
    it.unit = (pl * PH + ph) * PWU + pd * XVEC;
    it.pl8 = pl * 8;
    it.flags = (active ? 1 : 0) | (inside ? 2 : 0);
    return it;
}

template <int XVEC, bool CALIGN>
__device__ __forceinline__ void load_patch_item(const uint16_t *xcb, const PatchItem &it, int c0,
                                                int Cg, int HW, uint32_t (&d)[8])
{
    const bool inside = (it.flags & 2) != 0;
    if (CALIGN) {
        const bool ok = inside && (c0 + it.pl8 < Cg);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            uint32_t v = 0;
            if (ok) {
                if (XVEC == 2) v = *reinterpret_cast<const uint32_t *>(xcb + it.goff + j * HW);
                else v = xcb[it.goff + j * HW];
            }
            d[j] = v;
        }
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            uint32_t v = 0;
            if (inside && (c0 + it.pl8 + j < Cg)) {
                if (XVEC == 2) v = *reinterpret_cast<const uint32_t *>(xcb + it.goff + j * HW);
                else v = xcb[it.goff + j * HW];
            }
            d[j] = v;
        }
    }
}

template <int XVEC>
__device__ __forceinline__ void store_patch_item(u32x4 *xl, const PatchItem &it, const uint32_t (&d)[8])
{
    if (!(it.flags & 1)) return;
    u32x4 u0;
    u0.x = pack_lo(d[0], d[1]); u0.y = pack_lo(d[2], d[3]);
    u0.z = pack_lo(d[4], d[5]); u0.w = pack_lo(d[6], d[7]);
    xl[it.unit] = u0;
    if (XVEC == 2) {
        u32x4 u1;
        u1.x = pack_hi(d[0], d[1]); u1.y = pack_hi(d[2], d[3]);
        u1.z = pack_hi(d[4], d[5]); u1.w = pack_hi(d[6], d[7]);
        xl[it.unit + 1] = u1;
    }
}

// KS: kernel extent.  A, B: 32x32 accumulator blocks per wave along channels and
// pixels.  WAVES_M: waves along channels (4 waves per workgroup).  NPL: 8-channel
// planes per K step.  XVEC: input pixels per global load (2 needs even W and a
// 4-byte aligned base).  CALIGN: Cg % 8 == 0 and a 16-byte aligned weight base.
// MAXR: staging rounds of the patch that are prefetched through registers.
// SPLITK: write FP32 partial sums of a slice of the channel blocks.
template <int KS, int A, int B, int WAVES_M, int NPL, int XVEC, bool CALIGN, int MAXR, bool SPLITK>
__global__ __launch_bounds__(256) void igemm_kernel(const ConvArgs p)
{
    constexpr int WAVES_N = 4 / WAVES_M;
    constexpr int BM = 32 * A * WAVES_M;
    constexpr int BN = 32 * B * WAVES_N;
    constexpr int T = KS * KS;
    constexpr int CB = 8 * NPL;
    constexpr int W_UNITS = T * NPL * BM;
    constexpr int W_ITEMS = BM * NPL;
    constexpr int WR = (W_ITEMS + 255) / 256;
    constexpr bool WPREFETCH = CALIGN && (T * WR <= 9);
    static_assert(NPL % 2 == 0, "planes come in pairs (16 channels per MFMA)");

    extern __shared__ u32x4 lds[];
    u32x4 *wl = lds;              // [T][NPL][BM]
    u32x4 *xl = lds + W_UNITS;    // [NPL][PH][PWU]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WAVES_M;
    const int wn = wave / WAVES_M;
    const int l32 = lane & 31;
    const int lh = lane >> 5;

    int bid = blockIdx.x;
    const int tm = bid % p.tiles_m; bid /= p.tiles_m;
    const int twi = bid % p.tiles_w; bid /= p.tiles_w;
    const int thi = bid % p.tiles_h; bid /= p.tiles_h;
    const int g = bid % p.G; bid /= p.G;
    const int n = bid % p.N; bid /= p.N;
    const int ksl = bid;

    const int TW = 1 << p.log2_tw;
    const int TH = BN >> p.log2_tw;
    const int oh0 = thi * TH, ow0 = twi * TW;
    const int m0 = tm * BM;
    const int s = p.stride;
    const int ih0 = oh0 * s - p.pad;
    const int iw0 = ow0 * s - p.pad;
    const int iwa = (XVEC == 2) ? (iw0 & ~1) : iw0;
    const int cofs = iw0 - iwa;
    const int PH = p.PH, PWU = p.PWU;
    const int HW = p.H * p.W;
    const int Cg = p.Cg, Mg = p.Mg;

    // ---- staging maps (do not depend on the K step) ----
    const int ipr = PWU / XVEC;                 // items per patch row
    const int total_items = NPL * PH * ipr;
    const int rounds = (total_items + 255) >> 8;
    PatchItem pit[MAXR];
#pragma unroll
    for (int r = 0; r < MAXR; ++r)
        pit[r] = decode_patch_item<XVEC>(r * 256 + tid, total_items, ipr, PH, PWU, ih0, iwa, p.H, p.W, HW);

    const uint16_t *xg = p.x + ((size_t)n * p.C + (size_t)g * Cg) * HW;
    const uint16_t *wg = p.w + (size_t)g * Mg * Cg * T;

    uint32_t xreg[MAXR][8];
    u32x4 wreg[WPREFETCH ? WR : 1][T];

    auto load_x = [&](int st) {
        const uint16_t *xcb = xg + (size_t)st * CB * HW;
#pragma unroll
        for (int r = 0; r < MAXR; ++r)
            load_patch_item<XVEC, CALIGN>(xcb, pit[r], st * CB, Cg, HW, xreg[r]);
    };
    auto store_x = [&](int st) {
#pragma unroll
        for (int r = 0; r < MAXR; ++r) store_patch_item<XVEC>(xl, pit[r], xreg[r]);
        // patches larger than the prefetch capacity: remaining rounds, not pipelined
        if (rounds > MAXR) {
            const uint16_t *xcb = xg + (size_t)st * CB * HW;
            for (int r = MAXR; r < rounds; ++r) {
                PatchItem it = decode_patch_item<XVEC>(r * 256 + tid, total_items, ipr, PH, PWU,
                                                       ih0, iwa, p.H, p.W, HW);
                uint32_t d[8];
                load_patch_item<XVEC, CALIGN>(xcb, it, st * CB, Cg, HW, d);
                store_patch_item<XVEC>(xl, it, d);
            }
        }
    };

    // weights: item = (row m of the tile, plane); T taps x 8 channels each
    auto load_w_vec = [&](int st, int r, u32x4 (&wv)[T]) {
        const int id = r * 256 + tid;
        const int m = id % BM, pl = id / BM;
        const bool ok = (id < W_ITEMS) && (m0 + m < Mg) && (st * CB + pl * 8 < Cg);
        const u32x4 *src = reinterpret_cast<const u32x4 *>(
            wg + ((size_t)(m0 + m) * Cg + st * CB + pl * 8) * T);
#pragma unroll
        for (int t = 0; t < T; ++t) {
            u32x4 v = {0u, 0u, 0u, 0u};
            if (ok) v = src[t];
            wv[t] = v;
        }
    };
    auto store_w_vec = [&](int r, const u32x4 (&wv)[T]) {
        const int id = r * 256 + tid;
        if (id >= W_ITEMS) return;
        const int m = id % BM, pl = id / BM;
        // wv as 4T dwords holds halves e = c*T + tap (c = 0..7); regroup per tap
#pragma unroll
        for (int t = 0; t < T; ++t) {
            uint32_t o[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int ea = (2 * i) * T + t, eb = (2 * i + 1) * T + t;
                const int da = ea >> 1, db = eb >> 1;
                const uint32_t va = wv[da >> 2][da & 3];
                const uint32_t vb = wv[db >> 2][db & 3];
                const uint32_t sel = ((ea & 1) ? 0x0302u : 0x0100u) | (((eb & 1) ? 0x0706u : 0x0504u) << 16);
                o[i] = __builtin_amdgcn_perm(vb, va, sel);
            }
            u32x4 u = {o[0], o[1], o[2], o[3]};
            wl[(t * NPL + pl) * BM + m] = u;
        }
    };
    auto stage_w_scalar = [&](int st) {    // any Cg, any alignment: 2-byte loads
        for (int r = 0; r < WR; ++r) {
            const int id = r * 256 + tid;
            if (id >= W_ITEMS) continue;
            const int m = id % BM, pl = id / BM;
            const bool rowok = (m0 + m < Mg);
            const int c0 = st * CB + pl * 8;
            const uint16_t *src = wg + ((size_t)(m0 + m) * Cg + c0) * T;
            for (int t = 0; t < T; ++t) {
                uint32_t h[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    uint32_t v = 0;
                    if (rowok && (c0 + j < Cg)) v = src[j * T + t];
                    h[j] = v;
                }
                u32x4 u = {h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
                wl[(t * NPL + pl) * BM + m] = u;
            }
        }
    };
    auto load_w = [&](int st) {
        if (WPREFETCH) {
#pragma unroll
            for (int r = 0; r < WR; ++r) load_w_vec(st, r, wreg[r]);
        }
    };
    auto store_w = [&](int st) {
        if (WPREFETCH) {
#pragma unroll
            for (int r = 0; r < WR; ++r) store_w_vec(r, wreg[r]);
        } else if (CALIGN) {
            for (int r = 0; r < WR; ++r) {
                u32x4 wv[T];
                load_w_vec(st, r, wv);
                store_w_vec(r, wv);
            }
        } else {
            stage_w_scalar(st);
        }
    };

    // ---- MFMA operand addresses ----
    int xb[B];
#pragma unroll
    for (int j = 0; j < B; ++j) {
        const int pix = (wn * B + j) * 32 + l32;
        const int th = pix >> p.log2_tw, tw = pix & (TW - 1);
        xb[j] = (lh * PH + th * s) * PWU + tw * s + cofs;
    }
    const int ab = lh * BM + wm * (32 * A) + l32;
    const int plane_pair_stride = 2 * PH * PWU;

    floatx16 acc[A][B];
#pragma unroll
    for (int i = 0; i < A; ++i)
#pragma unroll
        for (int j = 0; j < B; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    auto compute = [&]() {
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const int r = t / KS, q = t % KS;
            const int toff = r * PWU + q;
#pragma unroll
            for (int pp = 0; pp < NPL / 2; ++pp) {
                half8 af[A], bf[B];
#pragma unroll
                for (int i = 0; i < A; ++i)
                    af[i] = __builtin_bit_cast(half8, wl[(t * NPL + pp * 2) * BM + ab + i * 32]);
#pragma unroll
                for (int j = 0; j < B; ++j)
                    bf[j] = __builtin_bit_cast(half8, xl[xb[j] + toff + pp * plane_pair_stride]);
#pragma unroll
                for (int i = 0; i < A; ++i)
#pragma unroll
                    for (int j = 0; j < B; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[i], bf[j], acc[i][j], 0, 0, 0);
            }
        }
    };

    // ---- K loop over channel blocks ----
    int st0 = 0, st1 = p.nsteps;
    if (SPLITK) {
        st0 = ksl * p.steps_per_split;
        st1 = min(p.nsteps, st0 + p.steps_per_split);
    }
    if (st0 < st1) {
        load_x(st0);
        load_w(st0);
    }
    for (int st = st0; st < st1; ++st) {
        __syncthreads();
        store_x(st);
        store_w(st);
        __syncthreads();
        if (st + 1 < st1) {
            load_x(st + 1);
            load_w(st + 1);
        }
        compute();
    }

    // ---- epilogue: accumulator register e of lane (l32, lh) in block (i, j) is
    // channel row 8*(e/4) + 4*lh + e%4 and pixel column l32 of that block ----
    const int HoWo = p.Ho * p.Wo;
#pragma unroll
    for (int j = 0; j < B; ++j) {
        const int pix = (wn * B + j) * 32 + l32;
        const int oh = oh0 + (pix >> p.log2_tw), ow = ow0 + (pix & (TW - 1));
        const bool pix_ok = (oh < p.Ho) && (ow < p.Wo);
#pragma unroll
        for (int i = 0; i < A; ++i) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int ml = m0 + wm * (32 * A) + i * 32 + 8 * (e >> 2) + 4 * lh + (e & 3);
                if (pix_ok && ml < Mg) {
                    const int mg = g * Mg + ml;
                    float v = acc[i][j][e];
                    if (SPLITK) {
                        p.ws[(((size_t)ksl * p.N + n) * p.M + mg) * HoWo + oh * p.Wo + ow] = v;
                    } else {
                        if (p.bias) {
                            _Float16 hb = __builtin_bit_cast(_Float16, p.b[mg]);
                            v += (float)hb;
                        }
                        if (p.relu) v = fmaxf(v, 0.0f);
                        _Float16 hv = (_Float16)v;
                        p.y[((size_t)n * p.M + mg) * HoWo + oh * p.Wo + ow] = __builtin_bit_cast(uint16_t, hv);
                    }
                }
            }
        }
    }
}

// LDS beyond 64 KB per workgroup has to be requested per kernel; remember the
// largest request so the attribute is set at most a few times per process.
template <typename Kern>
static hipError_t ensure_lds(Kern kern, size_t lds, std::atomic<size_t> &granted)
{
    if (lds <= 64 * 1024 || lds <= granted.load(std::memory_order_acquire)) return hipSuccess;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e == hipSuccess) granted.store(lds, std::memory_order_release);
    return e;
}

template <int KS, int A, int B, int WAVES_M, int NPL, int XVEC, bool CALIGN, int MAXR>
static hipError_t launch_igemm(const ConvArgs &a, dim3 grid, hipStream_t stream)
{
    constexpr int W_UNITS = KS * KS * NPL * 32 * A * WAVES_M;
    const size_t lds = (size_t)(W_UNITS + NPL * a.PH * a.PWU) * 16;
    hipError_t e;
    if (a.split_k > 1) {
        static std::atomic<size_t> granted{0};
        auto kern = igemm_kernel<KS, A, B, WAVES_M, NPL, XVEC, CALIGN, MAXR, true>;
        if ((e = ensure_lds(kern, lds, granted)) != hipSuccess) return e;
        hipLaunchKernelGGL(kern, grid, dim3(256), lds, stream, a);
    } else {
        static std::atomic<size_t> granted{0};
        auto kern = igemm_kernel<KS, A, B, WAVES_M, NPL, XVEC, CALIGN, MAXR, false>;
        if ((e = ensure_lds(kern, lds, granted)) != hipSuccess) return e;
        hipLaunchKernelGGL(kern, grid, dim3(256), lds, stream, a);
    }
    return hipGetLastError();
}

#define HGC_VARIANT(KS, A, B, WM, NPL, XVEC, CAL, MAXR)                                        \
    {KS, A, B, WM, NPL, XVEC, CAL, MAXR, KS * KS * NPL * 32 * A * WM * 16,                      \
     &launch_igemm<KS, A, B, WM, NPL, XVEC, (CAL != 0), MAXR>}

// For each kernel extent: vector-load and scalar-load forms of each tile shape.
static const IgemmVariant g_variants[] = {
    //          KS  A  B  WM NPL XVEC CAL MAXR
    HGC_VARIANT(3, 2, 4, 2, 2, 2, 1, 3),   // 128 ch x 256 px
    HGC_VARIANT(3, 2, 4, 2, 2, 1, 1, 3),
    HGC_VARIANT(3, 2, 4, 2, 2, 2, 0, 3),
    HGC_VARIANT(3, 2, 4, 2, 2, 1, 0, 3),
    HGC_VARIANT(3, 2, 2, 1, 2, 2, 1, 3),   //  64 ch x 256 px
    HGC_VARIANT(3, 2, 2, 1, 2, 1, 1, 3),
    HGC_VARIANT(3, 2, 2, 1, 2, 2, 0, 3),
    HGC_VARIANT(3, 2, 2, 1, 2, 1, 0, 3),
    HGC_VARIANT(1, 2, 4, 2, 8, 2, 1, 4),   // pointwise: 64 channels per step
    HGC_VARIANT(1, 2, 4, 2, 8, 1, 1, 4),
    HGC_VARIANT(1, 2, 4, 2, 8, 2, 0, 4),
    HGC_VARIANT(1, 2, 4, 2, 8, 1, 0, 4),
    HGC_VARIANT(1, 2, 2, 1, 8, 2, 1, 4),
    HGC_VARIANT(1, 2, 2, 1, 8, 1, 1, 4),
    HGC_VARIANT(1, 2, 2, 1, 8, 2, 0, 4),
    HGC_VARIANT(1, 2, 2, 1, 8, 1, 0, 4),
    HGC_VARIANT(5, 2, 2, 1, 2, 2, 1, 3),
    HGC_VARIANT(5, 2, 2, 1, 2, 1, 1, 3),
    HGC_VARIANT(5, 2, 2, 1, 2, 2, 0, 3),
    HGC_VARIANT(5, 2, 2, 1, 2, 1, 0, 3),
    HGC_VARIANT(7, 1, 2, 1, 2, 2, 0, 3),   // stem-like: 32 ch x 256 px
    HGC_VARIANT(7, 1, 2, 1, 2, 1, 0, 3),
};

const IgemmVariant *igemm_variants(int *count)
{
    *count = (int)(sizeof(g_variants) / sizeof(g_variants[0]));
    return g_variants;
}

}  // namespace hgc
