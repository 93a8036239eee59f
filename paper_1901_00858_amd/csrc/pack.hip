// One-time re-layout of convolution weights for the implicit-GEMM kernels.
// The paper's engine pays conversion costs once, offline, and never on the
// inference path (Section 3.3: FP16 weight files, model converter); this is the
// same idea applied to the weight layout: pure data movement, no arithmetic.
#include "hgc_internal.h"

namespace hgc {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

PackedLayout packed_layout(const Geometry &g)
{
    PackedLayout pl;
    const int T = g.k * g.k;
    pl.MB8 = (g.Mg + 7) / 8;
    pl.NP8 = (g.Cg + 7) / 8;
    pl.raw_bytes = 2LL * g.M * g.Kg;
    pl.igemm_off = (pl.raw_bytes + 255) / 256 * 256;
    const long long units = (long long)g.G * pl.MB8 * pl.NP8 * T * 8;
    pl.zero_off = pl.igemm_off + (units * 16 + 255) / 256 * 256;
    pl.total = pl.zero_off + 1024;
    pl.c4_off = 0;
    pl.c4_mpad = 0;
    if (g.G == 1 && g.Cg <= 4 && (g.k == 3 || g.k == 5 || g.k == 7 || g.k == 11)) {
        pl.c4_off = pl.total;
        pl.c4_mpad = (g.M + 63) / 64 * 64;
        const long long c4_units = (long long)g.k * ((g.k + 1) / 2) * pl.c4_mpad;
        pl.total = pl.c4_off + (c4_units * 16 + 255) / 256 * 256;
    }
    return pl;
}

// One thread per 16-byte unit: the 8 channels of one (row, tap) of one plane.
__global__ __launch_bounds__(256) void pack_weights_kernel(const uint16_t *w, uint8_t *packed, int G, int Mg,
                                                           int Cg, int T, int MB8, int NP8, long long raw_bytes,
                                                           long long igemm_off, long long zero_off,
                                                           long long total, long long c4_off, int c4_mpad, int ks)
{
    const long long units = (long long)G * MB8 * NP8 * T * 8;
    const long long tid = (long long)blockIdx.x * 256 + threadIdx.x;
    const long long stride = (long long)gridDim.x * 256;
    u32x4 *out = reinterpret_cast<u32x4 *>(packed + igemm_off);
    for (long long u = tid; u < units; u += stride) {
        const int r = (int)(u % 8);
        long long v = u / 8;
        const int t = (int)(v % T); v /= T;
        const int pl = (int)(v % NP8); v /= NP8;
        const int mb = (int)(v % MB8);
        const int g = (int)(v / MB8);
        const int m = mb * 8 + r;
        uint32_t h[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int c = pl * 8 + j;
            h[j] = (m < Mg && c < Cg) ? w[(((size_t)g * Mg + m) * Cg + c) * T + t] : 0u;
        }
        u32x4 o = {h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
        out[u] = o;
    }
    // verbatim copy (used by the non-MFMA kernels) and the zero regions
    uint16_t *raw = reinterpret_cast<uint16_t *>(packed);
    for (long long i = tid; i < raw_bytes / 2; i += stride) raw[i] = w[i];
    for (long long i = raw_bytes / 2 + tid; i < igemm_off / 2; i += stride) raw[i] = 0;
    const long long tail_end = c4_off ? c4_off : total;
    for (long long i = (igemm_off + units * 16) / 2 + tid; i < tail_end / 2; i += stride) raw[i] = 0;
    if (c4_off) {
        // first-layer section: unit (r, qp, m) = taps (r, 2qp) and (r, 2qp+1), 4 channels each
        const int qpn = (ks + 1) / 2;
        const long long c4_units = (long long)ks * qpn * c4_mpad;
        u32x4 *c4 = reinterpret_cast<u32x4 *>(packed + c4_off);
        for (long long u = tid; u < (total - c4_off) / 16; u += stride) {
            uint32_t h[8] = {0, 0, 0, 0, 0, 0, 0, 0};
            if (u < c4_units) {
                const int m = (int)(u % c4_mpad);
                const int qp = (int)((u / c4_mpad) % qpn), r = (int)(u / c4_mpad / qpn);
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int q = 2 * qp + (j >> 2), c = j & 3;
                    if (m < Mg && c < Cg && q < ks) h[j] = w[(((size_t)m * Cg + c) * ks + r) * ks + q];
                }
            }
            u32x4 o = {h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
            c4[u] = o;
        }
    }
}

hipError_t launch_pack_weights(const Geometry &g, const PackedLayout &pl, const uint16_t *w, uint8_t *packed,
                               hipStream_t stream)
{
    const long long units = (long long)g.G * pl.MB8 * pl.NP8 * g.k * g.k * 8;
    long long blocks = (units + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(pack_weights_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, w, packed, g.G, g.Mg,
                       g.Cg, g.k * g.k, pl.MB8, pl.NP8, pl.raw_bytes, pl.igemm_off, pl.zero_off, pl.total, pl.c4_off,
                       pl.c4_mpad, g.k);
    return hipGetLastError();
}

}  // namespace hgc
