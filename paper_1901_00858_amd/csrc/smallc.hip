// First-layer convolutions (at most 4 input channels, one group) on FP16 MFMA for gfx950.
//
// With C = 3 the general kernel pads the channels of every tap to 16 for one MFMA and
// wastes four fifths of its loads and MFMAs.  Here the taps are folded into the reduction
// instead: the reduction index of one MFMA (16 values) is two pairs of horizontally adjacent
// taps x 4 channels.  The input halo patch is staged in LDS with 8-byte units = the 4
// channels of one pixel, so the operand of a tap pair (r, 2*qp), (r, 2*qp+1) for a pixel is
// the 16 bytes of two adjacent patch pixels: one read, whatever the stride.  The weights come
// from the packed buffer's first-layer section (pack.hip): 16-byte units [tap row r][pair
// qp][output channel] = {tap 2qp: c0..c3, tap 2qp+1: c0..c3}, zero past C, k and M; the
// caller-layout form (PACKED = false) gathers the same units from w[m][c][r][q] itself.  The
// whole reduction (k*ceil(k/2) units of 8) fits LDS at once, so there is no K loop: stage,
// one barrier, MFMAs, epilogue.  Same arithmetic as everywhere: FP16 products, FP32
// accumulation starting from the bias, one rounding (paper Sections 3.1 and 3.3).
#include <atomic>

#include "hgc_internal.h"
#include "tile_store.h"

namespace hgc {

typedef uint32_t u32x2s __attribute__((ext_vector_type(2)));
typedef u32x2s __attribute__((may_alias)) u32x2_alias;

// KS: kernel extent.  A: 32-row blocks of output channels (BM = 32*A), B: 32-pixel blocks per
// wave; 4 waves along the pixels (BN = 128*B).  XV: input pixels per global load (2 or 1).
template <int KS, int A, int B, int XV, bool PACKED>
__global__ __launch_bounds__(256) void smallc_kernel(const ConvArgs p)
{
    constexpr int NW = 4;
    constexpr int BM = 32 * A, BN = 32 * B * NW;
    constexpr int QP = (KS + 1) / 2;             // tap pairs per kernel row
    constexpr int NG = KS * QP;                  // 8-value units of the reduction
    constexpr int NT2 = (NG + 1) / 2;            // MFMAs per accumulator block (two units each)
    constexpr int NGP = 2 * NT2;
    constexpr int BIAS_UNITS = NW * 8 * A;
    constexpr int W_UNITS = NGP * BM;

    extern __shared__ u32x4 lds_raw[];
    u32x4 *const wl = lds_raw + BIAS_UNITS;
    u32x2_alias *const xl = reinterpret_cast<u32x2_alias *>(wl + W_UNITS);   // 8-byte units: one pixel

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, lh = lane >> 5;
    const int nblk = p.grid_blocks;
    int bid;
    {
        const int per = (nblk + 7) >> 3;         // contiguous tile ranges per XCD
        bid = (blockIdx.x & 7) * per + (blockIdx.x >> 3);
        if (bid >= nblk) return;
    }
    int q = (int)fast_div((uint32_t)bid, p.fd_tiles_m);
    const int tm = bid - q * p.tiles_m; bid = q;
    q = (int)fast_div((uint32_t)bid, p.fd_tiles_w);
    const int twi = bid - q * p.tiles_w; bid = q;
    const int n = (int)fast_div((uint32_t)bid, p.fd_tiles_h);
    const int thi = bid - n * p.tiles_h;
    const int TW = 1 << p.log2_tw;               // one image per tile: log2_ti = 0, 2^log2_thi = BN / TW rows
    const int oh0 = thi << p.log2_thi, ow0 = twi * TW, m0 = tm * BM;
    const int s = p.stride;
    const int ih0 = oh0 * s - p.pad, iw0 = ow0 * s - p.pad;
    const int iwa = iw0 & ~(XV - 1), cofs = iw0 - iwa;
    const int PH = p.PH, PWU = p.PWU;            // patch rows, pixels per patch row (even)
    const int HW = p.H * p.W;

    const __amdgpu_buffer_rsrc_t rx = make_rsrc(p.x, p.x_bytes);
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(p.w, p.w_bytes);

    // bias of the wave's rows, fetched early (see init below)
    constexpr int BROWS = (BM + 63) / 64;
    float bias_row[BROWS];
    const __amdgpu_buffer_rsrc_t rb = make_rsrc(p.bias ? (const void *)p.b : (const void *)p.x, p.bias ? 2u * (uint32_t)p.M : 0u);
#pragma unroll
    for (int r = 0; r < BROWS; ++r) {
        const int ml = m0 + lane + 64 * r;
        // range-checked (zero where there is no bias or no such row); no branch, no wait of its own
        const bool want = lane + 64 * r < BM && ml < p.M;
        const uint16_t raw = __builtin_amdgcn_raw_buffer_load_b16(rb, want ? 2u * (uint32_t)ml : kNoLoad, 0, 0);
        bias_row[r] = (float)__builtin_bit_cast(_Float16, raw);
    }

    if constexpr (PACKED) {
        // ---- weights: LDS-direct loads of whole 64-unit runs, already in operand order ----
        constexpr int WROUNDS = (W_UNITS / 64 + NW - 1) / NW;
#pragma unroll
        for (int k = 0; k < WROUNDS; ++k) {
            const int run = k * NW + wave;       // 64 units: BM/64... rows of one unit index (or two, BM = 32)
            const int u = run * 64 + lane;
            const int kg = u / BM, row = u % BM;
            const bool real = (run * 64 < W_UNITS) && kg < NG;
            const uint32_t vo = real ? p.wp_off + 16u * (uint32_t)(kg * p.MB8 + m0 + row) : p.wp_zero;
            if (run * 64 < W_UNITS)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, (lds_ptr_t)(wl + run * 64), 16, vo, 0, 0, 0);
        }
    } else {
        // ---- weights in the caller's layout w[m][c][r][q]: unit (r, qp, row) gathers taps (r, 2qp) and
        // (r, 2qp+1) of its row's (up to) 4 channels, eight 2-byte range-checked loads (zero past C, k, M
        // and for the padding unit); WU units per thread in flight at a time ----
        constexpr int WU = 2;
        for (int u0 = tid; u0 < W_UNITS; u0 += 256 * WU) {
            uint32_t h[WU][8];
#pragma unroll
            for (int uu = 0; uu < WU; ++uu) {
                const int u = u0 + 256 * uu;
                const int kg = u / BM, row = u % BM;
                const int r = kg / QP, qp = kg % QP, m = m0 + row;
                const bool unit_ok = u < W_UNITS && kg < NG && m < p.M;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int q = 2 * qp + (j >> 2), c = j & 3;
                    const bool ok = unit_ok && c < p.C && q < KS;
                    const uint32_t off = ok ? 2u * (uint32_t)(((m * p.C + c) * KS + r) * KS + q) : kNoLoad;
                    h[uu][j] = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rw, off, 0, 0);
                }
            }
#pragma unroll
            for (int uu = 0; uu < WU; ++uu) {
                const int u = u0 + 256 * uu;
                if (u >= W_UNITS) continue;
                const u32x4 v = {h[uu][0] | (h[uu][1] << 16), h[uu][2] | (h[uu][3] << 16), h[uu][4] | (h[uu][5] << 16),
                                 h[uu][6] | (h[uu][7] << 16)};
                wl[u] = v;
            }
        }
    }

    // ---- input patch: XV pixels x 4 channels per item, transposed to pixel-major units ----
    const int ipr = PWU / XV;
    const int items = PH * ipr;
    const uint32_t img_off = 2u * (uint32_t)(n * p.C * HW);
    // U items per thread and round, the loads of all of them issued before the first is stored (large
    // kernels with a stride have patches of thousands of items: one round trip per item would dominate).
    // An item past the end loads from an out-of-range offset and stores nothing.
    constexpr int U = KS >= 7 ? 4 : 1;
    for (int id0 = tid; id0 < items; id0 += 256 * U) {
        uint32_t d[U][4];
        int ph[U], pd[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int id = id0 + 256 * u;
            ph[u] = (int)fast_div((uint32_t)id, p.fd_ipr);
            pd[u] = id - ph[u] * ipr;
            const int ih = ih0 + ph[u], iw = iwa + pd[u] * XV;
            const bool inside = id < items && ih >= 0 && ih < p.H && iw >= 0 && iw < p.W;
            const uint32_t vo = inside ? img_off + 2u * (uint32_t)(ih * p.W + iw) : kNoLoad;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t vc = c < p.C ? vo : kNoLoad;
                if (XV == 2) d[u][c] = __builtin_amdgcn_raw_buffer_load_b32(rx, vc, 2u * (uint32_t)(c * HW), 0);
                else d[u][c] = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rx, vc, 2u * (uint32_t)(c * HW), 0);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (id0 + 256 * u >= items) continue;
            if (XV == 2) {
                const u32x4 v = {pack_lo(d[u][0], d[u][1]), pack_lo(d[u][2], d[u][3]), pack_hi(d[u][0], d[u][1]),
                                 pack_hi(d[u][2], d[u][3])};
                *reinterpret_cast<u32x4_alias *>(xl + ph[u] * PWU + pd[u] * 2) = v;     // PWU is even: 16-byte aligned
            } else {
                const u32x2s v = {d[u][0] | (d[u][1] << 16), d[u][2] | (d[u][3] << 16)};
                xl[ph[u] * PWU + pd[u]] = v;
            }
        }
    }

    // ---- operand addresses ----
    int xb[B];
#pragma unroll
    for (int j = 0; j < B; ++j) {
        const int pix = (wave * B + j) * 32 + l32;
        xb[j] = ((pix >> p.log2_tw) * s) * PWU + (pix & (TW - 1)) * s + cofs;
    }
    int toff[NT2];                               // this lane's tap-pair offset for MFMA t (lanes 32..63: the odd unit)
#pragma unroll
    for (int t = 0; t < NT2; ++t) {
        const int k0 = 2 * t, k1 = (2 * t + 1 < NG) ? 2 * t + 1 : 0;      // a padding unit has zero weights
        const int o0 = (k0 / QP) * PWU + 2 * (k0 % QP), o1 = (k1 / QP) * PWU + 2 * (k1 % QP);
        toff[t] = lh ? o1 : o0;
    }

    // accumulators start from the bias: through the wave's private LDS words to the lanes that own the rows
    floatx16 acc[A][B];
    {
        typedef float __attribute__((ext_vector_type(4), may_alias)) floatx4;
        f32_alias *bw = reinterpret_cast<f32_alias *>(lds_raw) + wave * BM;
#pragma unroll
        for (int r = 0; r < BROWS; ++r)
            if (lane + 64 * r < BM) bw[lane + 64 * r] = bias_row[r];
        asm volatile("" ::: "memory");
#pragma unroll
        for (int i = 0; i < A; ++i) {
            floatx4 bv[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) bv[q] = *reinterpret_cast<const floatx4 *>(bw + 32 * i + 8 * q + 4 * lh);
#pragma unroll
            for (int j = 0; j < B; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = bv[e >> 2][e & 3];
        }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);           // the LDS-direct weight loads have landed
    __syncthreads();

    // ---- the whole reduction: NT2 MFMAs per accumulator block ----
#pragma unroll
    for (int t = 0; t < NT2; ++t) {
        half8 af[A], bf[B];
#pragma unroll
        for (int i = 0; i < A; ++i) af[i] = __builtin_bit_cast(half8, wl[(2 * t + lh) * BM + i * 32 + l32]);
#pragma unroll
        for (int j = 0; j < B; ++j) {
            const u32x2_alias *src = xl + xb[j] + toff[t];
            const u32x2s lo = src[0], hi = src[1];
            const u32x4 v = {lo.x, lo.y, hi.x, hi.y};
            bf[j] = __builtin_bit_cast(half8, v);
        }
#pragma unroll
        for (int i = 0; i < A; ++i)
#pragma unroll
            for (int j = 0; j < B; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[i], bf[j], acc[i][j], 0, 0, 0);
    }
    mfma_drain();
    __syncthreads();                              // the transpose tiles reuse the operand buffers
    store_tile<A, B>(p, acc, wl, wave, 0, wave, lane, n, 0, m0, oh0, ow0);
}

template <int KS, int A, int B, int XV, bool PACKED>
static hipError_t launch_one(const ConvArgs &a, size_t lds, hipStream_t stream)
{
    static std::atomic<size_t> granted{0};
    auto kern = smallc_kernel<KS, A, B, XV, PACKED>;
    if (lds > 64 * 1024 && lds > granted.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        granted.store(lds, std::memory_order_release);
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)(((a.grid_blocks + 7) / 8) * 8)), dim3(256), lds, stream, a);
    return hipGetLastError();
}

template <int KS, int B, bool PACKED>
static hipError_t launch_ks(const ConvArgs &a, int blocks_m, int xv, size_t lds, hipStream_t s)
{
    if (blocks_m == 2)
        return xv == 2 ? launch_one<KS, 2, B, 2, PACKED>(a, lds, s) : launch_one<KS, 2, B, 1, PACKED>(a, lds, s);
    return xv == 2 ? launch_one<KS, 1, B, 2, PACKED>(a, lds, s) : launch_one<KS, 1, B, 1, PACKED>(a, lds, s);
}

template <int B, bool PACKED>
static hipError_t launch_layout(const ConvArgs &a, int blocks_m, int xv, size_t lds, hipStream_t stream)
{
    switch (a.ks) {
    case 3: return launch_ks<3, B, PACKED>(a, blocks_m, xv, lds, stream);
    case 5: return launch_ks<5, B, PACKED>(a, blocks_m, xv, lds, stream);
    case 7: return launch_ks<7, B, PACKED>(a, blocks_m, xv, lds, stream);
    case 11: return launch_ks<11, B, PACKED>(a, blocks_m, xv, lds, stream);
    default: return hipErrorInvalidValue;
    }
}

long long smallc_lds_bytes(int ks, int blocks_m, int PH, int PWU)
{
    const int qp = (ks + 1) / 2, ngp = 2 * ((ks * qp + 1) / 2), bm = 32 * blocks_m;
    const long long bias = 16LL * 4 * 8 * blocks_m;
    const long long main = 16LL * ngp * bm + 8LL * PH * PWU + 16;
    const long long epi = 80LL * 32 * blocks_m * 4;
    return bias + (main > epi ? main : epi);
}

hipError_t launch_smallc(const ConvArgs &a, int blocks_m, int blocks_n, int xv, size_t lds, bool packed,
                         hipStream_t stream)
{
    if (blocks_n == 1)
        return packed ? launch_layout<1, true>(a, blocks_m, xv, lds, stream)
                      : launch_layout<1, false>(a, blocks_m, xv, lds, stream);
    return packed ? launch_layout<2, true>(a, blocks_m, xv, lds, stream)
                  : launch_layout<2, false>(a, blocks_m, xv, lds, stream);
}

}  // namespace hgc
