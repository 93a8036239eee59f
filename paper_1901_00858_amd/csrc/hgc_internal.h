// Internal declarations shared by the host dispatcher and the HIP kernels of
// libhgc.  Not part of the public ABI (that is include/hgc.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hgc.h"

namespace hgc {

// Problem geometry derived from a validated descriptor.  Notation follows the
// layer definition: M = num_output, G = group, Mg = M/G, Cg = C/G,
// Kg = Cg*k*k (reduction length per group), P = N*Ho*Wo (output pixels).
struct Geometry {
    int N, C, H, W, M, k, s, p, G, bias, relu;
    int Ho, Wo, Cg, Mg;
    long long Kg, P;
    bool flat;           // pointwise layer presented to the kernels as 1 x (H*W) images
};

// Division of 0 <= n < 2^31 by a divisor fixed on the host, as multiply-high, add and shift
// (round-up method: s = ceil(log2 d), m = floor(2^32 (2^s - d) / d) + 1, n / d = (mulhi(n, m) + n) >> s;
// mulhi(n, m) < n < 2^31, so the sum stays below 2^32).  A runtime integer division costs the
// kernels some thirty instructions each, at the head of every workgroup.
struct FastDiv {
    uint32_t d, m, s;
};
inline FastDiv make_fastdiv(uint32_t d)
{
    FastDiv f;
    f.d = d;
    f.s = 0;
    while ((1ull << f.s) < d) ++f.s;
    f.m = (uint32_t)(((1ull << 32) * ((1ull << f.s) - d)) / d + 1);
    return f;
}
__host__ __device__ inline uint32_t fast_div(uint32_t n, const FastDiv &f)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return (__umulhi(n, f.m) + n) >> f.s;
#else
    return (uint32_t)((((unsigned long long)n * f.m) >> 32) + n) >> f.s;
#endif
}

// Arguments of every kernel: tensors + geometry + the tiling chosen on the host.
struct ConvArgs {
    const uint16_t *x;
    const uint16_t *w;
    const uint16_t *b;
    uint16_t *y;
    float *ws;           // FP32 partial sums [split_k][N][M][Ho][Wo] (split-K only)
    int N, C, H, W, M, Ho, Wo;
    int Cg, Mg, G;
    int ks, stride, pad;
    int bias, relu;
    // implicit-GEMM tiling
    int log2_tw;         // a tile is 2^log2_ti images x 2^log2_thi rows x 2^log2_tw columns = BN pixels
    int log2_thi, log2_ti;
    int tiles_n;         // image tiles: ceil(N / 2^log2_ti)
    int tiles_w, tiles_h, tiles_m;
    int PH, PWU;         // input halo patch: rows, and 16-byte units (pixels) per row
    int nsteps;          // channel blocks of CB channels per group: ceil(Cg / CB)
    uint32_t x_bytes;    // size of x and w (or the packed weight buffer) in bytes (buffer-load range checks)
    uint32_t w_bytes;
    uint32_t wp_off;     // packed weights: byte offset of the implicit-GEMM layout, and of the zero page
    uint32_t wp_zero;
    int MB8, NP8;        // packed weights: 8-row blocks per group, 8-channel planes per group
    int out_vec;         // output pixels per store (8, 4, 2 or 1): divides Wo and tile_w, fits y's alignment
    int grid_blocks;     // workgroups that have work (the launch pads to a multiple of 8)
    FastDiv fd_tiles_m, fd_tiles_w, fd_tiles_h, fd_G, fd_tiles_n;   // workgroup id -> tile coordinates
    FastDiv fd_ipr, fd_PH;                                     // staging item -> patch coordinates
    int split_k;         // reduction slices (1 = none)
    int steps_per_split; // channel blocks per slice
};

// LDS units (16 bytes) of one weight buffer: every wave owns a slice that holds
// its BM/NW rows, rounded up so that each lane of each 64-lane load round lands inside.
constexpr int igemm_w_units(int ks, int wm_blocks, int waves_m, int stage_waves, int npl)
{
    const int nw = stage_waves;
    const int rpw = 32 * wm_blocks * waves_m / nw;
    const int wch = rpw * npl * ks * ks;
    return nw * (((wch + 63) / 64) * 64 + (rpw == 8 ? 8 : 0));    // 8-row slices sit half a bank row apart
}

// One instantiation of the implicit-GEMM kernel.
struct IgemmVariant {
    int ks;              // compile-time kernel extent (1, 3, 5, 7)
    int wm_blocks;       // 32-row blocks of output channels per wave
    int wn_blocks;       // 32-pixel blocks per wave
    int waves_m;         // waves along output channels
    int waves_n;         // waves along pixels
    int npl;             // 8-channel planes per K step (CB = 8 * npl)
    int xvec;            // pixels per global load of the input (1 or 2)
    int calign;          // 1: Cg % 8 == 0, weights fetched as 16-byte vectors
    int packed;          // 1: weights in the pre-packed layout
    int nstage;          // LDS buffers (2 = double buffered; 3 = loads two steps ahead)
    int max_rounds;      // patch staging rounds pipelined through registers
    int prod_waves;      // waves that only stage operands (0: every wave stages and runs MFMAs)
    hipError_t (*launch)(const ConvArgs &, size_t lds_bytes, hipStream_t stream);
    int BM() const { return 32 * wm_blocks * waves_m; }
    int BN() const { return 32 * wn_blocks * waves_n; }
    int threads() const { return 64 * (waves_m * waves_n + prod_waves); }
    int stage_waves() const { return prod_waves ? prod_waves : waves_m * waves_n; }
    // LDS of a launch: stages of {weights, patch + 8 dump units}; the epilogue reuses it
    long long lds_bytes(int PH, int PWU, int images = 1) const
    {
        const long long wu = igemm_w_units(ks, wm_blocks, waves_m, stage_waves(), npl);
        const long long xu = (long long)images * npl * PH * PWU + 8;
        // nstage 3: three weight buffers, two patch buffers (the patch waits in registers one step longer)
        const long long main = 16LL * (nstage == 3 ? 3 * wu + 2 * xu : nstage * (wu + xu));
        const long long epi = 80LL * 32 * wm_blocks * waves_m * waves_n;   // transpose tile per wave
        const long long bias = 128LL * wm_blocks * waves_m * waves_n;      // FP32 bias of each wave's rows
        return bias + (main > epi ? main : epi);
    }
};

const IgemmVariant *igemm_variants_raw(int *count);
const IgemmVariant *igemm_variants_packed(int *count);

// Layout of a packed weight buffer (all offsets in bytes, multiples of 256):
// [0, raw) the caller's weights verbatim, [igemm_off, zero_off) 16-byte units
// [G][ceil(Mg/8)][ceil(Cg/8)][k*k][8 rows] of 8 channels, zero filled past Mg and Cg,
// [zero_off, zero_off + 1024) a page of zeros, then the first-layer section if there is one.
struct PackedLayout {
    long long raw_bytes, igemm_off, zero_off, total;
    int MB8, NP8;
    // first-layer section (one group, at most 4 input channels, k in {3, 5, 7, 11}; else c4_off = 0):
    // 16-byte units [k rows][ceil(k/2) tap pairs][c4_mpad output channels] of
    // {tap 2qp: channels 0..3, tap 2qp+1: channels 0..3}, zero past C, k and M
    long long c4_off;
    int c4_mpad;
};
PackedLayout packed_layout(const Geometry &g);
hipError_t launch_pack_weights(const Geometry &g, const PackedLayout &pl, const uint16_t *w, uint8_t *packed,
                               hipStream_t stream);

// 1x1 / stride 1 / unpadded / one-group layers as a GEMM over all images' pixels (pointwise.hip):
// whether the kernel takes the layer (alignments in bytes), its tile (64 a rows x 64 b pixels), the launch
bool pointwise_eligible(const ConvArgs &c, int x_align, int y_align, bool w_al16);
void pointwise_tile(const ConvArgs &c, int *a, int *b);
hipError_t launch_pointwise(const ConvArgs &c, int a, int b, hipStream_t stream);

// records the runtime error behind the calling thread's latest HGC_ERR_LAUNCH (hgc_last_launch_error)
void set_last_hip_error(hipError_t e);

hipError_t launch_direct(const ConvArgs &a, hipStream_t stream);
hipError_t launch_depthwise(const ConvArgs &a, hipStream_t stream);
hipError_t launch_splitk_reduce(const ConvArgs &a, hipStream_t stream);
// first-layer kernel (smallc.hip): blocks_m = 32-row blocks of output channels per workgroup (1 or 2),
// blocks_n = 32-pixel blocks per wave (2 or 1: 256 or 128 pixels per workgroup),
// xv = input pixels per load (2 or 1); packed: a.wp_off = byte offset of the first-layer section, a.MB8 = c4_mpad
// (else a.w is the caller's layout),
// a.PWU = pixels per patch row (even)
long long smallc_lds_bytes(int ks, int blocks_m, int PH, int PWU);
hipError_t launch_smallc(const ConvArgs &a, int blocks_m, int blocks_n, int xv, size_t lds, bool packed,
                         hipStream_t stream);

}  // namespace hgc
