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
};

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
    int log2_tw;         // tile_w = 1 << log2_tw output columns; tile_h = BN >> log2_tw rows
    int tiles_w, tiles_h, tiles_m;
    int PH, PWU;         // input halo patch: rows, and 16-byte units (pixels) per row
    int nsteps;          // channel blocks of CB channels per group: ceil(Cg / CB)
    int out_vec;         // output pixels per store (8, 4, 2 or 1): divides Wo and tile_w, fits y's alignment
    int grid_blocks;     // workgroups that have work (the launch pads to a multiple of 8)
    int split_k;         // reduction slices (1 = none)
    int steps_per_split; // channel blocks per slice
};

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
    int nstage;          // LDS buffers (2 = double buffered)
    int max_rounds;      // patch staging rounds pipelined through registers
    hipError_t (*launch)(const ConvArgs &, hipStream_t stream);
    int BM() const { return 32 * wm_blocks * waves_m; }
    int BN() const { return 32 * wn_blocks * waves_n; }
    int threads() const { return 64 * waves_m * waves_n; }
    long long w_lds_bytes() const { return 16LL * ks * ks * npl * BM(); }
    long long epilogue_lds_bytes() const { return 80LL * 32 * wm_blocks * waves_m * waves_n; }
};

const IgemmVariant *igemm_variants(int *count);

hipError_t launch_direct(const ConvArgs &a, hipStream_t stream);
hipError_t launch_depthwise(const ConvArgs &a, hipStream_t stream);
hipError_t launch_splitk_reduce(const ConvArgs &a, hipStream_t stream);

}  // namespace hgc
