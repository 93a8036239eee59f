// Pieces shared by the MFMA convolution kernels: vector types, the wait states before the
// accumulators are read, and the epilogue that turns a wave's accumulator blocks into
// wide FP16 stores.
#pragma once
#include "hgc_internal.h"

namespace hgc {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void *lds_ptr_t;
// the epilogue writes its LDS tile as halves and floats and reads it back as vectors:
// these accesses must be allowed to alias
typedef uint16_t __attribute__((may_alias)) u16_alias;
typedef float __attribute__((may_alias)) f32_alias;
typedef u32x4 __attribute__((may_alias)) u32x4_alias;


constexpr uint32_t kNoLoad = 0xFFFFFFFFu;       // buffer offset that is always out of range

__device__ __forceinline__ uint32_t pack_lo(uint32_t a, uint32_t b)   // a.lo | b.lo << 16
{
    return __builtin_amdgcn_perm(b, a, 0x05040100u);
}
__device__ __forceinline__ uint32_t pack_hi(uint32_t a, uint32_t b)   // a.hi | b.hi << 16
{
    return __builtin_amdgcn_perm(b, a, 0x07060302u);
}

// Workgroup barrier for data exchanged through LDS only.  __syncthreads() also waits
// for every outstanding vector-memory operation (vmcnt(0)), which would drain the loads
// that are deliberately left in flight across K steps; LDS operations are counted by
// lgkmcnt alone, and LDS-direct loads are waited for explicitly where they are consumed.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, uint32_t bytes)
{
    // raw buffer, stride 0, 32-bit data format: offsets >= bytes read as zero
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, bytes, 0x00020000);
}

// The last MFMAs may still be in flight when a kernel turns to its accumulators.  The compiler
// pads MFMA -> accumulator-read hazards along the fall-through path only; a taken branch just
// before the epilogue reached the first accumulator read too early and saw it without the
// last MFMA's contribution.  32 wait states cover the longest MFMA on any path.
__device__ __forceinline__ void mfma_drain()
{
    __builtin_amdgcn_sched_barrier(0);           // nothing, MFMAs included, moves across the padding
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

// Epilogue of a wave that holds A x B accumulator blocks of 32 channel rows x 32 pixels:
// accumulator register e of lane (l32, lh) in block (i, j) is channel row 8*(e/4) + 4*lh + e%4
// and pixel column l32.  Rows start at m0 + wm*32*A (within group g), pixel blocks at
// (wn*B + j)*32 of the workgroup's tile: 2^log2_ti images starting at image n, of each a window
// of 2^log2_thi rows x 2^log2_tw columns with origin (oh0, ow0).
// lds: at least 80*32*A bytes per wave, indexed by `wave`.
template <int A, int B>
__device__ __forceinline__ void store_tile(const ConvArgs &p, floatx16 (&acc)[A][B], u32x4 *lds, int wave, int wm,
                                           int wn, int lane, int n, int g, int m0, int oh0, int ow0)
{
    const int l32 = lane & 31, lh = lane >> 5;
    const int HoWo = p.Ho * p.Wo;
    const int Mg = p.Mg;
    const int TW = 1 << p.log2_tw;
    // pixel index of the workgroup's tile -> (image of the tile, row and column of its window)
    const int img_shift = p.log2_tw + p.log2_thi, th_mask = (1 << p.log2_thi) - 1;
    const size_t img_stride = (size_t)p.M * HoWo;
    auto locate = [&](int pix, bool &ok) -> size_t {
        const int img = pix >> img_shift;
        const int oh = oh0 + ((pix >> p.log2_tw) & th_mask), ow = ow0 + (pix & (TW - 1));
        ok = oh < p.Ho && ow < p.Wo && n + img < p.N;
        return img * img_stride + (size_t)(oh * p.Wo + ow);
    };
    // The bias is already in the accumulators.  One rounding to FP16 (two rows per packed
    // conversion), ReLU as a packed maximum; then each wave transposes its tile through LDS
    // (2-byte writes, 16-byte reads) so that a lane holds 8 consecutive pixels of one
    // output row and the global stores are 16, 8 or 4 bytes wide.  Everything that does
    // not depend on the accumulator block is computed once per wave.
    constexpr int EP = 40;                       // halves per LDS row: 32 pixels + pad (80 bytes)
    u16_alias *el = reinterpret_cast<u16_alias *>(lds) + wave * (32 * A * EP);
    typedef _Float16 half2v __attribute__((ext_vector_type(2)));
    typedef float float2v __attribute__((ext_vector_type(2)));
    const _Float16 floor_h = p.relu ? (_Float16)0.0f : (_Float16)(-__builtin_inff());
    const half2v floor2 = {floor_h, floor_h};
    u16_alias *elw = el + (4 * lh) * EP + l32;    // this lane's column of the transpose tile
    const int row0 = lane >> 2, chunk = lane & 3;
    const u16_alias *elr = el + row0 * EP + chunk * 8;
    const int ml0 = m0 + wm * (32 * A) + row0;
    uint16_t *ybase = p.y + ((size_t)n * p.M + (size_t)g * Mg + ml0) * HoWo;
    const size_t kstride = (size_t)16 * HoWo;    // 16 rows further per read round
    const int ov = p.out_vec;                    // pixels per store: divides Wo, tile_w and the base alignment
#pragma unroll
    for (int j = 0; j < B; ++j) {
#pragma unroll
        for (int i = 0; i < A; ++i)
#pragma unroll
            for (int e = 0; e < 16; e += 2) {
                // two rows at a time: one packed conversion (RNE) and one packed max
                const float2v v = {acc[i][j][e], acc[i][j][e + 1]};
                const half2v h = __builtin_elementwise_max(__builtin_convertvector(v, half2v), floor2);
                const uint32_t bits = __builtin_bit_cast(uint32_t, h);
                elw[(i * 32 + 8 * (e >> 2) + (e & 3)) * EP] = (uint16_t)bits;
                elw[(i * 32 + 8 * (e >> 2) + (e & 3) + 1) * EP] = (uint16_t)(bits >> 16);
            }
        asm volatile("" ::: "memory");          // the reads below see the writes above
        const int pix0 = (wn * B + j) * 32 + chunk * 8;
        if (ov == 8) {
            bool ok;
            uint16_t *dst = ybase + locate(pix0, ok);
#pragma unroll
            for (int k = 0; k < 2 * A; ++k) {
                const u32x4 v = *reinterpret_cast<const u32x4_alias *>(elr + k * 16 * EP);
                if (ok && ml0 + 16 * k < Mg) *reinterpret_cast<u32x4 *>(dst + k * kstride) = v;
            }
        } else if (ov == 4) {
            bool ok[2];
            uint16_t *dst[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                dst[h] = ybase + locate(pix0 + 4 * h, ok[h]);
            }
#pragma unroll
            for (int k = 0; k < 2 * A; ++k) {
                const u32x4 v = *reinterpret_cast<const u32x4_alias *>(elr + k * 16 * EP);
#pragma unroll
                for (int h = 0; h < 2; ++h)
                    if (ok[h] && ml0 + 16 * k < Mg)
                        *reinterpret_cast<uint2 *>(dst[h] + k * kstride) = make_uint2(v[2 * h], v[2 * h + 1]);
            }
        } else if (ov == 2) {
            bool ok[4];
            uint16_t *dst[4];
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                dst[h] = ybase + locate(pix0 + 2 * h, ok[h]);
            }
#pragma unroll
            for (int k = 0; k < 2 * A; ++k) {
                const u32x4 v = *reinterpret_cast<const u32x4_alias *>(elr + k * 16 * EP);
#pragma unroll
                for (int h = 0; h < 4; ++h)
                    if (ok[h] && ml0 + 16 * k < Mg) *reinterpret_cast<uint32_t *>(dst[h] + k * kstride) = v[h];
            }
        } else {
            for (int k = 0; k < 2 * A; ++k) {
                const u32x4 v = *reinterpret_cast<const u32x4_alias *>(elr + k * 16 * EP);
                if (ml0 + 16 * k >= Mg) continue;
#pragma unroll
                for (int h = 0; h < 8; ++h) {
                    bool ok;
                    const size_t at = locate(pix0 + h, ok);
                    if (ok) (ybase + k * kstride)[at] = (uint16_t)(v[h >> 1] >> (16 * (h & 1)));
                }
            }
        }
    }
}

}  // namespace hgc
