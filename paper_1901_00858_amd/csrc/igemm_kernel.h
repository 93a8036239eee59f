// Implicit-GEMM convolution forward on FP16 MFMA for gfx950: the kernel template and
// its instantiation table.  Included by igemm_raw_<part>.hip and igemm_packed_<part>.hip, which set
// HGC_IGEMM_PACKED (0: weights in the caller's layout, 1: pre-packed weights) and
// HGC_IGEMM_ACCESSOR (the name of the function that returns the table).
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
//
// Staging is branch-free so that a whole K step is one basic block the scheduler
// can interleave with the MFMAs.  All global reads are buffer loads: a lane's
// byte offset is fixed for the kernel, the step only moves a scalar offset, and an
// offset of ~0 (padding pixel, channel or row outside the problem) makes the
// hardware return zero instead of a predicate.
//   Input: each item is XVEC pixels x 8 channels; eight loads (one per channel
// plane of NCHW, coalesced along W) are transposed in registers with v_perm_b32
// into XVEC units.  Items past the end of the patch write a dump unit.
//   Weights: each staging wave owns a share of the BM rows; it fetches their contiguous CB*k*k-half
// runs with 16-byte LDS-direct loads (buffer_load_dwordx4 ... lds) into its own
// slice of the LDS weight buffer, reads them back one (row, plane) per lane and
// writes the regrouped units over the same slice.  LDS operations of one wave
// execute in order, so no barrier is needed inside the wave.
// Pipelines over the K steps (NSTAGE, PW): 1 = one LDS buffer; 2 = double-buffered LDS,
// the loads of step s+1 are issued among the MFMAs of step s and stored to the other
// buffer; 3 = three weight and two patch buffers with the loads two steps ahead; PW > 0
// adds PW producer waves that only stage while the other waves only run MFMAs.
#pragma once
#include <atomic>
#include <type_traits>

#include "hgc_internal.h"
#include "tile_store.h"

namespace hgc {

// Decoded staging item of the input patch: XVEC pixels x 8 channels.
struct PatchItem {
    uint32_t voff;   // byte offset of (channel 0 of the plane, first pixel) in x at K step 0, or kNoLoad
    int unit;        // LDS unit index of the first pixel (the dump unit for items past the end)
    int pl8;         // first channel of the plane within a channel block (plane * 8)
};

template <int XVEC, int NPL>
__device__ __forceinline__ PatchItem decode_patch_item(int id, int total, const FastDiv &fd_ipr,
                                                       const FastDiv &fd_PH, int PH, int PWU,
                                                       int ih0, int iwa, int H, int W, int HW,
                                                       uint32_t plane0_off, int dump_unit,
                                                       int img_elems, int imgs_left)
{
    PatchItem it;
    const int t = (int)fast_div((uint32_t)id, fd_ipr);
    const int pd = id - t * (int)fd_ipr.d;
    const int t2 = (int)fast_div((uint32_t)t, fd_PH);
    const int ph = t - t2 * PH;
    const int pl = t2 % NPL, img = t2 / NPL;     // NPL is a compile-time power of two or small constant
    const int ih = ih0 + ph;
    const int iw = iwa + pd * XVEC;
    const bool active = id < total;
    const bool inside = active && ih >= 0 && ih < H && iw >= 0 && iw < W && img < imgs_left;
    it.voff = inside ? plane0_off + 2u * (uint32_t)(img * img_elems + pl * 8 * HW + ih * W + iw) : kNoLoad;
    it.unit = active ? ((img * NPL + pl) * PH + ph) * PWU + pd * XVEC : dump_unit;
    it.pl8 = pl * 8;
    return it;
}

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// XVEC pixels (XVEC*2 bytes) of each of the 8 channels of the item's plane.
// d[j][k]: channel j, dword k (two pixels per dword; one pixel when XVEC == 1).
template <int XVEC, bool CALIGN>
__device__ __forceinline__ void load_patch_chan(__amdgpu_buffer_rsrc_t rx, const PatchItem &it, int c0,
                                                int Cg, uint32_t soff, uint32_t chan_bytes, int j,
                                                uint32_t (&dj)[(XVEC + 1) / 2])
{
    const uint32_t vo = (c0 + it.pl8 + (CALIGN ? 0 : j) < Cg) ? it.voff : kNoLoad;
    const uint32_t so = soff + j * chan_bytes;
    if (XVEC == 8) {
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rx, vo, so, 0);
        dj[0] = v.x; dj[1 % ((XVEC + 1) / 2)] = v.y; dj[2 % ((XVEC + 1) / 2)] = v.z; dj[3 % ((XVEC + 1) / 2)] = v.w;
    } else if (XVEC == 4) {
        const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rx, vo, so, 0);
        dj[0] = v.x; dj[1 % ((XVEC + 1) / 2)] = v.y;
    } else if (XVEC == 2) {
        dj[0] = __builtin_amdgcn_raw_buffer_load_b32(rx, vo, so, 0);
    } else {
        dj[0] = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rx, vo, so, 0);
    }
}

template <int XVEC, bool CALIGN>
__device__ __forceinline__ void load_patch_item(__amdgpu_buffer_rsrc_t rx, const PatchItem &it, int c0,
                                                int Cg, uint32_t soff, uint32_t chan_bytes,
                                                uint32_t (&d)[8][(XVEC + 1) / 2])
{
#pragma unroll
    for (int j = 0; j < 8; ++j) load_patch_chan<XVEC, CALIGN>(rx, it, c0, Cg, soff, chan_bytes, j, d[j]);
}

// Transpose 8 channels x XVEC pixels into XVEC units of 8 channels.
template <int XVEC>
__device__ __forceinline__ void store_patch_item(u32x4 *xl, const PatchItem &it,
                                                 const uint32_t (&d)[8][(XVEC + 1) / 2])
{
#pragma unroll
    for (int px = 0; px < XVEC; ++px) {
        const int k = px >> 1;
        u32x4 u;
        if (px & 1) {
            u.x = pack_hi(d[0][k], d[1][k]); u.y = pack_hi(d[2][k], d[3][k]);
            u.z = pack_hi(d[4][k], d[5][k]); u.w = pack_hi(d[6][k], d[7][k]);
        } else {
            u.x = pack_lo(d[0][k], d[1][k]); u.y = pack_lo(d[2][k], d[3][k]);
            u.z = pack_lo(d[4][k], d[5][k]); u.w = pack_lo(d[6][k], d[7][k]);
        }
        xl[it.unit + px] = u;
    }
}

// Scheduling hints for a region that mixes MFMAs with staging work: one MFMA, then
// up to NV vector-memory, ND LDS and NA VALU instructions, N times.
template <int N, int NV, int ND, int NA>
__device__ __forceinline__ void interleave_hint()
{
#pragma unroll
    for (int i = 0; i < N; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (NV) __builtin_amdgcn_sched_group_barrier(0x020, NV, 0);
        if (ND) __builtin_amdgcn_sched_group_barrier(0x300, ND, 0);
        if (NA) __builtin_amdgcn_sched_group_barrier(0x002, NA, 0);
    }
}

// KS: kernel extent.  A, B: 32x32 accumulator blocks per wave along channels and
// pixels.  WAVES_M x WAVES_N waves per workgroup.  NPL: 8-channel planes per K
// step.  XVEC: input pixels per global load (1, 2, 4 or 8; W and the byte alignment
// of x must be multiples of it).  CALIGN: Cg % 8 == 0 and a 16-byte aligned weight base.
// PACKED: weights come from the pre-packed layout (see pack.hip) and need no regrouping.
// NSTAGE: LDS buffers (1, 2, or 3 = three weight and two patch buffers with the loads two steps ahead).  MAXR: patch staging rounds held in registers.  SPLITK: write
// FP32 partial sums of a slice of the channel blocks instead of the output.
template <int KS, int A, int B, int WAVES_M, int WAVES_N, int NPL, int XVEC, bool CALIGN, bool PACKED,
          int NSTAGE, int MAXR, int PW, bool SPLITK>
__global__ __launch_bounds__(64 * (WAVES_M * WAVES_N + PW)) void igemm_kernel(const ConvArgs p)
{
    constexpr int NW = WAVES_M * WAVES_N;        // waves that run the MFMAs
    constexpr int NWS = PW ? PW : NW;            // waves that stage the operands
    constexpr int NT = 64 * NWS;                 // staging threads
    constexpr int BM = 32 * A * WAVES_M;
    constexpr int BN = 32 * B * WAVES_N;
    constexpr int T = KS * KS;
    constexpr int CB = 8 * NPL;
    constexpr int RPW = BM / NWS;                // weight rows staged by one wave
    constexpr int CPR = NPL * T;                 // 16-byte chunks per row per step
    constexpr int WCH = RPW * CPR;               // chunks (= LDS units) of one wave's rows
    constexpr int WLR = (WCH + 63) / 64;         // LDS-direct load rounds per lane
    // LDS units of one wave's slice (every lane of every round lands inside).  Slices of 8 rows are
    // 128 bytes per (tap, plane) and a 16-lane group of an operand read spans two of them: half a
    // bank row apart (8 units more per slice) they do not collide.
    constexpr int WSL = WLR * 64 + (RPW == 8 ? 8 : 0);
    constexpr int W_UNITS = NWS * WSL;
    constexpr int WIT = RPW * NPL;               // (row, plane) items per wave
    constexpr int WIR = (WIT + 63) / 64;
    constexpr int TC = T < 9 ? T : 9;            // taps handled together by the scalar weight path
    static_assert(NPL % 2 == 0, "planes come in pairs (16 channels per MFMA)");
    static_assert(BM % NWS == 0 && (RPW & (RPW - 1)) == 0, "rows per wave must be a power of two");
    static_assert(W_UNITS == igemm_w_units(KS, A, WAVES_M, NWS, NPL), "host and kernel disagree on LDS");

    // LDS: [bias of every MFMA wave's rows, FP32][stage buffers ...]; the epilogue's transpose
    // tiles reuse the stage buffers
    constexpr int BIAS_UNITS = NW * 8 * A;       // 32*A floats per wave
    extern __shared__ u32x4 lds_raw[];
    u32x4 *const lds = lds_raw + BIAS_UNITS;
    const int IMG_UNITS = NPL * p.PH * p.PWU;    // patch of one image of the tile
    const int X_UNITS = (IMG_UNITS << p.log2_ti) + 8;   // + dump units (one item's worth) for staging items past the end
    const int stage_units = W_UNITS + X_UNITS;   // [stage]{ W[wave]{[T][NPL][RPW]} , X[NPL][PH][PWU], dump }
    const int dump_unit = X_UNITS - 8;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // with PW > 0 waves NW .. NW+PW-1 only stage (producers) and waves 0 .. NW-1 only
    // run MFMAs (consumers); otherwise every wave does both
    const int sw = PW ? wave - NW : wave;        // staging wave index (negative: not a staging wave)
    const int stid = PW ? tid - 64 * NW : tid;   // staging thread index
    const int wm = wave % WAVES_M;
    const int wn = wave / WAVES_M;
    const int l32 = lane & 31;
    const int lh = lane >> 5;

    // Workgroup ids are dealt round-robin to the 8 XCDs; renumber so that each XCD
    // (one L2) works on a contiguous range of tiles, which share patches and weights.
    const int nblk = p.grid_blocks;
    int bid;
    {
        const int per = (nblk + 7) >> 3;
        bid = (blockIdx.x & 7) * per + (blockIdx.x >> 3);
        if (bid >= nblk) return;                 // padding workgroups of the last XCD rows
    }
    int q = (int)fast_div((uint32_t)bid, p.fd_tiles_m);
    const int tm = bid - q * p.tiles_m; bid = q;
    q = (int)fast_div((uint32_t)bid, p.fd_tiles_w);
    const int twi = bid - q * p.tiles_w; bid = q;
    q = (int)fast_div((uint32_t)bid, p.fd_tiles_h);
    const int thi = bid - q * p.tiles_h; bid = q;
    q = (int)fast_div((uint32_t)bid, p.fd_G);
    const int g = bid - q * p.G; bid = q;
    const int ksl = (int)fast_div((uint32_t)bid, p.fd_tiles_n);
    const int n = (bid - ksl * p.tiles_n) << p.log2_ti;      // first image of the tile

    const int TW = 1 << p.log2_tw;
    const int oh0 = thi << p.log2_thi, ow0 = twi * TW;
    const int m0 = tm * BM;
    const int s = p.stride;
    const int ih0 = oh0 * s - p.pad;
    const int iw0 = ow0 * s - p.pad;
    const int iwa = iw0 & ~(XVEC - 1);           // aligned start of the patch rows (two's complement floor)
    const int cofs = iw0 - iwa;
    const int PH = p.PH, PWU = p.PWU;
    const int HW = p.H * p.W;
    const int Cg = p.Cg, Mg = p.Mg;

    const __amdgpu_buffer_rsrc_t rx = make_rsrc(p.x, p.x_bytes);
    const __amdgpu_buffer_rsrc_t rw = make_rsrc(p.w, p.w_bytes);   // raw weights, or the whole packed buffer

    // ---- K range of this workgroup ----
    int st0 = 0, st1 = p.nsteps;
    if (SPLITK) {
        st0 = ksl * p.steps_per_split;
        st1 = min(p.nsteps, st0 + p.steps_per_split);
    }

    // ---- weights ----
    const uint32_t wgrp_off = 2u * (uint32_t)(g * Mg * Cg * T);           // M*Kg < 2^31: fits
    constexpr bool WDMA = CALIGN || PACKED;      // weights arrive by LDS-direct loads
    uint32_t wvoff[WDMA ? WLR : 1];              // byte offset of this lane's chunk at K step 0
    int wpl8[WDMA ? WLR : 1];
    if (PACKED) {
        // packed layout: units [G][Mg/8][Cg/8][T][8 rows] of 8 channels; unit u of the
        // slice is (tap, plane, row) in the order the MFMA operand reads want
#pragma unroll
        for (int k = 0; k < WLR; ++k) {
            const int u = lane + 64 * k;
            const int t = u / (NPL * RPW), pl = (u / RPW) % NPL, r = u % RPW;
            const int m = m0 + sw * RPW + r;
            const bool ok = (u < WCH) && (m < p.MB8 * 8);
            wvoff[k] = ok ? p.wp_off + 16u * (uint32_t)((((g * p.MB8 + (m >> 3)) * p.NP8 + pl) * T + t) * 8 + (m & 7))
                          : p.wp_zero;
            wpl8[k] = pl;
        }
    } else if (CALIGN) {
#pragma unroll
        for (int k = 0; k < WLR; ++k) {
            const int id = lane + 64 * k;
            const int row = id / CPR, j = id % CPR;
            const int m = m0 + sw * RPW + row;
            wvoff[k] = (id < WCH && m < Mg) ? wgrp_off + 2u * (uint32_t)(m * Cg * T + j * 8) : kNoLoad;
            wpl8[k] = (j / T) * 8;
        }
    }
    // LDS-direct load round k of step st into this wave's slice of the weight buffer wl
    auto load_w_round = [&](int st, u32x4 *wl, int k) {
        u32x4 *mine = wl + sw * WSL;
        if (PACKED) {
            const uint32_t soff = 16u * (uint32_t)(st * NPL * T * 8);
            // planes past the last channel: read the zero page (the scalar offset must not move it)
            const bool inside = (wvoff[k] != p.wp_zero) && (st * NPL + wpl8[k] < p.NP8);
            const uint32_t vo = inside ? wvoff[k] : p.wp_zero - soff;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, (lds_ptr_t)(mine + 64 * k), 16, vo, soff, 0, 0);
        } else {
            const uint32_t soff = 2u * (uint32_t)(st * CB * T);
            const uint32_t vo = (st * CB + wpl8[k] < Cg) ? wvoff[k] : kNoLoad;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rw, (lds_ptr_t)(mine + 64 * k), 16, vo, soff, 0, 0);
        }
    };
    auto load_w = [&](int st, u32x4 *wl) {
        if (!WDMA) return;
#pragma unroll
        for (int k = 0; k < WLR; ++k) load_w_round(st, wl, k);
    };
    // the first step's weights need no index decode: get them under way before anything else
    // (single-buffered kernels load them inside the loop, after its first barrier)
    if (NSTAGE != 1 && (PW == 0 || wave >= NW)) load_w(st0, lds);

    // ---- staging maps (do not depend on the K step) ----
    const int ipr = PWU / XVEC;                  // items per patch row
    const int total_items = (NPL * PH * ipr) << p.log2_ti;
    const int rounds = (total_items + NT - 1) / NT;
    const uint32_t plane0_off = 2u * (uint32_t)((n * p.C + g * Cg) * HW);   // elements < 2^31: fits
    const uint32_t chan_bytes = 2u * (uint32_t)HW;
    PatchItem pit[MAXR];
#pragma unroll
    for (int r = 0; r < MAXR; ++r)
        pit[r] = decode_patch_item<XVEC, NPL>(r * NT + (stid < 0 ? 0 : stid), total_items, p.fd_ipr, p.fd_PH, PH, PWU,
                                              ih0, iwa, p.H, p.W, HW, plane0_off, dump_unit, p.C * HW, p.N - n);
    typedef uint32_t XRegs[MAXR][8][(XVEC + 1) / 2];
    XRegs xreg[NSTAGE == 3 ? 2 : 1];             // NSTAGE 3: two steps of loads in flight

    auto load_x = [&](int st, XRegs &xr) {
        const uint32_t soff = (uint32_t)(st * CB) * chan_bytes;
#pragma unroll
        for (int r = 0; r < MAXR; ++r)
            load_patch_item<XVEC, CALIGN>(rx, pit[r], st * CB, Cg, soff, chan_bytes, xr[r]);
    };
    auto store_x = [&](int st, u32x4 *xl, const XRegs &xr) {
#pragma unroll
        for (int r = 0; r < MAXR; ++r) store_patch_item<XVEC>(xl, pit[r], xr[r]);
        // patches larger than the register capacity: remaining rounds, not pipelined
        if (rounds > MAXR) {
            const uint32_t soff = (uint32_t)(st * CB) * chan_bytes;
            for (int r = MAXR; r < rounds; ++r) {
                PatchItem it = decode_patch_item<XVEC, NPL>(r * NT + stid, total_items, p.fd_ipr, p.fd_PH, PH, PWU, ih0,
                                                            iwa, p.H, p.W, HW, plane0_off, dump_unit, p.C * HW, p.N - n);
                uint32_t d[8][(XVEC + 1) / 2];
                load_patch_item<XVEC, CALIGN>(rx, it, st * CB, Cg, soff, chan_bytes, d);
                store_patch_item<XVEC>(xl, it, d);
            }
        }
    };

    // regroup items: lanes past the item count redo item (lane % WIT) and write the dump unit
    auto store_w = [&](int st, u32x4 *wl, u32x4 *xl) {
        u32x4 *mine = wl + sw * WSL;             // this wave's slice: final layout [T][NPL][RPW]
        if (PACKED) return;                      // already in the final layout
        if (CALIGN) {
            // the raw rows ([row][CPR] chunks) have landed (caller waited on vmcnt);
            // read back one (row, plane) per lane: halves e = c*T + tap, c = 0..7 ...
            u32x4 rr[WIR][T];
#pragma unroll
            for (int k = 0; k < WIR; ++k) {
                const int item = (lane + 64 * k) % WIT;
                const int row = item % RPW, pl = item / RPW;
#pragma unroll
                for (int t = 0; t < T; ++t) rr[k][t] = mine[row * CPR + pl * T + t];
            }
            // ... and write one unit per tap: the 8 channels of (row, tap)
#pragma unroll
            for (int k = 0; k < WIR; ++k) {
                const bool real = (WIT % 64 == 0) || (lane + 64 * k < WIT);
                const int item = (lane + 64 * k) % WIT;
                const int row = item % RPW, pl = item / RPW;
                const bool ok = (m0 + sw * RPW + row < Mg) && (st * CB + pl * 8 < Cg);
                u32x4 *dst = real ? mine + pl * RPW + row : xl + dump_unit;
                const int tstride = real ? NPL * RPW : 0;
#pragma unroll
                for (int t = 0; t < T; ++t) {
                    uint32_t o[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int ea = (2 * i) * T + t, eb = (2 * i + 1) * T + t;
                        const int da = ea >> 1, db = eb >> 1;
                        const uint32_t va = rr[k][da >> 2][da & 3];
                        const uint32_t vb = rr[k][db >> 2][db & 3];
                        const uint32_t sel = ((ea & 1) ? 0x0302u : 0x0100u) |
                                             (((eb & 1) ? 0x0706u : 0x0504u) << 16);
                        o[i] = ok ? __builtin_amdgcn_perm(vb, va, sel) : 0u;
                    }
                    u32x4 u = {o[0], o[1], o[2], o[3]};
                    dst[t * tstride] = u;
                }
            }
        } else {
            // any Cg, any alignment: 2-byte buffer loads straight into the final layout
            for (int k = 0; k < WIR; ++k) {
                const bool real = (WIT % 64 == 0) || (lane + 64 * k < WIT);
                const int item = (lane + 64 * k) % WIT;
                const int row = item % RPW, pl = item / RPW;
                const int m = m0 + sw * RPW + row;
                const int c0 = st * CB + pl * 8;
                const uint32_t vrow = (real && m < Mg) ? wgrp_off + 2u * (uint32_t)((m * Cg + c0) * T) : kNoLoad;
                u32x4 *dst = real ? mine + pl * RPW + row : xl + dump_unit;
                const int tstride = real ? NPL * RPW : 0;
                for (int t0 = 0; t0 < T; t0 += TC) {
                    uint32_t h[TC][8];
#pragma unroll
                    for (int tt = 0; tt < TC; ++tt)
#pragma unroll
                        for (int j = 0; j < 8; ++j) {
                            const uint32_t vo = (c0 + j < Cg && t0 + tt < T) ? vrow : kNoLoad;
                            h[tt][j] = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(
                                rw, vo, 2u * (uint32_t)(j * T + t0 + tt), 0);
                        }
#pragma unroll
                    for (int tt = 0; tt < TC; ++tt) {
                        u32x4 u = {h[tt][0] | (h[tt][1] << 16), h[tt][2] | (h[tt][3] << 16),
                                   h[tt][4] | (h[tt][5] << 16), h[tt][6] | (h[tt][7] << 16)};
                        if (t0 + tt < T) dst[(t0 + tt) * tstride] = u;
                    }
                }
            }
        }
    };

    // ---- MFMA operand addresses ----
    int xb[B];
#pragma unroll
    for (int j = 0; j < B; ++j) {
        const int pix = (wn * B + j) * 32 + l32;
        const int img = pix >> (p.log2_tw + p.log2_thi);
        const int th = (pix >> p.log2_tw) & ((1 << p.log2_thi) - 1), tw = pix & (TW - 1);
        xb[j] = img * IMG_UNITS + (lh * PH + th * s) * PWU + tw * s + cofs;
    }
    int ab[A];                                   // row -> (owning wave slice, row within it)
#pragma unroll
    for (int i = 0; i < A; ++i) {
        const int m = wm * (32 * A) + i * 32 + l32;
        ab[i] = (m / RPW) * WSL + lh * RPW + (m % RPW);
    }
    const int plane_pair_stride = 2 * PH * PWU;

    // The accumulators start from the bias (FP32), so the epilogue has no addition left.  A lane
    // fetches the bias of one of its wave's rows early; init_acc(), called once the first stage's
    // loads are under way, passes the values through the wave's private LDS words to the lanes
    // that hold those rows (LDS operations of one wave execute in order: no barrier).  A split
    // reduction adds the bias in its reduce kernel and starts from zero.
    typedef float __attribute__((ext_vector_type(4), may_alias)) floatx4;
    constexpr int BROWS = (32 * A + 63) / 64;
    float bias_row[BROWS];
    const __amdgpu_buffer_rsrc_t rb = make_rsrc(p.bias ? (const void *)p.b : (const void *)p.x, p.bias ? 2u * (uint32_t)p.M : 0u);
#pragma unroll
    for (int r = 0; r < BROWS; ++r) {
        const int ml = m0 + wm * (32 * A) + lane + 64 * r;
        // a range-checked load (zero where there is no bias or no such row): a load behind a
        // branch would be waited for on the spot, ahead of the first patch loads
        const bool want = !SPLITK && wave < NW && lane + 64 * r < 32 * A && ml < Mg;
        const uint16_t raw = __builtin_amdgcn_raw_buffer_load_b16(rb, want ? 2u * (uint32_t)(g * Mg + ml) : kNoLoad, 0, 0);
        bias_row[r] = (float)__builtin_bit_cast(_Float16, raw);
    }
    floatx16 acc[A][B];
    auto init_acc = [&]() {
        f32_alias *bw = reinterpret_cast<f32_alias *>(lds_raw) + (wave < NW ? wave : 0) * (32 * A);
#pragma unroll
        for (int r = 0; r < BROWS; ++r)
            if (lane + 64 * r < 32 * A) bw[lane + 64 * r] = bias_row[r];
        asm volatile("" ::: "memory");
#pragma unroll
        for (int i = 0; i < A; ++i) {
            floatx4 bv[4];                       // rows 32i + 8q + 4lh + (0..3)
#pragma unroll
            for (int q = 0; q < 4; ++q) bv[q] = *reinterpret_cast<const floatx4 *>(bw + 32 * i + 8 * q + 4 * lh);
#pragma unroll
            for (int j = 0; j < B; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = bv[e >> 2][e & 3];
        }
    };

    // One K step: T taps x NPL/2 plane pairs, walked in two halves.  An iteration of a
    // large tile (A*B >= 4 MFMAs) hides the latency of the next iteration's ds_reads, so
    // its fragments are double-buffered in registers.  An iteration of a small tile is one
    // or two MFMAs, far shorter than a ds_read_b128: there all fragments of a half are
    // read in one burst (BURST) and the MFMAs follow as the reads return in order.
    constexpr int NIT_ALL = T * (NPL / 2);
    constexpr int NIT_H = (NIT_ALL + 1) / 2;
    constexpr bool BURST = (A * B <= 2) && (NIT_H * (A + B) <= 27);
    auto compute = [&](const u32x4 *wl, const u32x4 *xl, int it0, int it1) {
        half8 af[2][A], bf[2][B];
        auto frag_load = [&](int it, half8 (&fa)[A], half8 (&fb)[B]) {
            const int t = it / (NPL / 2), pp = it % (NPL / 2);
            const int r = t / KS, q = t % KS;
            const int toff = r * PWU + q + pp * plane_pair_stride;
#pragma unroll
            for (int i = 0; i < A; ++i)
                fa[i] = __builtin_bit_cast(half8, wl[ab[i] + (t * NPL + pp * 2) * RPW]);
#pragma unroll
            for (int j = 0; j < B; ++j) fb[j] = __builtin_bit_cast(half8, xl[xb[j] + toff]);
        };
        frag_load(it0, af[it0 & 1], bf[it0 & 1]);
#pragma unroll
        for (int it = 0; it < NIT_ALL; ++it) {
            if (it < it0 || it >= it1) continue;
            if (it + 1 < it1) frag_load(it + 1, af[(it + 1) & 1], bf[(it + 1) & 1]);
#pragma unroll
            for (int i = 0; i < A; ++i)
#pragma unroll
                for (int j = 0; j < B; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[it & 1][i], bf[it & 1][j],
                                                                       acc[i][j], 0, 0, 0);
        }
    };
    // The small-tile step.  The texture-address unit of a CU accepts one wave-wide
    // vector-memory instruction every ~16 cycles and the issuing wave waits for it; with one
    // wave per SIMD nothing else would run meanwhile.  So the loads of a later step (LOADS:
    // 0 none, 1 the patch, 2 patch and weights; step stn into registers xr and weight buffer
    // wnext) are issued one or two at a time behind each MFMA, with scheduling fences
    // that keep them there.
    constexpr int NLD_X = 8 * MAXR, NLD_W = WDMA ? WLR : 0;
    auto burst_step = [&](const u32x4 *wl, const u32x4 *xl, auto loads, int stn, u32x4 *wnext, XRegs &xr) {
        constexpr int LOADS = decltype(loads)::value;
        constexpr int NM = NIT_ALL * A * B;
        constexpr int NLD = LOADS == 0 ? 0 : (LOADS == 1 ? NLD_X : NLD_X + NLD_W);
        const uint32_t xsoff = (uint32_t)(stn * CB) * chan_bytes;
        half8 af[NIT_H][A], bf[NIT_H][B];
#pragma unroll
        for (int h0 = 0; h0 < NIT_ALL; h0 += NIT_H) {
#pragma unroll
            for (int it = h0; it < h0 + NIT_H && it < NIT_ALL; ++it) {
                const int t = it / (NPL / 2), pp = it % (NPL / 2);
                const int toff = (t / KS) * PWU + (t % KS) + pp * plane_pair_stride;
#pragma unroll
                for (int i = 0; i < A; ++i)
                    af[it - h0][i] = __builtin_bit_cast(half8, wl[ab[i] + (t * NPL + pp * 2) * RPW]);
#pragma unroll
                for (int j = 0; j < B; ++j) bf[it - h0][j] = __builtin_bit_cast(half8, xl[xb[j] + toff]);
            }
            __builtin_amdgcn_sched_barrier(0);       // the reads of the half stay ahead of its MFMAs
#pragma unroll
            for (int it = h0; it < h0 + NIT_H && it < NIT_ALL; ++it)
#pragma unroll
                for (int i = 0; i < A; ++i)
#pragma unroll
                    for (int j = 0; j < B; ++j) {
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[it - h0][i], bf[it - h0][j],
                                                                           acc[i][j], 0, 0, 0);
                        const int m = (it * A + i) * B + j;
#pragma unroll
                        for (int slot = m * NLD / NM; slot < (m + 1) * NLD / NM; ++slot) {
                            if (slot < NLD_X)
                                load_patch_chan<XVEC, CALIGN>(rx, pit[slot / 8], stn * CB, Cg, xsoff, chan_bytes,
                                                              slot % 8, xr[slot / 8][slot % 8]);
                            else
                                load_w_round(stn, wnext, slot - NLD_X);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
        }
    };
    typedef std::integral_constant<int, 0> no_loads;
    typedef std::integral_constant<int, 1> patch_loads;
    typedef std::integral_constant<int, 2> all_loads;

    // ---- K loop over channel blocks ----
    // all outstanding vector-memory operations (patch loads and LDS-direct weight rows)
    auto wait_vmem = [&]() { __builtin_amdgcn_s_waitcnt(0x0F70); };
    if constexpr (PW > 0) {
        // Producer and consumer waves.  A wave that issues vector-memory instructions waits
        // on the CU's address unit and a wave that transposes and stores is not issuing
        // MFMAs; with one wave per SIMD these phases would add up.  Here PW waves only
        // stage (loads two steps ahead, three weight buffers, two patch buffers) and the
        // other waves only read fragments and issue MFMAs; both meet at one barrier per step.
        static_assert(PW == 0 || (NSTAGE == 3 && BURST && WDMA), "specialised waves use the two-steps-ahead pipeline");
        constexpr int NLD = 8 * MAXR + WLR;
        static_assert(NLD < 64, "vmcnt is a 6-bit counter");
        constexpr int WAIT_OLDER = (NLD & 15) | ((NLD >> 4) << 14) | 0x0F70;
        u32x4 *const xbuf0 = lds + 3 * W_UNITS;
        if (wave >= NW) {
            auto stage_step = [&](int st, int wi, auto parity) {
                constexpr int P = decltype(parity)::value;
                const bool has1 = st + 1 < st1, has2 = st + 2 < st1;
                const int w1 = wi == 2 ? 0 : wi + 1, w2 = w1 == 2 ? 0 : w1 + 1;
                if (has2) {
                    load_x(st + 2, xreg[P]);
                    load_w(st + 2, lds + w2 * W_UNITS);
                }
                __builtin_amdgcn_sched_barrier(0);
                if (has1) {
                    if (has2) __builtin_amdgcn_s_waitcnt(WAIT_OLDER); else wait_vmem();
                    u32x4 *xn_ = xbuf0 + (P ^ 1) * X_UNITS;
                    store_x(st + 1, xn_, xreg[P ^ 1]);
                    store_w(st + 1, lds + w1 * W_UNITS, xn_);
                }
                lds_barrier();
            };
            load_x(st0, xreg[0]);
            if (st0 + 1 < st1) {
                load_x(st0 + 1, xreg[1]);
                load_w(st0 + 1, lds + W_UNITS);
                __builtin_amdgcn_sched_barrier(0);
                __builtin_amdgcn_s_waitcnt(WAIT_OLDER);
            } else {
                wait_vmem();
            }
            store_x(st0, xbuf0, xreg[0]);
            store_w(st0, lds, xbuf0);
            lds_barrier();
            int wi = 0;
            for (int st = st0; st < st1; st += 2) {
                stage_step(st, wi, std::integral_constant<int, 0>());
                wi = wi == 2 ? 0 : wi + 1;
                if (st + 1 < st1) {
                    stage_step(st + 1, wi, std::integral_constant<int, 1>());
                    wi = wi == 2 ? 0 : wi + 1;
                }
            }
            return;                               // the epilogue belongs to the consumers
        }
        init_acc();
        lds_barrier();                          // the first step is staged
        int wi = 0, par = 0;
        for (int st = st0; st < st1; ++st) {
            burst_step(lds + wi * W_UNITS, xbuf0 + par * X_UNITS, no_loads(), 0, lds, xreg[0]);
            lds_barrier();                      // step st is consumed, step st + 1 is staged
            wi = wi == 2 ? 0 : wi + 1;
            par ^= 1;
        }
    } else if constexpr (NSTAGE == 3) {
        // Three weight buffers and two patch buffers in LDS, two register sets for the patch:
        // the loads of step s+2 are issued before the MFMAs of step s, so a load has a whole
        // step to arrive.  Vector-memory loads complete in order: waiting until only the
        // newest batch (NLD instructions) is outstanding means the older batch has landed.
        static_assert(NSTAGE != 3 || (BURST && WDMA), "prefetch distance 2 is for the small tiles");
        constexpr int NLD = 8 * MAXR + WLR;      // vector-memory instructions of one step's loads
        static_assert(NLD < 64, "vmcnt is a 6-bit counter");
        constexpr int WAIT_OLDER = (NLD & 15) | ((NLD >> 4) << 14) | 0x0F70;
        u32x4 *const xbuf0 = lds + 3 * W_UNITS;
        auto step = [&](int st, int wi, auto parity) {
            constexpr int P = decltype(parity)::value;
            const bool has1 = st + 1 < st1, has2 = st + 2 < st1;
            u32x4 *wl = lds + wi * W_UNITS, *xl = xbuf0 + P * X_UNITS;
            const int w1 = wi == 2 ? 0 : wi + 1, w2 = w1 == 2 ? 0 : w1 + 1;
            if (has2) burst_step(wl, xl, all_loads(), st + 2, lds + w2 * W_UNITS, xreg[P]);
            else burst_step(wl, xl, no_loads(), 0, lds, xreg[P]);
            if (has1) {
                if (has2) __builtin_amdgcn_s_waitcnt(WAIT_OLDER); else wait_vmem();
                u32x4 *xn_ = xbuf0 + (P ^ 1) * X_UNITS;
                store_x(st + 1, xn_, xreg[P ^ 1]);
                store_w(st + 1, lds + w1 * W_UNITS, xn_);
            }
            lds_barrier();
        };
        load_x(st0, xreg[0]);
        if (st0 + 1 < st1) {
            load_x(st0 + 1, xreg[1]);
            load_w(st0 + 1, lds + W_UNITS);
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_waitcnt(WAIT_OLDER);
        } else {
            wait_vmem();
        }
        store_x(st0, xbuf0, xreg[0]);
        store_w(st0, lds, xbuf0);
        init_acc();
        lds_barrier();
        int wi = 0;
        for (int st = st0; st < st1; st += 2) {
            step(st, wi, std::integral_constant<int, 0>());
            wi = wi == 2 ? 0 : wi + 1;
            if (st + 1 < st1) {
                step(st + 1, wi, std::integral_constant<int, 1>());
                wi = wi == 2 ? 0 : wi + 1;
            }
        }
    } else if constexpr (NSTAGE == 2) {
        load_x(st0, xreg[0]);
        wait_vmem();
        store_x(st0, lds + W_UNITS, xreg[0]);
        store_w(st0, lds, lds + W_UNITS);
        init_acc();
        lds_barrier();
        int cur = 0;
        for (int st = st0; st + 1 < st1; ++st, cur ^= 1) {
            u32x4 *wl = lds + cur * stage_units, *xl = wl + W_UNITS;
            u32x4 *wn_ = lds + (cur ^ 1) * stage_units, *xn_ = wn_ + W_UNITS;
            if constexpr (BURST) {
                burst_step(wl, xl, all_loads(), st + 1, wn_, xreg[0]);
                wait_vmem();
                store_x(st + 1, xn_, xreg[0]);
                store_w(st + 1, wn_, xn_);
            } else {
                // region 1: the next step's loads are issued between the first half of the MFMAs
                load_x(st + 1, xreg[0]);
                load_w(st + 1, wn_);
                compute(wl, xl, 0, NIT_H);
                interleave_hint<NIT_H * A * B, 1, 1, 2>();
                wait_vmem();
                // region 2: transposes, regroup and LDS stores between the second half
                store_x(st + 1, xn_, xreg[0]);
                store_w(st + 1, wn_, xn_);
                compute(wl, xl, NIT_H, NIT_ALL);
                interleave_hint<(NIT_ALL - NIT_H) * A * B, 0, 2, 3>();
            }
            lds_barrier();
        }
        if constexpr (BURST)
            burst_step(lds + cur * stage_units, lds + cur * stage_units + W_UNITS, no_loads(), 0, lds, xreg[0]);
        else
            compute(lds + cur * stage_units, lds + cur * stage_units + W_UNITS, 0, NIT_ALL);
        lds_barrier();                          // the buffers are reused by the epilogue
    } else {
        u32x4 *wl = lds, *xl = lds + W_UNITS;
        load_x(st0, xreg[0]);
        init_acc();
        for (int st = st0; st < st1; ++st) {
            lds_barrier();                      // everyone is done reading the buffers
            load_w(st, wl);
            wait_vmem();
            store_x(st, xl, xreg[0]);
            store_w(st, wl, xl);
            lds_barrier();
            if constexpr (BURST) {
                if (st + 1 < st1) burst_step(wl, xl, patch_loads(), st + 1, lds, xreg[0]);
                else burst_step(wl, xl, no_loads(), 0, lds, xreg[0]);
            } else {
                if (st + 1 < st1) load_x(st + 1, xreg[0]);
                compute(wl, xl, 0, NIT_ALL);
            }
        }
        lds_barrier();
    }

    // ---- epilogue: accumulator register e of lane (l32, lh) in block (i, j) is
    // channel row 8*(e/4) + 4*lh + e%4 and pixel column l32 of that block ----
    const int HoWo = p.Ho * p.Wo;
    mfma_drain();
    if (SPLITK) {
        // FP32 partial sums of this slice: 32 consecutive pixels per row and instruction
#pragma unroll
        for (int j = 0; j < B; ++j) {
            const int pix = (wn * B + j) * 32 + l32;
            const int img = pix >> (p.log2_tw + p.log2_thi);
            const int oh = oh0 + ((pix >> p.log2_tw) & ((1 << p.log2_thi) - 1)), ow = ow0 + (pix & (TW - 1));
            const bool pix_ok = (oh < p.Ho) && (ow < p.Wo) && (n + img < p.N);
            float *dst = p.ws + (((size_t)ksl * p.N + n + img) * p.M + (size_t)g * Mg) * HoWo + oh * p.Wo + ow;
#pragma unroll
            for (int i = 0; i < A; ++i)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int ml = m0 + wm * (32 * A) + i * 32 + 8 * (e >> 2) + 4 * lh + (e & 3);
                    if (pix_ok && ml < Mg) dst[(size_t)ml * HoWo] = acc[i][j][e];
                }
        }
        return;
    }
    store_tile<A, B>(p, acc, lds, wave, wm, wn, lane, n, g, m0, oh0, ow0);
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

template <int KS, int A, int B, int WM, int WN, int NPL, int XVEC, bool CALIGN, bool PACKED, int NSTAGE, int MAXR,
          int PW>
static hipError_t launch_igemm(const ConvArgs &a, size_t lds, hipStream_t stream)
{
    const dim3 grid((unsigned)(((a.grid_blocks + 7) / 8) * 8)), block(64 * (WM * WN + PW));
    hipError_t e;
    if (a.split_k > 1) {
        static std::atomic<size_t> granted{0};
        auto kern = igemm_kernel<KS, A, B, WM, WN, NPL, XVEC, CALIGN, PACKED, NSTAGE, MAXR, PW, true>;
        if ((e = ensure_lds(kern, lds, granted)) != hipSuccess) return e;
        hipLaunchKernelGGL(kern, grid, block, lds, stream, a);
    } else {
        static std::atomic<size_t> granted{0};
        auto kern = igemm_kernel<KS, A, B, WM, WN, NPL, XVEC, CALIGN, PACKED, NSTAGE, MAXR, PW, false>;
        if ((e = ensure_lds(kern, lds, granted)) != hipSuccess) return e;
        hipLaunchKernelGGL(kern, grid, block, lds, stream, a);
    }
    return hipGetLastError();
}

#define HGC_VP(KS, A, B, WM, WN, NPL, XVEC, CAL, NST, MAXR, PW)                                 \
    {KS, A, B, WM, WN, NPL, XVEC, CAL, HGC_IGEMM_PACKED, NST, MAXR, PW,                         \
     &launch_igemm<KS, A, B, WM, WN, NPL, XVEC, (CAL != 0), (HGC_IGEMM_PACKED != 0), NST, MAXR, PW>}
#define HGC_V1(KS, A, B, WM, WN, NPL, XVEC, CAL, NST, MAXR) HGC_VP(KS, A, B, WM, WN, NPL, XVEC, CAL, NST, MAXR, 0)
// aligned-channel forms with PW producer waves (the two-steps-ahead pipeline)
#define HGC_VS(KS, A, B, WM, WN, NPL, PW, R4, R2, R1)                                           \
    HGC_VP(KS, A, B, WM, WN, NPL, 4, 1, 3, R4, PW),                                             \
    HGC_VP(KS, A, B, WM, WN, NPL, 2, 1, 3, R2, PW), HGC_VP(KS, A, B, WM, WN, NPL, 1, 1, 3, R1, PW)
// aligned-channel forms of one tile shape for input loads of 4, 2 and 1 pixels
#define HGC_VX(KS, A, B, WM, WN, NPL, NST, R8, R4, R2, R1)                                      \
    HGC_V1(KS, A, B, WM, WN, NPL, 4, 1, NST, R4),                                               \
    HGC_V1(KS, A, B, WM, WN, NPL, 2, 1, NST, R2), HGC_V1(KS, A, B, WM, WN, NPL, 1, 1, NST, R1)
// ragged-channel forms (Cg % 8 != 0 or unaligned weights): 2- and 1-pixel input loads
#define HGC_VR(KS, A, B, WM, WN, NPL, NST, R2, R1)                                              \
    HGC_V1(KS, A, B, WM, WN, NPL, 2, 0, NST, R2), HGC_V1(KS, A, B, WM, WN, NPL, 1, 0, NST, R1)

// The table is compiled in four parts (HGC_IGEMM_PART 0..3, one translation unit each, so that the
// build uses several cores); igemm_tables.hip joins them in this order, which fixes the variant numbers.
static const IgemmVariant g_variants[] = {
    //     KS  A  B  WM WN NPL NST  patch rounds in registers per input-load width
#if HGC_IGEMM_PART == 0
    HGC_VX(3, 2, 4, 2, 4, 2, 2, 1, 1, 2, 2),    // 128 ch x 512 px, 8 waves: throughput tile
    HGC_VX(3, 4, 2, 2, 4, 2, 2, 1, 1, 1, 2),    // 256 ch x 256 px, 8 waves
    HGC_VX(3, 2, 4, 2, 2, 2, 2, 1, 2, 2, 4),    // 128 ch x 256 px
    HGC_VX(3, 2, 2, 2, 2, 2, 2, 1, 1, 2, 2),    // 128 ch x 128 px
    HGC_VX(3, 2, 2, 1, 4, 2, 2, 1, 1, 2, 4),    //  64 ch x 256 px
#elif HGC_IGEMM_PART == 1
    HGC_VR(3, 2, 2, 1, 4, 2, 2, 2, 4),
    HGC_VX(3, 2, 1, 1, 4, 4, 2, 1, 1, 2, 2),    //  64 ch x 128 px, 32 channels per step
    HGC_VX(3, 1, 2, 2, 2, 4, 2, 1, 1, 2, 2),    //  64 ch x 128 px, waves 2 x 2
    HGC_VX(3, 1, 2, 1, 4, 2, 2, 1, 1, 2, 4),    //  32 ch x 256 px
    HGC_VX(3, 1, 1, 1, 4, 4, 2, 1, 1, 2, 2),    //  32 ch x 128 px, 32 channels per step
    HGC_VR(3, 1, 2, 1, 4, 2, 2, 2, 4),
#elif HGC_IGEMM_PART == 2
    HGC_VX(1, 2, 4, 2, 2, 8, 2, 1, 1, 2, 4),    // pointwise 128 ch x 256 px, 64 channels per step
    HGC_VX(1, 2, 2, 1, 4, 8, 2, 1, 1, 2, 4),    // pointwise  64 ch x 256 px
    HGC_VR(1, 2, 2, 1, 4, 8, 2, 2, 4),
    HGC_VX(1, 2, 1, 1, 4, 8, 2, 1, 1, 2, 4),    // pointwise  64 ch x 128 px
    HGC_VX(1, 2, 2, 1, 4, 8, 1, 1, 1, 2, 4),    // pointwise  64 ch x 256 px, one LDS buffer (few channel blocks)
    HGC_VX(1, 2, 1, 1, 4, 8, 1, 1, 1, 2, 4),    // pointwise  64 ch x 128 px, one LDS buffer
    HGC_VX(1, 2, 2, 1, 4, 4, 1, 1, 1, 2, 4),    // pointwise  64 ch x 256 px, 32 channels per step, one LDS buffer
    HGC_VX(1, 4, 1, 1, 4, 8, 1, 1, 1, 2, 4),    // pointwise 128 ch x 128 px, one LDS buffer
    HGC_VX(1, 2, 4, 1, 4, 8, 1, 1, 4, 4, 4),    // pointwise  64 ch x 512 px: many loads in flight per wave
    HGC_VX(1, 2, 4, 1, 4, 4, 1, 1, 2, 4, 4),    // pointwise  64 ch x 512 px, 32 channels per step
    HGC_VX(1, 4, 4, 1, 4, 4, 1, 1, 2, 4, 4),    // pointwise 128 ch x 512 px, 32 channels per step
    HGC_VX(5, 2, 2, 1, 4, 2, 1, 1, 2, 3, 4),    // 5x5  64 ch x 256 px
    HGC_VR(5, 2, 2, 1, 4, 2, 1, 3, 4),
    HGC_VR(7, 1, 2, 1, 4, 2, 1, 3, 6),          // stem-like 7x7: 32 ch x 256 px
#elif HGC_IGEMM_PART == 3
    // small tiles with the loads two steps ahead (three weight buffers): few, latency-bound workgroups
    HGC_VX(3, 1, 1, 1, 4, 4, 3, 1, 1, 2, 2),    //  32 ch x 128 px, 32 channels per step
    HGC_VX(3, 1, 1, 1, 4, 2, 3, 1, 1, 1, 2),    //  32 ch x 128 px, 16 channels per step
    HGC_VX(3, 2, 1, 1, 4, 4, 3, 1, 1, 2, 2),    //  64 ch x 128 px, 32 channels per step
    HGC_VX(3, 1, 2, 1, 4, 2, 3, 1, 1, 2, 4),    //  32 ch x 256 px, 16 channels per step
    // the same with four producer waves beside the four MFMA waves
    HGC_VS(3, 1, 1, 1, 4, 4, 4, 1, 2, 2),       //  32 ch x 128 px, 32 channels per step
    HGC_VS(3, 1, 1, 1, 4, 2, 4, 1, 1, 2),       //  32 ch x 128 px, 16 channels per step
    HGC_VS(3, 2, 1, 1, 4, 4, 4, 1, 2, 2),       //  64 ch x 128 px, 32 channels per step
    HGC_VS(3, 1, 2, 1, 4, 2, 4, 1, 2, 4),       //  32 ch x 256 px, 16 channels per step
    HGC_VS(3, 1, 2, 1, 4, 4, 4, 2, 4, 4),       //  32 ch x 256 px, 32 channels per step
#else
#error "HGC_IGEMM_PART must be 0..3"
#endif
};

const IgemmVariant *HGC_IGEMM_ACCESSOR(int *count)
{
    *count = (int)(sizeof(g_variants) / sizeof(g_variants[0]));
    return g_variants;
}

}  // namespace hgc
