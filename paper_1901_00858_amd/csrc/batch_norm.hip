// Batch-norm layer forward in FP16 for gfx950 (BVLC Caffe's layer, optionally followed by its
// per-channel scale layer and a ReLU):
//   mean[c] = (1/L) sum x,  var[c] = (1/L) sum (x - mean[c])^2,  L = N*H*W,
//   y = act( gamma[c] * (x - mean[c]) / sqrt(var[c] + eps) + beta[c] ).
//
// The paper's FP16 engine keeps the two accumulations in range with two devices (Section 3.1):
// the mean of a long vector is taken as the mean of the means of its groups, and values are
// multiplied by a power of two before they are squared and scaled back afterwards.  What holds
// of that on this chip:
//  * the grouped mean is the natural shape of the reduction.  A group is a contiguous run of at
//    most 2048 values of one (image, channel) plane, owned by one wave, which keeps the whole
//    group in registers (32 values per lane): it sums them, forms the group's own mean, and then
//    sums the squared deviations from THAT mean out of the same registers, so x is read from
//    HBM once for both statistics and no square of a large raw value is ever formed.  A second
//    small kernel takes the (length-weighted) mean of the group means and combines the groups'
//    squared-deviation sums about it: M2 = sum_g [ M2_g + len_g (mean_g - mean)^2 ], in FP64.
//  * the power-of-two scale exists to keep FP16 accumulators finite.  Accumulators here are
//    FP32, as in the convolution; a multiplication by 2^-5 or 2^5 is exact in FP32 over the
//    whole range FP16 deviations and their squares can take (2^-48 .. 2^32), so the step would
//    change no bit of the result and is left out.
// Per-channel parameters and statistics are FP32 (the paper keeps scalars in float, Section 3.2);
// an FP16 variance could not even hold 255^2 of 8-bit image data.
//
// Three launches (statistics of groups; per-channel coefficients mean, a = gamma/sqrt(var+eps)
// and beta; then y = act((x - mean) a + beta) with one rounding to FP16 at the store); two with
// stored statistics.  The mean travels as an FP32 pair (high part + remainder) and is
// subtracted before the multiplication, so the output's error is relative to |x - mean|, not
// to |x| + |mean|, and a constant channel gives beta exactly.  The path is bound by HBM: two
// reads and one write of the tensor.
#include "hgc_internal.h"

namespace hgc {

typedef uint32_t bn_u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t bn_u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 bn_h2 __attribute__((ext_vector_type(2)));

constexpr uint32_t kBnNoLoad = 0xFFFFFFFFu;   // beyond any buffer: such a load returns zero
constexpr int kBnLaneVals = 32;               // values a lane holds: a group is at most 64 * 32 values
constexpr int kBnGroupMax = 64 * kBnLaneVals;

struct BnArgs {
    const uint16_t *x;
    uint16_t *y;
    float2 *part;            // [planes * gpp]  {group mean, group sum of squared deviations}
    float4 *coef;            // [C]             {mean high, mean low, a, beta}
    const float *mean_in, *var_in, *gamma, *beta;
    float *mean_out, *var_out;
    int N, C, HW;
    int gpp, gl;             // groups per plane, values per group (last group of a plane: the rest)
    uint32_t groups;         // N * C * gpp
    uint32_t nvec;           // vectors of the whole tensor in the apply kernel
    uint32_t x_bytes;
    float eps, stat_scale;
    int relu;
    FastDiv fd_gpp, fd_HW, fd_C;
};

__device__ __forceinline__ float bn_lo(uint32_t u) { return (float)__builtin_bit_cast(bn_h2, u).x; }
__device__ __forceinline__ float bn_hi(uint32_t u) { return (float)__builtin_bit_cast(bn_h2, u).y; }

// The statistics kernels are bound by instruction issue before they are bound by memory unless
// the FP16 -> FP32 conversions are folded into the arithmetic.  Sum of a pair of halves: one dot
// product with (1, 1), products and sum in FP32.  Deviation from a mean: the mixed-precision
// multiply-add, (float)half * 1.0 + (-mean), one instruction per value, result in FP32.
__device__ __forceinline__ float bn_add_pair(uint32_t w, float acc)
{
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(bn_h2, w), __builtin_bit_cast(bn_h2, 0x3C003C00u), acc, false);
}
__device__ __forceinline__ float bn_dev_lo(uint32_t w, float neg_mean)
{
    float d;
    asm("v_fma_mix_f32 %0, %1, 1.0, %2 op_sel_hi:[1,0,0]" : "=v"(d) : "v"(w), "v"(neg_mean));
    return d;
}
__device__ __forceinline__ float bn_dev_hi(uint32_t w, float neg_mean)
{
    float d;
    asm("v_fma_mix_f32 %0, %1, 1.0, %2 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(w), "v"(neg_mean));
    return d;
}

// One load of V halves into NW = max(V / 2, 1) registers (V = 1: the half in the low 16 bits, zero above).
template <int V>
__device__ __forceinline__ void bn_load(uint32_t *dst, const __amdgpu_buffer_rsrc_t rx, uint32_t off)
{
    if constexpr (V == 8) {
        const bn_u32x4 d = __builtin_amdgcn_raw_buffer_load_b128(rx, off, 0, 0);
        dst[0] = d.x; dst[1] = d.y; dst[2] = d.z; dst[3] = d.w;
    } else if constexpr (V == 4) {
        const bn_u32x2 d = __builtin_amdgcn_raw_buffer_load_b64(rx, off, 0, 0);
        dst[0] = d.x; dst[1] = d.y;
    } else if constexpr (V == 2) {
        dst[0] = __builtin_amdgcn_raw_buffer_load_b32(rx, off, 0, 0);
    } else {
        dst[0] = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rx, off, 0, 0);
    }
}
// sum of squared deviations of one load's values; neg_mean = 0 for a load beyond the group (its values are zero)
template <int V>
__device__ __forceinline__ float bn_sq_dev(const uint32_t *w, float neg_mean, float t)
{
#pragma unroll
    for (int i = 0; i < (V >= 2 ? V / 2 : 1); ++i) {
        const float d0 = bn_dev_lo(w[i], neg_mean);
        t = fmaf(d0, d0, t);
        if (V >= 2) {
            const float d1 = bn_dev_hi(w[i], neg_mean);
            t = fmaf(d1, d1, t);
        }
    }
    return t;
}

// Sums over the 64 lanes on the data-parallel-primitive path of the ALU (no LDS crossbar, a few
// cycles a step): four rotations within each row of 16 lanes leave the row's sum in all its lanes;
// for FP32 two row broadcasts (lane 15 into the next row, lane 31 into rows 2 and 3) then leave
// the wave's sum in lane 63, which is read as a scalar.  The order of the additions is fixed.
template <int CTRL, int ROWS = 0xF>
__device__ __forceinline__ float bn_dpp(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROWS, 0xF, false));
}
__device__ __forceinline__ float bn_row_sum(float v)
{
    v += bn_dpp<0x128>(v);          // row_ror:8
    v += bn_dpp<0x124>(v);          // row_ror:4
    v += bn_dpp<0x122>(v);          // row_ror:2
    v += bn_dpp<0x121>(v);          // row_ror:1
    return v;
}
__device__ __forceinline__ float bn_wave_sum(float v)
{
    v = bn_row_sum(v);
    v += bn_dpp<0x142, 0xA>(v);     // row_bcast:15 into rows 1 and 3 (the other rows add zero)
    v += bn_dpp<0x143, 0xC>(v);     // row_bcast:31 into rows 2 and 3
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}
__device__ __forceinline__ float bn_get_lane(float v, int lane)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}

template <int CTRL>
__device__ __forceinline__ double bn_dpp(double v)
{
    const uint64_t u = __builtin_bit_cast(uint64_t, v);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)u, CTRL, 0xF, 0xF, false);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(u >> 32), CTRL, 0xF, 0xF, false);
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ double bn_lane(double v, int lane)
{
    const uint64_t u = __builtin_bit_cast(uint64_t, v);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)u, lane);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(u >> 32), lane);
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ double bn_wave_sum(double v)
{
    v += bn_dpp<0x128>(v);
    v += bn_dpp<0x124>(v);
    v += bn_dpp<0x122>(v);
    v += bn_dpp<0x121>(v);
    return (bn_lane(v, 0) + bn_lane(v, 16)) + (bn_lane(v, 32) + bn_lane(v, 48));
}

// A wave takes PP consecutive groups, each of at most 64 * 32 / PP values, and issues the loads
// of all of them before any arithmetic: planes of 7x7 or 14x14 values are far too short to
// cover the memory latency one at a time, and at one plane a wave the kernel would be bound by
// instruction issue, not by memory.  The groups' sums are gathered into one register (group k in
// lane k), so that the division by the length and the store are done once for all of them.
// V = values per load (8, 4, 2, 1), chosen on the host from the alignment of the base and of the
// plane length, so that every load is naturally aligned and no vector straddles the end of a
// group (group lengths are then multiples of V).
template <int V, int PP>
__global__ __launch_bounds__(256) void bn_group_stats_kernel(const BnArgs p)
{
    constexpr int JP = kBnLaneVals / V / PP;                      // loads per lane and group
    static_assert(JP >= 1 && PP <= 32, "a group needs at least one load per lane");
    const uint32_t lane = threadIdx.x & 63;
    // the same for every lane of the wave: taken through a scalar register so that the tests on
    // the groups' lengths below are scalar branches
    const uint32_t g0 = __builtin_amdgcn_readfirstlane((blockIdx.x * 4 + (threadIdx.x >> 6)) * PP);
    if (g0 >= p.groups) return;
    const __amdgpu_buffer_rsrc_t rx =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(p.x), 0, p.x_bytes, 0x00020000);
    // A short group issues only the loads and the arithmetic it needs: load j of the lanes
    // covers values from j * 64 * V on.  Values stay packed as they arrive.
    constexpr int NW = V >= 2 ? V / 2 : 1;
    uint32_t v[PP][JP * NW];
    uint32_t len[PP];
#pragma unroll
    for (int k = 0; k < PP; ++k) {
        const uint32_t grp = g0 + k;
        const uint32_t plane = fast_div(grp, p.fd_gpp);
        const uint32_t e0 = (grp - plane * (uint32_t)p.gpp) * (uint32_t)p.gl;
        len[k] = grp < p.groups ? min((uint32_t)p.gl, (uint32_t)p.HW - e0) : 0u;
        const uint32_t base = 2u * (plane * (uint32_t)p.HW + e0);
#pragma unroll
        for (int j = 0; j < JP; ++j) {
#pragma unroll
            for (int i = 0; i < NW; ++i) v[k][j * NW + i] = 0u;
            if (JP == 1 || (uint32_t)j * 64u * V < len[k]) {
                const uint32_t e = ((uint32_t)j * 64u + lane) * V;
                bn_load<V>(&v[k][j * NW], rx, e < len[k] ? base + 2u * e : kBnNoLoad);   // beyond the group: zero
            }
        }
    }
    // lane k (k < PP) works out the length of group k for itself: the divisor of the means
    float lens;
    {
        const uint32_t grp = g0 + min(lane, (uint32_t)(PP - 1));
        const uint32_t plane = fast_div(grp, p.fd_gpp);
        const uint32_t e0 = (grp - plane * (uint32_t)p.gpp) * (uint32_t)p.gl;
        lens = grp < p.groups ? (float)min((uint32_t)p.gl, (uint32_t)p.HW - e0) : 1.0f;
    }
    float sums = 0.0f;
#pragma unroll
    for (int k = 0; k < PP; ++k) {
        float s = 0.0f;
#pragma unroll
        for (int j = 0; j < JP; ++j)
            if (JP == 1 || (uint32_t)j * 64u * V < len[k]) {
#pragma unroll
                for (int i = 0; i < NW; ++i) s = bn_add_pair(v[k][j * NW + i], s);
            }
        const float ws = bn_wave_sum(s);                          // by every lane: a wave-wide operation
        sums = lane == (uint32_t)k ? ws : sums;
    }
    const float means = sums / lens;                              // the groups' means, group k in lane k
    float m2 = 0.0f;
#pragma unroll
    for (int k = 0; k < PP; ++k) {
        const float nm = -bn_get_lane(means, k);
        float t = 0.0f;
#pragma unroll
        for (int j = 0; j < JP; ++j)
            if (JP == 1 || (uint32_t)j * 64u * V < len[k])
                t = bn_sq_dev<V>(&v[k][j * NW], ((uint32_t)j * 64u + lane) * V < len[k] ? nm : 0.0f, t);
        const float wt = bn_wave_sum(t);
        m2 = lane == (uint32_t)k ? wt : m2;
    }
    if (lane < PP && g0 + lane < p.groups) p.part[g0 + lane] = make_float2(means, m2);
}

// Planes of at most 256 values (7x7, 14x14, 16x16 feature maps; 1x1 after a global pooling): a
// plane per row of 16 lanes, four planes side by side in a wave and up to eight such sets one
// after the other, all loads first.  The rotations within a row are the whole reduction, each
// lane ends up with its own plane's sum, and the mean, the deviations and their squares stay
// ordinary per-lane arithmetic: no scalar detour, every instruction works on four planes.
// Here a group is the plane (one group per plane).  JP = loads per lane and plane.
template <int V, int JP>
__global__ __launch_bounds__(256) void bn_row_stats_kernel(const BnArgs p)
{
    constexpr int kSets = kBnLaneVals / (V * JP) < 8 ? kBnLaneVals / (V * JP) : 8;
    static_assert(kSets >= 1, "a plane must fit the 32 values a lane holds");
    const uint32_t lane = threadIdx.x & 63, row = lane >> 4, li = lane & 15;
    const uint32_t p0 = (blockIdx.x * 4 + (threadIdx.x >> 6)) * (4u * kSets);     // the wave's first plane
    if (p0 >= p.groups) return;
    const __amdgpu_buffer_rsrc_t rx =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(p.x), 0, p.x_bytes, 0x00020000);
    const uint32_t HW = (uint32_t)p.HW;
    constexpr int NW = V >= 2 ? V / 2 : 1;
    uint32_t v[kSets][JP * NW];
#pragma unroll
    for (int k = 0; k < kSets; ++k) {
        const uint32_t plane = p0 + 4u * k + row;
        const uint32_t base = 2u * plane * HW;
#pragma unroll
        for (int j = 0; j < JP; ++j) {
            const uint32_t e = ((uint32_t)j * 16u + li) * V;
            bn_load<V>(&v[k][j * NW], rx, (plane < p.groups && e < HW) ? base + 2u * e : kBnNoLoad);   // else zero
        }
    }
    const float flen = (float)HW;
#pragma unroll
    for (int k = 0; k < kSets; ++k) {
        float s = 0.0f;
#pragma unroll
        for (int i = 0; i < JP * NW; ++i) s = bn_add_pair(v[k][i], s);
        const float m = bn_row_sum(s) / flen;                     // this lane's plane's mean
        float t = 0.0f;
#pragma unroll
        for (int j = 0; j < JP; ++j)
            t = bn_sq_dev<V>(&v[k][j * NW], ((uint32_t)j * 16u + li) * V < HW ? -m : 0.0f, t);
        t = bn_row_sum(t);
        const uint32_t plane = p0 + 4u * k + row;
        if (li == 0 && plane < p.groups) p.part[plane] = make_float2(m, t);
    }
}

__device__ __forceinline__ float4 bn_coefficients(double mu, double var, double gamma, double beta, float eps)
{
    const float mh = (float)mu;
    return make_float4(mh, (float)(mu - (double)mh), (float)(gamma / sqrt(var + (double)eps)), (float)beta);
}

// One wave per channel: length-weighted mean of the group means, then the groups' squared
// deviations combined about it; FP64 (a few thousand terms at most).
__global__ __launch_bounds__(64) void bn_channel_kernel(const BnArgs p)
{
    const int c = blockIdx.x;
    const int lane = threadIdx.x;
    const int per = p.N * p.gpp;
    const double L = (double)p.N * (double)p.HW;
    double sw = 0.0;
    for (int i = lane; i < per; i += 64) {
        const int n = i / p.gpp, j = i - n * p.gpp;
        const int len = min(p.gl, p.HW - j * p.gl);
        sw += (double)len * (double)p.part[(size_t)(n * p.C + c) * p.gpp + j].x;
    }
    const double mu = bn_wave_sum(sw) / L;
    double m2 = 0.0;
    for (int i = lane; i < per; i += 64) {
        const int n = i / p.gpp, j = i - n * p.gpp;
        const int len = min(p.gl, p.HW - j * p.gl);
        const float2 g = p.part[(size_t)(n * p.C + c) * p.gpp + j];
        const double d = (double)g.x - mu;
        m2 += (double)g.y + (double)len * d * d;
    }
    const double var = bn_wave_sum(m2) / L;
    if (lane == 0) {
        const double gm = p.gamma ? (double)p.gamma[c] : 1.0;
        const double bt = p.beta ? (double)p.beta[c] : 0.0;
        p.coef[c] = bn_coefficients(mu, var, gm, bt, p.eps);
        if (p.mean_out) p.mean_out[c] = (float)mu;
        if (p.var_out) p.var_out[c] = (float)var;
    }
}

// Stored statistics: a thread per channel.
__global__ __launch_bounds__(256) void bn_stored_stats_kernel(const BnArgs p)
{
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= p.C) return;
    const double mu = (double)p.stat_scale * (double)p.mean_in[c];
    const double var = (double)p.stat_scale * (double)p.var_in[c];
    const double gm = p.gamma ? (double)p.gamma[c] : 1.0;
    const double bt = p.beta ? (double)p.beta[c] : 0.0;
    p.coef[c] = bn_coefficients(mu, var, gm, bt, p.eps);
}

__device__ __forceinline__ uint32_t bn_apply2(uint32_t u, const float4 k, bool relu)
{
    float lo = fmaf((bn_lo(u) - k.x) - k.y, k.z, k.w), hi = fmaf((bn_hi(u) - k.x) - k.y, k.z, k.w);
    if (relu) { lo = fmaxf(lo, 0.0f); hi = fmaxf(hi, 0.0f); }
    bn_h2 r;
    r.x = (_Float16)lo;
    r.y = (_Float16)hi;
    return __builtin_bit_cast(uint32_t, r);
}

// y = act((x - mean[c]) a[c] + beta[c]) over the tensor taken as one flat array of V-value vectors (a plane's
// length is a multiple of V, so a vector lies in one plane).  Each thread takes U vectors, 256
// vectors apart.  Loads and stores are range-checked buffer accesses (a vector past the end reads
// zero and its store is dropped), so the kernel has no branch and all of a thread's loads are in
// flight together; with an `if (inside)` around each the compiler waits for one before issuing the
// next.  y may be x itself.
template <int V>
__global__ __launch_bounds__(256) void bn_apply_kernel(const BnArgs p)
{
    constexpr int U = 4;
    constexpr int NW = V >= 2 ? V / 2 : 1;
    const __amdgpu_buffer_rsrc_t rx =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(p.x), 0, p.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(p.y, 0, p.x_bytes, 0x00020000);
    const uint32_t v0 = blockIdx.x * (256u * U) + threadIdx.x;
    uint32_t d[U][NW];
    float4 k[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t vi = v0 + (uint32_t)u * 256u;
        // past the end: the byte offset is beyond the buffer (nvec * V * 2 = its size; no wrap: vi < 2^29 + 2^20)
        bn_load<V>(d[u], rx, vi < p.nvec ? vi * (2u * V) : kBnNoLoad);
        const uint32_t plane = fast_div(min(vi, p.nvec - 1u) * V, p.fd_HW);
        k[u] = p.coef[plane - fast_div(plane, p.fd_C) * (uint32_t)p.C];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t vi = v0 + (uint32_t)u * 256u;
        const uint32_t off = vi < p.nvec ? vi * (2u * V) : kBnNoLoad;
        const bool relu = p.relu != 0;
        uint32_t r[NW];
#pragma unroll
        for (int i = 0; i < NW; ++i) r[i] = bn_apply2(d[u][i], k[u], relu);
        if constexpr (V == 8) {
            const bn_u32x4 o = {r[0], r[1], r[2], r[3]};
            __builtin_amdgcn_raw_buffer_store_b128(o, ry, off, 0, 0);
        } else if constexpr (V == 4) {
            const bn_u32x2 o = {r[0], r[1]};
            __builtin_amdgcn_raw_buffer_store_b64(o, ry, off, 0, 0);
        } else if constexpr (V == 2) {
            __builtin_amdgcn_raw_buffer_store_b32(r[0], ry, off, 0, 0);
        } else {
            __builtin_amdgcn_raw_buffer_store_b16((uint16_t)r[0], ry, off, 0, 0);
        }
    }
}

static int bn_groups_per_plane(long long HW) { return (int)((HW + kBnGroupMax - 1) / kBnGroupMax); }

static size_t bn_round256(size_t v) { return (v + 255) & ~(size_t)255; }

// Workspace: 256 bytes of slack to align the base, the C coefficient pairs, then the group partials.
static size_t bn_workspace_bytes(const hgc_batch_norm_desc *d)
{
    const long long HW = (long long)d->H * d->W;
    size_t need = 256 + bn_round256(16 * (size_t)d->C);
    if (!d->use_global_stats) need += 8 * (size_t)d->N * (size_t)d->C * (size_t)bn_groups_per_plane(HW);
    return need;
}

static hgc_status bn_check_desc(const hgc_batch_norm_desc *d)
{
    if (d->N < 1 || d->C < 1 || d->H < 1 || d->W < 1) return HGC_ERR_BAD_DESC;
    if ((d->use_global_stats != 0 && d->use_global_stats != 1) || (d->scale_bias != 0 && d->scale_bias != 1) ||
        (d->relu != 0 && d->relu != 1))
        return HGC_ERR_BAD_DESC;
    if (!(d->eps > 0.0f) || !(d->eps < 3.0e38f)) return HGC_ERR_BAD_DESC;
    if (d->use_global_stats && !(d->stat_scale > 0.0f && d->stat_scale < 3.0e38f)) return HGC_ERR_BAD_DESC;
    if ((long long)d->N * d->C * d->H * d->W > 0x7FFFFFFFLL) return HGC_ERR_TOO_LARGE;
    return HGC_OK;
}

template <int V, int PP>
static hipError_t bn_launch_stats(const BnArgs &a, hipStream_t s)
{
    const uint32_t waves = (a.groups + PP - 1) / PP;
    bn_group_stats_kernel<V, PP><<<dim3((waves + 3) / 4), dim3(256), 0, s>>>(a);
    return hipGetLastError();
}

template <int V, int JP>
static hipError_t bn_launch_rows(const BnArgs &a, hipStream_t s)
{
    if constexpr (V * JP <= kBnLaneVals) {
        constexpr int kSets = kBnLaneVals / (V * JP) < 8 ? kBnLaneVals / (V * JP) : 8;
        const uint32_t waves = (a.groups + 4 * kSets - 1) / (4 * kSets);
        bn_row_stats_kernel<V, JP><<<dim3((waves + 3) / 4), dim3(256), 0, s>>>(a);
        return hipGetLastError();
    } else {
        return hipErrorInvalidValue;                               // not reached: the caller checks the plane length
    }
}

constexpr int kBnRowPlaneMax = 256;     // planes up to this length go a plane per 16 lanes

template <int V>
static hipError_t bn_launch(const BnArgs &a, bool batch_stats, hipStream_t s)
{
    if (batch_stats && a.gpp == 1 && a.HW <= kBnRowPlaneMax) {
        const int need = (a.HW + 16 * V - 1) / (16 * V);            // loads per lane, rounded up to a power of two
        hipError_t e;
        if (need <= 1) e = bn_launch_rows<V, 1>(a, s);
        else if (need <= 2) e = bn_launch_rows<V, 2>(a, s);
        else if (need <= 4) e = bn_launch_rows<V, 4>(a, s);
        else if (need <= 8) e = bn_launch_rows<V, 8>(a, s);
        else e = bn_launch_rows<V, 16>(a, s);
        if (e != hipSuccess) return e;
        bn_channel_kernel<<<dim3(a.C), dim3(64), 0, s>>>(a);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    } else if (batch_stats) {
        // as many groups per wave as fit its 32 values per lane (a power of two, 32 / V at most)
        const int fit = 64 * kBnLaneVals / a.gl;
        hipError_t e;
        if (fit >= 32 && V == 1) e = bn_launch_stats<V, V == 1 ? 32 : 1>(a, s);
        else if (fit >= 16 && V <= 2) e = bn_launch_stats<V, V <= 2 ? 16 : 1>(a, s);
        else if (fit >= 8 && V <= 4) e = bn_launch_stats<V, V <= 4 ? 8 : 1>(a, s);
        else if (fit >= 4) e = bn_launch_stats<V, 4>(a, s);
        else if (fit >= 2) e = bn_launch_stats<V, 2>(a, s);
        else e = bn_launch_stats<V, 1>(a, s);
        if (e != hipSuccess) return e;
        bn_channel_kernel<<<dim3(a.C), dim3(64), 0, s>>>(a);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    } else {
        bn_stored_stats_kernel<<<dim3((a.C + 255) / 256), dim3(256), 0, s>>>(a);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    bn_apply_kernel<V><<<dim3((a.nvec + 1023) / 1024), dim3(256), 0, s>>>(a);
    return hipGetLastError();
}

// Offline folding of stored statistics into the convolution in front: one thread per weight (and
// one per bias), FP64 arithmetic, one rounding to FP16 per value.
struct FoldArgs {
    const uint16_t *w, *b;
    const float *mean, *var, *gamma, *beta;
    uint16_t *w_out, *b_out;
    uint32_t per, total;      // weights per output channel, all weights
    int M;
    float eps, stat_scale;
    FastDiv fd_per;
};

__device__ __forceinline__ double bn_fold_scale(const FoldArgs &a, int m)
{
    const double g = a.gamma ? (double)a.gamma[m] : 1.0;
    return g / sqrt((double)a.stat_scale * (double)a.var[m] + (double)a.eps);
}

__global__ __launch_bounds__(256) void bn_fold_kernel(const FoldArgs a)
{
    const uint32_t i = blockIdx.x * 256u + threadIdx.x;
    if (i < a.total) {
        const int m = (int)fast_div(i, a.fd_per);
        const double wv = (double)__builtin_bit_cast(_Float16, a.w[i]);
        a.w_out[i] = __builtin_bit_cast(uint16_t, (_Float16)(bn_fold_scale(a, m) * wv));
    }
    if (i < (uint32_t)a.M) {
        const double bv = a.b ? (double)__builtin_bit_cast(_Float16, a.b[i]) : 0.0;
        const double bt = a.beta ? (double)a.beta[i] : 0.0;
        const double r = bn_fold_scale(a, (int)i) * (bv - (double)a.stat_scale * (double)a.mean[i]) + bt;
        a.b_out[i] = __builtin_bit_cast(uint16_t, (_Float16)r);
    }
}

}  // namespace hgc

using namespace hgc;

extern "C" hgc_status hgc_batch_norm_fold(const hgc_conv2d_desc *conv, const void *w, const void *b, const float *mean,
                                          const float *var, float stat_scale, float eps, const float *gamma,
                                          const float *beta, void *w_out, void *b_out, void *stream)
{
    if (!conv || !w || !mean || !var || !w_out || !b_out) return HGC_ERR_NULL;
    if (conv->bias == 1 && !b) return HGC_ERR_NULL;
    if ((gamma == nullptr) != (beta == nullptr)) return HGC_ERR_NULL;
    if (conv->C < 1 || conv->num_output < 1 || conv->kernel < 1 || conv->group < 1 || conv->C % conv->group != 0 ||
        conv->num_output % conv->group != 0 || (conv->bias != 0 && conv->bias != 1))
        return HGC_ERR_BAD_DESC;
    if (!(eps > 0.0f && eps < 3.0e38f) || !(stat_scale > 0.0f && stat_scale < 3.0e38f)) return HGC_ERR_BAD_DESC;
    const long long per = (long long)(conv->C / conv->group) * conv->kernel * conv->kernel;
    if (per * conv->num_output > 0x7FFFFFFFLL) return HGC_ERR_TOO_LARGE;
    FoldArgs a;
    a.w = static_cast<const uint16_t *>(w);
    a.b = conv->bias ? static_cast<const uint16_t *>(b) : nullptr;
    a.mean = mean; a.var = var; a.gamma = gamma; a.beta = beta;
    a.w_out = static_cast<uint16_t *>(w_out);
    a.b_out = static_cast<uint16_t *>(b_out);
    a.per = (uint32_t)per;
    a.total = (uint32_t)(per * conv->num_output);
    a.M = conv->num_output;
    a.eps = eps; a.stat_scale = stat_scale;
    a.fd_per = make_fastdiv(a.per);
    const uint32_t threads = a.total > (uint32_t)a.M ? a.total : (uint32_t)a.M;
    bn_fold_kernel<<<dim3((threads + 255) / 256), dim3(256), 0, static_cast<hipStream_t>(stream)>>>(a);
    const hipError_t e = hipGetLastError();
    set_last_hip_error(e);
    return e == hipSuccess ? HGC_OK : HGC_ERR_LAUNCH;
}

extern "C" hgc_status hgc_batch_norm_workspace_size(const hgc_batch_norm_desc *desc, size_t *bytes)
{
    if (!desc || !bytes) return HGC_ERR_NULL;
    const hgc_status st = bn_check_desc(desc);
    if (st != HGC_OK) return st;
    *bytes = bn_workspace_bytes(desc);
    return HGC_OK;
}

extern "C" hgc_status hgc_batch_norm_forward(const hgc_batch_norm_desc *desc, const void *x, float *mean, float *var,
                                             const float *gamma, const float *beta, void *y, void *workspace,
                                             size_t workspace_bytes, void *stream)
{
    if (!desc || !x || !y) return HGC_ERR_NULL;
    if (desc->use_global_stats == 1 && (!mean || !var)) return HGC_ERR_NULL;
    if (desc->scale_bias == 1 && (!gamma || !beta)) return HGC_ERR_NULL;
    const hgc_status st = bn_check_desc(desc);
    if (st != HGC_OK) return st;
    if (!workspace || workspace_bytes < bn_workspace_bytes(desc)) return HGC_ERR_WORKSPACE;

    const long long HW = (long long)desc->H * desc->W;
    const long long total = (long long)desc->N * desc->C * HW;
    BnArgs a;
    a.x = static_cast<const uint16_t *>(x);
    a.y = static_cast<uint16_t *>(y);
    uint8_t *ws = reinterpret_cast<uint8_t *>(bn_round256((size_t)(uintptr_t)workspace));
    a.coef = reinterpret_cast<float4 *>(ws);
    a.part = reinterpret_cast<float2 *>(ws + bn_round256(16 * (size_t)desc->C));
    const bool batch_stats = desc->use_global_stats == 0;
    a.mean_in = batch_stats ? nullptr : mean;
    a.var_in = batch_stats ? nullptr : var;
    a.mean_out = batch_stats ? mean : nullptr;
    a.var_out = batch_stats ? var : nullptr;
    a.gamma = desc->scale_bias ? gamma : nullptr;
    a.beta = desc->scale_bias ? beta : nullptr;
    a.N = desc->N; a.C = desc->C; a.HW = (int)HW;
    a.gpp = bn_groups_per_plane(HW);
    a.gl = (int)((((HW + a.gpp - 1) / a.gpp) + 7) / 8 * 8);
    a.groups = (uint32_t)((long long)desc->N * desc->C * a.gpp);
    a.x_bytes = (uint32_t)(2 * total);
    a.eps = desc->eps; a.stat_scale = desc->stat_scale; a.relu = desc->relu;
    a.fd_gpp = make_fastdiv((uint32_t)a.gpp);
    a.fd_HW = make_fastdiv((uint32_t)HW);
    a.fd_C = make_fastdiv((uint32_t)desc->C);

    // widest vector every access is naturally aligned for
    const uintptr_t bits = (uintptr_t)x | (uintptr_t)y;
    int V = 1;
    if (HW % 8 == 0 && (bits & 15) == 0) V = 8;
    else if (HW % 4 == 0 && (bits & 7) == 0) V = 4;
    else if (HW % 2 == 0 && (bits & 3) == 0) V = 2;
    a.nvec = (uint32_t)(total / V);

    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e;
    switch (V) {
    case 8: e = bn_launch<8>(a, batch_stats, s); break;
    case 4: e = bn_launch<4>(a, batch_stats, s); break;
    case 2: e = bn_launch<2>(a, batch_stats, s); break;
    default: e = bn_launch<1>(a, batch_stats, s); break;
    }
    set_last_hip_error(e);
    return e == hipSuccess ? HGC_OK : HGC_ERR_LAUNCH;
}
