// Non-MFMA kernels of libhgc: the reference direct kernel (any descriptor), the
// depthwise streaming kernel and the split-K reduction.  All accumulate in FP32
// and round to FP16 once (paper Section 3.1 on accumulation; Section 3.3: no
// separate conversion pass).
#include "hgc_internal.h"

namespace hgc {

__device__ __forceinline__ float h2f(uint16_t bits)
{
    return (float)__builtin_bit_cast(_Float16, bits);
}
__device__ __forceinline__ uint16_t f2h(float v)
{
    return __builtin_bit_cast(uint16_t, (_Float16)v);
}

// One thread per output element, consecutive threads along ow.  Walks the
// reduction in the weight layout's order (c, r, q).
__global__ __launch_bounds__(256) void direct_kernel(const ConvArgs p)
{
    const long long total = (long long)p.N * p.M * p.Ho * p.Wo;
    for (long long o = (long long)blockIdx.x * 256 + threadIdx.x; o < total;
         o += (long long)gridDim.x * 256) {
        int ow = (int)(o % p.Wo);
        long long t = o / p.Wo;
        int oh = (int)(t % p.Ho); t /= p.Ho;
        int m = (int)(t % p.M);
        int n = (int)(t / p.M);
        int g = m / p.Mg;
        const uint16_t *xg = p.x + ((size_t)n * p.C + (size_t)g * p.Cg) * p.H * p.W;
        const uint16_t *wm = p.w + (size_t)m * p.Cg * p.ks * p.ks;
        float acc = 0.0f;
        for (int c = 0; c < p.Cg; ++c)
            for (int r = 0; r < p.ks; ++r) {
                int ih = oh * p.stride - p.pad + r;
                if (ih < 0 || ih >= p.H) continue;
                for (int q = 0; q < p.ks; ++q) {
                    int iw = ow * p.stride - p.pad + q;
                    if (iw < 0 || iw >= p.W) continue;
                    acc = fmaf(h2f(wm[(c * p.ks + r) * p.ks + q]),
                               h2f(xg[((size_t)c * p.H + ih) * p.W + iw]), acc);
                }
            }
        if (p.bias) acc += h2f(p.b[m]);
        if (p.relu) acc = fmaxf(acc, 0.0f);
        p.y[o] = f2h(acc);
    }
}

hipError_t launch_direct(const ConvArgs &a, hipStream_t stream)
{
    const long long total = (long long)a.N * a.M * a.Ho * a.Wo;
    long long blocks = (total + 255) / 256;
    if (blocks > 1048576) blocks = 1048576;
    hipLaunchKernelGGL(direct_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, a);
    return hipGetLastError();
}

// Depthwise (group == C == num_output): each output reads k*k inputs of its own
// channel; 1.8 - 4.5 FLOP per byte, so the kernel is a stream over x and y.
// A workgroup handles a strip of one (n, c) plane; threads run along ow so that
// loads and stores are contiguous, and the k*k weights of the channel sit in
// registers.
template <int KS>
__global__ __launch_bounds__(256) void depthwise_kernel(const ConvArgs p)
{
    const int HoWo = p.Ho * p.Wo;
    const int chunks = (HoWo + 255) / 256;
    const long long nblocks = (long long)p.N * p.C * chunks;
    for (long long bid = blockIdx.x; bid < nblocks; bid += gridDim.x) {
        const int chunk = (int)(bid % chunks);
        const long long nc = bid / chunks;
        const int c = (int)(nc % p.C);
        float wr[KS * KS];
#pragma unroll
        for (int t = 0; t < KS * KS; ++t) wr[t] = h2f(p.w[(size_t)c * KS * KS + t]);
        const float bv = p.bias ? h2f(p.b[c]) : 0.0f;
        const int o = chunk * 256 + threadIdx.x;
        if (o < HoWo) {
            const int oh = o / p.Wo, ow = o % p.Wo;
            const uint16_t *xp = p.x + (size_t)nc * p.H * p.W;
            float acc = 0.0f;
#pragma unroll
            for (int r = 0; r < KS; ++r) {
                const int ih = oh * p.stride - p.pad + r;
#pragma unroll
                for (int q = 0; q < KS; ++q) {
                    const int iw = ow * p.stride - p.pad + q;
                    float xv = 0.0f;
                    if (ih >= 0 && ih < p.H && iw >= 0 && iw < p.W) xv = h2f(xp[ih * p.W + iw]);
                    acc = fmaf(wr[r * KS + q], xv, acc);
                }
            }
            acc += bv;
            if (p.relu) acc = fmaxf(acc, 0.0f);
            p.y[(size_t)nc * HoWo + o] = f2h(acc);
        }
    }
}

// Depthwise 3x3, pad 1, vector form.  A thread produces RO rows x VO consecutive outputs
// from RO*STRIDE + 3 - STRIDE input rows; each input row is one aligned load of
// VI = VO*STRIDE pixels, and the two halo columns come from the neighbouring lanes by
// wavefront shuffles (lanes run along the row).  Only the first and last lane of a wave,
// when their neighbour pixel belongs to another wave, fetch the halo themselves.
// x and y are each touched once (rows shared by vertically adjacent threads hit in cache).
template <int STRIDE, int VO, int RO>
__global__ __launch_bounds__(256) void depthwise3_vec_kernel(const ConvArgs p)
{
    constexpr int VI = VO * STRIDE;
    constexpr int RI = (RO - 1) * STRIDE + 3;      // input rows per thread
    constexpr uint32_t kNone = 0xFFFFFFFFu;        // an offset beyond any buffer: such a load returns zero
    typedef uint16_t ho __attribute__((ext_vector_type(VO)));
    typedef uint32_t dw_u32x2 __attribute__((ext_vector_type(2)));
    typedef uint32_t dw_u32x4 __attribute__((ext_vector_type(4)));
    const uint32_t GW = p.fd_tiles_w.d;            // thread groups per output row (Wo / VO)
    const uint32_t GH = p.fd_tiles_h.d;            // row groups per plane
    const uint32_t items = (uint32_t)p.N * (uint32_t)p.C * GH * GW;
    const uint32_t lane = threadIdx.x & 63;
    const __amdgpu_buffer_rsrc_t rx =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(p.x), 0, p.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(p.bias ? p.b : p.x), 0, p.bias ? 2 * p.M : 0, 0x00020000);
    for (uint32_t t = blockIdx.x * 256u + threadIdx.x; t - lane < items; t += gridDim.x * 256u) {
        const bool live = t < items;               // whole waves stay in the loop: shuffles need every lane
        const uint32_t tt = live ? t : items - 1;
        const uint32_t u = fast_div(tt, p.fd_tiles_w);
        const int owg = (int)(tt - u * GW);
        const uint32_t nc = fast_div(u, p.fd_tiles_h);
        const int oh0 = (int)(u - nc * GH) * RO;
        const int c = (int)(nc - fast_div(nc, p.fd_G) * (uint32_t)p.C);
        float wr[9];
#pragma unroll
        for (int k = 0; k < 9; ++k) wr[k] = h2f(p.w[(size_t)c * 9 + k]);
        // range-checked (zero without a bias): no branch, no wait of its own
        const float bv = h2f((uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rb, 2u * (uint32_t)c, 0, 0));
        const int iw0 = owg * VI;                  // first input column of the vector; the window starts at iw0 - 1
        const uint32_t plane = 2u * nc * (uint32_t)(p.H * p.W);      // byte offset of the (n, c) plane
        // Every load of the item is issued before the first is used: the rows as range-checked buffer
        // loads (a row outside the image, or an item past the end: an out-of-range offset, which reads
        // zero), and the two halo pixels that the neighbouring lanes cannot supply (first and last lane
        // of the wave) the same way.  A branch around each load would make each a round trip of its own.
        // Two-pixel vectors at stride 1 (rows of 6, 10, 14 ... pixels): the window of a row is 4 pixels,
        // 8 bytes, and one load at a 2-byte aligned address brings all of it, halo included -- no
        // exchange between lanes, no separate halo loads.  The first group of a row loads from its own
        // first pixel and shifts one pixel up (the left halo is padding), the last loads one pixel
        // earlier and shifts down (the right halo is padding), so every load stays inside its row.
        constexpr bool kWide = (VI == 2 && STRIDE == 1);
        uint32_t raw[RI][kWide ? 2 : (VI >= 2 ? VI / 2 : 1)];
        uint32_t edge_l[RI], edge_r[RI];
        const bool first = owg == 0, last = owg == (int)GW - 1;
#pragma unroll
        for (int rr = 0; rr < RI; ++rr) {
            const int ih = oh0 * STRIDE - 1 + rr;
            const bool row_ok = live && ih >= 0 && ih < p.H;
            const uint32_t at = plane + 2u * (uint32_t)(ih * p.W + iw0);
            const uint32_t off = row_ok ? at : kNone;
            if constexpr (kWide) {
                const dw_u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rx, row_ok ? at - (first ? 0u : last ? 4u : 2u) : kNone, 0, 0);
                raw[rr][0] = v.x; raw[rr][1] = v.y;
                edge_l[rr] = edge_r[rr] = 0u;
            } else {
            if constexpr (VI == 8) {
                const dw_u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rx, off, 0, 0);
                raw[rr][0] = v.x; raw[rr][1] = v.y; raw[rr][2] = v.z; raw[rr][3] = v.w;
            } else if constexpr (VI == 4) {
                const dw_u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rx, off, 0, 0);
                raw[rr][0] = v.x; raw[rr][1] = v.y;
            } else if constexpr (VI == 2) {
                raw[rr][0] = __builtin_amdgcn_raw_buffer_load_b32(rx, off, 0, 0);
            } else {
                raw[rr][0] = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rx, off, 0, 0);
            }
            edge_l[rr] = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rx, (row_ok && lane == 0 && owg != 0) ? at - 2u : kNone, 0, 0);
            edge_r[rr] = STRIDE == 1
                ? (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rx, (row_ok && lane == 63 && owg != (int)GW - 1) ? at + 2u * VI : kNone, 0, 0)
                : 0u;
            }
        }
        float acc[RO][VO];
#pragma unroll
        for (int o = 0; o < RO; ++o)
#pragma unroll
            for (int j = 0; j < VO; ++j) acc[o][j] = bv;
#pragma unroll
        for (int rr = 0; rr < RI; ++rr) {
            float in[VI + 2];                      // columns iw0-1 .. iw0+VI
            if constexpr (kWide) {
                uint64_t v = ((uint64_t)raw[rr][1] << 32) | raw[rr][0];
                v = first ? (v << 16) : last ? (v >> 16) : v;
#pragma unroll
                for (int j = 0; j < 4; ++j) in[j] = h2f((uint16_t)(v >> (16 * j)));
            } else {
#pragma unroll
            for (int j = 0; j < VI; ++j) in[j + 1] = h2f((uint16_t)(raw[rr][j >> 1] >> (16 * (j & 1))));
            // halo columns: the neighbour lane holds the adjacent vector of the same row
            float left = __shfl_up(in[VI], 1);
            float right = __shfl_down(in[1], 1);
            // selects, not branches: a load that is used only inside a branch is moved there
            // and waited for on the spot, with every other load of the item
            const float el = h2f((uint16_t)edge_l[rr]), er = h2f((uint16_t)edge_r[rr]);
            left = lane == 0 ? el : left;
            left = owg == 0 ? 0.0f : left;         // padding column
            if (STRIDE == 1) {
                right = lane == 63 ? er : right;
                right = owg == (int)GW - 1 ? 0.0f : right;
            }
            in[0] = left;
            in[VI + 1] = right;
            }
            // input row rr is tap row kr of output row o when rr = o*STRIDE + kr
#pragma unroll
            for (int kr = 0; kr < 3; ++kr) {
                if (rr - kr < 0 || (rr - kr) % STRIDE != 0 || (rr - kr) / STRIDE >= RO) continue;
                const int o = (rr - kr) / STRIDE;
#pragma unroll
                for (int j = 0; j < VO; ++j)
#pragma unroll
                    for (int q = 0; q < 3; ++q)
                        acc[o][j] = fmaf(wr[kr * 3 + q], in[j * STRIDE + q], acc[o][j]);
            }
        }
        if (live) {
#pragma unroll
            for (int o = 0; o < RO; ++o) {
                if (oh0 + o >= p.Ho) continue;
                ho ov;
#pragma unroll
                for (int j = 0; j < VO; ++j) ov[j] = f2h(p.relu ? fmaxf(acc[o][j], 0.0f) : acc[o][j]);
                *reinterpret_cast<ho *>(p.y + ((size_t)nc * p.Ho + oh0 + o) * p.Wo + owg * VO) = ov;
            }
        }
    }
}

constexpr long long kDwSmallGrid = 256;

template <int STRIDE, int VO, int RO>
static hipError_t launch_dw3_rows(const ConvArgs &a, hipStream_t stream)
{
    const long long items = (long long)a.N * a.C * ((a.Ho + RO - 1) / RO) * (a.Wo / VO);
    long long blocks = (items + 255) / 256;
    if (blocks > 1048576) blocks = 1048576;
    ConvArgs b = a;                                // item index -> (plane, row group, column group), channel of a plane
    b.fd_tiles_w = make_fastdiv((uint32_t)(a.Wo / VO));
    b.fd_tiles_h = make_fastdiv((uint32_t)((a.Ho + RO - 1) / RO));
    b.fd_G = make_fastdiv((uint32_t)a.C);
    hipLaunchKernelGGL((depthwise3_vec_kernel<STRIDE, VO, RO>), dim3((unsigned)blocks), dim3(256), 0, stream, b);
    return hipGetLastError();
}

template <int STRIDE, int VO>
static hipError_t launch_dw3(const ConvArgs &a, hipStream_t stream)
{
    constexpr int RO = (VO >= 8) ? 2 : (VO >= 4 ? 4 : 8);   // output rows per thread: narrow vectors (small maps) take more rows
    // ... unless that leaves most compute units without a workgroup: then two rows per thread
    const long long items = (long long)a.N * a.C * ((a.Ho + RO - 1) / RO) * (a.Wo / VO);
    if (RO > 2 && items < 256 * kDwSmallGrid) return launch_dw3_rows<STRIDE, VO, 2>(a, stream);
    return launch_dw3_rows<STRIDE, VO, RO>(a, stream);
}

hipError_t launch_depthwise(const ConvArgs &a, hipStream_t stream)
{
    // vector form: 3x3, pad 1, stride 1 or 2, rows that split into aligned vectors
    if (a.ks == 3 && a.pad == 1 && (a.stride == 1 || a.stride == 2) && (a.stride == 1 || a.W % 2 == 0)) {
        const uintptr_t xa = (uintptr_t)a.x, ya = (uintptr_t)a.y;
        int vi = 8;                                 // input pixels per load
        while (vi > a.stride && (a.W % vi || xa % (2 * vi) || a.Wo % (vi / a.stride) || ya % (2 * vi / a.stride)))
            vi >>= 1;
        if (a.W % vi == 0 && xa % (2 * vi) == 0 && a.Wo % (vi / a.stride) == 0 && ya % (2 * vi / a.stride) == 0) {
            if (a.stride == 1) {
                if (vi == 8) return launch_dw3<1, 8>(a, stream);
                if (vi == 4) return launch_dw3<1, 4>(a, stream);
                if (vi == 2 && a.W >= 4) return launch_dw3<1, 2>(a, stream);   // its window loads span 4 pixels of a row
                return launch_dw3<1, 1>(a, stream);
            }
            if (vi == 8) return launch_dw3<2, 4>(a, stream);
            if (vi == 4) return launch_dw3<2, 2>(a, stream);
            if (vi == 2) return launch_dw3<2, 1>(a, stream);
        }
    }
    const int chunks = (a.Ho * a.Wo + 255) / 256;
    long long blocks = (long long)a.N * a.C * chunks;
    if (blocks > 1048576) blocks = 1048576;
    if (a.ks == 3)
        hipLaunchKernelGGL(depthwise_kernel<3>, dim3((unsigned)blocks), dim3(256), 0, stream, a);
    else if (a.ks == 5)
        hipLaunchKernelGGL(depthwise_kernel<5>, dim3((unsigned)blocks), dim3(256), 0, stream, a);
    else
        return launch_direct(a, stream);
    return hipGetLastError();
}

// Sum the FP32 slices of a split reduction in slice order (deterministic), then
// bias, ReLU and the one rounding to FP16.  The job is tiny and latency-bound: a thread
// owns V consecutive outputs and has the loads of S slices in flight at once (the
// additions still happen in slice order).  No load sits behind a branch, which would
// give it a wait of its own: past the last slice the last one is read again and a zero
// is added instead.
template <int V, int S>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const ConvArgs p)
{
    typedef float fvec __attribute__((ext_vector_type(V)));
    const long long total = (long long)p.N * p.M * p.Ho * p.Wo;
    const int HoWo = p.Ho * p.Wo;
    const long long o = ((long long)blockIdx.x * 256 + threadIdx.x) * V;
    if (o >= total) return;
    const fvec *src = reinterpret_cast<const fvec *>(p.ws + o);
    const size_t stride = (size_t)total / V;      // total % V == 0 (checked by the launcher)
    const int last = p.split_k - 1;
    // V consecutive outputs lie in one channel's plane when HoWo % V == 0 (checked by the launcher).
    // The bias is fetched with the slices (from the workspace, ignored, when there is none).
    const uint32_t m = ((uint32_t)o / (uint32_t)HoWo) % (uint32_t)p.M;
    const uint16_t bias_raw = *(p.bias ? p.b + m : reinterpret_cast<const uint16_t *>(p.ws));
    float acc[V];
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] = 0.0f;
    for (int k0 = 0; k0 < p.split_k; k0 += S) {
        fvec part[S];
#pragma unroll
        for (int k = 0; k < S; ++k) part[k] = src[(size_t)min(k0 + k, last) * stride];
#pragma unroll
        for (int k = 0; k < S; ++k) {
            const bool live = k0 + k <= last;
#pragma unroll
            for (int v = 0; v < V; ++v) {
                const float t = V == 1 ? ((const float *)&part[k])[0] : part[k][v];
                acc[v] += live ? t : 0.0f;
            }
        }
    }
    const float bias = p.bias ? h2f(bias_raw) : 0.0f;
    uint16_t out[V];
#pragma unroll
    for (int v = 0; v < V; ++v) {
        float r = acc[v] + bias;
        if (p.relu) r = fmaxf(r, 0.0f);
        out[v] = f2h(r);
    }
    if (V == 4) {
        *reinterpret_cast<uint2 *>(p.y + o) = make_uint2(out[0] | ((uint32_t)out[1 % V] << 16),
                                                         out[2 % V] | ((uint32_t)out[3 % V] << 16));
    } else {
#pragma unroll
        for (int v = 0; v < V; ++v) p.y[o + v] = out[v];
    }
}

template <int V>
static void launch_splitk_reduce_v(const ConvArgs &a, long long blocks, hipStream_t stream)
{
    if (a.split_k <= 2)
        hipLaunchKernelGGL((splitk_reduce_kernel<V, 2>), dim3((unsigned)blocks), dim3(256), 0, stream, a);
    else if (a.split_k <= 4)
        hipLaunchKernelGGL((splitk_reduce_kernel<V, 4>), dim3((unsigned)blocks), dim3(256), 0, stream, a);
    else
        hipLaunchKernelGGL((splitk_reduce_kernel<V, 8>), dim3((unsigned)blocks), dim3(256), 0, stream, a);
}

hipError_t launch_splitk_reduce(const ConvArgs &a, hipStream_t stream)
{
    const long long total = (long long)a.N * a.M * a.Ho * a.Wo;
    const bool vec = ((a.Ho * a.Wo) % 4 == 0) && (((uintptr_t)a.ws & 15) == 0) && (((uintptr_t)a.y & 7) == 0);
    if (vec)
        launch_splitk_reduce_v<4>(a, (total / 4 + 255) / 256, stream);
    else
        launch_splitk_reduce_v<1>(a, (total + 255) / 256, stream);
    return hipGetLastError();
}

}  // namespace hgc
