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

hipError_t launch_depthwise(const ConvArgs &a, hipStream_t stream)
{
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
// bias, ReLU and the one rounding to FP16.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const ConvArgs p)
{
    const long long total = (long long)p.N * p.M * p.Ho * p.Wo;
    const int HoWo = p.Ho * p.Wo;
    for (long long o = (long long)blockIdx.x * 256 + threadIdx.x; o < total;
         o += (long long)gridDim.x * 256) {
        float acc = 0.0f;
        for (int k = 0; k < p.split_k; ++k) acc += p.ws[(size_t)k * total + o];
        const int m = (int)((o / HoWo) % p.M);
        if (p.bias) acc += h2f(p.b[m]);
        if (p.relu) acc = fmaxf(acc, 0.0f);
        p.y[o] = f2h(acc);
    }
}

hipError_t launch_splitk_reduce(const ConvArgs &a, hipStream_t stream)
{
    const long long total = (long long)a.N * a.M * a.Ho * a.Wo;
    long long blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, a);
    return hipGetLastError();
}

}  // namespace hgc
