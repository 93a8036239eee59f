// Inner-product (fully connected) layer forward in FP16 for gfx950:
//   y[n][m] = act( b[m] + sum_{k<K} w[m][k] * x[n][k] ),  x [N][K], w [M][K], y [N][M].
// The paper names this layer as one where FP16 accumulation overflows (Section 3.1), so
// products are accumulated in FP32 and the result is rounded to FP16 once, at the store;
// weights are used as they arrive, no conversion pass (Section 3.3).
//
// At the batch sizes of inference the layer is bound by reading w once from HBM (2*M*K
// bytes against 2*N*M*K FLOP), so this is a streaming kernel, not a GEMM: a wave owns R
// rows of w and NB images; its 64 lanes walk K in 16-byte steps (one fully coalesced 1 KiB
// segment of a row per instruction), multiply with v_dot2_f32_f16 (FP32 accumulate) and
// reduce across the lanes at the end.  Rows of x are re-read by every wave; they stay
// in L2.  That form serves up to 8 images; from 4 images on (long layers) or 9 (all), the layer goes
// to the matrix cores (inner_product_mfma_kernel below), 32 images a pass.
#include "hgc_internal.h"

#include <atomic>

namespace hgc {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct IpArgs {
    const uint16_t *x, *w, *b;
    uint16_t *y;
    int N, K, M, n0, bias, relu;
    uint32_t x_bytes, w_bytes;
};

__device__ __forceinline__ float dot2(uint32_t a, uint32_t c, float acc)
{
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, a), __builtin_bit_cast(half2_t, c), acc, false);
}

__device__ __forceinline__ float dot8(const u32x4 a, const u32x4 c, float acc)
{
    acc = dot2(a.x, c.x, acc);
    acc = dot2(a.y, c.y, acc);
    acc = dot2(a.z, c.z, acc);
    return dot2(a.w, c.w, acc);
}

// NB images per pass, R rows per wave.  VEC: K % 8 == 0 and 16-byte aligned bases (16-byte
// loads), else element loads.
template <int NB, int R, bool VEC>
__global__ __launch_bounds__(256) void inner_product_kernel(const IpArgs p)
{
    const int lane = threadIdx.x & 63;
    const int wave = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int m0 = wave * R;
    if (m0 >= p.M) return;
    const int K = p.K;
    float acc[R][NB];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int i = 0; i < NB; ++i) acc[r][i] = 0.0f;
    // the rows' bias, fetched ahead of the reduction (range-checked: zero without a bias or past M);
    // loaded in the epilogue it would be a round trip of its own at the end of every wave
    const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(p.bias ? p.b : p.w), 0, p.bias ? 2 * p.M : 0, 0x00020000);
    float bias_row[R];
#pragma unroll
    for (int r = 0; r < R; ++r)
        bias_row[r] = (float)__builtin_bit_cast(
            _Float16, (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rb, m0 + r < p.M ? 2u * (uint32_t)(m0 + r) : 0xFFFFFFFFu, 0, 0));

    if (VEC) {
        // buffer loads: rows past M and images past N use an out-of-range offset and read zero
        const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(p.x), 0, p.x_bytes, 0x00020000);
        const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(p.w), 0, p.w_bytes, 0x00020000);
        uint32_t wo[R], xo[NB];
#pragma unroll
        for (int r = 0; r < R; ++r) wo[r] = (m0 + r < p.M) ? 2u * (uint32_t)((m0 + r) * K) : 0xFFFFFFFFu;
#pragma unroll
        for (int i = 0; i < NB; ++i) xo[i] = (p.n0 + i < p.N) ? 2u * (uint32_t)((p.n0 + i) * K) : 0xFFFFFFFFu;
        // the same number of iterations for every lane; a lane past the end of the row reads zeros
        const int iters = (K + 511) / 512;
#pragma unroll 2
        for (int it = 0; it < iters; ++it) {
            const int k = it * 512 + lane * 8;
            const bool in_row = k < K;
            const uint32_t ko = 2u * (uint32_t)k;
            u32x4 wv[R], xv[NB];
#pragma unroll
            for (int r = 0; r < R; ++r)
                wv[r] = __builtin_amdgcn_raw_buffer_load_b128(rw, (in_row && wo[r] != 0xFFFFFFFFu) ? wo[r] + ko : 0xFFFFFFFFu, 0, 0);
#pragma unroll
            for (int i = 0; i < NB; ++i)
                xv[i] = __builtin_amdgcn_raw_buffer_load_b128(rx, (in_row && xo[i] != 0xFFFFFFFFu) ? xo[i] + ko : 0xFFFFFFFFu, 0, 0);
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int i = 0; i < NB; ++i) acc[r][i] = dot8(wv[r], xv[i], acc[r][i]);
        }
    } else {
        for (int k = lane; k < K; k += 64) {
            float wv[R], xv[NB];
#pragma unroll
            for (int r = 0; r < R; ++r)
                wv[r] = (m0 + r < p.M) ? (float)__builtin_bit_cast(_Float16, p.w[(size_t)(m0 + r) * K + k]) : 0.0f;
#pragma unroll
            for (int i = 0; i < NB; ++i)
                xv[i] = (p.n0 + i < p.N) ? (float)__builtin_bit_cast(_Float16, p.x[(size_t)(p.n0 + i) * K + k]) : 0.0f;
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int i = 0; i < NB; ++i) acc[r][i] = fmaf(wv[r], xv[i], acc[r][i]);
        }
    }
    // sum over the 64 lanes (fixed butterfly order: results are deterministic)
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            float v = acc[r][i];
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
            acc[r][i] = v;
        }
    if (lane == 0) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int m = m0 + r;
            if (m >= p.M) continue;
            const float bv = bias_row[r];
#pragma unroll
            for (int i = 0; i < NB; ++i) {
                const int n = p.n0 + i;
                if (n >= p.N) continue;
                float v = acc[r][i] + bv;
                if (p.relu) v = fmaxf(v, 0.0f);
                p.y[(size_t)n * p.M + m] = __builtin_bit_cast(uint16_t, (_Float16)v);
            }
        }
    }
}

// Batches above eight images: the layer becomes a real contraction (every weight meets 9 or more
// images), so it goes to the matrix cores while staying a weight-streaming kernel.  A workgroup of
// 16 waves owns 16 rows of w and up to 32 images; its waves split K in 64-value blocks (wave i
// takes blocks i, i + 16, ...), each multiplies its blocks with v_mfma_f32_16x16x32_f16 (rows of w
// as the A operand, images as the B operand: a lane of either operand holds 8 consecutive k of one
// row, so w[M][K] and x[N][K] need no transposition of k), and the 16 partial tiles are added in
// wave order through LDS (deterministic).  4096 rows make 256 workgroups, one per compute unit.
// The operands want one row per lane, which read straight from memory costs an instruction that
// touches 32 cache lines; measured, that form was bound by the address path (time proportional
// to the number of load instructions, 3.9 TB/s at best).  So a wave loads its block of both
// operands in the coalesced order (8 lanes per 128-byte row segment, 8 rows an instruction), passes
// it through a private piece of LDS (rows 144 bytes apart: conflict-free for the operand reads) and
// reads the operands from there; the next block's loads are in flight meanwhile.  The order in which
// k is walked inside a block is free as long as both operands agree: lane group q of the
// instruction takes the 16 values from 16 q on, in two steps of 8.
typedef _Float16 ip_h8 __attribute__((ext_vector_type(8)));
typedef float ip_f4 __attribute__((ext_vector_type(4)));

constexpr int kIpRowBytes = 144;                   // 64 halves + 16 bytes of padding

template <int NF>
constexpr int ip_mfma_lds_bytes() { return 16 * (16 + 16 * NF) * kIpRowBytes; }

template <int NF>   // NF = 1: up to 16 images a pass, 2: up to 32
__global__ __launch_bounds__(1024) void inner_product_mfma_kernel(const IpArgs p)
{
    extern __shared__ u32x4 ip_lds[];
    constexpr int ROWS = 16 + 16 * NF;             // of a wave's piece: 16 rows of w, then the images
    constexpr int J = 2 + 2 * NF;                  // load instructions per block
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l16 = lane & 15, lq = lane >> 4;     // operand view: row / image, k group
    const int lr = lane >> 3, lp = lane & 7;       // load view: row within 8, 16-byte piece of the segment
    const int m0 = blockIdx.x * 16;
    const int K = p.K;
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(p.x), 0, p.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(p.w), 0, p.w_bytes, 0x00020000);
    char *mine = reinterpret_cast<char *>(ip_lds) + wave * (ROWS * kIpRowBytes);
    // rows past M and images past N use an out-of-range offset and read zero
    uint32_t go[J];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int m = m0 + 8 * i + lr;
        go[i] = (m < p.M) ? 2u * (uint32_t)(m * K) + 16u * (uint32_t)lp : 0xFFFFFFFFu;
    }
#pragma unroll
    for (int j = 2; j < J; ++j) {
        const int n = p.n0 + 8 * (j - 2) + lr;
        go[j] = (n < p.N) ? 2u * (uint32_t)(n * K) + 16u * (uint32_t)lp : 0xFFFFFFFFu;
    }
    u32x4 *put = reinterpret_cast<u32x4 *>(mine + lr * kIpRowBytes + 16 * lp);              // + 8 rows per instruction
    const u32x4 *get_a = reinterpret_cast<const u32x4 *>(mine + l16 * kIpRowBytes + 32 * lq);
    const u32x4 *get_b = reinterpret_cast<const u32x4 *>(mine + (16 + l16) * kIpRowBytes + 32 * lq);

    ip_f4 acc[NF];
#pragma unroll
    for (int f = 0; f < NF; ++f) acc[f] = ip_f4{0.0f, 0.0f, 0.0f, 0.0f};
    const int blocks = (K + 63) / 64;
    u32x4 cur[J], nxt[J];
    auto fetch = [&](u32x4 *dst, int kb) {
        const int k = kb * 64 + 8 * lp;
        const bool in_row = k < K;                                // K is a multiple of 8 here
        const uint32_t ko = 128u * (uint32_t)kb;
#pragma unroll
        for (int j = 0; j < J; ++j)
            dst[j] = __builtin_amdgcn_raw_buffer_load_b128(j < 2 ? rw : rx, (in_row && go[j] != 0xFFFFFFFFu) ? go[j] + ko : 0xFFFFFFFFu, 0, 0);
    };
    fetch(cur, wave);
    for (int kb = wave; kb < blocks; kb += 16) {
        if (kb + 16 < blocks) fetch(nxt, kb + 16);
#pragma unroll
        for (int j = 0; j < J; ++j) put[j * (8 * kIpRowBytes / 16)] = cur[j];
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");        // the wave's own writes, before its lanes read each other's
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
            const ip_h8 a = __builtin_bit_cast(ip_h8, get_a[s2]);
#pragma unroll
            for (int f = 0; f < NF; ++f)
                acc[f] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, __builtin_bit_cast(ip_h8, get_b[f * (16 * kIpRowBytes / 16) + s2]),
                                                                acc[f], 0, 0, 0);
        }
        asm volatile("" ::: "memory");                            // the next block's writes stay behind these reads
#pragma unroll
        for (int j = 0; j < J; ++j) cur[j] = nxt[j];
    }
    __syncthreads();                                              // the partial tiles reuse the operand space
    float *red = reinterpret_cast<float *>(ip_lds);               // [wave][f][e][lane]
#pragma unroll
    for (int f = 0; f < NF; ++f) {
        red[((wave * NF + f) * 4 + 0) * 64 + lane] = acc[f].x;
        red[((wave * NF + f) * 4 + 1) * 64 + lane] = acc[f].y;
        red[((wave * NF + f) * 4 + 2) * 64 + lane] = acc[f].z;
        red[((wave * NF + f) * 4 + 3) * 64 + lane] = acc[f].w;
    }
    __syncthreads();
    // element e of lane (l16, lq) of the result tile is row 4 lq + e of the 16 rows, image l16 of the 16
    const int t = threadIdx.x;
    if (t < 256 * NF) {
        const int f = t >> 8, e = (t >> 6) & 3, ln = t & 63;
        float v = 0.0f;
#pragma unroll
        for (int w = 0; w < 16; ++w) v += red[((w * NF + f) * 4 + e) * 64 + ln];
        const int m = m0 + 4 * (ln >> 4) + e;
        const int n = p.n0 + 16 * f + (ln & 15);
        if (m < p.M && n < p.N) {
            if (p.bias) v += (float)__builtin_bit_cast(_Float16, p.b[m]);
            if (p.relu) v = fmaxf(v, 0.0f);
            p.y[(size_t)n * p.M + m] = __builtin_bit_cast(uint16_t, (_Float16)v);
        }
    }
}

template <int NF>
static hipError_t launch_ip_mfma_nf(const IpArgs &a, hipStream_t s)
{
    static std::atomic<bool> granted{false};
    auto kern = inner_product_mfma_kernel<NF>;
    constexpr int lds = ip_mfma_lds_bytes<NF>();
    if (lds > 64 * 1024 && !granted.load(std::memory_order_acquire)) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        granted.store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)((a.M + 15) / 16)), dim3(1024), lds, s, a);
    return hipGetLastError();
}

static hipError_t launch_ip_mfma(const IpArgs &a, int images, hipStream_t s)
{
    return images > 16 ? launch_ip_mfma_nf<2>(a, s) : launch_ip_mfma_nf<1>(a, s);
}

template <int NB, int R, bool VEC>
static hipError_t launch_ip(const IpArgs &a, hipStream_t s)
{
    const int waves = (a.M + R - 1) / R;
    hipLaunchKernelGGL((inner_product_kernel<NB, R, VEC>), dim3((unsigned)((waves + 3) / 4)), dim3(256), 0, s, a);
    return hipGetLastError();
}

template <int NB>
static hipError_t launch_ip_nb(const IpArgs &a, bool vec, int rows, hipStream_t s)
{
    if (vec) return rows == 2 ? launch_ip<NB, 2, true>(a, s) : launch_ip<NB, 1, true>(a, s);
    return launch_ip<NB, 1, false>(a, s);
}

}  // namespace hgc

using namespace hgc;

extern "C" hgc_status hgc_inner_product_forward(const hgc_inner_product_desc *desc, const void *x, const void *w,
                                                const void *b, void *y, void *stream)
{
    if (!desc || !x || !w || !y) return HGC_ERR_NULL;
    if (desc->bias == 1 && !b) return HGC_ERR_NULL;
    if (desc->N < 1 || desc->K < 1 || desc->num_output < 1) return HGC_ERR_BAD_DESC;
    if ((desc->bias != 0 && desc->bias != 1) || (desc->relu != 0 && desc->relu != 1)) return HGC_ERR_BAD_DESC;
    const long long lim = 0x7FFFFFFFLL;
    const long long N = desc->N, K = desc->K, M = desc->num_output;
    if (N * K > lim || M * K > lim || N * M > lim) return HGC_ERR_TOO_LARGE;
    IpArgs a;
    a.x = static_cast<const uint16_t *>(x);
    a.w = static_cast<const uint16_t *>(w);
    a.b = static_cast<const uint16_t *>(b);
    a.y = static_cast<uint16_t *>(y);
    a.N = desc->N; a.K = desc->K; a.M = desc->num_output; a.n0 = 0; a.bias = desc->bias; a.relu = desc->relu;
    a.x_bytes = (uint32_t)(2 * N * K);
    a.w_bytes = (uint32_t)(2 * M * K);
    const bool vec = (K % 8 == 0) && (((uintptr_t)x | (uintptr_t)w) & 15) == 0;
    // two rows per wave once there are enough rows to fill the chip with one-row waves twice over
    const int rows = M >= 2048 ? 2 : 1;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = hipSuccess;
    // measured on VGG-16's fc6/fc7/fc8: the streaming form wins up to 3 images, and up to 8 on short layers
    if (vec && (desc->N > 8 || (desc->N >= 4 && desc->num_output >= 2048))) {
        // matrix cores, passes of 32 images (w is read once per pass)
        for (int n0 = 0; n0 < desc->N && e == hipSuccess; n0 += 32) {
            a.n0 = n0;
            e = launch_ip_mfma(a, desc->N - n0, s);
        }
        set_last_hip_error(e);
        return e == hipSuccess ? HGC_OK : HGC_ERR_LAUNCH;
    }
    for (int n0 = 0; n0 < desc->N && e == hipSuccess; n0 += 8) {
        a.n0 = n0;
        const int nb = desc->N - n0;
        if (nb >= 8) e = launch_ip_nb<8>(a, vec, rows, s);
        else if (nb > 2) e = nb > 4 ? launch_ip_nb<8>(a, vec, rows, s) : launch_ip_nb<4>(a, vec, rows, s);
        else e = nb == 2 ? launch_ip_nb<2>(a, vec, rows, s) : launch_ip_nb<1>(a, vec, rows, s);
    }
    set_last_hip_error(e);
    return e == hipSuccess ? HGC_OK : HGC_ERR_LAUNCH;
}
