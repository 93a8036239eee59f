// 1x1 convolutions (stride 1, no padding, one group) as a plain GEMM on the matrix cores:
//   y[n][m][p] = act( b[m] + sum_c w[m][c] * x[n][c][p] ),   p over the H*W pixels of an image.
// The layer is the paper's convolution (Caffe's, Sections 2 and 5) with k = 1; what makes it
// worth a kernel of its own is its shape: no halo, a short reduction (C = 32 .. 2048) and, in the
// nets built from it, small feature maps (14x14, 7x7) at which a tile cut out of one image is
// mostly ragged.  So the pixels of all images are taken as one axis q = n * P + p, cut in tiles
// of TP pixels regardless of image boundaries (a 4- or 8-pixel chunk never straddles one, since
// P is a multiple of the chunk), and the kernel is a two-stage pipelined GEMM:
//   * A operand (rows of w[M][C], Caffe's layout, 8 consecutive c per lane): staged through LDS
//     with coalesced 16-byte loads, rows 80 bytes apart (conflict-free 16-byte operand reads);
//   * B operand (x[n][c][p], pixels contiguous): staged as it lies in memory, [c][pixels], rows
//     2 TP + 64 bytes apart, and read with ds_read_b64_tr_b16, which hands each lane the four
//     k-consecutive values of its pixel column: no transposition pass anywhere;
//   * 32 channels a stage, the loads of the next four stages in flight in registers (a stage is
//     only 2 MFMA steps of work, a trip to memory takes many times that), two LDS buffers, one
//     barrier a stage;
//   * bias in the accumulators from the start, ReLU, one rounding to FP16, a transposition of each
//     32x32 block through LDS so that a lane stores 8 consecutive pixels of one channel.
// FP32 accumulation, one rounding (Section 3.1); weights are read as they are (Section 3.3).
#include "hgc_internal.h"

namespace hgc {

typedef _Float16 pw_h8 __attribute__((ext_vector_type(8)));
typedef _Float16 pw_h2 __attribute__((ext_vector_type(2)));
typedef float pw_f2 __attribute__((ext_vector_type(2)));
typedef float pw_f16 __attribute__((ext_vector_type(16)));
typedef short pw_s4 __attribute__((ext_vector_type(4)));
typedef uint32_t pw_u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t pw_u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) pw_s4 *pw_lds_s4;

constexpr uint32_t kPwNoLoad = 0xFFFFFFFFu;
constexpr int kPwKC = 32;           // channels a stage
constexpr int kPwWRow = 80;         // bytes between rows of the weight stage (64 of data)

struct PwArgs {
    const uint16_t *x, *w, *b;
    uint16_t *y;
    int C, M, P;                    // channels in, channels out, pixels per image
    uint32_t Q;                     // N * P
    uint32_t x_bytes, w_bytes;
    int tiles_m;
    uint32_t tiles;                 // workgroups with work
    int relu, bias;
    FastDiv fd_P, fd_tiles_m;
};

template <int V> struct PwChunk;
template <> struct PwChunk<8> { typedef pw_u32x4 type; };
template <> struct PwChunk<4> { typedef pw_u32x2 type; };

template <int V>
__device__ __forceinline__ typename PwChunk<V>::type pw_load(const __amdgpu_buffer_rsrc_t r, uint32_t off)
{
    if constexpr (V == 8) return __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 0);
    else return __builtin_amdgcn_raw_buffer_load_b64(r, off, 0, 0);
}

// A, B: 32-row / 32-pixel blocks per wave; the four waves form a 2 x 2 grid, so a workgroup owns
// 64 A output channels x 64 B pixels.  V: pixels per load and store (8, or 4 when P % 8 != 0).
template <int A, int B, int V, int D>
__global__ __launch_bounds__(256, (A * B >= 8 ? 2 : 3)) void pointwise_kernel(const PwArgs p)
{
    constexpr int TM = 64 * A, TP = 64 * B;
    constexpr int SX = 2 * TP + 64;                 // bytes between rows of the input stage
    constexpr int XBYTES = kPwKC * SX, WBYTES = TM * kPwWRow;
    constexpr int CPR = TP / V;                     // chunks per input row
    constexpr int RP = 256 / CPR;                   // input rows per pass of the 256 threads
    constexpr int NXP = kPwKC / RP;                 // passes per stage
    static_assert(256 % CPR == 0 && kPwKC % RP == 0, "stage shape");
    __shared__ __attribute__((aligned(16))) char lds[2 * (XBYTES + WBYTES)];
    typedef typename PwChunk<V>::type chunk_t;

    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, lh = lane >> 5;
    // Workgroups are handed to the eight XCDs in turn, and each XCD has its own L2: the workgroups of one
    // XCD (every eighth of the launch) take consecutive tiles, row tiles fastest, so that the row tiles
    // that share a pixel tile fetch it into one L2, once, instead of into several.
    const uint32_t tile_id = (blockIdx.x & 7u) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    if (tile_id >= p.tiles) return;                                               // the launch is padded to a multiple of 8
    const uint32_t tile_q = fast_div(tile_id, p.fd_tiles_m);
    const int m0 = (int)(tile_id - tile_q * (uint32_t)p.tiles_m) * TM;
    const uint32_t q0 = tile_q * TP;
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(p.x), 0, p.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(p.w), 0, p.w_bytes, 0x00020000);

    // this thread's share of a stage: NXP chunks of one pixel column block, A chunks of weights
    const int cc = t % CPR, xr0 = t / CPR;
    uint32_t xbase;
    {
        const uint32_t q = q0 + (uint32_t)cc * V;
        const uint32_t img = fast_div(q, p.fd_P);
        const uint32_t pp = q - img * (uint32_t)p.P;
        xbase = q < p.Q ? 2u * ((img * (uint32_t)p.C + (uint32_t)xr0) * (uint32_t)p.P + pp) : kPwNoLoad;
    }
    const uint32_t xrow_step = 2u * (uint32_t)RP * (uint32_t)p.P;               // RP channels further
    const uint32_t xstage_step = 2u * (uint32_t)kPwKC * (uint32_t)p.P;
    const int wc = t & 3, wr0 = t >> 2;
    uint32_t wbase[A];
#pragma unroll
    for (int i = 0; i < A; ++i) {
        const int m = m0 + wr0 + 64 * i;
        wbase[i] = m < p.M ? 2u * (uint32_t)(m * p.C) + 16u * (uint32_t)wc : kPwNoLoad;
    }
    char *xput = lds + xr0 * SX + cc * (2 * V);
    char *wput = lds + 2 * XBYTES + wr0 * kPwWRow + 16 * wc;
    // operand addresses within a stage
    const char *aget = lds + 2 * XBYTES + (wm * 32 * A + l32) * kPwWRow + 16 * lh;
    const int gi = lane >> 4, ii = lane & 15;
    const char *bget = lds + (8 * (gi >> 1) + (ii >> 2)) * SX + 2 * (wn * 32 * B + 16 * (gi & 1) + 4 * (ii & 3));

    // bias of the rows this lane's accumulator elements belong to: range-checked loads, all issued before
    // the first is waited for (no bias, or a row past M: an out-of-range offset, which reads zero)
    pw_f16 acc[A][B];
    {
        const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint16_t *>(p.bias ? p.b : p.x), 0, p.bias ? 2u * (uint32_t)p.M : 0u, 0x00020000);
        uint32_t bits[A][16];
#pragma unroll
        for (int i = 0; i < A; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int m = m0 + wm * 32 * A + 32 * i + 8 * (e >> 2) + 4 * lh + (e & 3);
                bits[i][e] = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rb, (p.bias && m < p.M) ? 2u * (uint32_t)m : kPwNoLoad, 0, 0);
            }
#pragma unroll
        for (int i = 0; i < A; ++i) {
            pw_f16 init;
#pragma unroll
            for (int e = 0; e < 16; ++e) init[e] = (float)__builtin_bit_cast(_Float16, (uint16_t)bits[i][e]);
#pragma unroll
            for (int j = 0; j < B; ++j) acc[i][j] = init;
        }
    }

    // Stage j waits in register set j % D from the moment its loads are issued, D stages ahead of its
    // use: one stage is only 2 MFMA steps of work, far less than a trip to memory, so the loads of
    // several stages have to be in flight at once.  D divides the number of stages and the loop is
    // unrolled by D, so the sets are plain registers and the loop body has no branch (the wait before
    // a stage's registers are used then counts exactly the younger loads that may stay in flight).
    // Loads past the last stage use an out-of-range offset; what they bring is never used.
    chunk_t xr[D][NXP];
    pw_u32x4 wr[D][A];
    const int stages = p.C / kPwKC;
    auto fetch = [&](int slot, int s) {
        const bool real = s < stages;
#pragma unroll
        for (int i = 0; i < NXP; ++i)
            xr[slot][i] = pw_load<V>(rx, (real && xbase != kPwNoLoad) ? xbase + (uint32_t)s * xstage_step + (uint32_t)i * xrow_step : kPwNoLoad);
#pragma unroll
        for (int i = 0; i < A; ++i)
            wr[slot][i] = __builtin_amdgcn_raw_buffer_load_b128(rw, (real && wbase[i] != kPwNoLoad) ? wbase[i] + 64u * (uint32_t)s : kPwNoLoad, 0, 0);
    };
    auto put = [&](int slot, int buf) {
#pragma unroll
        for (int i = 0; i < NXP; ++i)
            *reinterpret_cast<chunk_t *>(xput + buf * XBYTES + i * RP * SX) = xr[slot][i];
#pragma unroll
        for (int i = 0; i < A; ++i)
            *reinterpret_cast<pw_u32x4 *>(wput + buf * WBYTES + i * 64 * kPwWRow) = wr[slot][i];
    };

#pragma unroll
    for (int d = 0; d < D; ++d) fetch(d, d);
    put(0, 0);
    fetch(0, D);
    __syncthreads();
    for (int s0 = 0; s0 < stages; s0 += D) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const int s = s0 + d;
            const int buf = (D % 2 == 0) ? (d & 1) : (s & 1);
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                pw_h8 af[A], bf[B];
#pragma unroll
                for (int i = 0; i < A; ++i)
                    af[i] = *reinterpret_cast<const pw_h8 *>(aget + buf * WBYTES + i * 32 * kPwWRow + 32 * ks);
#pragma unroll
                for (int j = 0; j < B; ++j) {
                    const char *at = bget + buf * XBYTES + 16 * ks * SX + 64 * j;
                    const pw_s4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((pw_lds_s4)(at));
                    const pw_s4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((pw_lds_s4)(at + 4 * SX));
                    typedef short pw_s8 __attribute__((ext_vector_type(8)));
                    const pw_s8 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                    bf[j] = __builtin_bit_cast(pw_h8, both);
                }
#pragma unroll
                for (int i = 0; i < A; ++i)
#pragma unroll
                    for (int j = 0; j < B; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[i], bf[j], acc[i][j], 0, 0, 0);
            }
            put((d + 1) % D, buf ^ 1);                   // stage s + 1 (past the end: never read)
            fetch((d + 1) % D, s + 1 + D);               // its set is free again
            __syncthreads();
        }
    }

    // epilogue: per 32 x 32 block, FP16 through a wave-private LDS tile (40 halves a row), then a lane
    // holds 8 consecutive pixels of one channel
    constexpr int EP = 40;
    uint16_t *tile = reinterpret_cast<uint16_t *>(lds) + wave * (32 * EP);
    const _Float16 floor_h = p.relu ? (_Float16)0.0f : (_Float16)(-__builtin_inff());
    const pw_h2 floor2 = {floor_h, floor_h};
    const int row0 = lane >> 2, chunk = lane & 3;
#pragma unroll
    for (int i = 0; i < A; ++i)
#pragma unroll
        for (int j = 0; j < B; ++j) {
#pragma unroll
            for (int e = 0; e < 16; e += 2) {
                const pw_f2 v = {acc[i][j][e], acc[i][j][e + 1]};
                const pw_h2 h = __builtin_elementwise_max(__builtin_convertvector(v, pw_h2), floor2);
                const uint32_t bits = __builtin_bit_cast(uint32_t, h);
                const int r = 8 * (e >> 2) + 4 * lh + (e & 3);
                tile[r * EP + l32] = (uint16_t)bits;
                tile[(r + 1) * EP + l32] = (uint16_t)(bits >> 16);
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");     // the wave's own writes, before its lanes read each other's
            const uint32_t q = q0 + (uint32_t)(wn * 32 * B + 32 * j + 8 * chunk);
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const int r = row0 + 16 * k;
                const int m = m0 + wm * 32 * A + 32 * i + r;
                const pw_u32x4 v = *reinterpret_cast<const pw_u32x4 *>(tile + r * EP + 8 * chunk);
                if (m >= p.M) continue;
                if (V == 8) {
                    if (q < p.Q) {
                        const uint32_t img = fast_div(q, p.fd_P);
                        const uint32_t pp = q - img * (uint32_t)p.P;
                        *reinterpret_cast<pw_u32x4 *>(p.y + ((size_t)img * p.M + m) * p.P + pp) = v;
                    }
                } else {
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const uint32_t qh = q + 4u * h;
                        if (qh < p.Q) {
                            const uint32_t img = fast_div(qh, p.fd_P);
                            const uint32_t pp = qh - img * (uint32_t)p.P;
                            const pw_u32x2 half = {v[2 * h], v[2 * h + 1]};
                            *reinterpret_cast<pw_u32x2 *>(p.y + ((size_t)img * p.M + m) * p.P + pp) = half;
                        }
                    }
                }
            }
            asm volatile("" ::: "memory");                          // the next block's writes stay behind these reads
        }
}

template <int A, int B>
static hipError_t pw_launch(const PwArgs &a, int v, unsigned blocks, hipStream_t s)
{
    // stages in flight: what the registers allow, and a divisor of the number of stages
    constexpr int DMAX = (B >= 4 || A >= 4) ? 2 : 4;
    const int stages = a.C / kPwKC;
    const int d = (stages % 4 == 0 && DMAX >= 4) ? 4 : (stages % 2 == 0 ? 2 : 1);
    if (v == 8) {
        if (d == 4) pointwise_kernel<A, B, 8, DMAX><<<dim3(blocks), dim3(256), 0, s>>>(a);
        else if (d == 2) pointwise_kernel<A, B, 8, 2><<<dim3(blocks), dim3(256), 0, s>>>(a);
        else pointwise_kernel<A, B, 8, 1><<<dim3(blocks), dim3(256), 0, s>>>(a);
    } else {
        if (d == 4) pointwise_kernel<A, B, 4, DMAX><<<dim3(blocks), dim3(256), 0, s>>>(a);
        else if (d == 2) pointwise_kernel<A, B, 4, 2><<<dim3(blocks), dim3(256), 0, s>>>(a);
        else pointwise_kernel<A, B, 4, 1><<<dim3(blocks), dim3(256), 0, s>>>(a);
    }
    return hipGetLastError();
}

// Whether the kernel takes this layer, and with which tile (tile_m = 64 * a, tile_p = 64 * b).
bool pointwise_eligible(const ConvArgs &c, int x_align, int y_align, bool w_al16)
{
    const long long P = (long long)c.H * c.W;
    return c.ks == 1 && c.stride == 1 && c.pad == 0 && c.G == 1 && c.C % kPwKC == 0 && P % 4 == 0 && w_al16 &&
           x_align % 16 == 0 && y_align % 16 == 0 && c.M >= 32;
}

// below this many 128-row x 128-pixel tiles a layer takes 64-row tiles (measured: batch-1 stacks of ResNet-50 and
// MobileNet-v1 shapes 6 % and 10 % faster with 64 and with 160; 256 and 400 cost the large batches 1-2 %)
constexpr long long kPwSmallGrid = 160;
// below this many 64-row x 128-pixel tiles a layer takes 64-pixel tiles (measured: the same batch-1 stacks another 11 %
// faster with 128; 48 gains less, 256 and 512 cost ResNet-50 shapes at batch 32 half a percent)
constexpr long long kPwTinyGrid = 128;

void pointwise_tile(const ConvArgs &c, int *a, int *b)
{
    // the larger tile once it still leaves every compute unit more than one workgroup
    const long long Q = (long long)c.N * c.H * c.W;
    *a = c.M <= 64 ? 1 : 2;                         // 64 rows a workgroup when there are no more
    // ... or when 128-row tiles would leave most compute units without a workgroup
    if (*a == 2 && ((c.M + 127) / 128) * ((Q + 127) / 128) < kPwSmallGrid) *a = 1;
    const long long big = ((c.M + 64 * *a - 1) / (64 * *a)) * ((Q + 255) / 256);
    *b = big >= 512 ? 4 : 2;
    // 64-pixel tiles when even the 64-row x 128-pixel tiles are few
    if (*a == 1 && ((c.M + 63) / 64) * ((Q + 127) / 128) < kPwTinyGrid) *b = 1;
    // 256 rows x 128 pixels re-read x half as often from L2; measured to pay from about 1.5 workgroups per compute unit on
    if (*b == 2 && c.M >= 256 && ((c.M + 255) / 256) * ((Q + 127) / 128) >= 384) *a = 4;
}

hipError_t launch_pointwise(const ConvArgs &c, int a, int b, hipStream_t s)
{
    PwArgs p;
    p.x = c.x; p.w = c.w; p.b = c.b; p.y = c.y;
    p.C = c.C; p.M = c.M; p.P = c.H * c.W;
    p.Q = (uint32_t)((long long)c.N * p.P);
    p.x_bytes = c.x_bytes;
    p.w_bytes = (uint32_t)(2LL * c.M * c.C);
    p.relu = c.relu; p.bias = c.bias;
    const int TM = 64 * a, TP = 64 * b;
    p.tiles_m = (c.M + TM - 1) / TM;
    p.fd_P = make_fastdiv((uint32_t)p.P);
    p.fd_tiles_m = make_fastdiv((uint32_t)p.tiles_m);
    p.tiles = (uint32_t)(p.tiles_m * ((p.Q + TP - 1) / TP));
    const unsigned blocks = (p.tiles + 7u) / 8u * 8u;
    const int v = p.P % 8 == 0 ? 8 : 4;
    if (a == 1) return b == 4 ? pw_launch<1, 4>(p, v, blocks, s) : b == 1 ? pw_launch<1, 1>(p, v, blocks, s) : pw_launch<1, 2>(p, v, blocks, s);
    if (a == 4) return pw_launch<4, 2>(p, v, blocks, s);
    return b == 4 ? pw_launch<2, 4>(p, v, blocks, s) : pw_launch<2, 2>(p, v, blocks, s);
}

}  // namespace hgc
