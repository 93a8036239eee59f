/*
 * hgc -- FP16 convolution-layer forward pass for AMD MI355X (gfx950), C ABI.
 *
 * The operation is the convolution layer the paper's engine inherits from BVLC
 * Caffe (Section 2 "Modified from Caffe"; Section 5: same layers, same weight
 * layout), run in half precision on the GPU (Section 1, feature "half precision
 * for all layers"), forward only (feature "forward only mode"):
 *
 *   y[n][m][oh][ow] = act( b[m] + sum_{c<C/group, r<kernel, q<kernel}
 *        w[m][c][r][q] * x[n][g*(C/group) + c][oh*stride - pad + r][ow*stride - pad + q] )
 *
 *   g  = m / (num_output/group)            group of output channel m
 *   Ho = floor((H + 2*pad - kernel)/stride) + 1,  Wo likewise
 *   taps outside the image contribute zero; act = max(.,0) if relu else identity.
 *
 * It is a cross-correlation (no kernel flip).  Products are FP16 x FP16, sums are
 * kept in FP32 (Section 3.1: overflow and underflow arise during accumulation),
 * and the result is rounded to FP16 once, at the store.
 *
 * Boundary rules taken from the paper:
 *   - scalars are ordinary host scalars, tensors are half: the descriptor holds
 *     int32 values in host memory, callers never convert them (Section 3.2);
 *   - tensors, weights included, arrive in FP16 and are used as they are: there
 *     is no float<->half conversion on the path (Section 3.3).
 *
 * All tensors are dense, row-major FP16 in DEVICE memory of the GPU the stream
 * belongs to:  x[N][C][H][W], w[num_output][C/group][kernel][kernel],
 * b[num_output], y[N][num_output][Ho][Wo].  Base pointers need 2-byte alignment
 * only; 16-byte aligned bases (any allocator gives them) enable the fast paths.
 *
 * Ownership: the caller owns every buffer.  The library never allocates, frees,
 * copies to the host or synchronises; each call only enqueues kernels on
 * `stream` and returns (one documented exception: hgc_conv2d_tune).  x, w, b are read-only; every element of y is written
 * exactly once; y must not overlap x, w, b or the workspace.  The descriptor is
 * read during the call only.  Calls are thread-safe.
 */
#ifndef HGC_H
#define HGC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hgc_conv2d_desc {
    int32_t N, C, H, W;     /* input x: [N][C][H][W]                                   */
    int32_t num_output;     /* M; w: [M][C/group][kernel][kernel]                      */
    int32_t kernel;         /* square kernel extent, >= 1                              */
    int32_t stride;         /* >= 1, both axes                                         */
    int32_t pad;            /* >= 0, zeros, symmetric, both axes                       */
    int32_t group;          /* >= 1; C % group == 0 and num_output % group == 0        */
    int32_t bias;           /* 0 or 1; b may be NULL iff 0                             */
    int32_t relu;           /* 0 or 1; fused max(.,0) after the bias                   */
} hgc_conv2d_desc;

typedef int32_t hgc_status;
#define HGC_OK              0
#define HGC_ERR_NULL       (-1)  /* a required pointer is NULL                          */
#define HGC_ERR_BAD_DESC   (-2)  /* a field out of range, or the output would be empty  */
#define HGC_ERR_TOO_LARGE  (-3)  /* a tensor has more than 2^31 - 1 elements            */
#define HGC_ERR_WORKSPACE  (-4)  /* workspace NULL or smaller than required             */
#define HGC_ERR_LAUNCH     (-5)  /* the HIP runtime refused a launch                    */
#define HGC_ERR_ALIGNMENT  (-6)  /* a packed weight buffer is not 256-byte aligned      */

/* Algorithms (hgc_plan.path). */
#define HGC_PATH_AUTO       0    /* only as an argument of hgc_set_forced_path          */
#define HGC_PATH_DIRECT     1    /* one thread per output, FP32 FMA; any descriptor     */
#define HGC_PATH_IGEMM      2    /* implicit GEMM on FP16 MFMA, input halo tile in LDS  */
#define HGC_PATH_IGEMM_SPLITK 3  /* the same with the reduction split over workgroups;
                                    FP32 partial sums in the workspace + a reduce kernel */
#define HGC_PATH_DEPTHWISE  4    /* group == C == num_output streaming kernel           */
#define HGC_PATH_FIRST_LAYER 5   /* C <= 4, one group, kernel 3/5/7, packed weights: MFMA
                                    with horizontal tap pairs folded into the reduction  */
#define HGC_PATH_POINTWISE  6    /* kernel 1, stride 1, pad 0, one group, C % 32 == 0, H*W % 4 == 0,
                                    16-byte aligned tensors: GEMM over the pixels of all images */

/* What a call will do for a descriptor; filled by hgc_conv2d_plan. */
typedef struct hgc_plan {
    int32_t path;            /* HGC_PATH_*                                              */
    int32_t Ho, Wo;          /* output extent                                           */
    int32_t tile_m;          /* output channels per workgroup                           */
    int32_t tile_h, tile_w;  /* output pixels per workgroup and image: tile_h rows x tile_w
                                cols (1x1 stride-1 unpadded layers: of the image seen as
                                one row of H*W pixels; HGC_PATH_POINTWISE: tile_w pixels
                                of all images' pixels taken as one axis)                */
    int32_t split_k;         /* >= 1; number of reduction slices                        */
    int32_t variant;         /* kernel instantiation index (diagnostic)                 */
    int32_t grid;            /* workgroups of the main kernel                           */
    int32_t block;           /* threads per workgroup                                   */
    int64_t workspace_bytes; /* scratch the path needs (0 unless split_k > 1)           */
    int64_t lds_bytes;       /* LDS per workgroup                                       */
    int32_t tile_n;          /* images per workgroup (small feature maps share a tile)  */
    int32_t reserved;
} hgc_plan;

/*
 * Convolution forward, workspace-free algorithms only (operation: header comment).
 * desc: host. x, w, b, y: device. stream: a hipStream_t (NULL = default stream).
 * Errors, checked in this order and before any GPU work: HGC_ERR_NULL (desc, x, w
 * or y NULL; b NULL with bias = 1), HGC_ERR_BAD_DESC, HGC_ERR_TOO_LARGE; then
 * HGC_ERR_LAUNCH if the runtime rejects a launch.  On error nothing is enqueued.
 */
hgc_status hgc_conv2d_forward(const hgc_conv2d_desc *desc, const void *x, const void *w,
                              const void *b, void *y, void *stream);

/*
 * The same operation with a caller-owned device scratch buffer, which allows the
 * split-reduction algorithm for layers with few output pixels (the accumulation
 * stays in FP32 across slices, Section 3.1).  workspace_bytes must be at least
 * what hgc_conv2d_workspace_size reports (else HGC_ERR_WORKSPACE, checked after
 * the descriptor); workspace may be NULL when that is 0.  The workspace content
 * is undefined afterwards.  Results are deterministic for a given descriptor.
 */
hgc_status hgc_conv2d_forward_ws(const hgc_conv2d_desc *desc, const void *x, const void *w,
                                 const void *b, void *y, void *workspace,
                                 size_t workspace_bytes, void *stream);

/*
 * Scratch bytes hgc_conv2d_forward_ws wants for this descriptor (may be 0).
 * Host-only: touches no GPU.  Errors: HGC_ERR_NULL, HGC_ERR_BAD_DESC, HGC_ERR_TOO_LARGE.
 */
hgc_status hgc_conv2d_workspace_size(const hgc_conv2d_desc *desc, size_t *bytes_out);

/*
 * The algorithm and launch shape a call would use (16-byte aligned tensors assumed; a
 * shape remembered by hgc_conv2d_tune is reported).  with_workspace = 0 describes
 * hgc_conv2d_forward, 1 hgc_conv2d_forward_ws, 3 hgc_conv2d_forward_packed.  Host-only.
 */
hgc_status hgc_conv2d_plan(const hgc_conv2d_desc *desc, int32_t with_workspace, hgc_plan *plan_out);

/*
 * One-time weight re-layout.  The engine the paper describes converts weights once,
 * offline, so that no conversion work is left on the inference path (Section 3.3:
 * FP16 weight files and the model converter); hgc_conv2d_pack_weights applies the
 * same rule to the weight LAYOUT: it copies w into a device buffer that holds the
 * weights verbatim plus a copy ordered the way the MFMA kernels consume them
 * (16-byte units [group][8-row block][8-channel plane][tap][row] of 8 channels, zero
 * filled past num_output/group and C/group).  Pure data movement, bit-exact.
 *
 * hgc_conv2d_packed_weights_size: bytes of that buffer for a descriptor (host-only).
 * hgc_conv2d_pack_weights: enqueue the re-layout of w (device, caller's layout)
 *   into w_packed (device, 256-byte aligned, caller-owned, at least the size above).
 * hgc_conv2d_forward_packed: hgc_conv2d_forward_ws with w_packed in place of w; the
 *   descriptor must be the one the buffer was packed for.  Same results up to the
 *   stated tolerance, same error order; additionally HGC_ERR_ALIGNMENT.
 */
hgc_status hgc_conv2d_packed_weights_size(const hgc_conv2d_desc *desc, size_t *bytes_out);
hgc_status hgc_conv2d_pack_weights(const hgc_conv2d_desc *desc, const void *w, void *w_packed, void *stream);
hgc_status hgc_conv2d_forward_packed(const hgc_conv2d_desc *desc, const void *x, const void *w_packed,
                                     const void *b, void *y, void *workspace, size_t workspace_bytes,
                                     void *stream);

/*
 * Set-up-time measurement of the launch shape, the counterpart of packing the weights
 * once: work done before inference so that none of it is left on the path (Section 3.3).
 * Runs the implicit-GEMM launch shapes that the cost model ranks near its own choice on
 * the caller's buffers, a few launches each, and remembers the fastest for later calls of
 * hgc_conv2d_forward_ws (packed = 0) or hgc_conv2d_forward_packed (packed = 1, w = the
 * packed buffer) with the same descriptor and tensor alignment in this process; a later
 * call that brings a smaller workspace than the remembered shape needs falls back to the
 * model's choice.  Unlike every other call this one creates and destroys two events and
 * WAITS for the stream.  y and the workspace are overwritten; on return y holds the
 * layer's output.  chosen_out (may be NULL) receives the shape now in effect.  Same
 * errors, in the same order, as the forward call it tunes.  Descriptors that do not take
 * the implicit-GEMM path have nothing to measure: the layer is enqueued once as planned.  hgc_conv2d_tune_reset forgets every
 * remembered shape.  Both are thread-safe.
 */
hgc_status hgc_conv2d_tune(const hgc_conv2d_desc *desc, const void *x, const void *w, const void *b, void *y,
                           void *workspace, size_t workspace_bytes, int32_t packed, void *stream,
                           hgc_plan *chosen_out);
void hgc_conv2d_tune_reset(void);

/*
 * Restores a launch shape found earlier (hgc_plan.variant, log2 of hgc_plan.tile_w, log2 of
 * hgc_plan.tile_n, hgc_plan.split_k as reported by hgc_conv2d_tune), so that a process need not measure
 * again: remembered for calls with 16-byte aligned tensors like a shape that
 * hgc_conv2d_tune found.  Host-only.  HGC_ERR_BAD_DESC if the descriptor is invalid or the
 * shape is not one of its implicit-GEMM launch shapes.
 */
hgc_status hgc_conv2d_set_launch_shape(const hgc_conv2d_desc *desc, int32_t packed, int32_t variant,
                                       int32_t log2_tile_w, int32_t log2_tile_n, int32_t split_k);

/*
 * Test/diagnostic control: force one algorithm (HGC_PATH_*) for every later call
 * in this process where it applies, or HGC_PATH_AUTO to restore the heuristic.
 * A forced path that cannot run a descriptor falls back to HGC_PATH_DIRECT.
 * tile_variant >= 0 additionally forces the implicit-GEMM instantiation; -1 = automatic.
 * Returns the previous forced path.
 */
int32_t hgc_set_forced_path(int32_t path, int32_t tile_variant);

/*
 * Test/diagnostic control for the implicit-GEMM path: force the output window
 * width (tile_w = 2^log2_tile_w), the number of reduction slices and the images per
 * workgroup (tile_n = 2^log2_tile_n); -1 = automatic.
 * Combinations that do not fit are ignored (the planner then finds no candidate
 * and the call falls back to HGC_PATH_DIRECT).
 */
void hgc_set_forced_tiling(int32_t log2_tile_w, int32_t split_k, int32_t log2_tile_n);

/*
 * Inner-product (fully connected) layer forward, the other layer the paper names as
 * accumulating many values (Section 3.1), with the same rules as the convolution: FP16
 * tensors used as they are, FP32 accumulation, one rounding to FP16 at the store,
 * optional fused bias and ReLU:
 *
 *   y[n][m] = act( b[m] + sum_{k<K} w[m][k] * x[n][k] )
 *
 * x[N][K] (an image's values in memory order: a [N][C][H][W] tensor with K = C*H*W can be
 * passed as it is), w[num_output][K] (Caffe's layout), b[num_output], y[N][num_output]:
 * dense row-major FP16 in device memory, caller-owned; y must not overlap the inputs.
 * desc: host.  Enqueues on `stream` and returns; no workspace.  Errors, in this order and
 * before any GPU work: HGC_ERR_NULL (desc, x, w or y NULL; b NULL with bias = 1),
 * HGC_ERR_BAD_DESC (N, K or num_output < 1; bias or relu not 0/1), HGC_ERR_TOO_LARGE (a
 * tensor with more than 2^31 - 1 elements); then HGC_ERR_LAUNCH.  Results are
 * deterministic.  Bases need 2-byte alignment; 16-byte aligned bases with K % 8 == 0
 * take the fast path.
 */
typedef struct hgc_inner_product_desc {
    int32_t N;              /* images                                                   */
    int32_t K;              /* inputs per image                                         */
    int32_t num_output;     /* M                                                        */
    int32_t bias;           /* 0 or 1; b may be NULL iff 0                              */
    int32_t relu;           /* 0 or 1                                                   */
} hgc_inner_product_desc;
hgc_status hgc_inner_product_forward(const hgc_inner_product_desc *desc, const void *x, const void *w,
                                     const void *b, void *y, void *stream);

/*
 * Batch-norm layer forward (BVLC Caffe's layer as the paper keeps it, Sections 2 and 5,
 * optionally followed by Caffe's per-channel scale layer and a ReLU), the layer whose FP16
 * accumulations Section 3.1 discusses:
 *
 *   mean[c] = (1/L) sum_{n,h,w} x[n][c][h][w],   L = N*H*W
 *   var[c]  = (1/L) sum_{n,h,w} (x[n][c][h][w] - mean[c])^2            (biased)
 *   y[n][c][h][w] = act( gamma[c] * (x[n][c][h][w] - mean[c]) / sqrt(var[c] + eps) + beta[c] )
 *
 * The mean is formed the way Section 3.1 describes, as the mean of the means of groups (a
 * group is a run of at most 2048 consecutive values of one image's channel; groups are
 * weighted by their lengths so that the result is the mean itself), and each group's squared
 * deviations are taken from its own mean, then combined.  Accumulation is FP32 within a
 * group and FP64 across groups, so the power-of-two scaling that Section 3.1 puts around the
 * squares, which is exact in FP32, is not applied.  x is read twice and y written once.
 *
 * x, y: dense FP16 [N][C][H][W] in device memory, caller-owned; y may be x itself (in
 * place) and must not overlap it otherwise.  Per-channel arrays are FP32 [C] in device
 * memory (the paper keeps scalars in float, Section 3.2):
 *   use_global_stats = 0: statistics of this batch.  mean and var are outputs and may each be
 *     NULL; they receive the batch mean and the biased variance.
 *   use_global_stats = 1: mean and var are inputs (required); the layer uses
 *     stat_scale * mean[c] and stat_scale * var[c] (Caffe stores running sums and the
 *     reciprocal of stat_scale beside them; pass 1 for plain statistics).
 *   scale_bias = 1: gamma and beta are required; 0: they are ignored (1 and 0).
 * workspace: device memory of at least hgc_batch_norm_workspace_size bytes, any alignment,
 * caller-owned, free to reuse once the call's work has run.  desc: host.  Enqueues on
 * `stream` and returns.  Errors, in this order and before any GPU work: HGC_ERR_NULL (desc,
 * x or y NULL; a required array NULL), HGC_ERR_BAD_DESC (a dimension < 1; a flag not 0/1;
 * eps not a positive finite number; with use_global_stats = 1, stat_scale not a positive
 * finite number), HGC_ERR_TOO_LARGE (more than 2^31 - 1 elements), HGC_ERR_WORKSPACE; then
 * HGC_ERR_LAUNCH.  Results are deterministic.  Bases need 2-byte alignment; 16-byte
 * aligned bases with H*W % 8 == 0 take the widest loads.
 */
typedef struct hgc_batch_norm_desc {
    int32_t N, C, H, W;
    int32_t use_global_stats;   /* 0: statistics of this batch; 1: mean/var given            */
    int32_t scale_bias;         /* 0 or 1: gamma/beta given                                  */
    int32_t relu;               /* 0 or 1                                                    */
    float   eps;                /* > 0; Caffe's default is 1e-5                              */
    float   stat_scale;         /* use_global_stats = 1 only                                 */
} hgc_batch_norm_desc;
hgc_status hgc_batch_norm_workspace_size(const hgc_batch_norm_desc *desc, size_t *bytes);
hgc_status hgc_batch_norm_forward(const hgc_batch_norm_desc *desc, const void *x, float *mean, float *var,
                                  const float *gamma, const float *beta, void *y, void *workspace,
                                  size_t workspace_bytes, void *stream);

/*
 * Stored batch-norm statistics (and the scale layer) folded into the convolution in front of
 * them, once, before inference: the pattern of Section 3.3, where conversion work is paid
 * offline and none is left on the path.  With a[m] = gamma[m] / sqrt(stat_scale*var[m] + eps):
 *
 *   w_out[m][c][r][q] = a[m] * w[m][c][r][q]
 *   b_out[m]          = a[m] * (b[m] - stat_scale*mean[m]) + beta[m]
 *
 * so that the convolution with (w_out, b_out) and bias = 1 computes batch norm after the
 * convolution with (w, b), ReLU included if the folded layer's descriptor asks for it, at the
 * cost of one more FP16 rounding per weight.  conv: the convolution's descriptor (host; N, H, W,
 * stride, pad and relu are not used).  w, w_out: [num_output][C/group][kernel][kernel] FP16;
 * b (NULL iff conv->bias = 0, read as zero), b_out: [num_output] FP16; mean, var: FP32
 * [num_output]; gamma, beta: FP32 [num_output], both or neither (1 and 0); all in device memory,
 * caller-owned; w_out may be w and b_out may be b.  FP64 arithmetic, one rounding per value.
 * Enqueues on `stream` and returns.  Errors, in this order: HGC_ERR_NULL, HGC_ERR_BAD_DESC (C,
 * num_output, kernel or group < 1 or not divisible; bias not 0/1; eps or stat_scale not a
 * positive finite number), HGC_ERR_TOO_LARGE; then HGC_ERR_LAUNCH.
 */
hgc_status hgc_batch_norm_fold(const hgc_conv2d_desc *conv, const void *w, const void *b, const float *mean,
                               const float *var, float stat_scale, float eps, const float *gamma,
                               const float *beta, void *w_out, void *b_out, void *stream);

/*
 * Max-pooling layer forward: BVLC Caffe's MAX pooling, which sits between the convolutions of
 * the networks the paper runs (Section 4; the paper keeps Caffe's layers, Sections 2 and 5).
 * Square window `kernel`, stride, symmetric padding pad < kernel:
 *
 *   Ho = ceil((H + 2*pad - kernel) / stride) + 1, one less if pad > 0 and the last window
 *        would start at or beyond H + pad; Wo likewise (hgc_max_pool_output_size)
 *   y[n][c][oh][ow] = maximum of x[n][c] over the window at (oh*stride - pad, ow*stride - pad),
 *        clipped to the image: padding never takes part, the last window may hang over the edge
 *
 * x [N][C][H][W], y [N][C][Ho][Wo]: dense FP16 in device memory, caller-owned, not overlapping.
 * The result is one of the inputs, bit for bit (for +0 against -0: either); inputs are finite.
 * desc: host.  Enqueues on `stream` and returns; no workspace.  Errors, in this order and before
 * any GPU work: HGC_ERR_NULL, HGC_ERR_BAD_DESC (a dimension, kernel or stride < 1; pad < 0 or
 * pad >= kernel; a padded extent smaller than the window), HGC_ERR_TOO_LARGE (more than
 * 2^31 - 1 elements); then HGC_ERR_LAUNCH.  Bases need 2-byte alignment; the 2x2 / stride 2 /
 * pad 0 window with W % 8 == 0, a 16-byte aligned x and an 8-byte aligned y takes vector loads.
 */
typedef struct hgc_max_pool_desc {
    int32_t N, C, H, W;
    int32_t kernel, stride, pad;
} hgc_max_pool_desc;
hgc_status hgc_max_pool_output_size(const hgc_max_pool_desc *desc, int32_t *Ho, int32_t *Wo);
hgc_status hgc_max_pool_forward(const hgc_max_pool_desc *desc, const void *x, void *y, void *stream);

/* Static, NUL-terminated description of a status code. */
const char *hgc_status_string(hgc_status status);

/*
 * Runtime's description of the error behind the calling thread's most recent
 * HGC_ERR_LAUNCH ("no error" text if the last launch succeeded). Static string.
 */
const char *hgc_last_launch_error(void);

/*
 * Diagnostic: writes the template-argument prefix of implicit-GEMM instantiation
 * `variant` (hgc_plan.variant; packed = 1 for hgc_conv2d_forward_packed's table) as a
 * profiler prints it, e.g. "igemm_kernel<3, 1, 1, 1, 4, 4, 4, true, true, 2, 1, 0".
 * Returns the length, or -1 for a bad index or buffer.
 */
int32_t hgc_igemm_variant_name(int32_t packed, int32_t variant, char *buf, int32_t buf_len);

/* Library version: major * 10000 + minor * 100 + patch. */
int32_t hgc_version(void);

#ifdef __cplusplus
}
#endif
#endif /* HGC_H */
