/*
 * convnet_hotpath.h -- C ABI of the MI355X (gfx950) convolution hot path.
 *
 * The library computes the three passes of a convolutional layer that dominate
 * a synchronous-SGD training step of the ConvNet studied in "Multi-GPU
 * Training of ConvNets" (arXiv 1312.5853): the forward pass (a layer's filters
 * convolve its input -- model-parallelism paragraph), and the two halves of
 * back-propagation through it (gradients with respect to the layer input and
 * with respect to all filter parameters -- optimisation and data-parallelism
 * paragraphs).  One call handles one GPU's share: a data-parallel mini-batch
 * shard, or one model-parallel column (a subset of filters and channels).
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 *  - Layout: activations NCHW, filters KCRS, dense and contiguous unless a
 *    batch stride is given.  x, dx: [N][C][H][W];  w, dw: [K][C][R][S];
 *    y, dy: [N][K][P][Q] with P = floor((H + 2*pad - R)/stride) + 1 and Q
 *    likewise from W and S.  H and W are ALWAYS the layer's input extent, in all
 *    three passes (with stride > 1 they cannot be recovered from P and Q).
 *    One stride and one symmetric zero padding for both axes; no dilation, no
 *    groups, no bias, no filter flip (cross-correlation).
 *  - All tensor pointers are DEVICE pointers owned by the caller.  The library
 *    never allocates, frees or keeps them.  Scratch memory comes from the `ws`
 *    argument (device pointer, 256-byte aligned, at least
 *    conv_workspace_bytes() bytes); its contents are undefined afterwards.
 *  - Outputs are fully overwritten (no accumulation into the destination, every
 *    element written -- dx positions that no window touches receive 0).
 *  - dtype: CONV_DTYPE_F32  = fp32 tensors, fp32 MFMA arithmetic.
 *           CONV_DTYPE_BF16 = x, w, dy hold bfloat16 (2 bytes, already rounded
 *           by the caller); products accumulate in fp32; outputs (y, dx, dw)
 *           are fp32.
 *           CONV_DTYPE_BF16_OUT_BF16 = as CONV_DTYPE_BF16, but conv_fwd writes y
 *           and conv_bwd_data writes dx as bfloat16, each fp32 sum rounded once
 *           to nearest even, so that activations and gradients chain from layer
 *           to layer without a conversion call.  conv_bwd_filter treats it as
 *           CONV_DTYPE_BF16: dw is always fp32.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Work is enqueued; returning does not imply completion.  Calls on one
 *    stream that share a workspace are ordered by the stream; calls on
 *    different streams must not share a workspace.
 *  - Results are bit-for-bit reproducible from run to run (fixed reduction
 *    order, no floating-point atomics).
 *  - Return value: CONV_OK or a negative conv_status.  All argument checks run
 *    on the host before any GPU call; nothing is enqueued when a call fails a
 *    check.  No C++ exception crosses this boundary.
 *  - Limits: every tensor (including batch-strided spans) must occupy fewer
 *    than 2^31 bytes; tensor base pointers must be 16-byte aligned.
 */
#ifndef CONVNET_HOTPATH_H
#define CONVNET_HOTPATH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum conv_status {
    CONV_OK = 0,
    CONV_ERR_INVALID_ARG = -1,         /* null pointer, non-positive extent, stride <= 0, pad < 0, P or Q <= 0,
                                          batch stride smaller than one sample */
    CONV_ERR_TOO_LARGE = -2,           /* a tensor span reaches 2^31 bytes */
    CONV_ERR_BAD_DTYPE = -3,
    CONV_ERR_WORKSPACE_TOO_SMALL = -4, /* ws is NULL or ws_bytes < conv_workspace_bytes() while scratch is needed */
    CONV_ERR_MISALIGNED = -5,          /* tensor base not 16-byte aligned, or ws not 256-byte aligned */
    CONV_ERR_HIP = -6,                 /* the HIP runtime refused a launch; hipGetLastError() text via conv_last_hip_error() */
    CONV_ERR_SCRATCH_LIMIT = -7        /* conv_bwd_filter_noalloc: the pass needs more than CONV_NOALLOC_SCRATCH_BYTES */
} conv_status;

enum { CONV_DTYPE_F32 = 0, CONV_DTYPE_BF16 = 1, CONV_DTYPE_BF16_OUT_BF16 = 2 };
enum { CONV_OP_FWD = 0, CONV_OP_BWD_DATA = 1, CONV_OP_BWD_FILTER = 2 };

/*
 * Forward pass of a convolutional layer (the layer's K filters convolve its
 * input; model-parallelism paragraph):
 *   y[n,k,p,q] = sum_{c,r,s} x[n,c,p*stride-pad+r,q*stride-pad+s] * w[k,c,r,s]
 * with x read as zero outside its extent.
 *   x  in   device, [N][C][H][W]
 *   w  in   device, [K][C][R][S]
 *   y  out  device, [N][K][P][Q], fp32
 */
int conv_fwd(const void *x, const void *w, void *y,
             int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
             int dtype, void *ws, size_t ws_bytes, void *stream);

/*
 * Backward-data pass (back-propagation of the error to the layer input;
 * optimisation paragraph):
 *   dx[n,c,h,w] = sum over (k,p,q,r,s) with p*stride-pad+r = h and
 *                 q*stride-pad+s = w of dy[n,k,p,q] * w[k,c,r,s]
 *   dy in   device, [N][K][P][Q]
 *   w  in   device, [K][C][R][S]
 *   dx out  device, [N][C][H][W], fp32
 */
int conv_bwd_data(const void *dy, const void *w, void *dx,
                  int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                  int dtype, void *ws, size_t ws_bytes, void *stream);

/*
 * Backward-filter pass (gradient with respect to all filter parameters from
 * this GPU's subset of the samples; data-parallelism paragraph):
 *   dw[k,c,r,s] = sum_{n,p,q} dy[n,k,p,q] * x[n,c,p*stride-pad+r,q*stride-pad+s]
 *   x  in   device, [N][C][H][W]
 *   dy in   device, [N][K][P][Q]
 *   dw out  device, [K][C][R][S], fp32 (this shard's sum; adding the shards of
 *           a data-parallel step is the caller's all-reduce)
 */
int conv_bwd_filter(const void *x, const void *dy, void *dw,
                    int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                    int dtype, void *ws, size_t ws_bytes, void *stream);

/*
 * conv_bwd_filter for callers that cannot allocate and have no workspace to
 * pass: code under HIP graph capture, tight training or serving loops, harnesses
 * that forbid hipMalloc.  Same arithmetic, kernels, layouts and results (bit for
 * bit) as conv_bwd_filter with dense tensors; the scratch (tap table, partial
 * sums of the split reduction, packed bf16 copies) lives in a static device
 * array of CONV_NOALLOC_SCRATCH_BYTES inside the library, of which every GPU the
 * library runs on holds one copy until the process ends.  The call allocates
 * and frees nothing, on the device or through any library.
 *   - A pass whose conv_workspace_bytes(CONV_OP_BWD_FILTER, ...) exceeds
 *     CONV_NOALLOC_SCRATCH_BYTES returns CONV_ERR_SCRATCH_LIMIT before anything
 *     is enqueued.  fp32: the partial sums do not grow with N (at most 36 MB,
 *     the first layer's 256 partial results), and all five layers of the stack
 *     fit at any batch size.  bf16: the packed copies grow with N (the third
 *     layer needs 31 MB at N = 16, 46 MB at N = 64).
 *   - All calls on one GPU share that GPU's array: calls that overlap in time
 *     on one GPU (different streams or threads) race.  Calls on one stream are
 *     ordered.  The array keeps the previous call's contents; every call
 *     overwrites what it reads, nothing has to start at zero.
 *   - The first call on a device looks the array's address up
 *     (hipGetSymbolAddress); make that call before a stream capture begins.
 */
#define CONV_NOALLOC_SCRATCH_BYTES (48u << 20)
int conv_bwd_filter_noalloc(const void *x, const void *dy, void *dw,
                            int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                            int dtype, void *stream);

/*
 * Batch-strided variants: sample n of the activation tensor on the layer's
 * input side (x / dx) starts x_batch_stride ELEMENTS after sample n-1, and
 * likewise y_batch_stride for the output side (y / dy); within a sample the
 * [channel][row][col] block is dense.  They let one model-parallel column read
 * and write a channel slice of a wider NCHW tensor in place (the two-column
 * architecture of the model-parallelism paragraph).  Strides must be at least
 * one sample (C*H*W resp. K*P*Q); 0 means dense.
 */
int conv_fwd_ex(const void *x, const void *w, void *y,
                int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                int64_t x_batch_stride, int64_t y_batch_stride,
                int dtype, void *ws, size_t ws_bytes, void *stream);
int conv_bwd_data_ex(const void *dy, const void *w, void *dx,
                     int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                     int64_t x_batch_stride, int64_t y_batch_stride,
                     int dtype, void *ws, size_t ws_bytes, void *stream);
int conv_bwd_filter_ex(const void *x, const void *dy, void *dw,
                       int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                       int64_t x_batch_stride, int64_t y_batch_stride,
                       int dtype, void *ws, size_t ws_bytes, void *stream);

/*
 * Grouped (multi-column) layers: the two-column architecture of the
 * model-parallelism paragraph, where a column's filters read only the
 * column's own input channels (no cross-connection).  C and K are the TOTAL
 * channel and filter counts, both multiples of `groups`; column g owns input
 * channels g*C/groups .. and filters g*K/groups ..:
 *   x, dx  [N][C][H][W]      w, dw  [K][C/groups][R][S]      y, dy  [N][K][P][Q]
 * Each column is the corresponding ordinary pass on its channel slice; all
 * conventions above apply (dense tensors here).  With fp32 tensors and channel
 * counts per column that are multiples of 16 the columns share one launch;
 * otherwise they run one after the other on the stream (then every column's
 * slice must itself start 16-byte aligned: CONV_ERR_MISALIGNED if not).
 * groups = 1 is the ordinary layer.
 */
int conv_fwd_grouped(const void *x, const void *w, void *y,
                     int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int groups,
                     int dtype, void *ws, size_t ws_bytes, void *stream);
int conv_bwd_data_grouped(const void *dy, const void *w, void *dx,
                          int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int groups,
                          int dtype, void *ws, size_t ws_bytes, void *stream);
int conv_bwd_filter_grouped(const void *x, const void *dy, void *dw,
                            int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int groups,
                            int dtype, void *ws, size_t ws_bytes, void *stream);
size_t conv_workspace_bytes_grouped(int op, int N, int C, int H, int W, int K, int R, int S,
                                    int stride, int pad, int groups, int dtype);

/*
 * Convolution passes with the element-wise layer that follows them applied
 * where the sums are stored, so that the activation layer makes no pass of its
 * own over HBM (conv3 and conv4 of the stack are followed by a ReLU without
 * pooling; bias and ReLU belong to the Krizhevsky architecture the paper
 * trains).  Dense tensors, one column; workspace as for conv_fwd /
 * conv_bwd_data with the same extents.
 *   conv_fwd_bias_relu: y = f(conv_fwd(x, w) + bias[k]), f = max(., 0) if relu = 1,
 *       identity if relu = 0; bias is fp32 [K] on the device or NULL (no bias).
 *       The bias is added to the fp32 sum before any rounding to bfloat16.
 *   conv_bwd_data_relu: dx = conv_bwd_data(dy, w) where act > 0, else 0: the
 *       gradient with respect to the INPUT of the ReLU whose output (or input)
 *       act [N][C][H][W] is; act has the element type of dx and is only read.
 * Both give exactly what the separate calls give for fp32 outputs; for bfloat16
 * outputs the fused result is rounded once, after the bias.
 */
int conv_fwd_bias_relu(const void *x, const void *w, const void *bias, void *y,
                       int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int relu,
                       int dtype, void *ws, size_t ws_bytes, void *stream);
int conv_bwd_data_relu(const void *dy, const void *w, const void *act, void *dx,
                       int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                       int dtype, void *ws, size_t ws_bytes, void *stream);

/*
 * Scratch bytes the given pass needs for these extents (op = CONV_OP_*).
 * Pure host arithmetic; returns 0 for invalid arguments.  The figure depends
 * only on the arguments, never on the device or on earlier calls.
 */
size_t conv_workspace_bytes(int op, int N, int C, int H, int W, int K, int R, int S,
                            int stride, int pad, int dtype);

/*
 * Output extent of one axis, floor((in + 2*pad - filt) / stride) + 1: the P (from H, R) and Q (from W, S) every
 * entry point derives, for callers that size y / dy.  0 when no window fits or an argument is not positive
 * (pad may be 0).
 */
int conv_output_extent(int in, int filt, int stride, int pad);

/* Static, NUL-terminated description of a conv_status value. */
const char *conv_status_string(int status);

/* Text of the HIP error behind the calling thread's last CONV_ERR_HIP ("" if none). */
const char *conv_last_hip_error(void);

/*
 * Glue layers between the convolutions of the five-layer stack (they belong to
 * the Krizhevsky architecture the paper trains; the paper's text does not
 * spell them out).  Device pointers, fully overwritten outputs, same stream and
 * error conventions as above.  `dtype` names the element type of ALL tensors of
 * the call: CONV_DTYPE_F32 = fp32 (4-byte aligned); CONV_DTYPE_BF16 or
 * CONV_DTYPE_BF16_OUT_BF16 = bfloat16 (2-byte aligned): values are read exactly,
 * arithmetic is fp32, and a result that is not itself an input value (the sum of
 * up to four gradients in the pooling backward) is rounded once to nearest even.
 *
 *   relu_fwd:  y[i]  = x[i] > 0 ? x[i] : 0                     (y may alias x)
 *   relu_bwd:  dx[i] = x[i] > 0 ? dy[i] : 0   (x = forward input or output; dx may alias dy)
 *   maxpool3x3s2_fwd: per plane, y[i,j] = max of the 3x3 window at (2i, 2j); no padding;
 *                     output extent floor((H-3)/2)+1 per axis; `planes` = N*C.
 *   maxpool3x3s2_bwd: dx = 0, then every dy[i,j] is added to the window element the
 *                     forward pass selected (first maximum in row-major window order);
 *                     overlapping windows accumulate in a fixed order.
 */
int relu_fwd(const void *x, void *y, int64_t count, int dtype, void *stream);
int relu_bwd(const void *x, const void *dy, void *dx, int64_t count, int dtype, void *stream);
int maxpool3x3s2_fwd(const void *x, void *y, int64_t planes, int H, int W, int dtype, void *stream);
int maxpool3x3s2_bwd(const void *x, const void *dy, void *dx, int64_t planes, int H, int W, int dtype, void *stream);

/*
 * ReLU followed by the pooling above, fused (the conv1/conv2/conv5 tail of the
 * stack), so that the activation never makes a pass of its own over HBM.
 *   relu_maxpool3x3s2_fwd: y = maxpool3x3s2(relu(x)); x is the convolution
 *       output and is left untouched.
 *   relu_maxpool3x3s2_bwd: dx = relu_bwd(x, maxpool3x3s2_bwd(relu(x), dy)), the
 *       gradient with respect to the convolution output x, from x itself.
 * Both give exactly what the separate calls give.
 */
int relu_maxpool3x3s2_fwd(const void *x, void *y, int64_t planes, int H, int W, int dtype, void *stream);
int relu_maxpool3x3s2_bwd(const void *x, const void *dy, void *dx, int64_t planes, int H, int W, int dtype,
                          void *stream);

/*
 * Bias of a convolutional layer: one fp32 value per filter.
 *   bias_fwd: y[n][k][:] += b[k], in place on y [N][K][PQ] (dtype = element type
 *             of y as for the glue layers; b is always fp32).
 *   bias_bwd: db[k] = sum over n and positions of dy[n][k][:], fp32, summed in a
 *             fixed order; needs bias_bwd_workspace_bytes(N, K) bytes of scratch
 *             (256-byte aligned).  N*K*PQ must stay below 2^31.
 */
int bias_fwd(void *y, const void *b, int N, int K, int PQ, int dtype, void *stream);
int bias_bwd(const void *dy, void *db, int N, int K, int PQ, int dtype, void *ws, size_t ws_bytes, void *stream);
size_t bias_bwd_workspace_bytes(int N, int K);

/*
 * fp32 -> bfloat16 with round-to-nearest-even, for callers that hold fp32 data
 * (network input, filters after an fp32 update, fp32 results of CONV_DTYPE_BF16
 * passes) and feed bf16 layers.  dst holds `count` 2-byte values; device pointers.
 */
int convert_f32_to_bf16(const void *src, void *dst, int64_t count, void *stream);

/*
 * Fully connected layers (the top layers of the network, where the columns of
 * the model-parallel architecture are cross-connected; model-parallelism
 * paragraph).  Row-major fp32 device tensors: x, dx [N][I] (a sample per row),
 * w, dw [O][I] (an output neuron per row), y, dy [N][O].
 *   fc_fwd:        y[n][o]  = f(sum_i x[n][i] * w[o][i] + bias[o]); bias fp32 [O] or
 *                  NULL; f = max(., 0) if relu = 1, identity if relu = 0
 *   fc_bwd_data:   dx[n][i] = sum_o dy[n][o] * w[o][i]
 *   fc_bwd_filter: dw[o][i] = sum_n dy[n][o] * x[n][i]   (this shard's sum)
 * Outputs are fully overwritten; sums accumulate in fp32 in a fixed order.
 * I and O must be multiples of 4 (CONV_ERR_INVALID_ARG otherwise), every tensor
 * below 2^31 elements, pointers 16-byte aligned, dtype CONV_DTYPE_F32
 * (CONV_ERR_BAD_DTYPE otherwise).  Scratch: fc_workspace_bytes(op, ...) bytes
 * (op = CONV_OP_*; 0 for invalid arguments), 256-byte aligned.  Stream, ownership
 * and error conventions as for the convolution passes.
 */
int fc_fwd(const void *x, const void *w, const void *bias, void *y, int N, int I, int O, int relu,
           int dtype, void *ws, size_t ws_bytes, void *stream);
int fc_bwd_data(const void *dy, const void *w, void *dx, int N, int I, int O,
                int dtype, void *ws, size_t ws_bytes, void *stream);
int fc_bwd_filter(const void *x, const void *dy, void *dw, int N, int I, int O,
                  int dtype, void *ws, size_t ws_bytes, void *stream);
size_t fc_workspace_bytes(int op, int N, int I, int O, int dtype);

/*
 * One step of synchronous mini-batch stochastic gradient descent (training-
 * procedure paragraph; the paper fixes no hyper-parameters beyond "the same
 * set-up" as the network it trains, whose rule this is), in place on fp32
 * device arrays of `count` parameters:
 *   vel[i] = momentum * vel[i] - lr * (weight_decay * w[i] + grad_scale * dw[i])
 *   w[i]  += vel[i]
 * grad_scale = 1 / mini-batch size turns the summed gradients the backward-
 * filter passes produce into the mean; momentum = weight_decay = 0 is plain
 * SGD (vel then only receives the step).  dw is only read.  4-byte aligned
 * pointers (16-byte aligned ones take the vector path); count = 0 is a no-op.
 */
int sgd_update(void *w, const void *dw, void *vel, int64_t count, float lr, float momentum,
               float weight_decay, float grad_scale, void *stream);

/*
 * The same update (same formula, same training-procedure paragraph) for
 * `ntensors` parameter tensors in one call: w, dw, vel and counts are HOST arrays
 * of `ntensors` device pointers / element counts, read before the call returns.
 * One kernel launch per 24 tensors instead of one per tensor; every parameter
 * gets bit for bit what sgd_update gives it.  Tensors with count 0 are skipped
 * (their pointers may be NULL); the argument checks of sgd_update apply to each
 * tensor, and nothing is launched if one fails.
 */
int sgd_update_multi(void *const *w, const void *const *dw, void *const *vel, const int64_t *counts,
                     int ntensors, float lr, float momentum, float weight_decay, float grad_scale,
                     void *stream);

#ifdef __cplusplus
}
#endif
#endif /* CONVNET_HOTPATH_H */
