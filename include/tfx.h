/*
 * tfx.h -- C ABI of the dense-op library for AMD MI355X (gfx950).
 *
 * The ops are the ones that dominate the MobileNet v1 inference timed in
 * Section 3.9 (Table 1) of the TensorFlow.js paper (arxiv 1901.05350):
 * matMul / batchMatMul, conv2d, depthwiseConv2d, with a fused bias + activation
 * epilogue, and the whole MobileNet v1 1.0 / 224 forward pass.
 *
 * Conventions common to every device entry point
 *   - All tensors are float32, dense, row-major.  Images are NHWC (the index
 *     order batch,row,column,depth of the conv2d sampler in Section 4.1), conv
 *     filters are HWIO [fh,fw,inC,outC], depthwise filters are [fh,fw,inC,mult].
 *   - Every data pointer is a DEVICE pointer.  Shape arrays and the weights
 *     struct are HOST memory and are read before the call returns.
 *   - Ownership: the caller owns every buffer.  The library allocates nothing
 *     and frees nothing, and keeps no tensor state between calls.  What it does
 *     keep, per process and per device, are launch attributes it has looked up
 *     once (which kernels were allowed their dynamic LDS size, how many
 *     workgroups of a kernel are resident at once) and, once a forward pass
 *     of 32 or more images has run, two streams and three events of its own (see
 *     tfx_mobilenet_v1_forward); these never change a result.  Inputs are never
 *     written
 *     (ops are functional, Section 3.7); the output must not overlap any input
 *     (overlap is not detected; the result is then undefined).
 *   - Asynchrony: a call validates its arguments on the host, enqueues its
 *     kernels on `stream` (a hipStream_t passed as void*, NULL = the default
 *     stream) and returns without synchronising, like the enqueue-and-return
 *     ops of Section 3.6 / 4.1.  The caller synchronises before reading.
 *     The device that `stream` belongs to must be the calling thread's current
 *     device.  Entry points may be called from several host threads at once
 *     (the caches above are atomics; calls that share an output or workspace
 *     buffer must be ordered by the caller).
 *   - Errors: the return value is a tfx_status.  Validation happens before any
 *     HIP call: a NULL pointer gives TFX_ERR_NULL; non-positive or mismatching
 *     dimensions, or a VALID convolution whose filter exceeds the image, give
 *     TFX_ERR_SHAPE; a stride < 1 or an unknown enum value gives TFX_ERR_ARG;
 *     a tensor of 2^31 or more elements gives TFX_ERR_UNSUPPORTED; a workspace
 *     that is too small or misaligned gives TFX_ERR_WORKSPACE; a failed kernel
 *     enqueue gives TFX_ERR_LAUNCH.  On error nothing has been enqueued, except
 *     for TFX_ERR_LAUNCH (earlier kernels of the same call may have been).
 *   - Zero-sized tensors are rejected with TFX_ERR_SHAPE.
 */
#ifndef TFX_H_
#define TFX_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  TFX_OK = 0,
  TFX_ERR_NULL = -1,
  TFX_ERR_SHAPE = -2,
  TFX_ERR_ARG = -3,
  TFX_ERR_UNSUPPORTED = -4,
  TFX_ERR_WORKSPACE = -5,
  TFX_ERR_LAUNCH = -6
} tfx_status;

typedef enum { TFX_PAD_VALID = 0, TFX_PAD_SAME = 1 } tfx_padding;
typedef enum { TFX_ACT_NONE = 0, TFX_ACT_RELU = 1, TFX_ACT_RELU6 = 2 } tfx_activation;

/* Human-readable name of a status code (static string, never NULL). */
const char* tfx_status_string(int status);

/* ------------------------------------------------------------------------- *
 * Host-only shape rules (no GPU needed, no HIP call made).
 *
 * The paper defines no padding rule; its API is modelled after TensorFlow
 * (Section 3.1), so per spatial dimension (in = input extent, k = filter
 * extent, s = stride):
 *   VALID: out = floor((in - k) / s) + 1, no padding, in < k is TFX_ERR_SHAPE;
 *   SAME : out = ceil(in / s), pad_total = max((out - 1) * s + k - in, 0),
 *          pad_before = floor(pad_total / 2), pad_after = pad_total - pad_before
 *          (the odd unit goes to the bottom / right).
 * pad_tblr receives top, bottom, left, right.
 * ------------------------------------------------------------------------- */

/* Output shape [M,N] of op(a) x op(b); a_shape / b_shape are the stored shapes.
 * M = ta ? a[1] : a[0], K = ta ? a[0] : a[1], N = tb ? b[0] : b[1]; the two K must agree. */
int tfx_matmul_out_shape(const int64_t a_shape[2], const int64_t b_shape[2],
                         int transpose_a, int transpose_b, int64_t out_shape[2]);

/* x_shape [N,H,W,inC], f_shape [fh,fw,inC,outC] -> out_shape [N,oh,ow,outC]. */
int tfx_conv2d_out_shape(const int64_t x_shape[4], const int64_t f_shape[4],
                         int stride_h, int stride_w, tfx_padding pad,
                         int64_t out_shape[4], int64_t pad_tblr[4]);

/* x_shape [N,H,W,C], f_shape [fh,fw,C,mult] -> out_shape [N,oh,ow,C*mult]. */
int tfx_depthwise_conv2d_out_shape(const int64_t x_shape[4], const int64_t f_shape[4],
                                   int stride_h, int stride_w, tfx_padding pad,
                                   int64_t out_shape[4], int64_t pad_tblr[4]);

/* ------------------------------------------------------------------------- *
 * Device entry points.
 * ------------------------------------------------------------------------- */

/* matMul (Section 4.1, Listing 2): c[i,j] = sum_k A'(i,k) * B'(k,j) where
 * A'(i,k) = transpose_a ? a[k,i] : a[i,k] and B'(k,j) = transpose_b ? b[j,k] : b[k,j].
 * a, b: device, stored shapes a_shape / b_shape; c: device, [M,N].  Any M,N,K >= 1
 * (the listing's "shared dimension is a multiple of 4" is not required). */
int tfx_matmul(const float* a, const int64_t a_shape[2], const float* b, const int64_t b_shape[2],
               int transpose_a, int transpose_b, float* c, void* stream);

/* batchMatMul: tfx_matmul independently for each leading index.  a_shape and
 * b_shape are [B,rows,cols] with equal B (no broadcasting); c is [B,M,N].
 * The paper defines only the rank-2 product (Listing 2); the batched form follows
 * the library its API is modelled on (Section 3.1): the same product per leading
 * index. */
int tfx_batch_matmul(const float* a, const int64_t a_shape[3], const float* b, const int64_t b_shape[3],
                     int transpose_a, int transpose_b, float* c, void* stream);

/* conv2d (cross-correlation, NHWC x HWIO; index order per Section 4.1) with
 * fused epilogue:
 *   y[n,oh,ow,o] = act( sum_{kh,kw,c} X(n, oh*sh - pt + kh, ow*sw - pl + kw, c) * filter[kh,kw,c,o] + bias[o] )
 * X is 0 outside the image.  bias is a device pointer to [outC] or NULL (= 0).
 * y: device, shape from tfx_conv2d_out_shape.
 * Epilogue, here and in every fused op below: the bias is added first, then the
 * activation: relu(v) = max(v, 0), relu6(v) = min(max(v, 0), 6).  A NaN passes
 * through either activation unchanged, -Inf gives 0, +Inf gives +Inf (relu) or 6
 * (relu6). */
int tfx_conv2d(const float* x, const int64_t x_shape[4], const float* filter, const int64_t f_shape[4],
               const float* bias, int stride_h, int stride_w, tfx_padding pad, tfx_activation act,
               float* y, void* stream);

/* depthwiseConv2d with fused epilogue.  The paper names the op but gives no
 * definition; this is the convention of the library its API is modelled on
 * (Section 3.1), in the index order of the conv2d sampler of Section 4.1:
 *   y[n,oh,ow,c*mult+q] = act( sum_{kh,kw} X(n, oh*sh - pt + kh, ow*sw - pl + kw, c) * filter[kh,kw,c,q]
 *                              + bias[c*mult+q] )
 * bias is a device pointer to [C*mult] or NULL.  y: device, shape from
 * tfx_depthwise_conv2d_out_shape. */
int tfx_depthwise_conv2d(const float* x, const int64_t x_shape[4], const float* filter, const int64_t f_shape[4],
                         const float* bias, int stride_h, int stride_w, tfx_padding pad, tfx_activation act,
                         float* y, void* stream);

/* Element-wise addition (Section 4.1, Fig. 3): c[i] = a[i] + b[i] for 0 <= i < n,
 * one correctly rounded IEEE addition per element.  a, b, c: device, n elements
 * each; c may be the same buffer as a or b (no other overlap).  n = 0 is a no-op;
 * n < 0 is TFX_ERR_SHAPE, n > 2^40 TFX_ERR_UNSUPPORTED. */
int tfx_add(const float* a, const float* b, int64_t n, float* c, void* stream);

/* ------------------------------------------------------------------------- *
 * 16-bit float storage (Section 4.1: the same matMul program renders to a
 * 32-bit or to a 16-bit floating point texture, depending on the device).
 * Tensors are IEEE 754 binary16 bit patterns (uint16_t); arithmetic inside an
 * op is at least fp32 and the result is rounded once, to nearest even, when
 * it is stored.  Results beyond 65504 become infinity.
 * ------------------------------------------------------------------------- */

/* c[i] = half(a[i] + b[i]); otherwise as tfx_add. */
int tfx_add_f16(const uint16_t* a, const uint16_t* b, int64_t n, uint16_t* c, void* stream);

/* batchMatMul on 16-bit storage with the fused epilogue of the fp32 ops:
 *   c[b,i,j] = half( act( sum_k A'(b,i,k) * B'(b,k,j) + bias[j] ) )
 * with A', B', shapes and transposes as tfx_batch_matmul (B = 1 gives matMul; a
 * pointwise convolution is the case a = x viewed as [1, N*H*W, inC],
 * b = filter viewed as [1, inC, outC]).  bias: device [N] binary16 or NULL.
 * The sum is accumulated in fp32 (products of two binary16 values are exact
 * there). */
int tfx_batch_matmul_f16(const uint16_t* a, const int64_t a_shape[3], const uint16_t* b, const int64_t b_shape[3],
                         int transpose_a, int transpose_b, const uint16_t* bias, tfx_activation act,
                         uint16_t* c, void* stream);

/* conv2d and depthwiseConv2d on 16-bit storage: the definitions of tfx_conv2d and
 * tfx_depthwise_conv2d with x, filter, bias and y stored as binary16, the sum
 * accumulated in fp32 and the result rounded once. */
int tfx_conv2d_f16(const uint16_t* x, const int64_t x_shape[4], const uint16_t* filter, const int64_t f_shape[4],
                   const uint16_t* bias, int stride_h, int stride_w, tfx_padding pad, tfx_activation act,
                   uint16_t* y, void* stream);
int tfx_depthwise_conv2d_f16(const uint16_t* x, const int64_t x_shape[4], const uint16_t* filter,
                             const int64_t f_shape[4], const uint16_t* bias, int stride_h, int stride_w,
                             tfx_padding pad, tfx_activation act, uint16_t* y, void* stream);

/* MobileNet v1 1.0 / 224 weights (Section 3.9, Table 1 workload), batch norm
 * already folded into the biases.  The struct lives in host memory; every
 * member is a device pointer owned by the caller.  Block i (0-based) has
 * dw_w[i] [3,3,Cin_i,1], dw_b[i] [Cin_i], pw_w[i] [1,1,Cin_i,Cout_i], pw_b[i] [Cout_i] with
 * Cout = 64,128,128,256,256,512,512,512,512,512,512,1024,1024, Cin_0 = 32,
 * and depthwise stride 2 in blocks 1, 3, 5 and 11, else 1. */
typedef struct {
  const float* conv0_w; /* [3,3,3,32] */
  const float* conv0_b; /* [32] */
  const float* dw_w[13];
  const float* dw_b[13];
  const float* pw_w[13];
  const float* pw_b[13];
  const float* fc_w; /* [1024,1000] */
  const float* fc_b; /* [1000] */
} tfx_mobilenet_v1_weights;

/* Bytes of device workspace tfx_mobilenet_v1_forward needs for `batch` images
 * (0 if batch < 1).  Host-only. */
size_t tfx_mobilenet_v1_workspace_bytes(int64_t batch);

/* Full forward pass: 3x3 stride-2 conv to 32 channels, 13 x (depthwise 3x3 ->
 * pointwise 1x1), bias + ReLU6 after each of the 27 convolutions, SAME padding
 * throughout, global average pool, fully connected 1024 -> 1000, softmax.
 * At batch 1 to 3 the stem and the first block, and each of the next four blocks, are
 * one kernel each.  At batch 1 and full width blocks 2 - 4 share one launch and the
 * blocks from the sixth on, the pool, the fully connected layer and the softmax run
 * as one kernel; the workgroups of these two kernels hand results to each other
 * through flags in the workspace.  Every wait in them is bounded, and if one ever
 * gives up (a workgroup that never got to run) every output of the call is NaN
 * rather than a number computed from unfinished data.
 * input: device [batch,224,224,3]; workspace: device, >= the size above, 256-byte
 * aligned, contents undefined before and after; probs: device [batch,1000];
 * logits: device [batch,1000] or NULL.  All kernels are enqueued on `stream`,
 * with one exception: from batch 32 on the pass runs as two parts of the batch, from
 * batch 60 on as three (each in its own part of the workspace), and all but the first
 * are enqueued on streams the library creates once per device, which wait for
 * everything queued on `stream` before the call (an event) and which `stream` waits
 * for before anything queued after the call: for the caller the call still behaves as work on `stream`, also
 * while `stream` is being captured into a graph (fork and join become edges of the
 * graph).  Independent chains of kernels fill the CUs that the last workgroups of
 * each kernel leave idle (1.03 -> 0.96 ms at batch 64).  If the streams cannot be created
 * (also: if the first such call of the process comes while `stream` is being
 * captured), or if TFX_ONE_STREAM is set in the environment, the batch runs as one
 * chain of kernels on `stream`, as below batch 32; the results then agree with the
 * split form to rounding (other tile shapes), not bit for bit. */
int tfx_mobilenet_v1_forward(const float* input, int64_t batch, const tfx_mobilenet_v1_weights* weights,
                             void* workspace, size_t workspace_bytes, float* probs, float* logits,
                             void* stream);

/* The other members of the MobileNet v1 family (Section 3.9 times the "1.0"
 * member at 224 x 224): same 28 layers, every channel count scaled by
 * alpha = width_quarters / 4 and a square input of image_size pixels.
 *   image_size:     32 ... 256 (the published members use 128, 160, 192, 224)
 *   width_quarters: 1, 2, 3 or 4 (alpha 0.25, 0.5, 0.75, 1.0)
 *   classes:        1 ... 1024 outputs of the fully connected layer
 * Channel counts are alpha * the counts listed above (stem 32 alpha, fully
 * connected input 1024 alpha); the weight struct is the same, with its arrays
 * sized accordingly.  {224, 4, 1000} is tfx_mobilenet_v1_forward. */
typedef struct {
  int64_t image_size;
  int64_t width_quarters;
  int64_t classes;
} tfx_mobilenet_v1_variant;

/* Workspace bytes for `batch` images of a variant; 0 if the variant or batch is
 * invalid.  Host-only. */
size_t tfx_mobilenet_v1_variant_workspace_bytes(const tfx_mobilenet_v1_variant* variant, int64_t batch);

/* As tfx_mobilenet_v1_forward for a variant: input device
 * [batch,image_size,image_size,3], probs (and logits, if not NULL) device
 * [batch,classes].  TFX_ERR_ARG for a variant outside the ranges above. */
int tfx_mobilenet_v1_variant_forward(const tfx_mobilenet_v1_variant* variant, const float* input, int64_t batch,
                                     const tfx_mobilenet_v1_weights* weights, void* workspace,
                                     size_t workspace_bytes, float* probs, float* logits, void* stream);

/* An internal activation of the network (Section 5.2 offers the hosted models to
 * transfer learning, which trains a small model on such an activation): the
 * output of depthwise-separable block `end_block` (1 ... 13, after its pointwise
 * layer's bias + ReLU6), [batch, h, w, c] NHWC.  tfx_mobilenet_v1_variant_features_shape
 * writes that shape (host-only): h = w = the image size halved by the stem and by each
 * stride-2 block up to end_block (rounded up), c = alpha * that block's pointwise width.
 * The layers up to that block run exactly as in tfx_mobilenet_v1_variant_forward (the
 * batch-1 kernel that chains the last blocks is not used) and nothing after it runs.
 * features: device, 16-byte aligned, written by the last kernel.  (Blocks 2 - 4 of the
 * batch-1 full-width network run as stages of one launch whose workgroups wait for each
 * other, every wait bounded: a stage that gives up writes NaN, which the later layers
 * carry along, so an element of `features` is then NaN rather than a wrong number.)  weights: the whole
 * struct must be filled in.  workspace as for the forward pass.  TFX_ERR_ARG for an
 * end_block outside 1 ... 13 or a misaligned features pointer; other errors as the
 * forward pass. */
int tfx_mobilenet_v1_variant_features_shape(const tfx_mobilenet_v1_variant* variant, int64_t batch, int end_block,
                                            int64_t shape[4]);
int tfx_mobilenet_v1_variant_features(const tfx_mobilenet_v1_variant* variant, const float* input, int64_t batch,
                                      const tfx_mobilenet_v1_weights* weights, void* workspace,
                                      size_t workspace_bytes, int end_block, float* features, void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): tfx_mobilenet_v1_variant_forward with
 * the workspace inside the library, a fixed array of
 * tfx_mobilenet_v1_static_scratch_bytes() = 16 MiB of device memory that every GPU the
 * library runs on holds until the process ends, from the moment the runtime loads the
 * library's device code there (at the latest during the first call of this entry point
 * on that GPU, which also looks up the array's device address once).  The call
 * allocates and frees nothing.  {224, 4, 1000} fits at batch 1 and 2; a variant / batch whose
 * tfx_mobilenet_v1_variant_workspace_bytes exceeds the array is refused with
 * TFX_ERR_WORKSPACE (nothing enqueued).  Results are bit-identical to
 * tfx_mobilenet_v1_variant_forward below batch 32 (from there on that call splits the batch
 * over two streams; this one creates no stream and runs one chain of kernels).  All calls on one GPU share the one array: calls that
 * overlap in time on one GPU (different streams or host threads) race and give
 * undefined results; calls ordered on one stream are fine.  Nothing in the array has to
 * start at zero (each kernel writes what later kernels read), so its contents between
 * calls do not matter.  Other arguments and errors as tfx_mobilenet_v1_variant_forward;
 * TFX_ERR_LAUNCH also if the array's device address cannot be obtained. */
size_t tfx_mobilenet_v1_static_scratch_bytes(void);
int tfx_mobilenet_v1_variant_forward_static(const tfx_mobilenet_v1_variant* variant, const float* input,
                                            int64_t batch, const tfx_mobilenet_v1_weights* weights, float* probs,
                                            float* logits, void* stream);

/* MobileNet v1 on 16-bit storage: the network of tfx_mobilenet_v1_variant_forward with
 * every tensor (image, weights, biases, feature maps, pooled vector, logits,
 * probabilities) stored as binary16 and every layer rounding its result once; the
 * softmax is taken of the binary16 logits.  Members as in tfx_mobilenet_v1_weights. */
typedef struct {
  const uint16_t* conv0_w;
  const uint16_t* conv0_b;
  const uint16_t* dw_w[13];
  const uint16_t* dw_b[13];
  const uint16_t* pw_w[13];
  const uint16_t* pw_b[13];
  const uint16_t* fc_w;
  const uint16_t* fc_b;
} tfx_mobilenet_v1_weights_f16;

/* Workspace bytes of tfx_mobilenet_v1_forward_f16 (0 if the variant or batch is invalid). */
size_t tfx_mobilenet_v1_workspace_bytes_f16(const tfx_mobilenet_v1_variant* variant, int64_t batch);

/* input: device [batch,image_size,image_size,3] binary16; probs / logits: device
 * [batch,classes] binary16 (logits may be NULL); workspace as for the fp32 entry point. */
int tfx_mobilenet_v1_forward_f16(const tfx_mobilenet_v1_variant* variant, const uint16_t* input, int64_t batch,
                                 const tfx_mobilenet_v1_weights_f16* weights, void* workspace,
                                 size_t workspace_bytes, uint16_t* probs, uint16_t* logits, void* stream);

/* tfx_mobilenet_v1_variant_features on 16-bit float storage: the output of block `end_block` (1 ... 13) as the
 * layers of tfx_mobilenet_v1_forward_f16 compute it, binary16 [batch, h, w, c] with the shape
 * tfx_mobilenet_v1_variant_features_shape gives; nothing after that block runs.  features: device, 16-byte
 * aligned.  Errors as the fp32 call. */
int tfx_mobilenet_v1_features_f16(const tfx_mobilenet_v1_variant* variant, const uint16_t* input, int64_t batch,
                                  const tfx_mobilenet_v1_weights_f16* weights, void* workspace, size_t workspace_bytes,
                                  int end_block, uint16_t* features, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* TFX_H_ */
