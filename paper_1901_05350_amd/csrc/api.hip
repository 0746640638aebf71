// C ABI of libtfx: argument validation, shape rules and kernel selection.
// Every entry point validates on the host before any HIP call and then only enqueues
// kernels on the caller's stream (enqueue-and-return, as the ops of Section 3.6 / 4.1);
// the fp32 forward pass of 32 or more images also uses one or two streams of the library's
// own, forked from and joined to the caller's (forward_whole).
#include <cstdlib>
#include <mutex>

#include "tfx_internal.h"

namespace tfx {

int out_extent(int64_t in, int64_t k, int64_t s, int pad, int64_t* out, int64_t* before, int64_t* after) {
  if (in < 1 || k < 1) return TFX_ERR_SHAPE;
  if (s < 1) return TFX_ERR_ARG;
  if (pad == TFX_PAD_VALID) {
    if (in < k) return TFX_ERR_SHAPE;
    *out = (in - k) / s + 1;
    *before = *after = 0;
    return TFX_OK;
  }
  if (pad != TFX_PAD_SAME) return TFX_ERR_ARG;
  const int64_t o = (in + s - 1) / s;
  const int64_t need = (o - 1) * s + k - in;
  const int64_t total = need > 0 ? need : 0;
  *out = o;
  *before = total >> 1;
  *after = total - (total >> 1);
  return TFX_OK;
}

namespace {

constexpr int64_t kMaxElems = (int64_t(1) << 31) - 1;

bool valid_act(int act) { return act == TFX_ACT_NONE || act == TFX_ACT_RELU || act == TFX_ACT_RELU6; }

// numel, or -1 if it does not fit below 2^31
int64_t numel(const int64_t* d, int rank) {
  int64_t p = 1;
  for (int i = 0; i < rank; ++i) {
    if (d[i] > kMaxElems) return -1;
    p *= d[i];
    if (p > kMaxElems) return -1;
  }
  return p;
}

struct ConvGeom {
  int64_t out[4];
  int64_t pad[4];
};

int conv_geometry(const int64_t x[4], const int64_t f[4], int sh, int sw, int pad, bool depthwise, ConvGeom* g) {
  for (int i = 0; i < 4; ++i)
    if (x[i] < 1 || f[i] < 1) return TFX_ERR_SHAPE;
  if (x[3] != f[2]) return TFX_ERR_SHAPE;
  if (sh < 1 || sw < 1) return TFX_ERR_ARG;
  if (pad != TFX_PAD_VALID && pad != TFX_PAD_SAME) return TFX_ERR_ARG;
  int rc = out_extent(x[1], f[0], sh, pad, &g->out[1], &g->pad[0], &g->pad[1]);
  if (rc) return rc;
  rc = out_extent(x[2], f[1], sw, pad, &g->out[2], &g->pad[2], &g->pad[3]);
  if (rc) return rc;
  g->out[0] = x[0];
  g->out[3] = depthwise ? x[3] * f[3] : f[3];
  return TFX_OK;
}

int matmul_geometry(const int64_t a[2], const int64_t b[2], int ta, int tb, int64_t* m, int64_t* n, int64_t* k) {
  if (a[0] < 1 || a[1] < 1 || b[0] < 1 || b[1] < 1) return TFX_ERR_SHAPE;
  *m = ta ? a[1] : a[0];
  *k = ta ? a[0] : a[1];
  const int64_t kb = tb ? b[1] : b[0];
  *n = tb ? b[0] : b[1];
  return *k == kb ? TFX_OK : TFX_ERR_SHAPE;
}

int batch_matmul_impl(const float* a, const int64_t* a_shape, const float* b, const int64_t* b_shape, int64_t batch,
                      int ta, int tb, float* c, void* stream) {
  int64_t m, n, k;
  int rc = matmul_geometry(a_shape, b_shape, ta, tb, &m, &n, &k);
  if (rc) return rc;
  const int64_t da[3] = {batch, m, k}, db[3] = {batch, n, k}, dc[3] = {batch, m, n};
  if (numel(da, 3) < 0 || numel(db, 3) < 0 || numel(dc, 3) < 0) return TFX_ERR_UNSUPPORTED;
  // stored [M,K] (not transposed) means K is contiguous for A; stored [N,K] (transposed) for B
  return launch_gemm(a, b, c, nullptr, (int)batch, (int)m, (int)n, (int)k, !ta, tb != 0, TFX_ACT_NONE,
                     static_cast<hipStream_t>(stream));
}

// MobileNet v1 1.0 / 224 architecture (Section 3.9, Table 1 workload).
constexpr int kBlocks = 13;
constexpr int kChannels[kBlocks] = {64, 128, 128, 256, 256, 512, 512, 512, 512, 512, 512, 1024, 1024};
constexpr int kStrides[kBlocks] = {1, 2, 1, 2, 1, 2, 1, 1, 1, 1, 1, 2, 1};
constexpr int kImage = 224, kStemChannels = 32, kClasses = 1000, kFeatures = 1024;
constexpr size_t kAlign = 256;

size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct NetPlan {
  size_t act_floats;  // per ping-pong buffer
  size_t off_buf[2], off_partial, off_chain, off_head, bytes;
  bool chain;         // the batch-1 full-width network: room for the chained small-map kernel (chain.hip)
  bool head;          // and for blocks 2 - 4 as stages of one launch (block.hip): their three outputs at once
};

bool valid_variant(const tfx_mobilenet_v1_variant* v) {
  return v && v->image_size >= 32 && v->image_size <= 256 && v->width_quarters >= 1 && v->width_quarters <= 4 &&
         v->classes >= 1 && v->classes <= 1024;
}

NetPlan plan_net(const tfx_mobilenet_v1_variant& v, int64_t batch, size_t elem_bytes = sizeof(float)) {
  NetPlan p{};
  // largest feature map: the output of the first pointwise layer (half the image size, 64 alpha channels)
  const size_t half = (size_t)(v.image_size + 1) / 2;
  p.act_floats = (size_t)batch * half * half * (size_t)(kChannels[0] * v.width_quarters / 4);
  size_t off = 0;
  for (int i = 0; i < 2; ++i) {
    p.off_buf[i] = off;
    off = align_up(off + p.act_floats * elem_bytes);
  }
  p.off_partial = off;  // K-slice partial sums of the fully connected layer
  off = align_up(off + fc_partial_floats((int)batch, (int)(kFeatures * v.width_quarters / 4), (int)v.classes) * sizeof(float));
  p.off_chain = off;
  p.chain = elem_bytes == sizeof(float) && chain_supported((int)v.image_size, (int)v.width_quarters, (int)v.classes, batch);
  if (p.chain) off = align_up(off + chain_workspace_bytes((int)v.image_size, (int)v.classes, (int)v.width_quarters));
  // blocks 2 - 4 in one launch: the outputs of blocks 2 and 3 share the second ping-pong buffer, the output of block 4
  // (1/8-size map, 256 channels) gets a region of its own, because block 2 is still reading the first buffer; the
  // output of block 5 (a launch of its own) goes behind it
  const size_t quarter = (half + 1) / 2, eighth = (quarter + 1) / 2;
  p.off_head = off;
  p.head = p.chain && v.width_quarters == 4 && 2 * quarter * quarter * 128 <= p.act_floats;
  if (p.head) off = align_up(off + 2 * eighth * eighth * 256 * sizeof(float));  // outputs of blocks 4 and 5
  p.bytes = off;
  return p;
}

constexpr tfx_mobilenet_v1_variant kBaseVariant = {kImage, 4, kClasses};

// Workspace of tfx_mobilenet_v1_variant_forward_static: it lives in the library's code object, one copy per
// GPU, from the moment the library is loaded on that GPU until the process ends.
constexpr size_t kStaticScratchBytes = size_t(16) << 20;
constexpr int kMaxDevices = 64;

}  // namespace
}  // namespace tfx

static __device__ __align__(256) unsigned char scratch[tfx::kStaticScratchBytes];

namespace tfx {
namespace {

// Device address of `scratch` on the calling thread's current device.  In host code the array's name is only a
// handle for the runtime; the address kernels can use is looked up once per device and kept.  Returns null if the
// lookup fails.  Safe to call from several threads (the lookup is idempotent).
void* static_scratch() {
  static std::atomic<void*> ptr[kMaxDevices];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  void* p = ptr[dev].load(std::memory_order_acquire);
  if (p) return p;
  if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
  ptr[dev].store(p, std::memory_order_release);
  return p;
}

// From batch 32 on the fp32 forward pass runs as two parts of the batch, from batch 60 on as three, all but the first
// on streams of the library's own that are forked from the caller's stream and joined back to it with events: the
// layers of such a batch are kernels of 10 - 90 us whose last workgroups leave most CUs idle, and independent chains
// of them fill each other's tails (measured: batch 64 1.03 -> 0.975 ms with two chains, 0.96 with three; batch 128
// 1.87 -> 1.76 either way; at batch 48 three are no better than two; nothing to gain on binary16 storage).
constexpr int64_t kSplitBatch = 32, kThreeChains = 60;
constexpr int kMaxChains = 3;

int net_chains(int64_t batch) { return batch < kSplitBatch ? 1 : batch < kThreeChains ? 2 : 3; }
// images of part i of `chains`: the first batch % chains parts take one more
int64_t part_images(int64_t batch, int chains, int i) { return batch / chains + (i < batch % chains ? 1 : 0); }

size_t net_workspace_bytes(const tfx_mobilenet_v1_variant& v, int64_t batch) {  // enough for either form
  const size_t whole = plan_net(v, batch).bytes;
  const int chains = net_chains(batch);
  if (chains == 1) return whole;
  size_t parts = 0;
  for (int i = 0; i < chains; ++i) parts += align_up(plan_net(v, part_images(batch, chains, i)).bytes);
  return parts > whole ? parts : whole;
}

// The library's own streams and events, one set per device, created on the first call that wants them and kept
// until the process ends.  Calls that use them hold the lock while they enqueue.
struct SideStreams {
  hipStream_t stream[kMaxChains - 1];
  hipEvent_t fork, join[kMaxChains - 1];
};
std::mutex g_side_lock;
SideStreams* side_streams(hipStream_t caller) {  // with g_side_lock held; null: none to be had
  static SideStreams table[kMaxDevices];
  static int state[kMaxDevices];  // 0 not tried, 1 there, 2 failed
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  if (state[dev] == 0) {
    // nothing is created while the caller's stream is being captured into a graph (creation calls are not allowed
    // then); a later call outside a capture creates them
    hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(caller, &capturing) != hipSuccess || capturing != hipStreamCaptureStatusNone) {
      (void)hipGetLastError();
      return nullptr;
    }
    SideStreams& t = table[dev];
    bool ok = hipEventCreateWithFlags(&t.fork, hipEventDisableTiming) == hipSuccess;
    for (int i = 0; i < kMaxChains - 1 && ok; ++i)
      ok = hipStreamCreateWithFlags(&t.stream[i], hipStreamNonBlocking) == hipSuccess &&
           hipEventCreateWithFlags(&t.join[i], hipEventDisableTiming) == hipSuccess;
    if (!ok) (void)hipGetLastError();
    state[dev] = ok ? 1 : 2;
  }
  return state[dev] == 1 ? &table[dev] : nullptr;
}

}  // namespace
}  // namespace tfx

using namespace tfx;

extern "C" {

const char* tfx_status_string(int status) {
  switch (status) {
    case TFX_OK: return "TFX_OK";
    case TFX_ERR_NULL: return "TFX_ERR_NULL: null pointer argument";
    case TFX_ERR_SHAPE: return "TFX_ERR_SHAPE: non-positive or mismatching dimensions";
    case TFX_ERR_ARG: return "TFX_ERR_ARG: bad stride or enum value";
    case TFX_ERR_UNSUPPORTED: return "TFX_ERR_UNSUPPORTED: tensor too large";
    case TFX_ERR_WORKSPACE: return "TFX_ERR_WORKSPACE: workspace too small or misaligned";
    case TFX_ERR_LAUNCH: return "TFX_ERR_LAUNCH: kernel enqueue failed";
    default: return "unknown tfx status";
  }
}

int tfx_matmul_out_shape(const int64_t a_shape[2], const int64_t b_shape[2], int transpose_a, int transpose_b,
                         int64_t out_shape[2]) {
  if (!a_shape || !b_shape || !out_shape) return TFX_ERR_NULL;
  int64_t m, n, k;
  int rc = matmul_geometry(a_shape, b_shape, transpose_a, transpose_b, &m, &n, &k);
  if (rc) return rc;
  out_shape[0] = m;
  out_shape[1] = n;
  return TFX_OK;
}

int tfx_conv2d_out_shape(const int64_t x_shape[4], const int64_t f_shape[4], int stride_h, int stride_w,
                         tfx_padding pad, int64_t out_shape[4], int64_t pad_tblr[4]) {
  if (!x_shape || !f_shape || !out_shape || !pad_tblr) return TFX_ERR_NULL;
  ConvGeom g;
  int rc = conv_geometry(x_shape, f_shape, stride_h, stride_w, (int)pad, false, &g);
  if (rc) return rc;
  for (int i = 0; i < 4; ++i) {
    out_shape[i] = g.out[i];
    pad_tblr[i] = g.pad[i];
  }
  return TFX_OK;
}

int tfx_depthwise_conv2d_out_shape(const int64_t x_shape[4], const int64_t f_shape[4], int stride_h, int stride_w,
                                   tfx_padding pad, int64_t out_shape[4], int64_t pad_tblr[4]) {
  if (!x_shape || !f_shape || !out_shape || !pad_tblr) return TFX_ERR_NULL;
  ConvGeom g;
  int rc = conv_geometry(x_shape, f_shape, stride_h, stride_w, (int)pad, true, &g);
  if (rc) return rc;
  for (int i = 0; i < 4; ++i) {
    out_shape[i] = g.out[i];
    pad_tblr[i] = g.pad[i];
  }
  return TFX_OK;
}

int tfx_matmul(const float* a, const int64_t a_shape[2], const float* b, const int64_t b_shape[2], int transpose_a,
               int transpose_b, float* c, void* stream) {
  if (!a || !b || !c || !a_shape || !b_shape) return TFX_ERR_NULL;
  return batch_matmul_impl(a, a_shape, b, b_shape, 1, transpose_a, transpose_b, c, stream);
}

int tfx_batch_matmul(const float* a, const int64_t a_shape[3], const float* b, const int64_t b_shape[3],
                     int transpose_a, int transpose_b, float* c, void* stream) {
  if (!a || !b || !c || !a_shape || !b_shape) return TFX_ERR_NULL;
  if (a_shape[0] < 1 || a_shape[0] != b_shape[0]) return TFX_ERR_SHAPE;
  return batch_matmul_impl(a, a_shape + 1, b, b_shape + 1, a_shape[0], transpose_a, transpose_b, c, stream);
}

int tfx_conv2d(const float* x, const int64_t x_shape[4], const float* filter, const int64_t f_shape[4],
               const float* bias, int stride_h, int stride_w, tfx_padding pad, tfx_activation act, float* y,
               void* stream) {
  if (!x || !filter || !y || !x_shape || !f_shape) return TFX_ERR_NULL;
  ConvGeom g;
  int rc = conv_geometry(x_shape, f_shape, stride_h, stride_w, (int)pad, false, &g);
  if (rc) return rc;
  if (!valid_act((int)act)) return TFX_ERR_ARG;
  if (numel(x_shape, 4) < 0 || numel(f_shape, 4) < 0 || numel(g.out, 4) < 0) return TFX_ERR_UNSUPPORTED;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int n = (int)x_shape[0], h = (int)x_shape[1], w = (int)x_shape[2], ci = (int)x_shape[3];
  const int fh = (int)f_shape[0], fw = (int)f_shape[1], co = (int)f_shape[3];
  const int oh = (int)g.out[1], ow = (int)g.out[2];
  if (fh == 1 && fw == 1 && stride_h == 1 && stride_w == 1) {
    // pointwise convolution = [N*H*W, Ci] x [Ci, Co] with the epilogue fused into the GEMM
    if (pointwise_stream_supported(n * h * w, ci, co, x, filter, bias, y))
      return launch_pointwise_stream(x, filter, bias, y, n * h * w, ci, co, (int)act, s);
    return launch_gemm(x, filter, y, bias, 1, n * h * w, co, ci, true, false, (int)act, s);
  }
  const bool aligned = reinterpret_cast<uintptr_t>(y) % 16 == 0;
  if (conv2d_stem_supported(ci, fh, fw, co, stride_h, stride_w) && aligned)
    return launch_conv2d_stem(x, filter, bias, y, n, h, w, co, oh, ow, stride_h, stride_w, (int)g.pad[0], (int)g.pad[2],
                              (int)act, s);
  // enough input channels and filters to fill matrix-core tiles: implicit GEMM; else one thread per output
  if (ci >= 8 && co >= 8)
    return launch_conv2d_gemm(x, filter, bias, y, n, h, w, ci, fh, fw, co, oh, ow, stride_h, stride_w, (int)g.pad[0],
                              (int)g.pad[2], (int)act, s);
  return launch_conv2d_direct(x, filter, bias, y, n, h, w, ci, fh, fw, co, oh, ow, stride_h, stride_w, (int)g.pad[0],
                              (int)g.pad[2], (int)act, s);
}

int tfx_depthwise_conv2d(const float* x, const int64_t x_shape[4], const float* filter, const int64_t f_shape[4],
                         const float* bias, int stride_h, int stride_w, tfx_padding pad, tfx_activation act, float* y,
                         void* stream) {
  if (!x || !filter || !y || !x_shape || !f_shape) return TFX_ERR_NULL;
  ConvGeom g;
  int rc = conv_geometry(x_shape, f_shape, stride_h, stride_w, (int)pad, true, &g);
  if (rc) return rc;
  if (!valid_act((int)act)) return TFX_ERR_ARG;
  if (numel(x_shape, 4) < 0 || numel(f_shape, 4) < 0 || numel(g.out, 4) < 0) return TFX_ERR_UNSUPPORTED;
  return launch_depthwise(x, filter, bias, y, (int)x_shape[0], (int)x_shape[1], (int)x_shape[2], (int)x_shape[3],
                          (int)f_shape[0], (int)f_shape[1], (int)f_shape[3], (int)g.out[1], (int)g.out[2], stride_h,
                          stride_w, (int)g.pad[0], (int)g.pad[2], (int)act, static_cast<hipStream_t>(stream));
}

int tfx_add(const float* a, const float* b, int64_t n, float* c, void* stream) {
  if (n < 0) return TFX_ERR_SHAPE;
  if (n == 0) return TFX_OK;
  if (!a || !b || !c) return TFX_ERR_NULL;
  if (n > (int64_t(1) << 40)) return TFX_ERR_UNSUPPORTED;
  return launch_add_f32(a, b, c, n, static_cast<hipStream_t>(stream));
}

int tfx_add_f16(const uint16_t* a, const uint16_t* b, int64_t n, uint16_t* c, void* stream) {
  if (n < 0) return TFX_ERR_SHAPE;
  if (n == 0) return TFX_OK;
  if (!a || !b || !c) return TFX_ERR_NULL;
  if (n > (int64_t(1) << 40)) return TFX_ERR_UNSUPPORTED;
  return launch_add_f16(a, b, c, n, static_cast<hipStream_t>(stream));
}

int tfx_batch_matmul_f16(const uint16_t* a, const int64_t a_shape[3], const uint16_t* b, const int64_t b_shape[3],
                         int transpose_a, int transpose_b, const uint16_t* bias, tfx_activation act, uint16_t* c,
                         void* stream) {
  if (!a || !b || !c || !a_shape || !b_shape) return TFX_ERR_NULL;
  if (!valid_act((int)act)) return TFX_ERR_ARG;
  if (a_shape[0] < 1 || a_shape[0] != b_shape[0]) return TFX_ERR_SHAPE;
  int64_t m, n, k;
  int rc = matmul_geometry(a_shape + 1, b_shape + 1, transpose_a, transpose_b, &m, &n, &k);
  if (rc) return rc;
  const int64_t batch = a_shape[0];
  const int64_t da[3] = {batch, m, k}, db[3] = {batch, n, k}, dc[3] = {batch, m, n};
  if (numel(da, 3) < 0 || numel(db, 3) < 0 || numel(dc, 3) < 0) return TFX_ERR_UNSUPPORTED;
  return launch_gemm_f16(a, b, c, bias, (int)batch, (int)m, (int)n, (int)k, !transpose_a, transpose_b != 0, (int)act,
                         static_cast<hipStream_t>(stream));
}

int tfx_conv2d_f16(const uint16_t* x, const int64_t x_shape[4], const uint16_t* filter, const int64_t f_shape[4],
                   const uint16_t* bias, int stride_h, int stride_w, tfx_padding pad, tfx_activation act, uint16_t* y,
                   void* stream) {
  if (!x || !filter || !y || !x_shape || !f_shape) return TFX_ERR_NULL;
  if (!valid_act((int)act)) return TFX_ERR_ARG;
  ConvGeom g;
  int rc = conv_geometry(x_shape, f_shape, stride_h, stride_w, (int)pad, false, &g);
  if (rc) return rc;
  if (numel(x_shape, 4) < 0 || numel(f_shape, 4) < 0 || numel(g.out, 4) < 0) return TFX_ERR_UNSUPPORTED;
  const int n = (int)x_shape[0], h = (int)x_shape[1], w = (int)x_shape[2], ci = (int)x_shape[3];
  const int fh = (int)f_shape[0], fw = (int)f_shape[1], co = (int)f_shape[3];
  const int oh = (int)g.out[1], ow = (int)g.out[2];
  hipStream_t s = static_cast<hipStream_t>(stream);
  // a 1x1 stride-1 convolution is the matMul of the pixel rows [n*h*w, ci] with the filter [ci, co]
  if (fh == 1 && fw == 1 && stride_h == 1 && stride_w == 1)
    return launch_gemm_f16(x, filter, y, bias, 1, n * h * w, co, ci, true, false, (int)act, s);
  if (conv2d_stem_f16_supported(ci, fh, fw, co, y))
    return launch_conv2d_stem_f16(x, filter, bias, y, n, h, w, co, oh, ow, stride_h, stride_w, (int)g.pad[0],
                                  (int)g.pad[2], (int)act, s);
  if (conv3x3_stream_f16_supported((long long)n * oh * ow, numel(x_shape, 4), ci, fh, fw, co, stride_h, stride_w, x,
                                   filter, y))
    return launch_conv3x3_stream_f16(x, filter, bias, y, n, h, w, ci, co, oh, ow, (int)g.pad[0], (int)g.pad[2],
                                     (int)act, s);
  if (conv2d_gemm_f16_supported(x, filter, ci, fh, fw, co))
    return launch_conv2d_gemm_f16(x, filter, bias, y, n, h, w, ci, fh, fw, co, oh, ow, stride_h, stride_w,
                                  (int)g.pad[0], (int)g.pad[2], (int)act, s);
  return launch_conv2d_direct_f16(x, filter, bias, y, n, h, w, ci, fh, fw, co, oh, ow, stride_h, stride_w,
                                  (int)g.pad[0], (int)g.pad[2], (int)act, s);
}

int tfx_depthwise_conv2d_f16(const uint16_t* x, const int64_t x_shape[4], const uint16_t* filter,
                             const int64_t f_shape[4], const uint16_t* bias, int stride_h, int stride_w,
                             tfx_padding pad, tfx_activation act, uint16_t* y, void* stream) {
  if (!x || !filter || !y || !x_shape || !f_shape) return TFX_ERR_NULL;
  if (!valid_act((int)act)) return TFX_ERR_ARG;
  ConvGeom g;
  int rc = conv_geometry(x_shape, f_shape, stride_h, stride_w, (int)pad, true, &g);
  if (rc) return rc;
  if (numel(x_shape, 4) < 0 || numel(f_shape, 4) < 0 || numel(g.out, 4) < 0) return TFX_ERR_UNSUPPORTED;
  return launch_depthwise_f16(x, filter, bias, y, (int)x_shape[0], (int)x_shape[1], (int)x_shape[2], (int)x_shape[3],
                              (int)f_shape[0], (int)f_shape[1], (int)f_shape[3], (int)g.out[1], (int)g.out[2], stride_h,
                              stride_w, (int)g.pad[0], (int)g.pad[2], (int)act, static_cast<hipStream_t>(stream));
}

size_t tfx_mobilenet_v1_workspace_bytes(int64_t batch) {
  if (batch < 1 || batch > 1024) return 0;
  return net_workspace_bytes(kBaseVariant, batch);
}

int tfx_mobilenet_v1_forward(const float* input, int64_t batch, const tfx_mobilenet_v1_weights* weights,
                             void* workspace, size_t workspace_bytes, float* probs, float* logits, void* stream) {
  return tfx_mobilenet_v1_variant_forward(&kBaseVariant, input, batch, weights, workspace, workspace_bytes, probs,
                                          logits, stream);
}

size_t tfx_mobilenet_v1_variant_workspace_bytes(const tfx_mobilenet_v1_variant* variant, int64_t batch) {
  if (!valid_variant(variant) || batch < 1 || batch > 1024) return 0;
  return net_workspace_bytes(*variant, batch);
}

namespace {
// The checks of a forward pass's arguments that come before the workspace's, in their order.
int check_net_args(const tfx_mobilenet_v1_variant* variant, const float* input, int64_t batch,
                   const tfx_mobilenet_v1_weights* weights, const void* workspace, const void* out) {
  if (!variant || !input || !weights || !workspace || !out) return TFX_ERR_NULL;
  if (!weights->conv0_w || !weights->conv0_b || !weights->fc_w || !weights->fc_b) return TFX_ERR_NULL;
  for (int i = 0; i < kBlocks; ++i)
    if (!weights->dw_w[i] || !weights->dw_b[i] || !weights->pw_w[i] || !weights->pw_b[i]) return TFX_ERR_NULL;
  if (!valid_variant(variant)) return TFX_ERR_ARG;
  if (batch < 1) return TFX_ERR_SHAPE;
  if (batch > 1024) return TFX_ERR_UNSUPPORTED;
  return TFX_OK;
}

// The forward pass; end_block = 0: the whole network into probs / logits; end_block = 1 .. 13: stop after that
// depthwise-separable block, whose output goes to `features` instead of the workspace.
int forward_impl(const tfx_mobilenet_v1_variant* variant, const float* input, int64_t batch,
                 const tfx_mobilenet_v1_weights* weights, void* workspace, size_t workspace_bytes, float* probs,
                 float* logits, int end_block, float* features, void* stream) {
  if (const int bad = check_net_args(variant, input, batch, weights, workspace,
                                     end_block == 0 ? (const void*)probs : (const void*)features))
    return bad;
  const NetPlan plan = plan_net(*variant, batch);
  if (workspace_bytes < plan.bytes || reinterpret_cast<uintptr_t>(workspace) % kAlign != 0) return TFX_ERR_WORKSPACE;
  const int q = (int)variant->width_quarters;

  char* ws = static_cast<char*>(workspace);
  float* buf[2] = {reinterpret_cast<float*>(ws + plan.off_buf[0]), reinterpret_cast<float*>(ws + plan.off_buf[1])};
  float* partial = reinterpret_cast<float*>(ws + plan.off_partial);

  // Batch 1: the blocks from the last 1/8-size map on, the pool, the fully connected layer and the
  // softmax run as one persistent kernel (chain.hip) when every pointer allows its vector loads and 256 of its
  // workgroups are resident at once on this device; its task flags are cleared by the first kernel of the pass
  // (the stem, alone or fused with block 1).
  bool flags_ok = plan.chain;  // the workspace has the flag region, and the kernels that use it may run
  if (flags_ok) {
    auto al16 = [](const void* p) { return reinterpret_cast<uintptr_t>(p) % 16 == 0; };
    flags_ok = al16(input) && al16(weights->conv0_b) && al16(weights->fc_w) && al16(weights->fc_b);
    for (int i = 0; i < kBlocks && flags_ok; ++i)
      flags_ok = al16(weights->dw_w[i]) && al16(weights->dw_b[i]) && al16(weights->pw_w[i]) && al16(weights->pw_b[i]);
    flags_ok = flags_ok && chain_resident(q);
  }
  const bool chain = flags_ok && end_block == 0;
  // blocks 2 - 4 as stages of one launch and block 5 as a launch (block.hip): in the whole pass and when block 4's
  // or block 5's output is asked for
  const bool head_chain = flags_ok && plan.head && (end_block == 0 || end_block == 4 || end_block == 5);
  void* chain_ws = ws + plan.off_chain;

  // stem: 3x3 stride-2 convolution to 32 alpha channels, then the 13 depthwise-separable blocks
  int64_t shape[4] = {batch, variant->image_size, variant->image_size, 3};
  const int64_t f0[4] = {3, 3, 3, kStemChannels * q / 4};
  ConvGeom g;
  conv_geometry(shape, f0, 2, 2, TFX_PAD_SAME, false, &g);
  int rc;
  int first_block = 0;
  const int64_t c0 = kChannels[0] * q / 4;
  if (kStrides[0] == 1 &&
      stem_block_supported(batch, (int)shape[1], (int)shape[2], (int)f0[3], (int)c0, input, weights->conv0_w,
                           weights->conv0_b, weights->dw_w[0], weights->dw_b[0], weights->pw_w[0], weights->pw_b[0],
                           end_block == 1 ? features : buf[0])) {
    // batch 1 to 3: stem and first block in one launch (block.hip); it also clears the chain's task flags
    rc = launch_stem_block(input, weights->conv0_w, weights->conv0_b, weights->dw_w[0], weights->dw_b[0],
                           weights->pw_w[0], weights->pw_b[0], end_block == 1 ? features : buf[0], (int)batch, (int)shape[1],
                           (int)shape[2], (int)g.out[1],
                           (int)g.out[2], (int)g.pad[0], (int)g.pad[2], (int)c0, TFX_ACT_RELU6,
                           static_cast<hipStream_t>(stream), chain || head_chain ? static_cast<int*>(chain_ws) : nullptr,
                           chain || head_chain ? chain_flag_words((int)variant->image_size, (int)variant->classes, q) : 0,
                           chain_flag_stride());
    first_block = 1;
  } else if (chain)
    rc = launch_conv2d_stem(input, weights->conv0_w, weights->conv0_b, buf[0], 1, (int)shape[1], (int)shape[2],
                            (int)f0[3], (int)g.out[1], (int)g.out[2], 2, 2, (int)g.pad[0], (int)g.pad[2], TFX_ACT_RELU6,
                            static_cast<hipStream_t>(stream), static_cast<int*>(chain_ws),
                            chain_flag_words((int)variant->image_size, (int)variant->classes, q), chain_flag_stride());
  else
    rc = tfx_conv2d(input, shape, weights->conv0_w, f0, weights->conv0_b, 2, 2, TFX_PAD_SAME, TFX_ACT_RELU6, buf[0],
                    stream);
  if (rc) return rc;
  for (int i = 0; i < 4; ++i) shape[i] = g.out[i];
  if (first_block == 1) shape[3] = c0;
  if (first_block == 1 && end_block == 1) return TFX_OK;
  int cur = 0;
  const int head_flags = block_chain_flag_words((int)shape[1], (int)shape[2]);
  if (head_chain && first_block == 1) {
    // blocks 2 - 4 as three stages of one launch, block 5 as a launch of its own, then the chained kernel from block 6
    // on; flags (cleared by the first kernel) and failure word are shared with it
    const size_t quarter = (size_t)((shape[1] + 1) / 2), eighth = (quarter + 1) / 2;
    float* const region = reinterpret_cast<float*>(ws + plan.off_head);
    float* const b2_out = buf[1];
    float* const b3_out = buf[1] + quarter * quarter * 128;
    float* const b4_out = end_block == 4 ? features : region;
    float* const b5_out = end_block == 5 ? features : region + eighth * eighth * 256;
    const bool with_b5 = end_block != 4 && separable_block_supported(1, (int)eighth, (int)eighth, 256, 256, 1, b4_out,
                                                                  weights->dw_w[4], weights->dw_b[4], weights->pw_w[4],
                                                                  weights->pw_b[4], b5_out);
    if (block_chain_supported(buf[0], b2_out, b3_out, b4_out, weights) && (with_b5 || end_block == 4)) {
      struct Head {
        const float* x;
        float *b2, *b3, *b4, *b5;
        int h, w, eighth;
        bool with_b5;
        const tfx_mobilenet_v1_weights* wt;
        int* flags;
        int flag_base;
        hipStream_t stream;
      } head{buf[0], b2_out, b3_out, b4_out, b5_out, (int)shape[1], (int)shape[2], (int)eighth, with_b5, weights,
             static_cast<int*>(chain_ws), chain_head_flag_base((int)variant->image_size, (int)variant->classes),
             static_cast<hipStream_t>(stream)};
      auto launch_head = [](void* p) -> int {
        const Head& a = *static_cast<const Head*>(p);
        const int rc = launch_block_chain(a.x, a.b2, a.b3, a.b4, a.h, a.w, a.wt, a.flags, a.flag_base, chain_spin_limit(), a.stream);
        if (rc != TFX_OK || !a.with_b5) return rc;
        // 28 x 28 x 256 -> 256, stride 1, SAME: one zero row / column before the map
        return launch_separable_block(a.b4, a.wt->dw_w[4], a.wt->dw_b[4], a.wt->pw_w[4], a.wt->pw_b[4], a.b5, 1, a.eighth, a.eighth,
                                      256, 256, a.eighth, a.eighth, 1, 1, 1, TFX_ACT_RELU6, TFX_ACT_RELU6, a.stream);
      };
      if (end_block != 0) return launch_ordered(static_cast<hipStream_t>(stream), launch_head, &head);
      return launch_chain(b5_out, (int)eighth, weights, chain_ws, head_flags, probs, logits, (int)variant->classes, q,
                          static_cast<hipStream_t>(stream), launch_head, &head, 5);
    }
  }
  for (int b = first_block; b < kBlocks; ++b) {
    float* const block_out = end_block == b + 1 ? features : buf[cur ^ 1];
    if (chain && b == 4)
      return launch_chain(buf[cur], (int)shape[1], weights, chain_ws, head_flags, probs, logits, (int)variant->classes, q,
                          static_cast<hipStream_t>(stream));
    const int64_t fd[4] = {3, 3, shape[3], 1};
    const int64_t cout = kChannels[b] * q / 4;
    // batch 1 to 3, thin block: depthwise and pointwise layer in one launch (block.hip)
    if (separable_block_supported(batch, (int)shape[1], (int)shape[2], (int)shape[3], (int)cout, kStrides[b], buf[cur],
                                  weights->dw_w[b], weights->dw_b[b], weights->pw_w[b], weights->pw_b[b], block_out)) {
      conv_geometry(shape, fd, kStrides[b], kStrides[b], TFX_PAD_SAME, true, &g);
      rc = launch_separable_block(buf[cur], weights->dw_w[b], weights->dw_b[b], weights->pw_w[b], weights->pw_b[b],
                                  block_out, (int)batch, (int)shape[1], (int)shape[2], (int)shape[3], (int)cout, (int)g.out[1],
                                  (int)g.out[2], kStrides[b], (int)g.pad[0], (int)g.pad[2], TFX_ACT_RELU6, TFX_ACT_RELU6,
                                  static_cast<hipStream_t>(stream));
      if (rc) return rc;
      if (end_block == b + 1) return TFX_OK;
      for (int i = 0; i < 3; ++i) shape[i] = g.out[i];
      shape[3] = cout;
      cur ^= 1;
      continue;
    }
    // large batch, early block: depthwise and pointwise layer in one filter-stationary launch (block_stream.hip)
    conv_geometry(shape, fd, kStrides[b], kStrides[b], TFX_PAD_SAME, true, &g);
    if (separable_stream_supported((int)batch, (int)shape[1], (int)shape[2], (int)shape[3], (int)cout, kStrides[b],
                                   (int)g.out[1], (int)g.out[2], buf[cur], weights->dw_w[b], weights->dw_b[b],
                                   weights->pw_w[b], weights->pw_b[b], block_out)) {
      rc = launch_separable_stream(buf[cur], weights->dw_w[b], weights->dw_b[b], weights->pw_w[b], weights->pw_b[b],
                                   block_out, (int)batch, (int)shape[1], (int)shape[2], (int)shape[3], (int)cout,
                                   (int)g.out[1], (int)g.out[2], kStrides[b], (int)g.pad[0], (int)g.pad[2], TFX_ACT_RELU6,
                                   TFX_ACT_RELU6, static_cast<hipStream_t>(stream));
      if (rc) return rc;
      if (end_block == b + 1) return TFX_OK;
      for (int i = 0; i < 3; ++i) shape[i] = g.out[i];
      shape[3] = cout;
      cur ^= 1;
      continue;
    }
    rc = tfx_depthwise_conv2d(buf[cur], shape, weights->dw_w[b], fd, weights->dw_b[b], kStrides[b], kStrides[b],
                              TFX_PAD_SAME, TFX_ACT_RELU6, buf[cur ^ 1], stream);
    if (rc) return rc;
    for (int i = 0; i < 4; ++i) shape[i] = g.out[i];
    cur ^= 1;
    const int64_t fp[4] = {1, 1, shape[3], cout};
    rc = tfx_conv2d(buf[cur], shape, weights->pw_w[b], fp, weights->pw_b[b], 1, 1, TFX_PAD_SAME, TFX_ACT_RELU6,
                    end_block == b + 1 ? features : buf[cur ^ 1], stream);
    if (rc) return rc;
    if (end_block == b + 1) return TFX_OK;
    shape[3] = cout;
    cur ^= 1;
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  return launch_pool_fc_softmax(buf[cur], weights->fc_w, weights->fc_b, partial, logits, probs, (int)batch,
                                (int)(shape[1] * shape[2]), (int)shape[3], (int)variant->classes, s);
}
}  // namespace

namespace {
// The whole forward pass: one chain of kernels on the caller's stream, or, from kSplitBatch on and if a second stream
// is to be had, two half batches, each with its own part of the workspace, on two streams.
int forward_whole(const tfx_mobilenet_v1_variant* variant, const float* input, int64_t batch,
                  const tfx_mobilenet_v1_weights* weights, void* workspace, size_t workspace_bytes, float* probs,
                  float* logits, void* stream, bool may_fork) {
  // TFX_ONE_STREAM in the environment: no stream of the library's in this process (also for per-kernel profiles:
  // overlapped kernels stretch each other's durations)
  if (batch < kSplitBatch || !may_fork || std::getenv("TFX_ONE_STREAM") != nullptr)
    return forward_impl(variant, input, batch, weights, workspace, workspace_bytes, probs, logits, 0, nullptr, stream);
  if (const int bad = check_net_args(variant, input, batch, weights, workspace, probs)) return bad;
  if (workspace_bytes < net_workspace_bytes(*variant, batch) || reinterpret_cast<uintptr_t>(workspace) % kAlign != 0)
    return TFX_ERR_WORKSPACE;
  hipStream_t main_stream = static_cast<hipStream_t>(stream);
  const int chains = net_chains(batch);
  std::unique_lock<std::mutex> guard(g_side_lock);
  SideStreams* const side = side_streams(main_stream);
  bool forked = side != nullptr && hipEventRecord(side->fork, main_stream) == hipSuccess;
  int waiting = 0;  // side streams that have joined the caller's stream (or the graph it is being captured into)
  for (; forked && waiting < chains - 1; ++waiting)
    if (hipStreamWaitEvent(side->stream[waiting], side->fork, 0) != hipSuccess) break;
  const bool all = forked && waiting == chains - 1;
  const size_t image = (size_t)variant->image_size * variant->image_size * 3;
  int rc = TFX_OK;
  if (all) {
    int64_t first = 0;
    char* ws = static_cast<char*>(workspace);
    for (int i = 0; i < chains && rc == TFX_OK; ++i) {
      const int64_t n = part_images(batch, chains, i);
      const size_t bytes = align_up(plan_net(*variant, n).bytes);
      rc = forward_impl(variant, input + first * image, n, weights, ws, bytes, probs + first * variant->classes,
                        logits ? logits + first * variant->classes : nullptr, 0, nullptr,
                        i == 0 ? main_stream : side->stream[i - 1]);
      first += n;
      ws += bytes;
    }
  } else {
    // no streams of the library's (creation failed, or this first large call comes inside a graph capture), or a
    // wait could not be enqueued: one chain on the caller's stream
    (void)hipGetLastError();
    rc = forward_impl(variant, input, batch, weights, workspace, workspace_bytes, probs, logits, 0, nullptr, stream);
  }
  // every stream that waits for the fork is joined whatever happened in between, so that the caller's stream (or the
  // graph it is being captured into) never ends with a side stream still forked
  for (int i = 0; i < waiting; ++i)
    if (hipEventRecord(side->join[i], side->stream[i]) != hipSuccess ||
        hipStreamWaitEvent(main_stream, side->join[i], 0) != hipSuccess) {
      (void)hipGetLastError();
      if (rc == TFX_OK) rc = TFX_ERR_LAUNCH;
    }
  return rc;
}
}  // namespace

int tfx_mobilenet_v1_variant_forward(const tfx_mobilenet_v1_variant* variant, const float* input, int64_t batch,
                                     const tfx_mobilenet_v1_weights* weights, void* workspace,
                                     size_t workspace_bytes, float* probs, float* logits, void* stream) {
  return forward_whole(variant, input, batch, weights, workspace, workspace_bytes, probs, logits, stream, true);
}

int tfx_mobilenet_v1_variant_features_shape(const tfx_mobilenet_v1_variant* variant, int64_t batch, int end_block,
                                            int64_t shape[4]) {
  if (!variant || !shape) return TFX_ERR_NULL;
  if (!valid_variant(variant) || end_block < 1 || end_block > kBlocks) return TFX_ERR_ARG;
  if (batch < 1) return TFX_ERR_SHAPE;
  int64_t hw = (variant->image_size + 1) / 2;  // the stem halves the image (stride 2, SAME padding)
  for (int b = 0; b < end_block; ++b) hw = (hw + kStrides[b] - 1) / kStrides[b];
  shape[0] = batch, shape[1] = hw, shape[2] = hw, shape[3] = kChannels[end_block - 1] * variant->width_quarters / 4;
  return TFX_OK;
}

int tfx_mobilenet_v1_variant_features(const tfx_mobilenet_v1_variant* variant, const float* input, int64_t batch,
                                      const tfx_mobilenet_v1_weights* weights, void* workspace, size_t workspace_bytes,
                                      int end_block, float* features, void* stream) {
  if (end_block < 1 || end_block > kBlocks) return variant && input && weights && workspace && features ? TFX_ERR_ARG : TFX_ERR_NULL;
  if (features && reinterpret_cast<uintptr_t>(features) % 16 != 0) return TFX_ERR_ARG;
  return forward_impl(variant, input, batch, weights, workspace, workspace_bytes, nullptr, nullptr, end_block, features,
                      stream);
}

size_t tfx_mobilenet_v1_static_scratch_bytes(void) { return kStaticScratchBytes; }

int tfx_mobilenet_v1_variant_forward_static(const tfx_mobilenet_v1_variant* variant, const float* input, int64_t batch,
                                            const tfx_mobilenet_v1_weights* weights, float* probs, float* logits,
                                            void* stream) {
  if (!variant || !input || !weights || !probs) return TFX_ERR_NULL;
  if (!valid_variant(variant)) return TFX_ERR_ARG;
  if (batch < 1) return TFX_ERR_SHAPE;
  if (batch > 1024) return TFX_ERR_UNSUPPORTED;
  if (net_workspace_bytes(*variant, batch) > kStaticScratchBytes) return TFX_ERR_WORKSPACE;
  void* ws = static_scratch();
  if (!ws) return TFX_ERR_LAUNCH;
  // Every kernel of the forward pass writes the part of the workspace it later reads (feature maps, the fully
  // connected layer's partial sums), so nothing has to be cleared between calls.
  // (no second stream here -- creating one allocates: one chain of kernels at every batch)
  return forward_whole(variant, input, batch, weights, ws, kStaticScratchBytes, probs, logits, stream, false);
}

size_t tfx_mobilenet_v1_workspace_bytes_f16(const tfx_mobilenet_v1_variant* variant, int64_t batch) {
  if (!valid_variant(variant) || batch < 1 || batch > 1024) return 0;
  return plan_net(*variant, batch, sizeof(uint16_t)).bytes;
}

}  // extern "C"

namespace {

// end_block = 0: the whole network; else stop after that block and write its output to `features`
int forward_f16_impl(const tfx_mobilenet_v1_variant* variant, const uint16_t* input, int64_t batch,
                     const tfx_mobilenet_v1_weights_f16* weights, void* workspace, size_t workspace_bytes,
                     uint16_t* probs, uint16_t* logits, int end_block, uint16_t* features, void* stream) {
  if (!variant || !input || !weights || !workspace || !(end_block ? (void*)features : (void*)probs)) return TFX_ERR_NULL;
  if (!weights->conv0_w || !weights->conv0_b || !weights->fc_w || !weights->fc_b) return TFX_ERR_NULL;
  for (int i = 0; i < kBlocks; ++i)
    if (!weights->dw_w[i] || !weights->dw_b[i] || !weights->pw_w[i] || !weights->pw_b[i]) return TFX_ERR_NULL;
  if (!valid_variant(variant)) return TFX_ERR_ARG;
  if (batch < 1) return TFX_ERR_SHAPE;
  if (batch > 1024) return TFX_ERR_UNSUPPORTED;
  const NetPlan plan = plan_net(*variant, batch, sizeof(uint16_t));
  if (workspace_bytes < plan.bytes || reinterpret_cast<uintptr_t>(workspace) % kAlign != 0) return TFX_ERR_WORKSPACE;
  const int q = (int)variant->width_quarters;

  char* ws = static_cast<char*>(workspace);
  uint16_t* buf[2] = {reinterpret_cast<uint16_t*>(ws + plan.off_buf[0]), reinterpret_cast<uint16_t*>(ws + plan.off_buf[1])};
  float* partial = reinterpret_cast<float*>(ws + plan.off_partial);

  int64_t shape[4] = {batch, variant->image_size, variant->image_size, 3};
  const int64_t f0[4] = {3, 3, 3, kStemChannels * q / 4};
  int rc = tfx_conv2d_f16(input, shape, weights->conv0_w, f0, weights->conv0_b, 2, 2, TFX_PAD_SAME, TFX_ACT_RELU6,
                          buf[0], stream);
  if (rc) return rc;
  ConvGeom g;
  conv_geometry(shape, f0, 2, 2, TFX_PAD_SAME, false, &g);
  for (int i = 0; i < 4; ++i) shape[i] = g.out[i];
  int cur = 0;
  for (int b = 0; b < kBlocks; ++b) {
    const int64_t fd[4] = {3, 3, shape[3], 1};
    const int64_t cout = kChannels[b] * q / 4;
    uint16_t* const block_out = end_block == b + 1 ? features : buf[cur ^ 1];
    conv_geometry(shape, fd, kStrides[b], kStrides[b], TFX_PAD_SAME, true, &g);
    // large batch, early block: depthwise and pointwise layer in one filter-stationary launch (block_stream_f16.hip)
    if (separable_stream_f16_supported((int)batch, (int)shape[1], (int)shape[2], (int)shape[3], (int)cout, kStrides[b],
                                       (int)g.out[1], (int)g.out[2], buf[cur], weights->dw_w[b], weights->dw_b[b],
                                       weights->pw_w[b], weights->pw_b[b], block_out)) {
      rc = launch_separable_stream_f16(buf[cur], weights->dw_w[b], weights->dw_b[b], weights->pw_w[b], weights->pw_b[b],
                                       block_out, (int)batch, (int)shape[1], (int)shape[2], (int)shape[3], (int)cout,
                                       (int)g.out[1], (int)g.out[2], kStrides[b], (int)g.pad[0], (int)g.pad[2],
                                       TFX_ACT_RELU6, TFX_ACT_RELU6, static_cast<hipStream_t>(stream));
      if (rc) return rc;
      if (end_block == b + 1) return TFX_OK;
      for (int i = 0; i < 3; ++i) shape[i] = g.out[i];
      shape[3] = cout;
      cur ^= 1;
      continue;
    }
    rc = tfx_depthwise_conv2d_f16(buf[cur], shape, weights->dw_w[b], fd, weights->dw_b[b], kStrides[b], kStrides[b],
                                  TFX_PAD_SAME, TFX_ACT_RELU6, buf[cur ^ 1], stream);
    if (rc) return rc;
    for (int i = 0; i < 4; ++i) shape[i] = g.out[i];
    cur ^= 1;
    const int64_t fp[4] = {1, 1, shape[3], cout};
    rc = tfx_conv2d_f16(buf[cur], shape, weights->pw_w[b], fp, weights->pw_b[b], 1, 1, TFX_PAD_SAME, TFX_ACT_RELU6,
                        end_block == b + 1 ? features : buf[cur ^ 1], stream);
    if (rc) return rc;
    if (end_block == b + 1) return TFX_OK;
    shape[3] = cout;
    cur ^= 1;
  }
  return launch_pool_fc_softmax_f16(buf[cur], weights->fc_w, weights->fc_b, partial, logits, probs, (int)batch,
                                    (int)(shape[1] * shape[2]), (int)shape[3], (int)variant->classes,
                                    static_cast<hipStream_t>(stream));
}

}  // namespace

extern "C" {

int tfx_mobilenet_v1_forward_f16(const tfx_mobilenet_v1_variant* variant, const uint16_t* input, int64_t batch,
                                 const tfx_mobilenet_v1_weights_f16* weights, void* workspace,
                                 size_t workspace_bytes, uint16_t* probs, uint16_t* logits, void* stream) {
  return forward_f16_impl(variant, input, batch, weights, workspace, workspace_bytes, probs, logits, 0, nullptr, stream);
}

int tfx_mobilenet_v1_features_f16(const tfx_mobilenet_v1_variant* variant, const uint16_t* input, int64_t batch,
                                  const tfx_mobilenet_v1_weights_f16* weights, void* workspace, size_t workspace_bytes,
                                  int end_block, uint16_t* features, void* stream) {
  if (end_block < 1 || end_block > kBlocks) return TFX_ERR_ARG;
  if (features && reinterpret_cast<uintptr_t>(features) % 16 != 0) return TFX_ERR_ARG;
  return forward_f16_impl(variant, input, batch, weights, workspace, workspace_bytes, nullptr, nullptr, end_block, features,
                          stream);
}

}  // extern "C"
