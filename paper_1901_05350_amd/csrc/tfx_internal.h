// Internal declarations shared by the HIP translation units of libtfx.
// Nothing here is part of the public ABI (that is include/tfx.h).
#ifndef TFX_INTERNAL_H_
#define TFX_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "../../include/tfx.h"

namespace tfx {

// Fused epilogue: bias first, then activation.  relu and relu6 are clamps ([0, +inf] and [0, 6]);
// kernels turn the enum into an on/off flag and an upper bound once and apply max / min per
// element.  With no activation the value passes through untouched (NaN and Inf included).  A NaN also
// passes through relu and relu6 (the hardware's max / min would return the other operand, i.e. turn a NaN
// into 0): an activation must not hide a poisoned value from the layers behind it, which is what the
// debug mode of Section 3.8 looks for.  -Inf clamps to 0, +Inf to the upper bound.
struct ActClamp {
  bool on;
  float hi;
};
__device__ __forceinline__ ActClamp make_act(int act) {
  ActClamp c;
  c.on = act != TFX_ACT_NONE;
  c.hi = act == TFX_ACT_RELU6 ? 6.0f : INFINITY;
  return c;
}
__device__ __forceinline__ float apply_act(float v, const ActClamp& c) {
  const float t = fminf(fmaxf(v, 0.0f), c.hi);
  return (c.on && v == v) ? t : v;
}
__device__ __forceinline__ float apply_act(float v, int act) { return apply_act(v, make_act(act)); }

typedef float floatx4 __attribute__((ext_vector_type(4)));

// Value held by the lane 8 places away within the lane's group of 16 (l % 16 <-> (l % 16) ^ 8): DPP row rotate by 8.
__device__ __forceinline__ float swap8(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x128, 0xf, 0xf, false));
}

// Bias + activation + store of NBLK 16-column blocks (NBLK even) of one 16-row slab.  After the MFMAs lane
// (li = l % 16, q = l / 16) holds columns 16j + 4q .. + 3 of row li for every block j; stored like that, an
// instruction would write 64-byte pieces of 16 rows (measured: half-line pieces cost 12 us of 72 on the
// 32 -> 64 layer).  Lanes li and li ^ 8 therefore trade blocks 2h + 1 / 2h first, so that the lanes with
// li < 8 hold block 2h of rows li and li + 8 and the others block 2h + 1 of rows li - 8 and li: two store
// instructions per block pair, each writing whole 128-byte lines of 8 rows.  bv[h]: bias of the lane's 4
// columns 32h + (li < 8 ? 0 : 16) + 4q .. + 3; yc: y + first column of block 0.
// CHECK = false: all 16 rows exist; the stores are then unconditional, which also lets the compiler count them
// when it waits for a later load (stores and loads share one in-order counter: behind stores it cannot count,
// every wait for a load would also wait for all earlier stores to be acknowledged).
template <int NBLK, bool CHECK>
__device__ __forceinline__ void store_slab(const floatx4 (&acc)[NBLK], const float4 (&bv)[NBLK / 2], float* yc, int n,
                                           int row0, int M, int li, int q, const ActClamp& clamp) {
  static_assert(NBLK % 2 == 0, "blocks are stored in pairs");
  const bool lo = li < 8;
  const int ra = row0 + (li & 7), rb = ra + 8;
#pragma unroll
  for (int h = 0; h < NBLK / 2; ++h) {
    float got[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) got[v] = swap8(lo ? acc[2 * h + 1][v] : acc[2 * h][v]);
    float4 oa, ob;
    oa.x = apply_act((lo ? acc[2 * h][0] : got[0]) + bv[h].x, clamp);
    oa.y = apply_act((lo ? acc[2 * h][1] : got[1]) + bv[h].y, clamp);
    oa.z = apply_act((lo ? acc[2 * h][2] : got[2]) + bv[h].z, clamp);
    oa.w = apply_act((lo ? acc[2 * h][3] : got[3]) + bv[h].w, clamp);
    ob.x = apply_act((lo ? got[0] : acc[2 * h + 1][0]) + bv[h].x, clamp);
    ob.y = apply_act((lo ? got[1] : acc[2 * h + 1][1]) + bv[h].y, clamp);
    ob.z = apply_act((lo ? got[2] : acc[2 * h + 1][2]) + bv[h].z, clamp);
    ob.w = apply_act((lo ? got[3] : acc[2 * h + 1][3]) + bv[h].w, clamp);
    const int col = 32 * h + (lo ? 0 : 16) + 4 * q;
    if (!CHECK || ra < M) *reinterpret_cast<float4*>(yc + (size_t)ra * n + col) = oa;
    if (!CHECK || rb < M) *reinterpret_cast<float4*>(yc + (size_t)rb * n + col) = ob;
  }
}

// The same store for accumulators that already hold the bias (they started from it).  The clamp is one
// median-of-three per value; that instruction, like max and min, drops a NaN, so NaNs are looked for on the side
// (one compare per pair of values, collected in scalar registers) and a block pair that holds one takes the exact
// form, through which a NaN passes.
// ya / yb: where this lane's two rows start (first column of block 0); oka / okb: whether they exist.
template <int NBLK>
__device__ __forceinline__ void store_rows_biased(const floatx4 (&acc)[NBLK], float* ya, float* yb, bool oka, bool okb,
                                                  int li, int q, const ActClamp& clamp) {
  static_assert(NBLK % 2 == 0, "blocks are stored in pairs");
  const bool lo = li < 8;
  const float lo_bound = clamp.on ? 0.f : -INFINITY;
  float a[NBLK / 2][4], b[NBLK / 2][4];
  unsigned long long nan = 0;
#pragma unroll
  for (int h = 0; h < NBLK / 2; ++h)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const float got = swap8(lo ? acc[2 * h + 1][v] : acc[2 * h][v]);
      a[h][v] = lo ? acc[2 * h][v] : got;
      b[h][v] = lo ? got : acc[2 * h + 1][v];
      nan |= __builtin_amdgcn_ballot_w64(__builtin_isunordered(a[h][v], b[h][v]));
    }
  auto store = [&](auto act1) {
#pragma unroll
    for (int h = 0; h < NBLK / 2; ++h) {
      const float4 oa = make_float4(act1(a[h][0]), act1(a[h][1]), act1(a[h][2]), act1(a[h][3]));
      const float4 ob = make_float4(act1(b[h][0]), act1(b[h][1]), act1(b[h][2]), act1(b[h][3]));
      const int col = 32 * h + (lo ? 0 : 16) + 4 * q;
      if (oka) *reinterpret_cast<float4*>(ya + col) = oa;
      if (okb) *reinterpret_cast<float4*>(yb + col) = ob;
    }
  };
  if (nan == 0) store([&](float v) { return __builtin_amdgcn_fmed3f(v, lo_bound, clamp.hi); });
  else store([&](float v) { return apply_act(v, clamp); });
}
template <int NBLK, bool CHECK>
__device__ __forceinline__ void store_slab_biased(const floatx4 (&acc)[NBLK], float* yc, int n, int row0, int M, int li,
                                                  int q, const ActClamp& clamp) {
  const int ra = row0 + (li & 7), rb = ra + 8;
  store_rows_biased<NBLK>(acc, yc + (size_t)ra * n, yc + (size_t)rb * n, !CHECK || ra < M, !CHECK || rb < M, li, q, clamp);
}

// ds_read_b128 serves 32 lanes at a time and is free of bank conflicts when their 16-byte pieces differ modulo 32
// (measured on gfx950: such patterns read at twice the rate of ones that only differ modulo 16 within 16 lanes).
// `piece(li, q)` is the piece index of lane (li = lane % 16, q = lane / 16) up to a constant: the fragment layouts of
// the 16 x 16 MFMAs read one row or pixel per li and consecutive pieces per q.
template <typename F>
constexpr bool conflict_free(F piece) {
  for (int half = 0; half < 2; ++half) {
    unsigned seen = 0;
    for (int li = 0; li < 16; ++li)
      for (int q = 2 * half; q < 2 * half + 2; ++q) {
        const unsigned bit = 1u << (piece(li, q) % 32);
        if (seen & bit) return false;
        seen |= bit;
      }
  }
  return true;
}

// Shape rule of one spatial dimension (see include/tfx.h); returns a tfx_status.
int out_extent(int64_t in, int64_t k, int64_t s, int pad, int64_t* out, int64_t* before, int64_t* after);

// C[b] = act(op(A[b]) * op(B[b]) + bias[col]) for b < batch.  a_kc: A is stored [M,K] (K contiguous),
// else [K,M].  b_kc: B is stored [N,K] (K contiguous), else [K,N].  bias may be null.
// Dimensions are validated by the callers; all fit in int32.
int launch_gemm(const float* a, const float* b, float* c, const float* bias, int batch, int m, int n, int k,
                bool a_kc, bool b_kc, int act, hipStream_t stream);

// conv2d as an implicit GEMM on the matrix cores: M = n*oh*ow, K = fh*fw*ci, N = co (any filter / stride).
int launch_conv2d_gemm(const float* x, const float* w, const float* bias, float* y, int n, int h, int wd, int ci, int fh,
                       int fw, int co, int oh, int ow, int sh, int sw, int pt, int pl, int act, hipStream_t stream);

// Filter-stationary pointwise conv for thin filters (K*N*4 <= 128 KB) and large M.
bool pointwise_stream_supported(int m, int k, int n, const void* x, const void* w, const void* bias, const void* y);
int launch_pointwise_stream(const float* x, const float* w, const float* bias, float* y, int m, int k, int n, int act,
                            hipStream_t stream);

// Direct convolution for any filter size / stride (one thread per output element).
int launch_conv2d_direct(const float* x, const float* w, const float* bias, float* y, int n, int h, int wd, int ci,
                         int fh, int fw, int co, int oh, int ow, int sh, int sw, int pt, int pl, int act,
                         hipStream_t stream);

// 3x3 stride-2 convolution with 3 input channels (the MobileNet stem).
bool conv2d_stem_supported(int ci, int fh, int fw, int co, int sh, int sw);
// zero_words / zero_count / zero_stride: optional: the kernel also clears zero_count 32-bit words, zero_stride
// words apart (matrix-core form only: 32 filters, 16-byte aligned y and bias).
int launch_conv2d_stem(const float* x, const float* w, const float* bias, float* y, int n, int h, int wd, int co,
                       int oh, int ow, int sh, int sw, int pt, int pl, int act, hipStream_t stream,
                       int* zero_words = nullptr, int zero_count = 0, int zero_stride = 1);

// The 28 x 28 ... 7 x 7 blocks, pool, fully connected layer and softmax of the batch-1 network (any of the four
// widths) as one persistent kernel (chain.hip).  chain_ws: chain_workspace_bytes() bytes, 256-byte aligned; its first
// chain_flag_words() words at a spacing of chain_flag_stride() words are zero when the kernel starts.  in0: the
// output of block 4 (in_hw x in_hw x 64 width_quarters).
bool chain_supported(int image_size, int width_quarters, int classes, long long batch);
bool chain_resident(int width_quarters);
size_t chain_workspace_bytes(int image_size, int classes, int width_quarters);
int chain_flag_words(int image_size, int classes, int width_quarters);
int chain_head_flag_base(int image_size, int classes);  // full width only: where the flags of blocks 2 - 4 as stages begin
int chain_flag_stride();
int chain_spin_limit();
// head_flags: flag words behind the chain kernel's own at the start of chain_ws (block_chain_flag_words).
// before(before_arg), if given, enqueues a launch that has to stay directly in front of the chain kernel on `stream`
// (it is called once the stream has been ordered behind other streams' chain kernels) and returns a tfx_status.
// first_block: 4 (the chain starts with block 5, in0 = the output of block 4) or 5 (block 6, in0 = output of block 5).
int launch_chain(const float* in0, int in_hw, const tfx_mobilenet_v1_weights* w, void* chain_ws, int head_flags,
                 float* probs, float* logits, int classes, int width_quarters, hipStream_t stream,
                 int (*before)(void*) = nullptr, void* before_arg = nullptr, int first_block = 4);
// fn(arg) enqueues a kernel of waiting workgroups on `stream`; the stream is first ordered behind the last such
// kernel of any other stream (two of them side by side could each hold the CUs the other's producers need).
int launch_ordered(hipStream_t stream, int (*fn)(void*), void* arg);

// Blocks 2 - 4 of a single full-width image (64 -> 128 /2, 128 -> 128, 128 -> 256 /2) as three stages of one launch
// that hand results over through flags (block.hip).  x: [h, w, 64]; b2_out, b3_out: [ceil(h/2), ceil(w/2), 128];
// y: [ceil(h/4), ceil(w/4), 256] (halvings round up).  flags: word 0 = failure word; block_chain_flag_words(h, w)
// words from flag_base on, block_chain_flag_stride() words apart, zero when the kernel starts.
int block_chain_flag_stride();
int block_chain_flag_words(int h, int w);
bool block_chain_supported(const void* x, const void* b2_out, const void* b3_out, const void* y,
                           const tfx_mobilenet_v1_weights* w);
int launch_block_chain(const float* x, float* b2_out, float* b3_out, float* y, int h, int w,
                       const tfx_mobilenet_v1_weights* wt, int* flags, int flag_base, int spin_limit, hipStream_t stream);

// One depthwise-separable block (depthwise 3x3 + bias + clamp, pointwise 1x1 + bias + clamp) of up to three images in
// one launch (block.hip): 32, 64 or 128 input channels (256 at stride 1), n a multiple of 64, 16-byte aligned pointers.
bool separable_block_supported(long long batch, int h, int w, int c, int n, int stride, const void* x, const void* dw_w,
                               const void* dw_b, const void* pw_w, const void* pw_b, const void* y);
int launch_separable_block(const float* x, const float* dw_w, const float* dw_b, const float* pw_w, const float* pw_b,
                           float* y, int batch, int h, int w, int c, int n, int oh, int ow, int stride, int pt, int pl,
                           int dw_act, int pw_act, hipStream_t stream);

// The stem (3x3 stride-2 convolution of the image [ih, iw, 3] to 32 channels, [h, w, 32]) and the first
// depthwise-separable block (stride 1, 32 -> n = 64 channels) of up to three images in one launch; every layer with
// bias + the activation `act`.  zero_words: as for launch_conv2d_stem.
bool stem_block_supported(long long batch, int ih, int iw, int stem_filters, int n, const void* image, const void* st_w,
                          const void* st_b, const void* dw_w, const void* dw_b, const void* pw_w, const void* pw_b,
                          const void* y);
int launch_stem_block(const float* image, const float* st_w, const float* st_b, const float* dw_w, const float* dw_b,
                      const float* pw_w, const float* pw_b, float* y, int batch, int ih, int iw, int h, int w, int st_pt,
                      int st_pl, int n, int act, hipStream_t stream, int* zero_words, int zero_count, int zero_stride);

// Depthwise convolution: generic kernel and the 3x3 / multiplier-1 / C%4==0 fast path.
int launch_depthwise(const float* x, const float* w, const float* bias, float* y, int n, int h, int wd, int c,
                     int fh, int fw, int mult, int oh, int ow, int sh, int sw, int pt, int pl, int act,
                     hipStream_t stream);

// MobileNet tail: global average pool of a [n,hw,k] map fused into the fully connected layer
// (split over K into `partial`), then bias + softmax.  logits may be null.
int launch_pool_fc_softmax(const float* a, const float* w, const float* bias, float* partial, float* logits,
                           float* probs, int n, int hw, int k, int classes, hipStream_t stream);
size_t fc_partial_floats(int n, int k, int classes);

// Element-wise c[i] = a[i] + b[i] for i < n, fp32 and IEEE binary16 storage (c may alias a or b).
int launch_add_f32(const float* a, const float* b, float* c, long long n, hipStream_t stream);
int launch_add_f16(const uint16_t* a, const uint16_t* b, uint16_t* c, long long n, hipStream_t stream);

// batchMatMul on IEEE binary16 storage with fp32 accumulation; arguments as launch_gemm, bias binary16.
int launch_gemm_f16(const uint16_t* a, const uint16_t* b, uint16_t* c, const uint16_t* bias, int batch, int m, int n,
                    int k, bool a_kc, bool b_kc, int act, hipStream_t stream);

// conv2d, depthwiseConv2d and the MobileNet tail on IEEE binary16 storage (fp32 accumulation).
int launch_conv2d_direct_f16(const uint16_t* x, const uint16_t* w, const uint16_t* bias, uint16_t* y, int n, int h,
                             int wd, int ci, int fh, int fw, int co, int oh, int ow, int sh, int sw, int pt, int pl,
                             int act, hipStream_t stream);
// conv2d on binary16 storage as an implicit GEMM on the matrix cores: channel counts multiples of 8, at most 32
// filter taps, 16-byte aligned x and filter.
bool conv2d_gemm_f16_supported(const void* x, const void* w, int ci, int fh, int fw, int co);
int launch_conv2d_gemm_f16(const uint16_t* x, const uint16_t* w, const uint16_t* bias, uint16_t* y, int n, int h, int wd,
                           int ci, int fh, int fw, int co, int oh, int ow, int sh, int sw, int pt, int pl, int act,
                           hipStream_t stream);
bool conv2d_stem_f16_supported(int ci, int fh, int fw, int co, const void* y);
int launch_conv2d_stem_f16(const uint16_t* x, const uint16_t* w, const uint16_t* bias, uint16_t* y, int n, int h,
                           int wd, int co, int oh, int ow, int sh, int sw, int pt, int pl, int act,
                           hipStream_t stream);
int launch_depthwise_f16(const uint16_t* x, const uint16_t* w, const uint16_t* bias, uint16_t* y, int n, int h, int wd,
                         int c, int fh, int fw, int mult, int oh, int ow, int sh, int sw, int pt, int pl, int act,
                         hipStream_t stream);
int launch_pool_fc_softmax_f16(const uint16_t* a, const uint16_t* w, const uint16_t* bias, float* partial,
                               uint16_t* logits, uint16_t* probs, int n, int hw, int k, int classes,
                               hipStream_t stream);

// Filter-stationary pointwise conv on binary16 storage for thin filters and large M.
bool pointwise_stream_f16_supported(int m, int k, int n, const void* x, const void* w, const void* y);
int launch_pointwise_stream_f16(const uint16_t* x, const uint16_t* w, const uint16_t* bias, uint16_t* y, int m, int k,
                                int n, int act, hipStream_t stream);
// The same with a filter too large for LDS or fewer rows (K = 64, 128, 256 or 512; N = 1, 2, 4, 8 or 16 slabs of 128
// columns; from 1536 rows on): a workgroup keeps one column slab (pointwise_slab_f16.hip).
bool pointwise_slab_f16_supported(int m, int k, int n, const void* x, const void* w, const void* y);
int launch_pointwise_slab_f16(const uint16_t* x, const uint16_t* w, const uint16_t* bias, uint16_t* y, int m, int k,
                              int n, int act, hipStream_t stream);

// 3x3 stride-1 conv2d on binary16 storage with the whole filter resident in LDS (few channels, many output pixels).
bool conv3x3_stream_f16_supported(long long m, long long x_elems, int ci, int fh, int fw, int co, int sh, int sw,
                                  const void* x, const void* w, const void* y);
int launch_conv3x3_stream_f16(const uint16_t* x, const uint16_t* w, const uint16_t* bias, uint16_t* y, int n, int h,
                              int wd, int ci, int co, int oh, int ow, int pt, int pl, int act, hipStream_t stream);

// A depthwise-separable block at large batch as one filter-stationary kernel (block_stream.hip).
bool separable_stream_supported(int batch, int h, int w, int c, int n, int stride, int oh, int ow, const void* x,
                                const void* dw_w, const void* dw_b, const void* pw_w, const void* pw_b, const void* y);
int launch_separable_stream(const float* x, const float* dw_w, const float* dw_b, const float* pw_w, const float* pw_b,
                            float* y, int batch, int h, int w, int c, int n, int oh, int ow, int stride, int pt, int pl,
                            int dw_act, int pw_act, hipStream_t stream);

// The same on binary16 storage (block_stream_f16.hip).
bool separable_stream_f16_supported(int batch, int h, int w, int c, int n, int stride, int oh, int ow, const void* x,
                                    const void* dw_w, const void* dw_b, const void* pw_w, const void* pw_b,
                                    const void* y);
int launch_separable_stream_f16(const uint16_t* x, const uint16_t* dw_w, const uint16_t* dw_b, const uint16_t* pw_w,
                                const uint16_t* pw_b, uint16_t* y, int batch, int h, int w, int c, int n, int oh, int ow,
                                int stride, int pt, int pl, int dw_act, int pw_act, hipStream_t stream);

inline int check_launch() { return hipGetLastError() == hipSuccess ? TFX_OK : TFX_ERR_LAUNCH; }

// A kernel that uses more than 64 KB of dynamic LDS has to be allowed to, once per device (the attribute
// belongs to the kernel's code object on the current device).  `done` is the caller's per-kernel bitmask of
// the devices already set up; callers launch on the current device.  Safe to call from several threads.
inline int allow_dynamic_lds(const void* kernel, size_t bytes, std::atomic<uint64_t>& done) {
  if (bytes <= 64 * 1024) return TFX_OK;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return TFX_ERR_LAUNCH;
  const uint64_t bit = (dev >= 0 && dev < 64) ? (1ull << dev) : 0;  // devices past 63 are set up on every call
  if (bit != 0 && (done.load(std::memory_order_acquire) & bit) != 0) return TFX_OK;
  if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess)
    return TFX_ERR_LAUNCH;
  done.fetch_or(bit, std::memory_order_release);
  return TFX_OK;
}

}  // namespace tfx

#endif  // TFX_INTERNAL_H_
