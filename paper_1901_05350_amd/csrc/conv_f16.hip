// conv2d (direct and 3-channel stem), depthwiseConv2d and the MobileNet tail on 16-bit float
// storage for gfx950 (Section 4.1: 16-bit floating point textures; Section 3.9 for the network).
// Tensors are IEEE binary16; every kernel accumulates in fp32 and rounds its result once when it
// stores it.  The structure of each kernel is that of its fp32 counterpart with 8 channels
// (16 bytes) per lane instead of 4; products of two binary16 values use the mixed-precision FMA
// (binary16 operands, fp32 accumulator), so no separate conversions are issued.
#include "tfx_internal.h"

namespace tfx {
namespace {

typedef _Float16 half_t;
typedef _Float16 h8 __attribute__((ext_vector_type(8)));

constexpr int kXcds = 8;

__device__ __forceinline__ half_t to_half(float v) { return (half_t)v; }  // round to nearest even

// ---- general kernels: one thread per output element, any shape --------------------------------
__global__ __launch_bounds__(256) void conv2d_direct_f16_kernel(const half_t* __restrict__ x,
                                                                const half_t* __restrict__ w,
                                                                const half_t* __restrict__ bias,
                                                                half_t* __restrict__ y, int N, int H, int W, int Ci,
                                                                int fh, int fw, int Co, int OH, int OW, int sh, int sw,
                                                                int pt, int pl, int act, long long total) {
  for (long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (long long)gridDim.x * blockDim.x) {
    const int oc = (int)(idx % Co);
    long long r = idx / Co;
    const int ow = (int)(r % OW);
    r /= OW;
    const int oh = (int)(r % OH);
    const int n = (int)(r / OH);
    float acc = 0.f;
    for (int kh = 0; kh < fh; ++kh) {
      const int ih = oh * sh - pt + kh;
      if (ih < 0 || ih >= H) continue;
      for (int kw = 0; kw < fw; ++kw) {
        const int iw = ow * sw - pl + kw;
        if (iw < 0 || iw >= W) continue;
        const half_t* xp = x + (((size_t)n * H + ih) * W + iw) * Ci;
        const half_t* wp = w + ((size_t)(kh * fw + kw) * Ci) * Co + oc;
        for (int c = 0; c < Ci; ++c) acc = fmaf((float)xp[c], (float)wp[(size_t)c * Co], acc);
      }
    }
    if (bias) acc += (float)bias[oc];
    y[idx] = to_half(apply_act(acc, act));
  }
}

__global__ __launch_bounds__(256) void depthwise_generic_f16_kernel(const half_t* __restrict__ x,
                                                                    const half_t* __restrict__ w,
                                                                    const half_t* __restrict__ bias,
                                                                    half_t* __restrict__ y, int N, int H, int W, int C,
                                                                    int fh, int fw, int mult, int OH, int OW, int sh,
                                                                    int sw, int pt, int pl, int act, long long total) {
  const int OC = C * mult;
  for (long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (long long)gridDim.x * blockDim.x) {
    const int oc = (int)(idx % OC);
    long long r = idx / OC;
    const int ow = (int)(r % OW);
    r /= OW;
    const int oh = (int)(r % OH);
    const int n = (int)(r / OH);
    const int c = oc / mult, q = oc % mult;
    float acc = 0.f;
    for (int kh = 0; kh < fh; ++kh) {
      const int ih = oh * sh - pt + kh;
      if (ih < 0 || ih >= H) continue;
      for (int kw = 0; kw < fw; ++kw) {
        const int iw = ow * sw - pl + kw;
        if (iw < 0 || iw >= W) continue;
        acc = fmaf((float)x[(((size_t)n * H + ih) * W + iw) * C + c],
                   (float)w[((size_t)(kh * fw + kw) * C + c) * mult + q], acc);
      }
    }
    if (bias) acc += (float)bias[oc];
    y[idx] = to_half(apply_act(acc, act));
  }
}

// ---- depthwise 3x3, multiplier 1, C % 8 == 0, stride S in both dims ----------------------------
// A lane owns 8 consecutive channels of one output column and RS consecutive output rows; all
// (RS-1)*S+3 input rows x 3 taps are loaded (16 bytes each) before the first multiply.
template <int S, int RS>
__global__ __launch_bounds__(256) void depthwise3x3_f16_kernel(const half_t* __restrict__ x,
                                                               const half_t* __restrict__ w,
                                                               const half_t* __restrict__ bias, half_t* __restrict__ y,
                                                               int H, int W, int C8, int OH, int OW, int pt, int pl,
                                                               int act, int strips, int total) {
  constexpr int IR = (RS - 1) * S + 3;
  int bid = blockIdx.x;
  {
    const int nb = gridDim.x, q = nb / kXcds, rem = nb % kXcds;
    const int xcd = bid % kXcds;
    bid = xcd * q + (xcd < rem ? xcd : rem) + bid / kXcds;
  }
  const int idx = bid * 256 + threadIdx.x;
  if (idx >= total) return;
  const int c8 = idx % C8;
  int r = idx / C8;
  const int ow = r % OW;
  r /= OW;
  const int strip = r % strips;
  const int n = r / strips;
  const int C = C8 * 8;

  const half_t* xn = x + (size_t)n * H * W * C + 8 * c8;
  const int iw0 = ow * S - pl;
  const bool in0 = iw0 >= 0 && iw0 < W, in1 = iw0 + 1 >= 0 && iw0 + 1 < W, in2 = iw0 + 2 >= 0 && iw0 + 2 < W;
  const int oh0 = strip * RS;
  const int ih0 = oh0 * S - pt;

  h8 win[IR][3];
  const h8 z = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
  for (int i = 0; i < IR; ++i) {
    const int ih = ih0 + i;
    const bool rok = ih >= 0 && ih < H;
    const half_t* p = xn + ((long long)ih * W + iw0) * C;
    win[i][0] = (rok && in0) ? *reinterpret_cast<const h8*>(p) : z;
    win[i][1] = (rok && in1) ? *reinterpret_cast<const h8*>(p + C) : z;
    win[i][2] = (rok && in2) ? *reinterpret_cast<const h8*>(p + 2 * C) : z;
  }
  typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
  u32x4 wraw[9];
#pragma unroll
  for (int t = 0; t < 9; ++t) wraw[t] = *reinterpret_cast<const u32x4*>(w + (size_t)t * C + 8 * c8);
  h8 bv = z;
  if (bias) bv = *reinterpret_cast<const h8*>(bias + 8 * c8);
  const ActClamp clamp = make_act(act);

#pragma unroll
  for (int o = 0; o < RS; ++o) {
    if (oh0 + o >= OH) break;
    // The filter stays packed (36 registers): the empty asm makes its value opaque per output row, so the
    // binary16 -> fp32 conversions are not hoisted into 72 more registers; the mixed FMA reads binary16 directly.
    h8 wt[9];
#pragma unroll
    for (int t = 0; t < 9; ++t) {
      asm volatile("" : "+v"(wraw[t]));
      wt[t] = __builtin_bit_cast(h8, wraw[t]);
    }
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = (float)bv[e];
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
      for (int kw = 0; kw < 3; ++kw)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = fmaf((float)win[o * S + kh][kw][e], (float)wt[kh * 3 + kw][e], acc[e]);
    h8 out;
#pragma unroll
    for (int e = 0; e < 8; ++e) out[e] = to_half(apply_act(acc[e], clamp));
    *reinterpret_cast<h8*>(y + (((size_t)n * OH + oh0 + o) * OW + ow) * C + 8 * c8) = out;
  }
}

template <int S, int RS>
int launch_dw3x3_f16(const half_t* x, const half_t* w, const half_t* bias, half_t* y, int n, int h, int wd, int c8,
                     int oh, int ow, int pt, int pl, int act, hipStream_t stream) {
  const int strips = (oh + RS - 1) / RS;
  const long long total = (long long)n * strips * ow * c8;
  if (total > 0x7fffff00LL) return TFX_ERR_UNSUPPORTED;
  const unsigned blocks = (unsigned)((total + 255) / 256);
  hipLaunchKernelGGL((depthwise3x3_f16_kernel<S, RS>), dim3(blocks), dim3(256), 0, stream, x, w, bias, y, h, wd, c8, oh,
                     ow, pt, pl, act, strips, (int)total);
  return check_launch();
}

// ---- stem: 3x3 filter, 3 input channels, CO output channels (CO % 8 == 0, CO <= 64) ------------
// A thread computes 8 consecutive output channels of one output pixel (one 16-byte store); the
// 27 x CO filter is converted to fp32 once and kept in LDS; the 27 input values are fetched with
// unconditional loads from clamped addresses.
template <int CO>
__global__ __launch_bounds__(256) void conv2d_stem_f16_kernel(const half_t* __restrict__ x,
                                                              const half_t* __restrict__ w,
                                                              const half_t* __restrict__ bias, half_t* __restrict__ y,
                                                              int N, int H, int W, int OH, int OW, int sh, int sw,
                                                              int pt, int pl, int act, int total) {
  constexpr int G = CO / 8;
  constexpr int WPT = (27 * CO + 255) / 256;
  __shared__ __align__(16) float wl[27 * CO];
  int idx = blockIdx.x * 256 + threadIdx.x;
  const bool live = idx < total;
  if (!live) idx = total - 1;
  const int g = idx % G;
  int r = idx / G;
  const int ow = r % OW;
  r /= OW;
  const int oh = r % OH;
  const int n = r / OH;

  half_t wreg[WPT];
#pragma unroll
  for (int i = 0; i < WPT; ++i) {
    const int e = threadIdx.x + i * 256;
    wreg[i] = w[e < 27 * CO ? e : 27 * CO - 1];
  }
  float acc[8];
#pragma unroll
  for (int o = 0; o < 8; ++o) acc[o] = bias ? (float)bias[8 * g + o] : 0.f;
  float xv[27];
#pragma unroll
  for (int kh = 0; kh < 3; ++kh) {
    const int ih = oh * sh - pt + kh;
    const int ihc = min(max(ih, 0), H - 1);
#pragma unroll
    for (int kw = 0; kw < 3; ++kw) {
      const int iw = ow * sw - pl + kw;
      const int iwc = min(max(iw, 0), W - 1);
      const bool ok = ih == ihc && iw == iwc;
      const half_t* xp = x + (((size_t)n * H + ihc) * W + iwc) * 3;
#pragma unroll
      for (int c = 0; c < 3; ++c) {
        const float v = (float)xp[c];
        xv[(kh * 3 + kw) * 3 + c] = ok ? v : 0.f;
      }
    }
  }
#pragma unroll
  for (int i = 0; i < WPT; ++i) {
    const int e = threadIdx.x + i * 256;
    if (e < 27 * CO) wl[e] = (float)wreg[i];
  }
  __syncthreads();
  if (!live) return;

#pragma unroll
  for (int t = 0; t < 27; ++t) {
    const float4 w0 = *reinterpret_cast<const float4*>(&wl[t * CO + 8 * g]);
    const float4 w1 = *reinterpret_cast<const float4*>(&wl[t * CO + 8 * g + 4]);
    acc[0] = fmaf(xv[t], w0.x, acc[0]);
    acc[1] = fmaf(xv[t], w0.y, acc[1]);
    acc[2] = fmaf(xv[t], w0.z, acc[2]);
    acc[3] = fmaf(xv[t], w0.w, acc[3]);
    acc[4] = fmaf(xv[t], w1.x, acc[4]);
    acc[5] = fmaf(xv[t], w1.y, acc[5]);
    acc[6] = fmaf(xv[t], w1.z, acc[6]);
    acc[7] = fmaf(xv[t], w1.w, acc[7]);
  }
  h8 out;
#pragma unroll
  for (int o = 0; o < 8; ++o) out[o] = to_half(apply_act(acc[o], act));
  *reinterpret_cast<h8*>(y + (((size_t)n * OH + oh) * OW + ow) * CO + 8 * g) = out;
}

// The stem on the matrix cores for 32 filters: K = 27 padded to 32 is one v_mfma_f32_16x16x32_f16 per 16 output
// channels and 16-pixel slab of an output row (channels as the first operand's rows, pixels as the second's
// columns).  Lane (li = l % 16, q = l / 16) keeps filter values k = 8q .. 8q + 7 of channels li and 16 + li in
// registers and loads input values k = 8q .. 8q + 7 of pixel li's 3 x 3 x 3 window (k = (kh * 3 + kw) * 3 + c)
// straight from memory: slabs whose windows lie inside the image with unconditional loads at constant per-lane
// offsets, slabs on a border with per-tap checks.  A wavefront walks over slabs with a scalar (n, oh, segment)
// counter advanced with carries.  Its 16 x 32 results pass through a private LDS strip and leave as one 16-byte
// store per lane (1 KB contiguous per slab).
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void conv2d_stem_mfma_f16_kernel(const half_t* __restrict__ x,
                                                                   const half_t* __restrict__ w,
                                                                   const half_t* __restrict__ bias,
                                                                   half_t* __restrict__ y, int N, int H, int W, int OH,
                                                                   int OW, int sh, int sw, int pt, int pl, int act) {
  constexpr int CO = 32, LS = CO + 8;
  __shared__ __align__(16) half_t strips[4][16 * LS];
  const int lane = threadIdx.x % 64, li = lane % 16, q = lane / 16;
  const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x / 64);
  half_t* strip = strips[wave];
  const int segs = (OW + 15) / 16;
  const int stride = (int)gridDim.x * 4;
  const int first = (int)blockIdx.x * 4 + wave;
  int seg = first % segs, oh = (first / segs) % OH, n = first / segs / OH;
  const int d_seg = stride % segs, d_oh = (stride / segs) % OH, d_n = stride / segs / OH;

  int kh[8], kw[8], dk[8];
  h8 wr[2];
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    const int k = 8 * q + t;
    const bool valid = k < 27;
    const int kc = valid ? k : 26;
    kh[t] = kc / 9;
    kw[t] = (kc % 9) / 3;
    dk[t] = (kh[t] * W + kw[t]) * 3 + kc % 3;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const half_t v = w[kc * CO + 16 * j + li];
      wr[j][t] = valid ? v : (half_t)0.f;
    }
  }
  float bv[2][4];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int e = 0; e < 4; ++e) bv[j][e] = bias ? (float)bias[16 * j + 4 * q + e] : 0.f;
  const ActClamp clamp = make_act(act);

  while (n < N) {
    const long long row = (long long)n * OH + oh;
    const int ow = min(seg * 16 + li, OW - 1);  // pixels past the row's end repeat the last one (not stored)
    const int ih0 = oh * sh - pt, iw0 = ow * sw - pl;
    const half_t* xb = x + (((long long)n * H + ih0) * W + iw0) * 3;  // tap (0, 0); outside x on a border
    const int iw_first = seg * 16 * sw - pl, iw_last = min(seg * 16 + 15, OW - 1) * sw - pl + 2;
    const bool interior = ih0 >= 0 && ih0 + 2 < H && iw_first >= 0 && iw_last < W;
    h8 xv;
    if (interior) {
#pragma unroll
      for (int t = 0; t < 8; ++t) xv[t] = xb[dk[t]];
#pragma unroll
      for (int t = 3; t < 8; ++t) xv[t] = q == 3 ? (half_t)0.f : xv[t];  // padding k = 27 .. 31: zero, not 0 * x
    } else {
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const int ih = ih0 + kh[t], iw = iw0 + kw[t];
        const bool ok = ih >= 0 && ih < H && iw >= 0 && iw < W && !(t >= 3 && q == 3);
        const half_t v = *(ok ? xb + dk[t] : x);
        xv[t] = ok ? v : (half_t)0.f;
      }
    }
    f32x4 acc[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
      acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wr[j], xv, zero, 0, 0, 0);
    }
    // lane (li, q) holds channels 16j + 4q .. + 3 of pixel li: through the strip to whole lines
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      h4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = to_half(apply_act(acc[j][e] + bv[j][e], clamp));
      *reinterpret_cast<h4*>(strip + li * LS + 16 * j + 4 * q) = o;
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    {
      const int r = lane / 4, c = 8 * (lane % 4);
      const h8 v = *reinterpret_cast<const h8*>(strip + r * LS + c);
      if (seg * 16 + r < OW) *reinterpret_cast<h8*>(y + ((row * OW + seg * 16 + r) * CO + c)) = v;
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    seg += d_seg;
    const int c1 = seg >= segs ? 1 : 0;
    seg -= c1 * segs;
    oh += d_oh + c1;
    const int c2 = oh >= OH ? 1 : 0;
    oh -= c2 * OH;
    n += d_n + c2;
  }
}

// ---- MobileNet tail: global average pool (rounded to binary16) fused into the fully connected
// layer, split over K into fp32 partial sums; then bias, logits (binary16) and softmax of those --
constexpr int kFcSlices = 32;
constexpr int kFcKMax = 32;
constexpr int kFcBatchMax = 4;

__global__ __launch_bounds__(256) void pool_fc_partial_f16_kernel(const half_t* __restrict__ a,
                                                                  const half_t* __restrict__ w,
                                                                  float* __restrict__ partial, int n, int hw, int k,
                                                                  int classes, int kslice) {
  const int j = blockIdx.x * 256 + threadIdx.x;
  const int slice = blockIdx.y;
  const int n0 = blockIdx.z * kFcBatchMax;
  const int nb = min(kFcBatchMax, n - n0);
  const int k0 = slice * kslice;
  const int kn = min(kslice, k - k0);
  __shared__ float ps[kFcBatchMax][kFcKMax];

  float wv[kFcKMax];
#pragma unroll
  for (int kk = 0; kk < kFcKMax; ++kk)
    wv[kk] = (kk < kn && j < classes) ? (float)w[(size_t)(k0 + kk) * classes + j] : 0.f;

  {
    constexpr int kPixPerLane = 8;  // hw <= 64
    const int kk = threadIdx.x % kFcKMax, p0 = threadIdx.x / kFcKMax;
    __shared__ float red[kFcBatchMax][8][kFcKMax];
    const int kc = kk < kn ? kk : 0;
#pragma unroll
    for (int b = 0; b < kFcBatchMax; ++b) {
      const int bc = b < nb ? b : 0;
      const half_t* ap = a + ((size_t)(n0 + bc) * hw) * k + k0 + kc;
      float v[kPixPerLane];
#pragma unroll
      for (int q = 0; q < kPixPerLane; ++q) {
        const int p = p0 + 8 * q;
        v[q] = (float)ap[(size_t)(p < hw ? p : hw - 1) * k];
      }
      float acc = 0.f;
#pragma unroll
      for (int q = 0; q < kPixPerLane; ++q) acc += (p0 + 8 * q < hw) ? v[q] : 0.f;
      red[b][p0][kk] = (b < nb && kk < kn) ? acc : 0.f;
    }
    __syncthreads();
    if (threadIdx.x < kFcBatchMax * kFcKMax) {
      const int b = threadIdx.x / kFcKMax, c = threadIdx.x % kFcKMax;
      float s = 0.f;
#pragma unroll
      for (int q = 0; q < 8; ++q) s += red[b][q][c];
      ps[b][c] = (float)to_half(s / (float)hw);  // the pooled vector is a binary16 tensor
    }
    __syncthreads();
  }
  if (j >= classes) return;
  float acc[kFcBatchMax];
#pragma unroll
  for (int b = 0; b < kFcBatchMax; ++b) acc[b] = 0.f;
#pragma unroll
  for (int kk = 0; kk < kFcKMax; ++kk) {
#pragma unroll
    for (int b = 0; b < kFcBatchMax; ++b) acc[b] = fmaf(ps[b][kk], wv[kk], acc[b]);
  }
  for (int b = 0; b < nb; ++b) partial[((size_t)slice * n + n0 + b) * classes + j] = acc[b];
}

__device__ __forceinline__ float block_reduce(float v, bool is_max, float* scratch) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const float o = __shfl_xor(v, off, 64);
    v = is_max ? fmaxf(v, o) : v + o;
  }
  const int wave = threadIdx.x / 64;
  __syncthreads();
  if (threadIdx.x % 64 == 0) scratch[wave] = v;
  __syncthreads();
  float r = scratch[0];
  for (int i = 1; i < 4; ++i) r = is_max ? fmaxf(r, scratch[i]) : r + scratch[i];
  return r;
}

// Global average pool alone, in front of the fully connected layer as a GEMM: workgroup
// (image, 256 channels), thread (pixel group p0 of 8, 8 channels): 16-byte loads, fp32 sums, one rounding.
__global__ __launch_bounds__(256) void pool_f16_kernel(const half_t* __restrict__ a, half_t* __restrict__ pooled, int hw,
                                                       int k) {
  typedef _Float16 h8 __attribute__((ext_vector_type(8)));
  __shared__ float red[8][32][8];
  const int img = blockIdx.y, c8 = threadIdx.x % 32, p0 = threadIdx.x / 32;
  const int ch = 256 * blockIdx.x + 8 * c8;
  const bool live = ch < k;  // k % 8 == 0
  const half_t* const ap = a + (size_t)img * hw * k + (live ? ch : 0);
  h8 v[8];  // hw <= 64
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int p = p0 + 8 * i;
    v[i] = *reinterpret_cast<const h8*>(ap + (size_t)(p < hw ? p : hw - 1) * k);
  }
  float s[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int i = 0; i < 8; ++i)
    if (p0 + 8 * i < hw) {
#pragma unroll
      for (int e = 0; e < 8; ++e) s[e] += (float)v[i][e];
    }
#pragma unroll
  for (int e = 0; e < 8; ++e) red[p0][c8][e] = s[e];
  __syncthreads();
  if (p0 == 0 && live) {
    h8 o;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float t = 0.f;
#pragma unroll
      for (int g = 0; g < 8; ++g) t += red[g][c8][e];
      o[e] = to_half(t / (float)hw);
    }
    *reinterpret_cast<h8*>(pooled + (size_t)img * k + ch) = o;
  }
}

constexpr int kMaxPerThread = 4;  // classes <= 1024
// logits_in == nullptr: the logits are the sum of the K-slice partial sums plus the bias, rounded to binary16 (and
// written to `logits` if asked for); otherwise they are read from logits_in.
__global__ __launch_bounds__(256) void softmax_f16_kernel(const float* __restrict__ partial,
                                                          const half_t* __restrict__ bias, half_t* __restrict__ logits,
                                                          half_t* __restrict__ probs, int n, int classes,
                                                          const half_t* __restrict__ logits_in) {
  __shared__ float scratch[4];
  const int img = blockIdx.x;
  float l[kMaxPerThread];
  float mx = -INFINITY;
#pragma unroll
  for (int i = 0; i < kMaxPerThread; ++i) {
    const int j = threadIdx.x + 256 * i;
    l[i] = -INFINITY;
    if (j < classes && logits_in != nullptr) {
      l[i] = (float)logits_in[(size_t)img * classes + j];
      mx = fmaxf(mx, l[i]);
    } else if (j < classes) {
      float part[kFcSlices];
#pragma unroll
      for (int s = 0; s < kFcSlices; ++s) part[s] = partial[((size_t)s * n + img) * classes + j];
      float v = bias ? (float)bias[j] : 0.f;
#pragma unroll
      for (int s = 0; s < kFcSlices; ++s) v += part[s];
      const half_t lh = to_half(v);  // the logits are a binary16 tensor; the softmax is taken of those
      if (logits) logits[(size_t)img * classes + j] = lh;
      l[i] = (float)lh;
      mx = fmaxf(mx, l[i]);
    }
  }
  mx = block_reduce(mx, true, scratch);
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < kMaxPerThread; ++i) {
    const int j = threadIdx.x + 256 * i;
    if (j < classes) {
      l[i] = __expf(l[i] - mx);
      sum += l[i];
    }
  }
  sum = block_reduce(sum, false, scratch);
  const float inv = 1.0f / sum;
#pragma unroll
  for (int i = 0; i < kMaxPerThread; ++i) {
    const int j = threadIdx.x + 256 * i;
    if (j < classes) probs[(size_t)img * classes + j] = to_half(l[i] * inv);
  }
}

inline const half_t* H(const uint16_t* p) { return reinterpret_cast<const half_t*>(p); }
inline half_t* H(uint16_t* p) { return reinterpret_cast<half_t*>(p); }

}  // namespace

int launch_conv2d_direct_f16(const uint16_t* x, const uint16_t* w, const uint16_t* bias, uint16_t* y, int n, int h,
                             int wd, int ci, int fh, int fw, int co, int oh, int ow, int sh, int sw, int pt, int pl,
                             int act, hipStream_t stream) {
  const long long total = (long long)n * oh * ow * co;
  long long blocks = (total + 255) / 256;
  if (blocks > 256 * 64) blocks = 256 * 64;
  hipLaunchKernelGGL(conv2d_direct_f16_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, H(x), H(w), H(bias), H(y),
                     n, h, wd, ci, fh, fw, co, oh, ow, sh, sw, pt, pl, act, total);
  return check_launch();
}

bool conv2d_stem_f16_supported(int ci, int fh, int fw, int co, const void* y) {
  return ci == 3 && fh == 3 && fw == 3 && (co == 8 || co == 16 || co == 24 || co == 32) &&
         reinterpret_cast<uintptr_t>(y) % 16 == 0;
}

int launch_conv2d_stem_f16(const uint16_t* x, const uint16_t* w, const uint16_t* bias, uint16_t* y, int n, int h,
                           int wd, int co, int oh, int ow, int sh, int sw, int pt, int pl, int act,
                           hipStream_t stream) {
  if (co == 32) {  // the matrix-core form (y is 16-byte aligned: conv2d_stem_f16_supported)
    const long long slabs = (long long)n * oh * ((ow + 15) / 16);
    if (slabs > 0x3fffffffLL) return TFX_ERR_UNSUPPORTED;
    long long blocks = (slabs + 3) / 4;
    if (blocks > 256 * 8) blocks = 256 * 8;  // 8 workgroups of 4 wavefronts per CU, then the slab loop
    hipLaunchKernelGGL(conv2d_stem_mfma_f16_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, H(x), H(w), H(bias),
                       H(y), n, h, wd, oh, ow, sh, sw, pt, pl, act);
    return check_launch();
  }
  const long long total = (long long)n * oh * ow * (co / 8);
  if (total > 0x7fffffffLL) return TFX_ERR_UNSUPPORTED;
  const unsigned blocks = (unsigned)((total + 255) / 256);
#define TFX_STEM16(CO)                                                                                          \
  hipLaunchKernelGGL(conv2d_stem_f16_kernel<CO>, dim3(blocks), dim3(256), 0, stream, H(x), H(w), H(bias), H(y), n, \
                     h, wd, oh, ow, sh, sw, pt, pl, act, (int)total)
  switch (co) {
    case 8: TFX_STEM16(8); break;
    case 16: TFX_STEM16(16); break;
    case 24: TFX_STEM16(24); break;
    case 32: TFX_STEM16(32); break;
    default: return TFX_ERR_UNSUPPORTED;
  }
#undef TFX_STEM16
  return check_launch();
}

int launch_depthwise_f16(const uint16_t* x16, const uint16_t* w16, const uint16_t* bias16, uint16_t* y16, int n, int h,
                         int wd, int c, int fh, int fw, int mult, int oh, int ow, int sh, int sw, int pt, int pl,
                         int act, hipStream_t stream) {
  const half_t *x = H(x16), *w = H(w16), *bias = H(bias16);
  half_t* y = H(y16);
  const bool aligned = reinterpret_cast<uintptr_t>(x) % 16 == 0 && reinterpret_cast<uintptr_t>(w) % 16 == 0 &&
                       reinterpret_cast<uintptr_t>(y) % 16 == 0 &&
                       (bias == nullptr || reinterpret_cast<uintptr_t>(bias) % 16 == 0);
  if (fh == 3 && fw == 3 && mult == 1 && c % 8 == 0 && sh == sw && (sh == 1 || sh == 2) && aligned) {
    const int c8 = c / 8;
    const long long px = (long long)n * oh * ow * c8;  // threads at one row per thread
    const long long want = 256LL * 256 * 4;            // about 4 workgroups per CU
    if (sh == 1) {
      if (px / 6 >= want) return launch_dw3x3_f16<1, 6>(x, w, bias, y, n, h, wd, c8, oh, ow, pt, pl, act, stream);
      if (px / 4 >= want) return launch_dw3x3_f16<1, 4>(x, w, bias, y, n, h, wd, c8, oh, ow, pt, pl, act, stream);
      if (px / 2 >= want / 4) return launch_dw3x3_f16<1, 2>(x, w, bias, y, n, h, wd, c8, oh, ow, pt, pl, act, stream);
      return launch_dw3x3_f16<1, 1>(x, w, bias, y, n, h, wd, c8, oh, ow, pt, pl, act, stream);
    }
    if (px / 2 >= want / 4) return launch_dw3x3_f16<2, 2>(x, w, bias, y, n, h, wd, c8, oh, ow, pt, pl, act, stream);
    return launch_dw3x3_f16<2, 1>(x, w, bias, y, n, h, wd, c8, oh, ow, pt, pl, act, stream);
  }
  const long long total = (long long)n * oh * ow * c * mult;
  long long blocks = (total + 255) / 256;
  if (blocks > 256 * 64) blocks = 256 * 64;
  hipLaunchKernelGGL(depthwise_generic_f16_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, x, w, bias, y, n, h,
                     wd, c, fh, fw, mult, oh, ow, sh, sw, pt, pl, act, total);
  return check_launch();
}

int launch_pool_fc_softmax_f16(const uint16_t* a, const uint16_t* w, const uint16_t* bias, float* partial,
                               uint16_t* logits, uint16_t* probs, int n, int hw, int k, int classes,
                               hipStream_t stream) {
  if (classes > 256 * kMaxPerThread) return TFX_ERR_UNSUPPORTED;
  // With a class count that is a multiple of 8 (16-byte rows of the weights): pool, then the fully connected layer as
  // a GEMM (bias and the rounding of the logits in its epilogue), then the softmax of the stored logits -- three
  // launches, faster than the two below at every batch (those re-read the weights once per 4 images and write 32 n
  // classes partial sums).  The pooled vectors, and the logits if the caller does not ask for them, live where the
  // partial sums would.
  const size_t partial_bytes = (size_t)kFcSlices * n * classes * sizeof(float);
  if (hw <= 64 && k % 8 == 0 && classes % 8 == 0 && reinterpret_cast<uintptr_t>(a) % 16 == 0 &&
      ((size_t)n * k + 127) / 128 * 256 + (size_t)n * classes * 2 <= partial_bytes) {
    uint16_t* const pooled = reinterpret_cast<uint16_t*>(partial);
    uint16_t* const lg = logits ? logits : pooled + (((size_t)n * k + 127) / 128) * 128;
    hipLaunchKernelGGL(pool_f16_kernel, dim3((k + 255) / 256, n), dim3(256), 0, stream, H(a), H(pooled), hw, k);
    int rc = check_launch();
    if (rc) return rc;
    rc = launch_gemm_f16(pooled, w, lg, bias, 1, n, classes, k, true, false, TFX_ACT_NONE, stream);
    if (rc) return rc;
    hipLaunchKernelGGL(softmax_f16_kernel, dim3(n), dim3(256), 0, stream, (const float*)nullptr, (const half_t*)nullptr,
                       (half_t*)nullptr, H(probs), n, classes, H(lg));
    return check_launch();
  }
  const int kslice = (k + kFcSlices - 1) / kFcSlices;
  if (kslice > kFcKMax || hw > 64) return TFX_ERR_UNSUPPORTED;
  dim3 grid((classes + 255) / 256, kFcSlices, (n + kFcBatchMax - 1) / kFcBatchMax);
  hipLaunchKernelGGL(pool_fc_partial_f16_kernel, grid, dim3(256), 0, stream, H(a), H(w), partial, n, hw, k, classes,
                     kslice);
  int rc = check_launch();
  if (rc) return rc;
  hipLaunchKernelGGL(softmax_f16_kernel, dim3(n), dim3(256), 0, stream, (const float*)partial, H(bias), H(logits),
                     H(probs), n, classes, (const half_t*)nullptr);
  return check_launch();
}

}  // namespace tfx
