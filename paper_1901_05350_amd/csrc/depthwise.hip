// depthwiseConv2d for gfx950, NHWC x [fh,fw,C,mult], fused bias + activation.
//
// The op does 9 multiply-adds per 8 bytes moved (3x3, stride 1), so it is bound by HBM
// traffic, not arithmetic: every input element should cross the memory bus once.
// Fast path (3x3, multiplier 1, C % 4 == 0, stride 1 or 2 in both dims): a lane owns four
// consecutive channels (one 128-bit load / store) of one output column and walks down a
// strip of output rows, keeping the 3x3 window of float4 values in registers so that each
// new output row needs only the new input rows.  Lanes are ordered channel-quad fastest,
// then output column, so a wavefront's load is one contiguous run of the NHWC row; the
// three horizontal taps of neighbouring lanes overlap and are served from the L1 / L2.
#include "tfx_internal.h"

namespace tfx {
namespace {

__global__ __launch_bounds__(256) void depthwise_generic_kernel(const float* __restrict__ x,
                                                                const float* __restrict__ w,
                                                                const float* __restrict__ bias, float* __restrict__ y,
                                                                int N, int H, int W, int C, int fh, int fw, int mult,
                                                                int OH, int OW, int sh, int sw, int pt, int pl,
                                                                int act, long long total) {
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
        acc = fmaf(x[(((size_t)n * H + ih) * W + iw) * C + c], w[((size_t)(kh * fw + kw) * C + c) * mult + q], acc);
      }
    }
    if (bias) acc += bias[oc];
    y[idx] = apply_act(acc, act);
  }
}

__device__ __forceinline__ float4 fma4(const float4& a, const float4& b, const float4& c) {
  return make_float4(fmaf(a.x, b.x, c.x), fmaf(a.y, b.y, c.y), fmaf(a.z, b.z, c.z), fmaf(a.w, b.w, c.w));
}

// S = stride (1 or 2).  RS = output rows per thread strip.
template <int S>
__global__ __launch_bounds__(256) void depthwise3x3_kernel(const float* __restrict__ x, const float* __restrict__ w,
                                                           const float* __restrict__ bias, float* __restrict__ y,
                                                           int H, int W, int C4, int OH, int OW, int pt, int pl,
                                                           int act, int rs, int strips, long long total) {
  const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const int c4 = (int)(idx % C4);
  long long r = idx / C4;
  const int ow = (int)(r % OW);
  r /= OW;
  const int strip = (int)(r % strips);
  const int n = (int)(r / strips);
  const int C = C4 * 4;

  float4 wt[9];
#pragma unroll
  for (int t = 0; t < 9; ++t) wt[t] = *reinterpret_cast<const float4*>(w + (size_t)t * C + 4 * c4);
  const float4 bv = bias ? *reinterpret_cast<const float4*>(bias + 4 * c4) : make_float4(0.f, 0.f, 0.f, 0.f);

  const float* xn = x + (size_t)n * H * W * C + 4 * c4;
  const int iw0 = ow * S - pl;
  const bool in0 = iw0 >= 0 && iw0 < W, in1 = iw0 + 1 >= 0 && iw0 + 1 < W, in2 = iw0 + 2 >= 0 && iw0 + 2 < W;

  auto load_row = [&](int ih, float4(&row)[3]) {
    const float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
    row[0] = z;
    row[1] = z;
    row[2] = z;
    if (ih >= 0 && ih < H) {
      const float* p = xn + ((long long)ih * W + iw0) * C;
      if (in0) row[0] = *reinterpret_cast<const float4*>(p);
      if (in1) row[1] = *reinterpret_cast<const float4*>(p + C);
      if (in2) row[2] = *reinterpret_cast<const float4*>(p + 2 * C);
    }
  };

  const int oh0 = strip * rs;
  const int oh1 = min(oh0 + rs, OH);
  float4 win[3][3];
  int ih = oh0 * S - pt;
  load_row(ih, win[0]);
  if (S == 1) load_row(ih + 1, win[1]);
  for (int oh = oh0; oh < oh1; ++oh) {
    ih = oh * S - pt;
    if (S == 1) {
      load_row(ih + 2, win[2]);
    } else {
      load_row(ih + 1, win[1]);
      load_row(ih + 2, win[2]);
    }
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
      for (int kw = 0; kw < 3; ++kw) acc = fma4(win[kh][kw], wt[kh * 3 + kw], acc);
    float4 o;
    o.x = apply_act(acc.x + bv.x, act);
    o.y = apply_act(acc.y + bv.y, act);
    o.z = apply_act(acc.z + bv.z, act);
    o.w = apply_act(acc.w + bv.w, act);
    *reinterpret_cast<float4*>(y + (((size_t)n * OH + oh) * OW + ow) * C + 4 * c4) = o;
    if (S == 1) {
#pragma unroll
      for (int k = 0; k < 3; ++k) {
        win[0][k] = win[1][k];
        win[1][k] = win[2][k];
      }
    } else {
#pragma unroll
      for (int k = 0; k < 3; ++k) win[0][k] = win[2][k];
    }
  }
}

}  // namespace

int launch_depthwise(const float* x, const float* w, const float* bias, float* y, int n, int h, int wd, int c, int fh,
                     int fw, int mult, int oh, int ow, int sh, int sw, int pt, int pl, int act, hipStream_t stream) {
  const bool aligned = reinterpret_cast<uintptr_t>(x) % 16 == 0 && reinterpret_cast<uintptr_t>(w) % 16 == 0 &&
                       reinterpret_cast<uintptr_t>(y) % 16 == 0 &&
                       (bias == nullptr || reinterpret_cast<uintptr_t>(bias) % 16 == 0);
  if (fh == 3 && fw == 3 && mult == 1 && c % 4 == 0 && sh == sw && (sh == 1 || sh == 2) && aligned) {
    const int c4 = c / 4;
    // Strip length: long strips re-read fewer halo rows, short strips give more threads.
    // Aim for at least ~8 wavefronts per CU (256 CUs) before lengthening the strip.
    int rs = 8;
    while (rs > 1 && (long long)n * ((oh + rs - 1) / rs) * ow * c4 < 256LL * 8 * 64) rs >>= 1;
    const int strips = (oh + rs - 1) / rs;
    const long long total = (long long)n * strips * ow * c4;
    const long long blocks = (total + 255) / 256;
    if (blocks > 0x7fffffffLL) return TFX_ERR_UNSUPPORTED;
    if (sh == 1)
      hipLaunchKernelGGL(depthwise3x3_kernel<1>, dim3((unsigned)blocks), dim3(256), 0, stream, x, w, bias, y, h, wd, c4,
                         oh, ow, pt, pl, act, rs, strips, total);
    else
      hipLaunchKernelGGL(depthwise3x3_kernel<2>, dim3((unsigned)blocks), dim3(256), 0, stream, x, w, bias, y, h, wd, c4,
                         oh, ow, pt, pl, act, rs, strips, total);
    return check_launch();
  }
  const long long total = (long long)n * oh * ow * c * mult;
  long long blocks = (total + 255) / 256;
  if (blocks > 256 * 64) blocks = 256 * 64;
  hipLaunchKernelGGL(depthwise_generic_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, x, w, bias, y, n, h, wd, c,
                     fh, fw, mult, oh, ow, sh, sw, pt, pl, act, total);
  return check_launch();
}

}  // namespace tfx
