// depthwiseConv2d for gfx950, NHWC x [fh,fw,C,mult], fused bias + activation.
//
// The op does 9 multiply-adds per 8 bytes moved (3x3, stride 1), so it is bound by HBM
// traffic and by how many bytes each CU keeps in flight, not by arithmetic.
// Fast path (3x3, multiplier 1, C % 4 == 0, stride 1 or 2 in both dims): a lane owns four
// consecutive channels (one 128-bit load / store) of one output column and RS consecutive
// output rows.  It issues all of its (RS-1)*S+3 input rows x 3 taps of loads up front -- the
// whole register window is in flight at once -- then computes and stores its RS outputs.
// Lanes are ordered channel-quad fastest, then output column, so every wave-wide load is one
// contiguous run of an NHWC row; the horizontal taps of neighbouring lanes overlap and hit in
// L1.  Workgroup ids are remapped so that each XCD works on a contiguous range of images:
// the halo rows shared by vertically adjacent strips are then re-read from that XCD's L2
// instead of HBM (HBM fetch = input size, measured).
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

constexpr int kXcds = 8;

typedef float v4f __attribute__((ext_vector_type(4)));  // native vector: keeps loads 128-bit

// S = stride (1 or 2), RS = output rows per thread.
template <int S, int RS>
__global__ __launch_bounds__(256) void depthwise3x3_kernel(const float* __restrict__ x, const float* __restrict__ w,
                                                           const float* __restrict__ bias, float* __restrict__ y,
                                                           int H, int W, int C4, int OH, int OW, int pt, int pl,
                                                           int act, int strips, int total) {
  constexpr int IR = (RS - 1) * S + 3;  // input rows feeding RS output rows
  // hardware workgroup id b runs on XCD b % 8: give each XCD a contiguous range of logical ids
  int bid = blockIdx.x;
  {
    const int nb = gridDim.x, q = nb / kXcds, rem = nb % kXcds;
    const int xcd = bid % kXcds;
    bid = xcd * q + (xcd < rem ? xcd : rem) + bid / kXcds;
  }
  const int idx = bid * 256 + threadIdx.x;
  if (idx >= total) return;
  const int c4 = idx % C4;
  int r = idx / C4;
  const int ow = r % OW;
  r /= OW;
  const int strip = r % strips;
  const int n = r / strips;
  const int C = C4 * 4;

  const float* xn = x + (size_t)n * H * W * C + 4 * c4;
  const int iw0 = ow * S - pl;
  const bool in0 = iw0 >= 0 && iw0 < W, in1 = iw0 + 1 >= 0 && iw0 + 1 < W, in2 = iw0 + 2 >= 0 && iw0 + 2 < W;
  const int oh0 = strip * RS;
  const int ih0 = oh0 * S - pt;

  v4f win[IR][3];
  const v4f z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int i = 0; i < IR; ++i) {
    const int ih = ih0 + i;
    const bool rok = ih >= 0 && ih < H;
    const float* p = xn + ((long long)ih * W + iw0) * C;
    win[i][0] = (rok && in0) ? *reinterpret_cast<const v4f*>(p) : z;
    win[i][1] = (rok && in1) ? *reinterpret_cast<const v4f*>(p + C) : z;
    win[i][2] = (rok && in2) ? *reinterpret_cast<const v4f*>(p + 2 * C) : z;
  }
  v4f wt[9];
#pragma unroll
  for (int t = 0; t < 9; ++t) wt[t] = *reinterpret_cast<const v4f*>(w + (size_t)t * C + 4 * c4);
  v4f bv = z;
  if (bias) bv = *reinterpret_cast<const v4f*>(bias + 4 * c4);
  const ActClamp clamp = make_act(act);

#pragma unroll
  for (int o = 0; o < RS; ++o) {
    if (oh0 + o >= OH) break;
    v4f acc = bv;
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
      for (int kw = 0; kw < 3; ++kw) acc += win[o * S + kh][kw] * wt[kh * 3 + kw];
    v4f out;
#pragma unroll
    for (int e = 0; e < 4; ++e) out[e] = apply_act(acc[e], clamp);
    *reinterpret_cast<v4f*>(y + (((size_t)n * OH + oh0 + o) * OW + ow) * C + 4 * c4) = out;
  }
}

template <int S, int RS>
int launch_dw3x3(const float* x, const float* w, const float* bias, float* y, int n, int h, int wd, int c4, int oh,
                 int ow, int pt, int pl, int act, hipStream_t stream) {
  const int strips = (oh + RS - 1) / RS;
  const long long total = (long long)n * strips * ow * c4;
  if (total > 0x7fffff00LL) return TFX_ERR_UNSUPPORTED;  // thread index is 32-bit in the kernel
  const unsigned blocks = (unsigned)((total + 255) / 256);
  hipLaunchKernelGGL((depthwise3x3_kernel<S, RS>), dim3(blocks), dim3(256), 0, stream, x, w, bias, y, h, wd, c4, oh,
                     ow, pt, pl, act, strips, (int)total);
  return check_launch();
}

}  // namespace

int launch_depthwise(const float* x, const float* w, const float* bias, float* y, int n, int h, int wd, int c, int fh,
                     int fw, int mult, int oh, int ow, int sh, int sw, int pt, int pl, int act, hipStream_t stream) {
  const bool aligned = reinterpret_cast<uintptr_t>(x) % 16 == 0 && reinterpret_cast<uintptr_t>(w) % 16 == 0 &&
                       reinterpret_cast<uintptr_t>(y) % 16 == 0 &&
                       (bias == nullptr || reinterpret_cast<uintptr_t>(bias) % 16 == 0);
  if (fh == 3 && fw == 3 && mult == 1 && c % 4 == 0 && sh == sw && (sh == 1 || sh == 2) && aligned) {
    const int c4 = c / 4;
    // Rows per thread: more rows = fewer halo re-reads and more bytes in flight per wavefront,
    // fewer rows = more wavefronts.  Measured best at large sizes: 6 or, when it divides the height (every map
    // of the 224-pixel network: no ragged last strip, a 7 x 7 map is a single strip), 7 (stride 1), 2 (stride 2);
    // small problems take fewer rows so that every CU still gets several wavefronts.
    const long long px = (long long)n * oh * ow * c4;  // threads at one row per thread
    const long long want = 256LL * 256 * 4;            // about 4 workgroups per CU
    if (sh == 1) {
      if (oh % 7 == 0 && (px / 7 >= want * 3 / 4 || (oh == 7 && px / 7 >= want / 4)))
        return launch_dw3x3<1, 7>(x, w, bias, y, n, h, wd, c4, oh, ow, pt, pl, act, stream);
      if (px / 6 >= want) return launch_dw3x3<1, 6>(x, w, bias, y, n, h, wd, c4, oh, ow, pt, pl, act, stream);
      if (px / 4 >= want / 4) return launch_dw3x3<1, 4>(x, w, bias, y, n, h, wd, c4, oh, ow, pt, pl, act, stream);
      if (px / 2 >= want / 4) return launch_dw3x3<1, 2>(x, w, bias, y, n, h, wd, c4, oh, ow, pt, pl, act, stream);
      return launch_dw3x3<1, 1>(x, w, bias, y, n, h, wd, c4, oh, ow, pt, pl, act, stream);
    }
    if (px / 2 >= want / 4) return launch_dw3x3<2, 2>(x, w, bias, y, n, h, wd, c4, oh, ow, pt, pl, act, stream);
    return launch_dw3x3<2, 1>(x, w, bias, y, n, h, wd, c4, oh, ow, pt, pl, act, stream);
  }
  const long long total = (long long)n * oh * ow * c * mult;
  long long blocks = (total + 255) / 256;
  if (blocks > 256 * 64) blocks = 256 * 64;
  hipLaunchKernelGGL(depthwise_generic_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, x, w, bias, y, n, h, wd, c,
                     fh, fw, mult, oh, ow, sh, sw, pt, pl, act, total);
  return check_launch();
}

}  // namespace tfx
