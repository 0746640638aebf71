// Direct convolutions for gfx950: a general conv2d for any filter / stride, and the
// 3x3 stride-s, 3-input-channel "stem" convolution of MobileNet v1 (K = 27 is too thin
// for the matrix cores; the layer is bound by its 2.2 MB of activations).
// Index order is NHWC (the batch,row,column,depth sampler of Section 4.1), filters HWIO.
#include "tfx_internal.h"

namespace tfx {
namespace {

// One thread per output element, output channel fastest so that filter reads and output
// writes are coalesced.  Correct for every shape; used when no specialised kernel applies.
__global__ __launch_bounds__(256) void conv2d_direct_kernel(const float* __restrict__ x, const float* __restrict__ w,
                                                            const float* __restrict__ bias, float* __restrict__ y,
                                                            int N, int H, int W, int Ci, int fh, int fw, int Co,
                                                            int OH, int OW, int sh, int sw, int pt, int pl, int act,
                                                            long long total) {
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
        const float* xp = x + (((size_t)n * H + ih) * W + iw) * Ci;
        const float* wp = w + ((size_t)(kh * fw + kw) * Ci) * Co + oc;
        for (int c = 0; c < Ci; ++c) acc = fmaf(xp[c], wp[(size_t)c * Co], acc);
      }
    }
    if (bias) acc += bias[oc];
    y[idx] = apply_act(acc, act);
  }
}

// Stem: 3x3 filter, 3 input channels, CO output channels (CO % 8 == 0, CO <= 64).
// A thread computes 8 consecutive output channels of one output pixel: the 27 x CO filter
// sits in LDS and is read as float4 pairs (only CO/8 distinct addresses per wave, so the
// reads broadcast); CO/8 neighbouring lanes write one pixel's CO floats as a contiguous run.
// All 27 input values of a pixel are fetched with unconditional loads from clamped addresses
// (out-of-image taps are zeroed afterwards), so they are all in flight at once.
template <int CO>
__global__ __launch_bounds__(256) void conv2d_stem_kernel(const float* __restrict__ x, const float* __restrict__ w,
                                                          const float* __restrict__ bias, float* __restrict__ y, int N,
                                                          int H, int W, int OH, int OW, int sh, int sw, int pt, int pl,
                                                          int act, int total, int* __restrict__ zero_words,
                                                          int zero_count, int zero_stride) {
  // optional: clear a small array of words for a later kernel of the same forward pass (its task flags)
  for (int i = (int)(blockIdx.x * 256 + threadIdx.x); i < zero_count; i += (int)gridDim.x * 256)
    zero_words[(size_t)i * zero_stride] = 0;
  constexpr int G = CO / 8;
  constexpr int WPT = (27 * CO + 255) / 256;  // filter floats staged per thread
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

  // issue the filter loads and the 27 input loads together, then stage the filter
  float wreg[WPT];
#pragma unroll
  for (int i = 0; i < WPT; ++i) {
    const int e = threadIdx.x + i * 256;
    wreg[i] = w[e < 27 * CO ? e : 27 * CO - 1];
  }
  float acc[8];
#pragma unroll
  for (int o = 0; o < 8; ++o) acc[o] = bias ? bias[8 * g + o] : 0.f;
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
      const float* xp = x + (((size_t)n * H + ihc) * W + iwc) * 3;
#pragma unroll
      for (int c = 0; c < 3; ++c) {
        const float v = xp[c];
        xv[(kh * 3 + kw) * 3 + c] = ok ? v : 0.f;
      }
    }
  }
#pragma unroll
  for (int i = 0; i < WPT; ++i) {
    const int e = threadIdx.x + i * 256;
    if (e < 27 * CO) wl[e] = wreg[i];
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
  float4 o0, o1;
  o0.x = apply_act(acc[0], act);
  o0.y = apply_act(acc[1], act);
  o0.z = apply_act(acc[2], act);
  o0.w = apply_act(acc[3], act);
  o1.x = apply_act(acc[4], act);
  o1.y = apply_act(acc[5], act);
  o1.z = apply_act(acc[6], act);
  o1.w = apply_act(acc[7], act);
  float* yp = y + (((size_t)n * OH + oh) * OW + ow) * CO + 8 * g;
  *reinterpret_cast<float4*>(yp) = o0;
  *reinterpret_cast<float4*>(yp + 4) = o1;
}

// The stem on the matrix cores, for a multiple of 32 filters (32 is instantiated).  K = 27 is thin, but the
// vector-ALU form above spends 27 x 8 FMAs plus 54 LDS reads per thread and is bound by that, not by its memory
// traffic; as a GEMM with
// v_mfma_f32_16x16x4_f32 (output channels as the A operand's rows, 16 output pixels as the B operand's columns, K
// padded to 28) a 16-pixel slab costs 7 MFMAs per 16 channels.  A wavefront keeps its lanes' filter values in
// registers (7 per column block) and walks over slabs of 16 consecutive pixels of one output row; lane
// (li = l % 16, q = l / 16) supplies, in step s, input value k = 4s + q of pixel li's 3 x 3 x 3 window (k = (kh * 3
// + kw) * 3 + c), loaded straight from memory.  Slabs whose windows lie inside the image take unconditional
// loads at constant per-lane offsets; slabs on a border check every tap.  The accumulators hold 4 consecutive
// channels per lane and leave through store_slab (whole 128-byte lines).
template <int CO>
__global__ __launch_bounds__(256) void conv2d_stem_mfma_kernel(const float* __restrict__ x, const float* __restrict__ w,
                                                               const float* __restrict__ bias, float* __restrict__ y,
                                                               int N, int H, int W, int OH, int OW, int sh, int sw, int pt,
                                                               int pl, int act, int* __restrict__ zero_words,
                                                               int zero_count, int zero_stride) {
  constexpr int NB = CO / 16;
  // optional: clear a small array of words for a later kernel of the same forward pass (its task flags)
  for (int i = (int)(blockIdx.x * 256 + threadIdx.x); i < zero_count; i += (int)gridDim.x * 256)
    zero_words[(size_t)i * zero_stride] = 0;
  static_assert(CO % 32 == 0, "column blocks are stored in pairs");
  const int lane = threadIdx.x % 64, li = lane % 16, q = lane / 16;
  const int segs = (OW + 15) / 16;
  // a wavefront's slabs: (n, oh, seg) of slab number first + t * stride, t = 0, 1, ..., kept in scalar registers and
  // advanced with carries (no division in the loop)
  const int stride = (int)gridDim.x * 4;
  const int first = (int)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane((int)threadIdx.x / 64);
  int seg = first % segs, oh = (first / segs) % OH, n = first / segs / OH;
  const int d_seg = stride % segs, d_oh = (stride / segs) % OH, d_n = stride / segs / OH;

  // this lane's 7 window positions and filter values
  int kh[7], kw[7], dk[7];
  float wr[7][NB];
#pragma unroll
  for (int s = 0; s < 7; ++s) {
    const int k = 4 * s + q;
    const bool valid = k < 27;
    const int kc = valid ? k : 26;
    kh[s] = kc / 9;
    kw[s] = (kc % 9) / 3;
    dk[s] = (kh[s] * W + kw[s]) * 3 + kc % 3;
#pragma unroll
    for (int j = 0; j < NB; ++j) wr[s][j] = valid ? w[kc * CO + 16 * j + li] : 0.f;
  }
  float4 bv[NB / 2];
#pragma unroll
  for (int h = 0; h < NB / 2; ++h)
    bv[h] = bias ? *reinterpret_cast<const float4*>(bias + 32 * h + (li < 8 ? 0 : 16) + 4 * q)
                 : make_float4(0.f, 0.f, 0.f, 0.f);
  const ActClamp clamp = make_act(act);
  const bool last_k = q == 3;  // step 6 of these lanes is the padding k = 27

  while (n < N) {
    const long long row = (long long)n * OH + oh;
    const int ow = min(seg * 16 + li, OW - 1);  // pixels past the row's end repeat the last one (not stored)
    const int ih0 = oh * sh - pt, iw0 = ow * sw - pl;
    const float* xb = x + (((long long)n * H + ih0) * W + iw0) * 3;  // tap (0, 0); outside x on a border
    // the whole slab's windows inside the image?  (uniform: the first and last pixel of the slab decide)
    const int iw_first = seg * 16 * sw - pl, iw_last = min(seg * 16 + 15, OW - 1) * sw - pl + 2;
    const bool interior = ih0 >= 0 && ih0 + 2 < H && iw_first >= 0 && iw_last < W;
    float xv[7];
    if (interior) {
#pragma unroll
      for (int s = 0; s < 7; ++s) xv[s] = xb[dk[s]];
      if (last_k) xv[6] = 0.f;  // not 0 * x: x may be Inf or NaN
    } else {
#pragma unroll
      for (int s = 0; s < 7; ++s) {
        const int ih = ih0 + kh[s], iw = iw0 + kw[s];
        const bool ok = ih >= 0 && ih < H && iw >= 0 && iw < W && !(s == 6 && last_k);
        const float v = *(ok ? xb + dk[s] : x);
        xv[s] = ok ? v : 0.f;
      }
    }
    floatx4 acc[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) acc[j][v] = 0.f;
#pragma unroll
    for (int s = 0; s < 7; ++s)
#pragma unroll
      for (int j = 0; j < NB; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(wr[s][j], xv[s], acc[j], 0, 0, 0);
    // rows of the output matrix [N * OH * OW, CO] covered by this slab
    const long long p0 = row * OW + seg * 16;
    const int valid_rows = min(16, OW - seg * 16);
    // store_slab addresses rows relative to y_slab; the row count guards the ragged last segment
    float* y_slab = y + p0 * CO;
    if (valid_rows == 16) store_slab<NB, false>(acc, bv, y_slab, CO, 0, 16, li, q, clamp);
    else store_slab<NB, true>(acc, bv, y_slab, CO, 0, valid_rows, li, q, clamp);
    seg += d_seg;
    const int c1 = seg >= segs ? 1 : 0;
    seg -= c1 * segs;
    oh += d_oh + c1;
    const int c2 = oh >= OH ? 1 : 0;
    oh -= c2 * OH;
    n += d_n + c2;
  }
}

}  // namespace

int launch_conv2d_direct(const float* x, const float* w, const float* bias, float* y, int n, int h, int wd, int ci,
                         int fh, int fw, int co, int oh, int ow, int sh, int sw, int pt, int pl, int act,
                         hipStream_t stream) {
  const long long total = (long long)n * oh * ow * co;
  long long blocks = (total + 255) / 256;
  if (blocks > 256 * 8) blocks = 256 * 8;  // grid-stride beyond 64 workgroups per CU
  hipLaunchKernelGGL(conv2d_direct_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, x, w, bias, y, n, h, wd, ci,
                     fh, fw, co, oh, ow, sh, sw, pt, pl, act, total);
  return check_launch();
}

bool conv2d_stem_supported(int ci, int fh, int fw, int co, int sh, int sw) {
  (void)sh;
  (void)sw;
  return ci == 3 && fh == 3 && fw == 3 && (co == 8 || co == 16 || co == 24 || co == 32);
}

int launch_conv2d_stem(const float* x, const float* w, const float* bias, float* y, int n, int h, int wd, int co,
                       int oh, int ow, int sh, int sw, int pt, int pl, int act, hipStream_t stream, int* zero_words,
                       int zero_count, int zero_stride) {
  // 32 filters, 16-byte aligned y and bias: the matrix-core form
  if (co == 32 && reinterpret_cast<uintptr_t>(y) % 16 == 0 && reinterpret_cast<uintptr_t>(bias) % 16 == 0) {
    const long long slabs = (long long)n * oh * ((ow + 15) / 16);
    if (slabs > 0x3fffffffLL) return TFX_ERR_UNSUPPORTED;
    long long blocks = (slabs + 3) / 4;
    if (blocks > 256 * 8) blocks = 256 * 8;  // 8 workgroups of 4 wavefronts per CU, then the slab loop
    hipLaunchKernelGGL(conv2d_stem_mfma_kernel<32>, dim3((unsigned)blocks), dim3(256), 0, stream, x, w, bias, y, n, h, wd,
                       oh, ow, sh, sw, pt, pl, act, zero_words, zero_count, zero_stride);
    return check_launch();
  }
  const long long total = (long long)n * oh * ow * (co / 8);
  if (total > 0x7fffffffLL) return TFX_ERR_UNSUPPORTED;
  const unsigned blocks = (unsigned)((total + 255) / 256);
#define TFX_STEM(CO)                                                                                              \
  hipLaunchKernelGGL(conv2d_stem_kernel<CO>, dim3(blocks), dim3(256), 0, stream, x, w, bias, y, n, h, wd, oh, ow, \
                     sh, sw, pt, pl, act, (int)total, zero_words, zero_count, zero_stride)
  switch (co) {
    case 8: TFX_STEM(8); break;
    case 16: TFX_STEM(16); break;
    case 24: TFX_STEM(24); break;
    case 32: TFX_STEM(32); break;
    default: return TFX_ERR_UNSUPPORTED;
  }
#undef TFX_STEM
  return check_launch();
}

}  // namespace tfx
