// One depthwise-separable block (depthwise 3x3 + bias + clamp, then pointwise 1x1 + bias + clamp) of one to three
// images as ONE kernel, for the early, thin blocks of the MobileNet v1 timed in Section 3.9 / Table 1 at batch 1, where
// the two layers are bound by being two dependent launches and not by traffic or arithmetic.  A second form also
// computes the network's stem inside the first block's kernel (STEM below).
//
// A workgroup owns a 4 x 4 patch of output pixels (= one 16-row matrix-core tile) and NS output channels.  It first
// copies the input window under the patch (6 x 6 or 9 x 9 pixels, all channels, zeros outside the image) into LDS,
// each element fetched once: the reads of the previous layer's output are the one long-latency step of the kernel
// (measured: 3 us per block when every lane fetched its own 9 taps from memory, 4 x redundantly; 0.6 us this way),
// so they are issued first and kept few.  The input channels are split over WK wavefronts; lane
// (li, q) of such a wavefront computes the depthwise output of pixel li for the 4 channels that are exactly its A
// operand of the 16x16x4 fp32 MFMA steps it issues, so the depthwise result goes from the filter arithmetic into the
// matrix cores without a second trip through LDS or memory; then a split-K reduction of the WK partial tiles
// through LDS with bias + clamp and the store.  The pointwise filter columns and the depthwise filter a lane needs
// are loaded straight into registers while the window is on its way.
//
// Workgroups that cover the same patch (the NS-wide slices of N) each recompute its depthwise output: 9 x 16 x C
// multiply-adds, nothing beside the 16 x C x NS of the pointwise product.
#include "tfx_internal.h"

namespace tfx {
namespace {

constexpr int kXcds = 8;
// images per call up to which the fused kernels beat the two single-op kernels (measured on the whole network:
// 6 us gained at batch 2 and 3, nothing at 4, a loss from 5 on, where the single-op kernels' larger tiles pay)
constexpr int kMaxFusedBatch = 3;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

struct BlockArgs {
  const float* x;     // [H, W, C]
  const float* dw_w;  // [3, 3, C]
  const float* dw_b;  // [C]
  const float* pw_w;  // [C, N]
  const float* pw_b;  // [N]
  float* y;           // [OH, OW, N]
  int H, W, OH, OW, pt, pl, N;
  int tiles_x, tiles_img, slices, total;  // patches per row and per image, column slices, workgroups
  long long x_img, y_img;                 // floats per input / output image
  int dw_act, pw_act;
  int batch;
  unsigned x_bytes;                       // bytes of one input image
  // STEM form: x is the image [IH, IW, 3]; the block's input [H, W, 32] is the 3x3 stride-2 convolution of the
  // image with st_w [3, 3, 3, 32] + st_b, clamped, and exists only as windows in LDS
  const float* st_w;
  const float* st_b;
  int IH, IW, st_pt, st_pl, st_act;
  int* zero_words;  // optional: zero_count words, zero_stride words apart, cleared by this kernel
  int zero_count, zero_stride;
};

__device__ __forceinline__ float f4_at(const float4& v, int i) { return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w; }

// C input channels, split over WK wavefronts; WN wavefronts side by side over the columns, CB column blocks of 16
// each: NS = 16 CB WN columns per workgroup.
// STEM: the block's input is computed from the image on the fly (see BlockArgs).
template <int C, int WK, int WN, int CB, int S, bool STEM = false>
__global__ __launch_bounds__(64 * WK * WN) void separable_block_kernel(const BlockArgs a) {
  constexpr int NT = 64 * WK * WN;
  constexpr int G = C / (16 * WK);  // groups of 16 channels per wavefront
  constexpr int NS = 16 * CB * WN;
  constexpr int EI = (256 * WN + NT - 1) / NT;  // epilogue items per thread
  static_assert(C % (16 * WK) == 0 && (CB == 2 || CB == 4), "tile shape");
  static_assert(!STEM || (C == 32 && S == 1 && NT == 256), "the stem form feeds the first block");
  constexpr int WH = 3 * S + 3;             // window edge: 3 (S) + 3 input pixels under 4 output pixels
  constexpr int P = C + 4;                   // floats between window pixels in LDS
  constexpr int WQ = WH * WH * (C / 4);      // float4 elements of the window
  constexpr int LI = (WQ + NT - 1) / NT;     // of which a thread copies at most LI
  constexpr int kRed = WK * WN * CB * 4 * 64, kWin = WH * WH * P;
  // the window, and after the MFMAs the partial tiles [wk][wn][j][v][lane]
  __shared__ __align__(16) float lds[kRed > kWin ? kRed : kWin];
  float* const red = lds;

  // workgroups are dealt to the XCDs round robin: give every XCD a contiguous run of patches (shared halos and
  // the slices of one patch then meet in one L2)
  const int bid = blockIdx.x;
  const int q8 = a.total / kXcds, rem = a.total % kXcds;
  const int xcd = bid % kXcds;
  const int vid = xcd * q8 + (xcd < rem ? xcd : rem) + bid / kXcds;
  const int slice = vid % a.slices, tile = vid / a.slices;
  const int img_n = tile / a.tiles_img, tile_i = tile % a.tiles_img;
  const int ty = tile_i / a.tiles_x, tx = tile_i % a.tiles_x;

  const int tid = threadIdx.x, wave = tid / 64, wk = wave % WK, wn = wave / WK;
  const int lane = tid % 64, li = lane % 16, q = lane / 16;
  const int N = a.N;
  const int n0 = slice * NS;

  // the input window: element i = (pixel i / (C/4) of the window, channel quad i % (C/4))
  const __amdgpu_buffer_rsrc_t xr =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(a.x + img_n * a.x_img), 0, (int)a.x_bytes, 0x00020000);
  u32x4 win[LI];
  // STEM: the 13 x 13 x 3 image pixels under the 6 x 6 window of stem outputs, rows of 39 floats; the stem filter
  constexpr int kImgRow = 40, kImgFloats = 13 * 39;
  __shared__ float img[STEM ? 13 * kImgRow : 1];
  constexpr int kWstRow = 48;  // floats between filter rows in LDS: lanes q and q + 1 read rows 16 banks apart
  __shared__ __align__(16) float wst[STEM ? 28 * kWstRow : 4];  // [27][32 of 48] filter, [32] bias
  float iv[2];
  float4 wv = make_float4(0.f, 0.f, 0.f, 0.f);
  const int sy0 = 4 * ty - a.pt, sx0 = 4 * tx - a.pl;  // STEM: first row / column of the window in the stem's output
  if constexpr (STEM) {
    const int gy0 = 2 * sy0 - a.st_pt, gx0 = 2 * sx0 - a.st_pl;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int e = tid + i * NT, gy = gy0 + e / 39, gx = gx0 + (e % 39) / 3;
      const bool in = e < kImgFloats && gy >= 0 && gy < a.IH && gx >= 0 && gx < a.IW;
      const unsigned off = in ? (unsigned)((gy * a.IW + gx) * 3 + e % 3) * 4u : 0x80000000u;
      iv[i] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(xr, (int)off, 0, 0));
    }
    if (tid < 27 * 8) wv = *reinterpret_cast<const float4*>(a.st_w + 4 * tid);
    else if (tid < 28 * 8) wv = *reinterpret_cast<const float4*>(a.st_b + 4 * (tid - 27 * 8));
    if (a.zero_count > 0)
      for (int i = bid * NT + tid; i < a.zero_count; i += a.total * NT) a.zero_words[(size_t)i * a.zero_stride] = 0;
  } else {
    const int wy0 = 4 * ty * S - a.pt, wx0 = 4 * tx * S - a.pl;
#pragma unroll
    for (int i = 0; i < LI; ++i) {
      const int e = tid + i * NT, p = e / (C / 4), cq = e % (C / 4);
      const int iy = wy0 + p / WH, ix = wx0 + p % WH;
      // outside the image (or past the window): past the end of the buffer, the hardware returns 0
      const bool in = e < WQ && iy >= 0 && iy < a.H && ix >= 0 && ix < a.W;
      const unsigned off = in ? (unsigned)((iy * a.W + ix) * C + 4 * cq) * 4u : 0x80000000u;
      win[i] = __builtin_amdgcn_raw_buffer_load_b128(xr, (int)off, 0, 0);
    }
  }
  (void)win;

  // pointwise filter columns of this lane: rows wk 16 G + 16 g + 4 q + s, columns n0 + 16 CB wn + CB li ...
  float b[G][4][CB];
  {
    const float* bp = a.pw_w + (size_t)(wk * 16 * G + 4 * q) * N + n0 + 16 * CB * wn + CB * li;
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const float* p = bp + (size_t)(16 * g + s) * N;
        if constexpr (CB == 4) {
          const float4 t = *reinterpret_cast<const float4*>(p);
          b[g][s][0] = t.x, b[g][s][1] = t.y, b[g][s][2] = t.z, b[g][s][3] = t.w;
        } else {
          const float2 t = *reinterpret_cast<const float2*>(p);
          b[g][s][0] = t.x, b[g][s][1] = t.y;
        }
      }
  }
  // epilogue item e < 256 WN: register v = (e / 64) % 4 of lane l = e % 64 of column group e / 256:
  // row 4 (l / 16) + v of the patch, columns n0 + 16 CB (e / 256) + CB (l % 16) ...
  float ebias[EI][CB];
#pragma unroll
  for (int i = 0; i < EI; ++i) {
    const int e = tid + i * NT;
    const float* p = a.pw_b + n0 + 16 * CB * (e / 256) + CB * (e % 16);
#pragma unroll
    for (int j = 0; j < CB; ++j) ebias[i][j] = e < 256 * WN ? p[j] : 0.f;
  }

  // depthwise filter and bias of the lane's channels c4 + 16 g ... + 3
  const int c4 = wk * 16 * G + 4 * q;
  float4 dwf[G][9], dwb[G];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    dwb[g] = *reinterpret_cast<const float4*>(a.dw_b + c4 + 16 * g);
#pragma unroll
    for (int t = 0; t < 9; ++t) dwf[g][t] = *reinterpret_cast<const float4*>(a.dw_w + t * C + c4 + 16 * g);
  }

  if constexpr (STEM) {
    // image pixels and stem filter -> LDS, then the stem's output for the window; window pixels outside the stem's
    // output map are the depthwise layer's zero padding
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int e = tid + i * NT;
      if (e < kImgFloats) img[(e / 39) * kImgRow + e % 39] = iv[i];
    }
    if (tid < 28 * 8) *reinterpret_cast<float4*>(wst + (tid / 8) * kWstRow + 4 * (tid % 8)) = wv;
    __syncthreads();
    // the 36 window pixels x 32 filters as a [48 (36 used), 36 (27 used)] x [36, 32] product on the matrix cores.
    // k = (kh, j): j runs along image row kh of the pixel's 3 x 3 x 3 patch (9 values), padded to 12 so that
    // every address is a per-lane base plus a constant -- with 3 - 4 workgroups per CU this phase is bound by
    // the number of instructions issued, not by the matrix cores.
    const ActClamp sclamp = make_act(a.st_act);
    const bool border = sy0 < 0 || sx0 < 0 || sy0 + WH > a.H || sx0 + WH > a.W;  // same for the whole workgroup
    for (int t = wave; t < 6; t += NT / 64) {
      const int rt = t % 3, cb = t / 3;
      const int p = min(16 * rt + li, WH * WH - 1);
      const float* ip = img + 2 * (p / WH) * kImgRow + 6 * (p % WH) + q;
      const float* fp = wst + q * kWstRow + 16 * cb + li;
      floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kk = 0; kk < 9; ++kk) {
        const int kh = kk / 3, j0 = 4 * (kk % 3);  // this lane's j = j0 + q: 8 + q > 8 is padding
        float av = ip[kh * kImgRow + j0], bv = fp[(kh * 9 + j0) * kWstRow];
        if (j0 == 8) av = q == 0 ? av : 0.f, bv = q == 0 ? bv : 0.f;
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bv, acc, 0, 0, 0);
      }
      const int c = 16 * cb + li;
      const float sb = wst[27 * kWstRow + c];
      if (rt < 2 || q == 0) {
        float* dst = lds + (16 * rt + 4 * q) * P + c;
#pragma unroll
        for (int v = 0; v < 4; ++v) dst[v * P] = apply_act(acc[v] + sb, sclamp);
        if (border) {
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const int pp = 16 * rt + 4 * q + v;
            const int sy = sy0 + pp / WH, sx = sx0 + pp % WH;
            if (sy < 0 || sy >= a.H || sx < 0 || sx >= a.W) dst[v * P] = 0.f;
          }
        }
      }
    }
  } else {
    // window -> LDS
#pragma unroll
    for (int i = 0; i < LI; ++i) {
      const int e = tid + i * NT;
      if (e < WQ) *reinterpret_cast<u32x4*>(lds + (e / (C / 4)) * P + 4 * (e % (C / 4))) = win[i];
    }
  }
  __syncthreads();

  // depthwise output of pixel li for the lane's channels
  const int oy = 4 * ty + li / 4, ox = 4 * tx + li % 4;
  const int iy0 = oy * S - a.pt, ix0 = ox * S - a.pl;
  float4 tap[G][9];
  bool ok[9];
#pragma unroll
  for (int kh = 0; kh < 3; ++kh)
#pragma unroll
    for (int kw = 0; kw < 3; ++kw) {
      const int iy = iy0 + kh, ix = ix0 + kw;
      ok[kh * 3 + kw] = iy >= 0 && iy < a.H && ix >= 0 && ix < a.W;
      const float* wp = lds + (((li / 4) * S + kh) * WH + (li % 4) * S + kw) * P + c4;
#pragma unroll
      for (int g = 0; g < G; ++g) tap[g][kh * 3 + kw] = *reinterpret_cast<const float4*>(wp + 16 * g);
    }
  // The filter is only used under the taps' in-image predicates; pinning it here keeps its loads where they
  // are written, ahead of the taps and all in flight together, instead of inside per-tap branches.
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int t = 0; t < 9; ++t)
      asm volatile("" : "+v"(dwf[g][t].x), "+v"(dwf[g][t].y), "+v"(dwf[g][t].z), "+v"(dwf[g][t].w));
  const ActClamp dclamp = make_act(a.dw_act);
  float4 av[G];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float4 acc = dwb[g];
#pragma unroll
    for (int t = 0; t < 9; ++t) {
      const float4 w = dwf[g][t];
      acc.x = ok[t] ? fmaf(tap[g][t].x, w.x, acc.x) : acc.x;
      acc.y = ok[t] ? fmaf(tap[g][t].y, w.y, acc.y) : acc.y;
      acc.z = ok[t] ? fmaf(tap[g][t].z, w.z, acc.z) : acc.z;
      acc.w = ok[t] ? fmaf(tap[g][t].w, w.w, acc.w) : acc.w;
    }
    av[g] = make_float4(apply_act(acc.x, dclamp), apply_act(acc.y, dclamp), apply_act(acc.z, dclamp), apply_act(acc.w, dclamp));
  }

  floatx4 acc[CB];
#pragma unroll
  for (int j = 0; j < CB; ++j)
#pragma unroll
    for (int v = 0; v < 4; ++v) acc[j][v] = 0.f;
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
      for (int j = 0; j < CB; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(f4_at(av[g], s), b[g][s][j], acc[j], 0, 0, 0);

  __syncthreads();  // everybody has read its taps: the window's LDS now takes the partial tiles
#pragma unroll
  for (int j = 0; j < CB; ++j)
#pragma unroll
    for (int v = 0; v < 4; ++v) red[(((wk * WN + wn) * CB + j) * 4 + v) * 64 + lane] = acc[j][v];
  __syncthreads();

  const ActClamp pclamp = make_act(a.pw_act);
#pragma unroll
  for (int i = 0; i < EI; ++i) {
    const int e = tid + i * NT;
    if (e >= 256 * WN) break;
    const int ewn = e / 256, ev = (e / 64) % 4, el = e % 64;
    const int row = 4 * (el / 16) + ev;
    const int py = 4 * ty + row / 4, px = 4 * tx + row % 4;
    float o[CB];
#pragma unroll
    for (int j = 0; j < CB; ++j) {
      float sum = ebias[i][j];
#pragma unroll
      for (int w = 0; w < WK; ++w) sum += red[(((w * WN + ewn) * CB + j) * 4 + ev) * 64 + el];
      o[j] = apply_act(sum, pclamp);
    }
    if (py < a.OH && px < a.OW) {
      float* dst = a.y + img_n * a.y_img + (size_t)(py * a.OW + px) * N + n0 + 16 * CB * ewn + CB * (el % 16);
      if constexpr (CB == 4) *reinterpret_cast<float4*>(dst) = make_float4(o[0], o[1], o[2], o[3]);
      else *reinterpret_cast<float2*>(dst) = make_float2(o[0], o[1]);
    }
  }
}

template <int C, int WK, int WN, int CB, int S, bool STEM = false>
int launch_cfg(BlockArgs a, hipStream_t stream) {
  constexpr int NS = 16 * CB * WN;
  a.tiles_x = (a.OW + 3) / 4;
  a.slices = a.N / NS;
  a.tiles_img = a.tiles_x * ((a.OH + 3) / 4);
  a.y_img = (long long)a.OH * a.OW * a.N;
  const long long total = (long long)a.batch * a.tiles_img * a.slices;
  if (total > 0x7fffffffLL) return TFX_ERR_UNSUPPORTED;
  a.total = (int)total;
  hipLaunchKernelGGL((separable_block_kernel<C, WK, WN, CB, S, STEM>), dim3((unsigned)a.total), dim3(64 * WK * WN), 0, stream, a);
  return check_launch();
}

}  // namespace

bool separable_block_supported(long long batch, int h, int w, int c, int n, int stride, const void* x, const void* dw_w,
                               const void* dw_b, const void* pw_w, const void* pw_b, const void* y) {
  auto al16 = [](const void* p) { return reinterpret_cast<uintptr_t>(p) % 16 == 0; };
  return batch >= 1 && batch <= kMaxFusedBatch && (c == 32 || c == 64 || c == 128) && n % 64 == 0 && n >= 64 && n <= 1024 &&
         (stride == 1 || stride == 2) && h >= 1 && w >= 1 && (long long)h * w * c * 4 < (1ll << 31) && al16(x) &&
         al16(dw_w) && al16(dw_b) && al16(pw_w) && al16(pw_b) && al16(y);
}

int launch_separable_block(const float* x, const float* dw_w, const float* dw_b, const float* pw_w, const float* pw_b,
                           float* y, int batch, int h, int w, int c, int n, int oh, int ow, int stride, int pt, int pl,
                           int dw_act, int pw_act, hipStream_t stream) {
  BlockArgs a;
  a.x = x, a.dw_w = dw_w, a.dw_b = dw_b, a.pw_w = pw_w, a.pw_b = pw_b, a.y = y;
  a.H = h, a.W = w, a.OH = oh, a.OW = ow, a.pt = pt, a.pl = pl, a.N = n;
  a.dw_act = dw_act, a.pw_act = pw_act;
  a.batch = batch;
  a.x_bytes = (unsigned)((long long)h * w * c * 4);
  a.x_img = (long long)h * w * c;
  a.tiles_x = a.tiles_img = a.slices = a.total = 0;
  a.y_img = 0;
  a.st_w = a.st_b = nullptr, a.IH = a.IW = a.st_pt = a.st_pl = a.st_act = 0;
  a.zero_words = nullptr, a.zero_count = 0, a.zero_stride = 1;
#define TFX_BLOCK_CASE(CC, WK, WN, CB)                                       \
  if (c == CC && stride == 1) return launch_cfg<CC, WK, WN, CB, 1>(a, stream); \
  if (c == CC && stride == 2) return launch_cfg<CC, WK, WN, CB, 2>(a, stream);
  TFX_BLOCK_CASE(32, 2, 2, 2)
  TFX_BLOCK_CASE(64, 4, 1, 4)
  TFX_BLOCK_CASE(128, 8, 1, 4)
#undef TFX_BLOCK_CASE
  return TFX_ERR_UNSUPPORTED;
}

bool stem_block_supported(long long batch, int ih, int iw, int stem_filters, int n, const void* image, const void* st_w,
                          const void* st_b, const void* dw_w, const void* dw_b, const void* pw_w, const void* pw_b,
                          const void* y) {
  auto al16 = [](const void* p) { return reinterpret_cast<uintptr_t>(p) % 16 == 0; };
  return batch >= 1 && batch <= kMaxFusedBatch && stem_filters == 32 && n == 64 && ih >= 1 && iw >= 1 && (long long)ih * iw * 3 * 4 < (1ll << 31) &&
         al16(image) && al16(st_w) && al16(st_b) && al16(dw_w) && al16(dw_b) && al16(pw_w) && al16(pw_b) && al16(y);
}

int launch_stem_block(const float* image, const float* st_w, const float* st_b, const float* dw_w, const float* dw_b,
                      const float* pw_w, const float* pw_b, float* y, int batch, int ih, int iw, int h, int w, int st_pt,
                      int st_pl, int n, int act, hipStream_t stream, int* zero_words, int zero_count, int zero_stride) {
  BlockArgs a;
  a.x = image, a.dw_w = dw_w, a.dw_b = dw_b, a.pw_w = pw_w, a.pw_b = pw_b, a.y = y;
  // the block: 3x3 stride-1 depthwise layer with SAME padding (one zero row / column before the map), then 32 -> n
  a.H = h, a.W = w, a.OH = h, a.OW = w, a.pt = 1, a.pl = 1, a.N = n;
  a.dw_act = act, a.pw_act = act;
  a.batch = batch;
  a.x_bytes = (unsigned)((long long)ih * iw * 3 * 4);
  a.x_img = (long long)ih * iw * 3;
  a.tiles_x = a.tiles_img = a.slices = a.total = 0;
  a.y_img = 0;
  a.st_w = st_w, a.st_b = st_b, a.IH = ih, a.IW = iw, a.st_pt = st_pt, a.st_pl = st_pl, a.st_act = act;
  a.zero_words = zero_words, a.zero_count = zero_count, a.zero_stride = zero_stride;
  return launch_cfg<32, 2, 2, 2, 1, true>(a, stream);
}

}  // namespace tfx
