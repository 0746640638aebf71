// One depthwise-separable block (depthwise 3x3 + bias + clamp, then pointwise 1x1 + bias + clamp) of one to three
// images as ONE kernel, for the early, thin blocks of the MobileNet v1 timed in Section 3.9 / Table 1 at batch 1, where
// the two layers are bound by being two dependent launches and not by traffic or arithmetic.  A second form also
// computes the network's stem inside the first block's kernel (STEM below); and blocks 2 - 4 of the batch-1 network
// run as three stages of one launch that hand their patches over through flags (separable_chain_kernel).
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
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
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

// Hand-over between blocks that run as stages of one launch (separable_chain_kernel): a workgroup's patch x slice
// has a flag word, kLinkFlagStride words apart; the producer sets it after its stores are acknowledged, the consumer
// polls the flags of the patches under its window.  Activations that move this way use device-coherent (sc1)
// stores and loads, as in chain.hip.  flags[0] is the failure word shared with the chained kernel that follows.
constexpr int kLinkFlagStride = 32;
constexpr int kSc1 = 16;
struct BlockLink {
  int* flags;
  int in_base, in_tiles_x, in_slices;  // producer stage: first flag, patches per row, column slices (in_base < 0: none)
  int out_base;                        // this stage's first flag (< 0: nobody waits for it inside the launch)
  int spin_limit;
};

__device__ __forceinline__ float f4_at(const float4& v, int i) { return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w; }

// C input channels, split over WK wavefronts; WN wavefronts side by side over the columns, CB column blocks of 16
// each: NS = 16 CB WN columns per workgroup.
// STEM: the block's input is computed from the image on the fly (see BlockArgs).
// LIN / LOUT: the input was written / the output will be read by another stage of the same launch (see BlockLink).
// lds: max(kRed, kWin) floats (BlockShape); img, wst: STEM only.
template <int C, int WK, int WN, int CB, int S>
struct BlockShape {
  static constexpr int WH = 3 * S + 3, P = C + 4;
  static constexpr int kRed = WK * WN * CB * 4 * 64, kWin = WH * WH * P;
  static constexpr int kLds = kRed > kWin ? kRed : kWin;
};
constexpr int kImgRow = 40, kImgFloats = 13 * 39;  // STEM: 13 x 13 x 3 image pixels under a window, rows of 39 floats
constexpr int kWstRow = 48;  // STEM: floats between filter rows in LDS: lanes q and q + 1 read rows 16 banks apart

template <int C, int WK, int WN, int CB, int S, bool STEM, bool LIN, bool LOUT>
__device__ __forceinline__ void block_body(const BlockArgs& a, const int bid, float* const lds, float* const img,
                                           float* const wst, const BlockLink& L, int* const gave_up) {
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
  static_assert(!(STEM && LIN), "the stem form reads the image");
  float* const red = lds;  // the window, and after the MFMAs the partial tiles [wk][wn][j][v][lane]

  // workgroups are dealt to the XCDs round robin: give every XCD a contiguous run of patches (shared halos and
  // the slices of one patch then meet in one L2)
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
  }
  const int wy0 = 4 * ty * S - a.pt, wx0 = 4 * tx * S - a.pl;
  auto load_window = [&]() {
#pragma unroll
    for (int i = 0; i < LI; ++i) {
      const int e = tid + i * NT, p = e / (C / 4), cq = e % (C / 4);
      const int iy = wy0 + p / WH, ix = wx0 + p % WH;
      // outside the image (or past the window): past the end of the buffer, the hardware returns 0
      const bool in = e < WQ && iy >= 0 && iy < a.H && ix >= 0 && ix < a.W;
      const unsigned off = in ? (unsigned)((iy * a.W + ix) * C + 4 * cq) * 4u : 0x80000000u;
      win[i] = __builtin_amdgcn_raw_buffer_load_b128(xr, (int)off, 0, LIN ? kSc1 : 0);
    }
  };
  if constexpr (!STEM && !LIN) load_window();  // first thing in flight; a linked stage fetches it after its wait
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

  if constexpr (LIN) {
    // the producer patches under the window (its rows and columns inside the map), every column slice: one flag per
    // lane of wavefront 0; bounded, a wait that gives up sets the failure word and ends every other wait
    if (wave == 0) {
      const int r_lo = max(wy0, 0) / 4, r_hi = min(wy0 + WH - 1, a.H - 1) / 4;
      const int c_lo = max(wx0, 0) / 4, c_hi = min(wx0 + WH - 1, a.W - 1) / 4;
      const int nc = c_hi - c_lo + 1, n = (r_hi - r_lo + 1) * nc * L.in_slices;
      const int rows_in = (a.H + 3) / 4;
      bool bad = false;
      for (int i = lane; i < n; i += 64) {
        const int r = r_lo + i / (nc * L.in_slices), c = c_lo + (i / L.in_slices) % nc, sl = i % L.in_slices;
        const int* f = L.flags + (size_t)(L.in_base + ((img_n * rows_in + r) * L.in_tiles_x + c) * L.in_slices + sl) * kLinkFlagStride;
        int spin = 0;
        while (__hip_atomic_load(f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0) {
          if (++spin > L.spin_limit) {
            __hip_atomic_store(L.flags, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            bad = true;
            break;
          }
          if ((spin & 255) == 0 && __hip_atomic_load(L.flags, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
            bad = true;
            break;
          }
          __builtin_amdgcn_s_sleep(1);
        }
      }
      const bool any_bad = __ballot(bad) != 0;
      if (lane == 0) *gave_up = any_bad ? 1 : 0;
    }
    __syncthreads();
    load_window();
  }
  // a stage that did not get all of its input writes NaN: every later layer then carries the NaN to the end of
  // the network (the clamps pass NaN on), so an unfinished hand-over cannot yield plausible numbers
  const bool poison = LIN ? *gave_up != 0 : false;

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
      o[j] = poison ? __uint_as_float(0x7fc00000u) : apply_act(sum, pclamp);
    }
    if (py < a.OH && px < a.OW) {
      const size_t at = (size_t)(py * a.OW + px) * N + n0 + 16 * CB * ewn + CB * (el % 16);
      float* dst = a.y + img_n * a.y_img + at;
      if constexpr (LOUT) {
        // device-coherent store (write-through: visible to the consumer's sc1 loads on any XCD)
        const __amdgpu_buffer_rsrc_t yr =
            __builtin_amdgcn_make_buffer_rsrc(a.y + img_n * a.y_img, 0, (int)(a.y_img * 4), 0x00020000);
        if constexpr (CB == 4) {
          u32x4 v;
          v.x = __float_as_uint(o[0]), v.y = __float_as_uint(o[1]), v.z = __float_as_uint(o[2]), v.w = __float_as_uint(o[3]);
          __builtin_amdgcn_raw_buffer_store_b128(v, yr, (int)(at * 4), 0, kSc1);
        } else {
          u32x2 v;
          v.x = __float_as_uint(o[0]), v.y = __float_as_uint(o[1]);
          __builtin_amdgcn_raw_buffer_store_b64(v, yr, (int)(at * 4), 0, kSc1);
        }
      } else {
        if constexpr (CB == 4) *reinterpret_cast<float4*>(dst) = make_float4(o[0], o[1], o[2], o[3]);
        else *reinterpret_cast<float2*>(dst) = make_float2(o[0], o[1]);
      }
    }
  }
  if constexpr (LOUT) {
    // stores acknowledged, everybody there, then the flag of (patch, slice)
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (tid == 0)
      __hip_atomic_store(L.flags + (size_t)(L.out_base + tile * a.slices + slice) * kLinkFlagStride, 1, __ATOMIC_RELAXED,
                         __HIP_MEMORY_SCOPE_AGENT);
  }
}

template <int C, int WK, int WN, int CB, int S, bool STEM = false>
__global__ __launch_bounds__(64 * WK * WN) void separable_block_kernel(const BlockArgs a) {
  __shared__ __align__(16) float lds[BlockShape<C, WK, WN, CB, S>::kLds];
  __shared__ float img[STEM ? 13 * kImgRow : 1];
  __shared__ __align__(16) float wst[STEM ? 28 * kWstRow : 4];  // [27][32 of 48] filter, [32] bias
  block_body<C, WK, WN, CB, S, STEM, false, false>(a, blockIdx.x, lds, img, wst, BlockLink{}, nullptr);
}

// Blocks 2, 3 and 4 of the batch-1 network (64 -> 128 at stride 2, 128 -> 128 at stride 1, 128 -> 256 at stride 2)
// as three stages of one launch: workgroups [0, first[1]) are block 2's, [first[1], first[2]) block 3's, the rest
// block 4's; a stage's workgroup waits for the flags of the patches under its window instead of for a kernel
// boundary, and has fetched its arguments and filters by then.  Workgroups start in the order of their ids, so a
// waiting workgroup never keeps its producers from starting; every wait is bounded all the same.
struct BlockChainArgs {
  BlockArgs blk[3];
  BlockLink link[3];
  int first[3];
};
constexpr int kChainLds = BlockShape<128, 8, 1, 4, 2>::kLds;
static_assert(kChainLds >= BlockShape<64, 4, 2, 2, 2>::kLds && kChainLds >= BlockShape<128, 8, 1, 4, 1>::kLds, "LDS of the widest stage");
__global__ __launch_bounds__(512) void separable_chain_kernel(const BlockChainArgs h) {
  __shared__ __align__(16) float lds[kChainLds];
  __shared__ int gave_up;
  const int bid = blockIdx.x;
  if (bid < h.first[1]) block_body<64, 4, 2, 2, 2, false, false, true>(h.blk[0], bid, lds, nullptr, nullptr, h.link[0], &gave_up);
  else if (bid < h.first[2])
    block_body<128, 8, 1, 4, 1, false, true, true>(h.blk[1], bid - h.first[1], lds, nullptr, nullptr, h.link[1], &gave_up);
  else block_body<128, 8, 1, 4, 2, false, true, false>(h.blk[2], bid - h.first[2], lds, nullptr, nullptr, h.link[2], &gave_up);
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
  // 256 channels: the 9 x 9 window of a stride-2 block would not fit the static LDS
  return batch >= 1 && batch <= kMaxFusedBatch && (c == 32 || c == 64 || c == 128 || (c == 256 && stride == 1)) &&
         n % 64 == 0 && n >= 64 && n <= 1024 &&
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
  if (c == 256 && stride == 1) return launch_cfg<256, 8, 1, 4, 1>(a, stream);
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

// ---- blocks 2 - 4 of a single full-width image as one launch ----
namespace {
BlockArgs plain_args(const float* x, const float* dw_w, const float* dw_b, const float* pw_w, const float* pw_b, float* y,
                     int h, int w, int c, int n, int stride, int ns) {
  BlockArgs a;
  a.x = x, a.dw_w = dw_w, a.dw_b = dw_b, a.pw_w = pw_w, a.pw_b = pw_b, a.y = y;
  a.H = h, a.W = w, a.OH = (h + stride - 1) / stride, a.OW = (w + stride - 1) / stride, a.N = n;
  // SAME padding of a 3-tap filter: the odd unit goes after the map
  const int need_h = (a.OH - 1) * stride + 3 - h, need_w = (a.OW - 1) * stride + 3 - w;
  a.pt = need_h > 0 ? need_h / 2 : 0, a.pl = need_w > 0 ? need_w / 2 : 0;
  a.dw_act = a.pw_act = TFX_ACT_RELU6;
  a.batch = 1;
  a.x_bytes = (unsigned)((long long)h * w * c * 4);
  a.x_img = (long long)h * w * c;
  a.tiles_x = (a.OW + 3) / 4;
  a.tiles_img = a.tiles_x * ((a.OH + 3) / 4);
  a.slices = n / ns;
  a.total = a.tiles_img * a.slices;
  a.y_img = (long long)a.OH * a.OW * n;
  a.st_w = a.st_b = nullptr, a.IH = a.IW = a.st_pt = a.st_pl = a.st_act = 0;
  a.zero_words = nullptr, a.zero_count = 0, a.zero_stride = 1;
  return a;
}
}  // namespace

int block_chain_flag_stride() { return kLinkFlagStride; }

// Flags the chained launch needs for a first map of h x w pixels: one per (patch, slice) of its first two stages.
int block_chain_flag_words(int h, int w) {
  const int oh = (h + 1) / 2, ow = (w + 1) / 2;
  return 2 * 2 * ((oh + 3) / 4) * ((ow + 3) / 4);
}

// x: [h, w, 64], the output of block 1; b2_out / b3_out: [ceil(h/2), ceil(w/2), 128]; y: the output of block 4,
// [ceil(h/4), ceil(w/4), 256] (sizes rounded up at each halving).  flags: block_chain_flag_words() words from index
// flag_base on, block_chain_flag_stride() words apart, zero when the kernel starts; word 0 is the failure word.
bool block_chain_supported(const void* x, const void* b2_out, const void* b3_out, const void* y,
                           const tfx_mobilenet_v1_weights* w) {
  auto al16 = [](const void* p) { return reinterpret_cast<uintptr_t>(p) % 16 == 0; };
  bool ok = al16(x) && al16(b2_out) && al16(b3_out) && al16(y);
  for (int i = 1; i <= 3 && ok; ++i) ok = al16(w->dw_w[i]) && al16(w->dw_b[i]) && al16(w->pw_w[i]) && al16(w->pw_b[i]);
  return ok;
}

int launch_block_chain(const float* x, float* b2_out, float* b3_out, float* y, int h, int w,
                       const tfx_mobilenet_v1_weights* wt, int* flags, int flag_base, int spin_limit,
                       hipStream_t stream) {
  BlockChainArgs c;
  c.blk[0] = plain_args(x, wt->dw_w[1], wt->dw_b[1], wt->pw_w[1], wt->pw_b[1], b2_out, h, w, 64, 128, 2, 64);
  const int h2 = c.blk[0].OH, w2 = c.blk[0].OW;
  c.blk[1] = plain_args(b2_out, wt->dw_w[2], wt->dw_b[2], wt->pw_w[2], wt->pw_b[2], b3_out, h2, w2, 128, 128, 1, 64);
  c.blk[2] = plain_args(b3_out, wt->dw_w[3], wt->dw_b[3], wt->pw_w[3], wt->pw_b[3], y, h2, w2, 128, 256, 2, 64);
  c.first[0] = 0, c.first[1] = c.blk[0].total, c.first[2] = c.blk[0].total + c.blk[1].total;
  const int f0 = flag_base, f1 = flag_base + c.blk[0].total;
  c.link[0] = BlockLink{flags, -1, 0, 0, f0, spin_limit};
  c.link[1] = BlockLink{flags, f0, c.blk[0].tiles_x, c.blk[0].slices, f1, spin_limit};
  c.link[2] = BlockLink{flags, f1, c.blk[1].tiles_x, c.blk[1].slices, -1, spin_limit};
  const int total = c.first[2] + c.blk[2].total;
  hipLaunchKernelGGL(separable_chain_kernel, dim3((unsigned)total), dim3(512), 0, stream, c);
  return check_launch();
}

}  // namespace tfx
