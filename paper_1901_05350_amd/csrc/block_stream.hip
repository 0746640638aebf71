// A depthwise-separable block of the Section 3.9 network at large batch in one launch (fp32):
//   y = relu6(pointwise(relu6(depthwise3x3(x) + dw_b)) + pw_b),  depthwise stride 1 or 2, SAME padding.
// At batch 64 the early blocks are bound by HBM, and as two kernels the depthwise layer's output makes a round
// trip through memory (103 MB out and in again for 56 x 56 x 128) that costs as much as the block's own input and
// output.  This is the filter-stationary pointwise kernel of pointwise.hip with its operand computed instead of
// loaded: the pointwise filter lives in LDS ([K][N + 4] floats), the 8 wavefronts of a workgroup take units of the
// output from a counter in LDS, and a unit is a 2 x 8 patch of output pixels of one image -- the 16 columns of the
// v_mfma_f32_16x16x4_f32 operand.  The wavefront copies the patch's input window, 32 channels at a time (whole
// 128-byte lines), into a private piece of LDS, and lane (li, q) -- pixel (li / 8, li % 8) of the patch, channels
// 16 g + 4 q ... + 3 of every group g of 16 -- forms its operand values as the depthwise result of its pixel: 9
// taps of 16 bytes from the window times the depthwise filter, also from LDS.  The next 32 channels of the window
// are on their way from memory into registers meanwhile.  (Taking the taps straight from memory instead was
// measured: 72 loads of 16 half lines each per unit make the texture path the limit.)
#include "tfx_internal.h"

#include <type_traits>

namespace tfx {
namespace {

constexpr int kThreads = 512, kWaves = kThreads / 64;
constexpr int kPatchH = 2, kPatchW = 8;  // output pixels of a unit
constexpr int kChunk = 32;               // channels of the window held in LDS at a time
typedef float v4f __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

struct WindowBlockGeom {
  int H, W, OH, OW, pt, pl;
  int tiles_c, tiles_r;  // patches per output row and column
  unsigned x_bytes;
};

// LDS layout of a window of 32 channels in 16-byte pieces: pixel stride PS >= 8 pieces, row stride RS >= WW * PS,
// the least ones for which the tap read of a wavefront (pixel (li / 8, li % 8) * S plus a constant, piece q) has
// no bank conflict.
template <int S>
struct WindowLayout {
  static constexpr int WH = (kPatchH - 1) * S + 3, WW = (kPatchW - 1) * S + 3;
  struct Piece {
    int ps, rs;
    constexpr int operator()(int li, int q) const { return (li / 8) * S * rs + (li % 8) * S * ps + q; }
  };
  static constexpr int pixel_stride() {
    for (int ps = kChunk / 4;; ++ps)
      for (int rs = WW * ps; rs < WW * ps + 32; ++rs)
        if (conflict_free(Piece{ps, rs})) return ps;
  }
  static constexpr int PS = pixel_stride();
  static constexpr int row_stride() {
    for (int rs = WW * PS;; ++rs)
      if (conflict_free(Piece{PS, rs})) return rs;
  }
  static constexpr int RS = row_stride();
  static constexpr int kFloats = WH * RS * 4;
  static constexpr int kPieces = WH * WW * (kChunk / 4), kLoads = (kPieces + 63) / 64;
};

template <int K, int N, int S>
__global__ __launch_bounds__(kThreads) void separable_window_kernel(const float* __restrict__ x,
                                                                    const float* __restrict__ dw_w,
                                                                    const float* __restrict__ dw_b,
                                                                    const float* __restrict__ pw_w,
                                                                    const float* __restrict__ pw_b,
                                                                    float* __restrict__ y, WindowBlockGeom g, int units,
                                                                    int dw_act, int pw_act) {
  using WL = WindowLayout<S>;
  constexpr int KG = K / 16, NB = N / 16, LD = N + 4, CH = K / kChunk;
  constexpr int NBP = NB < 8 ? NB : 8;  // 16-column blocks per pass
  constexpr int PS = WL::PS, RS = WL::RS, WW = WL::WW, LI = WL::kLoads, Q = kChunk / 4;
  static_assert((K * N / 4) % kThreads == 0 && N <= kThreads && 9 * K / 4 <= kThreads && NB % 2 == 0 && K % kChunk == 0,
                "staging");
  // pointwise filter [K][N + 4], its bias [N], depthwise filter [9][K], its bias [K], then one window per wavefront
  extern __shared__ __align__(16) float wl[];
  float* const pwb_l = wl + K * LD;
  float* const dww_l = pwb_l + N;
  float* const dwb_l = dww_l + 9 * K;
  __shared__ int next_unit;

  const int tid = threadIdx.x;
  const int lane = tid % 64, li = lane % 16, q = lane / 16;
  float* const win = dwb_l + K + (tid / 64) * WL::kFloats;
  const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(x), 0, (int)g.x_bytes, 0x00020000);
  const int u0 = (int)((long long)units * blockIdx.x / gridDim.x);
  const int u1 = (int)((long long)units * (blockIdx.x + 1) / gridDim.x);

  // This lane's pieces of a window chunk: piece e = lane + 64 i is 4 channels (cq) of window pixel (wr, wc).
  int wrc[LI], goff[LI], loff[LI];
#pragma unroll
  for (int i = 0; i < LI; ++i) {
    const int e = lane + 64 * i, p = e / Q, cq = e % Q, wr = p / WW, wc = p % WW;
    wrc[i] = wr | wc << 8 | (e < WL::kPieces ? 1 << 16 : 0);  // bit 16: the piece exists
    goff[i] = ((wr * g.W + wc) * K + 4 * cq) * 4;
    loff[i] = (wr * RS + wc * PS + cq) * 4;
  }
  // a unit's place: image, patch, and the byte offset of window pixel (0, 0), channel 0 (may lie outside x)
  struct Place {
    int n, tr, tc, ih0, iw0, base;
  };
  auto place_of = [&](int unit) {
    Place p;
    p.tc = unit % g.tiles_c;
    const int t1 = unit / g.tiles_c;
    p.tr = t1 % g.tiles_r;
    p.n = t1 / g.tiles_r;
    p.ih0 = kPatchH * p.tr * S - g.pt;
    p.iw0 = kPatchW * p.tc * S - g.pl;
    p.base = ((p.n * g.H + p.ih0) * g.W + p.iw0) * K * 4;
    return p;
  };
  // byte offsets of this lane's window pieces, channel 0; a piece outside the image (or of no unit) gets an offset
  // past the end of the buffer, from where the hardware returns 0
  struct Offsets {
    unsigned v[LI];
  };
  auto offsets_of = [&](const Place& p, bool live) {
    Offsets o;
#pragma unroll
    for (int i = 0; i < LI; ++i) {
      const int ih = p.ih0 + (wrc[i] & 0xff), iw = p.iw0 + ((wrc[i] >> 8) & 0xff);
      const bool in = live & (wrc[i] >> 16 != 0) & ((unsigned)ih < (unsigned)g.H) & ((unsigned)iw < (unsigned)g.W);
      o.v[i] = in ? (unsigned)(p.base + goff[i]) : 0x80000000u;
    }
    return o;
  };
  // window pieces of one chunk of 32 channels
  u32x4 wreg[LI];
  auto load_chunk = [&](const Offsets& o, int ch) {
#pragma unroll
    for (int i = 0; i < LI; ++i) wreg[i] = __builtin_amdgcn_raw_buffer_load_b128(xr, (int)o.v[i], kChunk * 4 * ch, 0);
  };

  // The first unit of a wavefront is fixed (the rest are handed out by the counter) and the first chunk of its
  // window is requested before the filters are staged.
  if (tid == 0) next_unit = kWaves;
  int cur = u0 + __builtin_amdgcn_readfirstlane(tid / 64);
  Place pc = place_of(cur < u1 ? cur : u0);
  Offsets oc = offsets_of(pc, cur < u1);
  load_chunk(oc, 0);
  {
    constexpr int PER = K * N / 4 / kThreads;
    float4 t[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) t[i] = reinterpret_cast<const float4*>(pw_w)[tid + i * kThreads];
    // (no branches around these loads: a thread past the end reads element 0 and its value is dropped)
    const float4 dwv = reinterpret_cast<const float4*>(dw_w)[tid < 9 * K / 4 ? tid : 0];
    const float pwb = (pw_b ? pw_b : pw_w)[tid < N ? tid : 0];
    const float dwb = (dw_b ? dw_b : pw_w)[tid < K ? tid : 0];
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int e = tid + i * kThreads;  // float4 index: row e / (N/4), column quad e % (N/4)
      *reinterpret_cast<float4*>(wl + (e / (N / 4)) * LD + 4 * (e % (N / 4))) = t[i];
    }
    if (tid < 9 * K / 4) reinterpret_cast<float4*>(dww_l)[tid] = dwv;
    if (tid < N) pwb_l[tid] = pw_b ? pwb : 0.f;
    if (tid < K) dwb_l[tid] = dw_b ? dwb : 0.f;
  }
  __syncthreads();

  const ActClamp dw_clamp = make_act(dw_act), pw_clamp = make_act(pw_act);
  const float dw_lo = dw_clamp.on ? 0.f : -INFINITY;
  // where this lane's taps start in a window: pixel (li / 8, li % 8) * S, piece q
  const float* const tap0 = win + ((li / 8) * S * RS + (li % 8) * S * PS + q) * 4;

  // W blocks of 16 columns, starting at block jb, of one unit whose operand values are in a[]
  auto columns = [&](auto wc_, const float4 (&a)[KG], float* ya, float* yb, bool oka, bool okb, int jb) {
    constexpr int W = decltype(wc_)::value;
    floatx4 acc[W];
#pragma unroll
    for (int j = 0; j < W; ++j) acc[j] = *reinterpret_cast<const floatx4*>(pwb_l + 16 * (jb + j) + 4 * q);
#pragma unroll
    for (int gg = 0; gg < KG; ++gg) {
      const float av[4] = {a[gg].x, a[gg].y, a[gg].z, a[gg].w};
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const float* wr = wl + (16 * gg + 4 * q + s) * LD + 16 * jb + li;
#pragma unroll
        for (int j = 0; j < W; ++j)
          acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(wr[16 * j], av[s], acc[j], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);  // keep later groups' LDS reads from being hoisted
    }
    store_rows_biased<W>(acc, ya + 16 * jb, yb + 16 * jb, oka, okb, li, q, pw_clamp);
  };

  // the first chunk of a unit's window is requested before the MFMAs of the unit before it
  while (cur < u1) {
    int ticket = 0;
    if (lane == 0) ticket = atomicAdd(&next_unit, 1);
    // depthwise layer, chunk by chunk: the chunk in the registers goes to LDS, the next one is requested, and the
    // two 16-channel groups of the chunk are reduced over the 9 taps.  The clamp is a median of three; that
    // instruction drops a NaN, so NaNs are looked for on the side and a wavefront that holds one repeats the
    // layer with the exact form.
    float4 a[KG];
    auto depthwise = [&](auto exact) {
      unsigned long long nan = 0;
      if constexpr (decltype(exact)::value) load_chunk(oc, 0);
#pragma unroll
      for (int ch = 0; ch < CH; ++ch) {
#pragma unroll
        for (int i = 0; i < LI; ++i)
          if (LI * 64 == WL::kPieces || i + 1 < LI || lane + 64 * i < WL::kPieces)
            *reinterpret_cast<u32x4*>(win + loff[i]) = wreg[i];
        if (ch + 1 < CH) load_chunk(oc, ch + 1);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int gl = 0; gl < kChunk / 16; ++gl) {
          const int gg = (kChunk / 16) * ch + gl;
          v4f acc = *reinterpret_cast<const v4f*>(dwb_l + 16 * gg + 4 * q);
#pragma unroll
          for (int t = 0; t < 9; ++t)
            acc += *reinterpret_cast<const v4f*>(tap0 + ((t / 3) * RS + (t % 3) * PS + 4 * gl) * 4) *
                   *reinterpret_cast<const v4f*>(dww_l + t * K + 16 * gg + 4 * q);
          if constexpr (decltype(exact)::value) {
            a[gg] = make_float4(apply_act(acc[0], dw_clamp), apply_act(acc[1], dw_clamp), apply_act(acc[2], dw_clamp),
                                apply_act(acc[3], dw_clamp));
          } else {
            nan |= __builtin_amdgcn_ballot_w64(__builtin_isunordered(acc[0], acc[1]) | __builtin_isunordered(acc[2], acc[3]));
            a[gg] = make_float4(__builtin_amdgcn_fmed3f(acc[0], dw_lo, dw_clamp.hi), __builtin_amdgcn_fmed3f(acc[1], dw_lo, dw_clamp.hi),
                                __builtin_amdgcn_fmed3f(acc[2], dw_lo, dw_clamp.hi), __builtin_amdgcn_fmed3f(acc[3], dw_lo, dw_clamp.hi));
          }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
      }
      return nan;
    };
    if (depthwise(std::false_type{}) != 0) depthwise(std::true_type{});

    const int nxt = u0 + __builtin_amdgcn_readfirstlane(ticket);
    const Place pn = place_of(nxt < u1 ? nxt : cur);
    const Offsets on = offsets_of(pn, nxt < u1);
    load_chunk(on, 0);

    // this lane's two output rows of the [pixels, N] matrix: patch pixels (0, li % 8) and (1, li % 8)
    const int oh = kPatchH * pc.tr, ow = kPatchW * pc.tc + (li & 7);
    float* const ya = y + ((size_t)(pc.n * g.OH + oh) * g.OW + ow) * N;
    float* const yb = ya + (size_t)g.OW * N;
    const bool oka = ow < g.OW, okb = oka && oh + 1 < g.OH;
#pragma unroll
    for (int pp = 0; pp < NB / NBP; ++pp)  // column passes of at most 128 columns keep the accumulators few
      columns(std::integral_constant<int, NBP>{}, a, ya, yb, oka, okb, NBP * pp);
    cur = nxt;
    pc = pn;
    oc = on;
  }
}

template <int K, int N, int S>
int launch_cfg(const float* x, const float* dw_w, const float* dw_b, const float* pw_w, const float* pw_b, float* y,
               const WindowBlockGeom& g, int units, int dw_act, int pw_act, hipStream_t stream) {
  constexpr size_t lds_bytes = ((size_t)K * (N + 4) + N + 10 * K + (size_t)kWaves * WindowLayout<S>::kFloats) * sizeof(float);
  static_assert(lds_bytes + 64 <= 160 * 1024, "LDS budget per workgroup");
  auto kern = separable_window_kernel<K, N, S>;
  static std::atomic<uint64_t> lds_allowed{0};
  if (allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds_bytes, lds_allowed) != TFX_OK) return TFX_ERR_LAUNCH;
  // as many workgroups as are resident at once: each loads the filters once
  static std::atomic<int> resident{0};
  int per_cu = resident.load(std::memory_order_relaxed);
  if (per_cu == 0) {
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, kThreads, lds_bytes) != hipSuccess || per_cu < 1)
      per_cu = 1;
    if (per_cu > 2) per_cu = 2;
    resident.store(per_cu, std::memory_order_relaxed);
  }
  int blocks = 256 * per_cu;
  if (blocks > (units + kWaves - 1) / kWaves) blocks = (units + kWaves - 1) / kWaves;
  hipLaunchKernelGGL(kern, dim3(blocks), dim3(kThreads), lds_bytes, stream, x, dw_w, dw_b, pw_w, pw_b, y, g, units,
                     dw_act, pw_act);
  return check_launch();
}

}  // namespace

// Blocks (channels -> filters, stride) of the full-width network's 112 x 112 and 56 x 56 maps, many output pixels
// (below that the two single-op kernels' tiles win), 16-byte aligned operands, an input below 2^31 bytes.
bool separable_stream_supported(int batch, int h, int w, int c, int n, int stride, int oh, int ow, const void* x,
                                const void* dw_w, const void* dw_b, const void* pw_w, const void* pw_b, const void* y) {
  const bool shape = (c == 128 && n == 128 && stride == 1) || (c == 64 && n == 128 && stride == 2) ||
                     (c == 32 && n == 64 && stride == 1);
  const void* ptrs[] = {x, dw_w, dw_b, pw_w, pw_b, y};
  bool aligned = true;
  for (const void* p : ptrs) aligned = aligned && reinterpret_cast<uintptr_t>(p) % 16 == 0;
  const long long m = (long long)batch * oh * ow, x_bytes = (long long)batch * h * w * c * 4;
  return shape && aligned && m >= 8192 && m <= 0x3fffffffLL && x_bytes < (1ll << 31);
}

int launch_separable_stream(const float* x, const float* dw_w, const float* dw_b, const float* pw_w, const float* pw_b,
                            float* y, int batch, int h, int w, int c, int n, int oh, int ow, int stride, int pt, int pl,
                            int dw_act, int pw_act, hipStream_t stream) {
  const WindowBlockGeom g{h, w, oh, ow, pt, pl, (ow + kPatchW - 1) / kPatchW, (oh + kPatchH - 1) / kPatchH,
                          (unsigned)((long long)batch * h * w * c * 4)};
  const long long units = (long long)batch * g.tiles_c * g.tiles_r;
  if (units > 0x3fffffffLL) return TFX_ERR_UNSUPPORTED;
#define TFX_WINDOW_BLOCK(C, NN, SS) \
  if (c == C && n == NN && stride == SS) \
    return launch_cfg<C, NN, SS>(x, dw_w, dw_b, pw_w, pw_b, y, g, (int)units, dw_act, pw_act, stream);
  TFX_WINDOW_BLOCK(128, 128, 1)
  TFX_WINDOW_BLOCK(64, 128, 2)
  TFX_WINDOW_BLOCK(32, 64, 1)
#undef TFX_WINDOW_BLOCK
  return TFX_ERR_UNSUPPORTED;
}

}  // namespace tfx
