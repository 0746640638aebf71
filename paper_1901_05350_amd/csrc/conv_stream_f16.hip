// 3x3 stride-1 conv2d with a small filter on 16-bit float storage for gfx950 (Section 4.1 storage format; the NHWC
// index order of the conv2d sampler):
//   y[M, N] = half(act(A[M, K] * w[K, N] + bias)),  M = n * oh * ow,  K = 9 * Ci,
// where row m of A is the 3 x 3 x Ci window of output pixel m, never materialised.
// With few channels the whole filter (K * N * 2 bytes, e.g. 74 KB for 64 -> 64) fits in LDS, and then the filter is
// the stationary operand, as in pointwise_f16.hip: a workgroup transposes w into LDS once (stream_f16.h) and its
// 8 wavefronts stream units of the output without meeting at a barrier again.  A unit is a 4 x 8 patch of output
// pixels of one image (two v_mfma_f32_16x16x32_f16 slabs of 2 x 8 pixels).  The wavefront copies the patch's 6 x 10
// input window into a private piece of LDS -- every input value crosses the vector memory path 1.9 times instead of
// 9 -- and reads each lane's MFMA operand (its pixel under one tap, 8 consecutive channels) from there with
// compile-time offsets; each filter fragment read from LDS serves both slabs.  The window of the wavefront's next
// unit is on its way from memory into registers while the current one is multiplied.  The filter's columns are
// stored in LDS in an order that leaves every lane with 8 consecutive output channels, so outputs go from the
// accumulators to memory as 16-byte pieces.
#include "stream_f16.h"

namespace tfx {
namespace {

using namespace f16s;

constexpr int kThreads = 512, kWaves = kThreads / 64;
constexpr int kPatchH = 4, kPatchW = 8;                      // output pixels of a unit
constexpr int kWinH = kPatchH + 2, kWinW = kPatchW + 2;      // its input window

struct WindowGeom {
  int H, W, OH, OW, pt, pl;
  int tiles_c, tiles_r;   // patches per output row and per output column
  unsigned x_bytes;
};

// LDS layout of a window in 16-byte pieces: a pixel takes Ci/8 pieces plus two of padding and a row of the window
// a multiple of 16 pieces that is not one of 32, which puts the 2 x 8 pixels of a slab, two k-groups each, into 32
// different columns (checked below).
template <int CI>
struct WindowShape {
  static constexpr int Q = CI / 8, PS = Q + 2;
  static constexpr int row_stride() {
    int v = kWinW * PS;
    while (v % 32 != 16) ++v;
    return v;
  }
  static constexpr int RS = row_stride();
  static constexpr int kHalfs = kWinH * RS * 8;
  static constexpr int kPieces = kWinH * kWinW * Q, kLoads = (kPieces + 63) / 64;
  static constexpr int piece(int li, int q) { return (li / 8) * RS + (li % 8) * PS + q; }
  static_assert(conflict_free(piece), "window layout");
};

template <int CI, int N>
__global__ __launch_bounds__(kThreads) void conv3x3_window_f16_kernel(const half_t* __restrict__ x,
                                                                      const half_t* __restrict__ w,
                                                                      const half_t* __restrict__ bias,
                                                                      half_t* __restrict__ y, WindowGeom g, int units,
                                                                      int act) {
  using WS = WindowShape<CI>;
  using Stage = FilterStage<9 * CI, N, kThreads>;
  constexpr int SPT = CI / 32, NB = N / 16, LD = Stage::LD;
  constexpr int Q = WS::Q, PS = WS::PS, RS = WS::RS, LI = WS::kLoads;
  static_assert(CI % 32 == 0 && N % 32 == 0 && NB <= 8, "filter shape");
  extern __shared__ __align__(16) half_t wl[];  // the filter, [N][LD], then one window per wavefront
  __shared__ int next_unit;

  const int tid = threadIdx.x;
  const int lane = tid % 64, li = lane % 16, q = lane / 16;
  half_t* const win = wl + N * LD + (tid / 64) * WS::kHalfs;
  const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(const_cast<half_t*>(x), 0, (int)g.x_bytes, 0x00020000);
  const int u0 = (int)((long long)units * blockIdx.x / gridDim.x);
  const int u1 = (int)((long long)units * (blockIdx.x + 1) / gridDim.x);

  // This lane's pieces of a window: piece e = lane + 64 i is 8 channels (cq) of window pixel (wr, wc).
  int wrc[LI], goff[LI], loff[LI];
#pragma unroll
  for (int i = 0; i < LI; ++i) {
    const int e = lane + 64 * i, p = e / Q, cq = e % Q, wr = p / kWinW, wc = p % kWinW;
    wrc[i] = wr | wc << 8 | (e < WS::kPieces ? 1 << 16 : 0);  // bit 16: the piece exists
    goff[i] = (wr * g.W + wc) * CI + 8 * cq;
    loff[i] = (wr * RS + wc * PS + cq) * 8;
  }
  u32x4 wreg[LI];
  // window loads of a unit; a piece outside the image (or no unit left) is fetched from past the end of the
  // buffer, where the hardware returns 0
  auto load_window = [&](int unit, bool live) {
    const int tc = unit % g.tiles_c, t = unit / g.tiles_c, tr = t % g.tiles_r, n = t / g.tiles_r;
    const int ih0 = kPatchH * tr - g.pt, iw0 = kPatchW * tc - g.pl;
    const int base = ((n * g.H + ih0) * g.W + iw0) * CI;
#pragma unroll
    for (int i = 0; i < LI; ++i) {
      const int ih = ih0 + (wrc[i] & 0xff), iw = iw0 + ((wrc[i] >> 8) & 0xff);
      const bool in = live & (wrc[i] >> 16 != 0) & ((unsigned)ih < (unsigned)g.H) & ((unsigned)iw < (unsigned)g.W);
      const unsigned off = in ? (unsigned)(base + goff[i]) * 2u : 0x80000000u;
      wreg[i] = __builtin_amdgcn_raw_buffer_load_b128(xr, (int)off, 0, 0);
    }
  };

  // the filter's loads and the bias's first, so that they are on their way while the window's are set up
  Stage stage;
  stage.fetch(w, tid);
  BiasRows<NB> bias_rows;
  bias_rows.fetch(bias, w, q);

  // the first unit of each wavefront is fixed, and its window is in flight while the filter is staged; the rest
  // are handed out by a counter in LDS
  int cur = u0 + __builtin_amdgcn_readfirstlane(tid / 64);
  if (tid == 0) next_unit = kWaves;
  load_window(cur, cur < u1);
  stage.store(wl, tid);
  const ActClamp clamp = make_act(act);
  // this lane's MFMA operand inside a window: pixel (li / 8, li % 8) of a slab, pieces q, q + 4, ...
  const half_t* const a_base = win + ((li / 8) * RS + (li % 8) * PS + q) * 8;
  const half_t* const w_base = wl + li * LD + 8 * q;
  __syncthreads();
  f32x4 bv[NB];
  bias_rows.get(bias != nullptr, bv);
  auto draw = [&]() {
    int ticket = 0;
    if (lane == 0) ticket = atomicAdd(&next_unit, 1);
    return ticket;
  };
  // the window in the registers goes to LDS and the registers are refilled with the window of `then`
  auto advance_window = [&](int then) {
#pragma unroll
    for (int i = 0; i < LI; ++i)
      if (LI * 64 == WS::kPieces || i + 1 < LI || lane + 64 * i < WS::kPieces)
        *reinterpret_cast<u32x4*>(win + loff[i]) = wreg[i];
    load_window(then, then < u1);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
  };
  // k-steps of 32: step s is channels 32 (s % SPT) ... of tap s / SPT.  The fragments of step s + 2 (s + 1 with
  // 128 output channels, for the registers' sake) are read from LDS before the MFMAs of step s are issued; the
  // scheduling barriers keep the compiler from moving the reads back to where their values are used.
  constexpr int STEPS = 9 * SPT, BUFS = NB > 4 ? 2 : 3, AHEAD = BUFS - 1;
  h8 fa[BUFS][2], fw[BUFS][NB];
  auto read_step = [&](int st, h8 (&a)[2], h8 (&f)[NB]) {
    const int t = st / SPT, ss = st % SPT;
    const int tap = ((t / 3) * RS + (t % 3) * PS + 4 * ss) * 8;
    a[0] = *reinterpret_cast<const h8*>(a_base + tap);
    a[1] = *reinterpret_cast<const h8*>(a_base + tap + 2 * RS * 8);
#pragma unroll
    for (int j = 0; j < NB; ++j) f[j] = *reinterpret_cast<const h8*>(w_base + 16 * j * LD + 32 * st);
  };
  auto read_first_steps = [&]() {
#pragma unroll
    for (int st = 0; st < AHEAD; ++st) read_step(st, fa[st], fw[st]);
  };

  // Per pass: the MFMAs of unit `cur`, whose window is in LDS and whose first fragments have been read; then the
  // window of `nxt` goes from the registers to LDS, the loads of the unit after it are issued and the first
  // fragments of `nxt` are read, all of which is in flight while the outputs of `cur` are clamped and stored.
  int nxt = u0 + __builtin_amdgcn_readfirstlane(draw());
  advance_window(nxt);
  read_first_steps();
  while (cur < u1) {
    const int ticket = draw();  // the unit after `nxt`; its number is not needed before the MFMAs are through
    f32x4 acc0[NB], acc1[NB];  // start from the bias
#pragma unroll
    for (int j = 0; j < NB; ++j) acc0[j] = acc1[j] = bv[j];
#pragma unroll
    for (int st = 0; st < STEPS; ++st) {
      if (st + AHEAD < STEPS) read_step(st + AHEAD, fa[(st + AHEAD) % BUFS], fw[(st + AHEAD) % BUFS]);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        acc0[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fw[st % BUFS][j], fa[st % BUFS][0], acc0[j], 0, 0, 0);
        acc1[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fw[st % BUFS][j], fa[st % BUFS][1], acc1[j], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    const int then = u0 + __builtin_amdgcn_readfirstlane(ticket);
    advance_window(then);
    read_first_steps();
    __builtin_amdgcn_sched_barrier(0);

    // Epilogue: activation, and one 16-byte store per lane, slab and 32 channels (a pixel's 4 lanes write
    // 64 consecutive bytes).
    const int tc = cur % g.tiles_c, tq = cur / g.tiles_c, tr = tq % g.tiles_r, n = tq / g.tiles_r;
    auto emit = [&](const f32x4 (&acc)[NB], int slab) {
      const int oh = kPatchH * tr + 2 * slab + li / 8, ow = kPatchW * tc + li % 8;
      half_t* const yp = y + ((size_t)(n * g.OH + oh) * g.OW + ow) * N + 8 * q;
      h8 o[NB / 2];
      activate_and_pack(acc, clamp, o);
      if (oh < g.OH && ow < g.OW) {
#pragma unroll
        for (int m = 0; m < NB / 2; ++m) *reinterpret_cast<h8*>(yp + 32 * m) = o[m];
      }
    };
    emit(acc0, 0);
    emit(acc1, 1);
    cur = nxt;
    nxt = then;
  }
}

template <int CI, int N>
constexpr size_t window_lds_bytes() {
  return ((size_t)N * filter_row_halfs(9 * CI) + (size_t)kWaves * WindowShape<CI>::kHalfs) * sizeof(half_t);
}

template <int CI, int N>
int launch_window(const half_t* x, const half_t* w, const half_t* bias, half_t* y, const WindowGeom& g, int units,
                  int act, hipStream_t stream) {
  constexpr size_t lds_bytes = window_lds_bytes<CI, N>();
  static_assert(lds_bytes + 64 <= 160 * 1024, "LDS budget per workgroup");
  auto kern = conv3x3_window_f16_kernel<CI, N>;
  static std::atomic<uint64_t> lds_allowed{0};
  if (allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds_bytes, lds_allowed) != TFX_OK) return TFX_ERR_LAUNCH;
  int blocks = 256;  // one workgroup per CU
  if (blocks > (units + kWaves - 1) / kWaves) blocks = (units + kWaves - 1) / kWaves;
  hipLaunchKernelGGL(kern, dim3(blocks), dim3(kThreads), lds_bytes, stream, x, w, bias, y, g, units, act);
  return check_launch();
}

}  // namespace

// 3 x 3 filters at stride 1 whose transposed copy fits in LDS beside the windows, many output pixels, 16-byte
// aligned operands, an input of fewer than 2^31 bytes (32-bit buffer offsets).
bool conv3x3_stream_f16_supported(long long m, long long x_elems, int ci, int fh, int fw, int co, int sh, int sw,
                                  const void* x, const void* w, const void* y) {
  const bool shape = fh == 3 && fw == 3 && sh == 1 && sw == 1 &&
                     ((ci == 32 && (co == 32 || co == 64 || co == 128)) || (ci == 64 && (co == 32 || co == 64)));
  const bool aligned = reinterpret_cast<uintptr_t>(x) % 16 == 0 && reinterpret_cast<uintptr_t>(w) % 16 == 0 &&
                       reinterpret_cast<uintptr_t>(y) % 16 == 0;
  return shape && aligned && m >= 16384 && m <= 0x3fffffffLL && x_elems * 2 < (1ll << 31);
}

int launch_conv3x3_stream_f16(const uint16_t* x16, const uint16_t* w16, const uint16_t* bias16, uint16_t* y16, int n, int h,
                              int wd, int ci, int co, int oh, int ow, int pt, int pl, int act, hipStream_t stream) {
  const half_t* x = reinterpret_cast<const half_t*>(x16);
  const half_t* w = reinterpret_cast<const half_t*>(w16);
  const half_t* bias = reinterpret_cast<const half_t*>(bias16);
  half_t* y = reinterpret_cast<half_t*>(y16);
  WindowGeom g{h, wd, oh, ow, pt, pl, (ow + kPatchW - 1) / kPatchW, (oh + kPatchH - 1) / kPatchH,
               (unsigned)((long long)n * h * wd * ci * 2)};
  const long long units = (long long)n * g.tiles_c * g.tiles_r;
  if (units > 0x3fffffffLL) return TFX_ERR_UNSUPPORTED;
#define TFX_WINDOW_CASE(CI, CO) \
  if (ci == CI && co == CO) return launch_window<CI, CO>(x, w, bias, y, g, (int)units, act, stream);
  TFX_WINDOW_CASE(32, 32)
  TFX_WINDOW_CASE(32, 64)
  TFX_WINDOW_CASE(32, 128)
  TFX_WINDOW_CASE(64, 32)
  TFX_WINDOW_CASE(64, 64)
#undef TFX_WINDOW_CASE
  return TFX_ERR_UNSUPPORTED;
}

}  // namespace tfx
