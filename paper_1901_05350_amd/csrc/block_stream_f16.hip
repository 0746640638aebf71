// A depthwise-separable block of the Section 3.9 network at large batch in one launch, on 16-bit float storage
// (Section 4.1):  y = half(relu6(pointwise(half(relu6(depthwise3x3(x) + dw_b))) + pw_b)),  stride 1 or 2, SAME.
// The fp32 kernel of block_stream.hip with the operand layout of pointwise_f16.hip: the pointwise filter is the
// stationary operand in LDS (stream_f16.h), a unit is a 4 x 8 patch of output pixels of one image = two
// v_mfma_f32_16x16x32_f16 slabs of 2 x 8 pixels (one slab, 2 x 8, for 128 -> 256 channels at stride 2, whose filter
// leaves less room for windows; its 256 output channels take two passes over the operands), the wavefront copies the patch's input window, 64 or 32 channels
// at a time, into its own piece of LDS, and lane (li, q) forms its operand of k-step s -- channels 32 s + 8 q ... + 7
// of slab pixel (li / 8, li % 8) -- as the depthwise result of that pixel: 9 taps of 16 bytes from the window times
// the depthwise filter (also in LDS), accumulated in fp32, clamped and rounded to binary16 exactly as the
// depthwise kernel rounds what it stores.  The next channels of the window (and, before the MFMAs, the first ones
// of the next unit) are on their way from memory into registers meanwhile.
#include "stream_f16.h"

#include <type_traits>

namespace tfx {
namespace {

using namespace f16s;

constexpr int kThreads = 512, kWaves = kThreads / 64;
constexpr int kPatchW = 8;  // a unit is PH x 8 output pixels: PH / 2 slabs of 2 x 8 (PH = 4; 2 where the windows of 4 rows do not fit)
template <int K, int N, int S>
constexpr int patch_rows() {
  return (K == 128 && N == 256 && S == 2) ? 2 : 4;
}

struct WindowBlockGeom16 {
  int H, W, OH, OW, pt, pl;
  int tiles_c, tiles_r;  // patches per output row and column
  unsigned x_bytes;
};

// LDS layout of a window chunk of CC channels in 16-byte pieces (8 channels each): pixel stride PS >= CC / 8 and
// row stride RS >= WW * PS, the least ones for which the tap read of a wavefront (pixel (li / 8, li % 8) * S plus a
// constant, piece q) has no bank conflict.
template <int S, int CC, int PH>
struct WindowLayout16 {
  static constexpr int WH = (PH - 1) * S + 3, WW = (kPatchW - 1) * S + 3, QC = CC / 8;
  struct Piece {
    int ps, rs;
    constexpr int operator()(int li, int q) const { return (li / 8) * S * rs + (li % 8) * S * ps + q; }
  };
  static constexpr int pixel_stride() {
    for (int ps = QC;; ++ps)
      for (int rs = WW * ps; rs < WW * ps + 32; ++rs)
        if (conflict_free(Piece{ps, rs})) return ps;
  }
  static constexpr int PS = pixel_stride();
  static constexpr int row_stride() {
    for (int rs = WW * PS;; ++rs)
      if (conflict_free(Piece{PS, rs})) return rs;
  }
  static constexpr int RS = row_stride();
  static constexpr int kHalfs = WH * RS * 8;
  static constexpr int kPieces = WH * WW * QC, kLoads = (kPieces + 63) / 64;
};

template <int K, int S>
constexpr int chunk_channels() {
  return (S == 1 && K >= 64) ? 64 : 32;
}

template <int K, int N, int S>
__global__ __launch_bounds__(kThreads) void separable_window_f16_kernel(const half_t* __restrict__ x,
                                                                        const half_t* __restrict__ dw_w,
                                                                        const half_t* __restrict__ dw_b,
                                                                        const half_t* __restrict__ pw_w,
                                                                        const half_t* __restrict__ pw_b,
                                                                        half_t* __restrict__ y, WindowBlockGeom16 g,
                                                                        int units, int dw_act, int pw_act) {
  constexpr int CC = chunk_channels<K, S>();
  constexpr int PH = patch_rows<K, N, S>(), SL = PH / 2;  // slabs per unit
  using WL = WindowLayout16<S, CC, PH>;
  using Stage = FilterStage<K, N, kThreads>;
  constexpr int KS = K / 32, NB = N / 16, LD = Stage::LD, CH = K / CC, SPC = CC / 32;  // k-steps, blocks, chunks, steps per chunk
  constexpr int PS = WL::PS, RS = WL::RS, WW = WL::WW, LI = WL::kLoads, QC = WL::QC;
  constexpr int NBP = NB < 8 ? NB : 8, PASSES = NB / NBP;  // 16-channel blocks per pass over the unit's operands
  static_assert(K % CC == 0 && N % 32 == 0 && NB % NBP == 0 && N <= kThreads && 9 * K / 8 <= kThreads, "shape");
  // pointwise filter [N][LD] halfs, its bias (N floats, in the filter's row order), depthwise filter [9][K] halfs,
  // its bias (K floats), then one window per wavefront
  extern __shared__ __align__(16) half_t wl[];
  float* const pwb_l = reinterpret_cast<float*>(wl + N * LD);
  half_t* const dww_l = reinterpret_cast<half_t*>(pwb_l + N);
  float* const dwb_l = reinterpret_cast<float*>(dww_l + 9 * K);
  half_t* const win = reinterpret_cast<half_t*>(dwb_l + K) + (threadIdx.x / 64) * WL::kHalfs;
  __shared__ int next_unit;

  const int tid = threadIdx.x;
  const int lane = tid % 64, li = lane % 16, q = lane / 16;
  const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(const_cast<half_t*>(x), 0, (int)g.x_bytes, 0x00020000);
  const int u0 = (int)((long long)units * blockIdx.x / gridDim.x);
  const int u1 = (int)((long long)units * (blockIdx.x + 1) / gridDim.x);

  // This lane's pieces of a window chunk: piece e = lane + 64 i is 8 channels (cq) of window pixel (wr, wc).
  int wrc[LI], goff[LI], loff[LI];
#pragma unroll
  for (int i = 0; i < LI; ++i) {
    const int e = lane + 64 * i, p = e / QC, cq = e % QC, wr = p / WW, wc = p % WW;
    wrc[i] = wr | wc << 8 | (e < WL::kPieces ? 1 << 16 : 0);  // bit 16: the piece exists
    goff[i] = ((wr * g.W + wc) * K + 8 * cq) * 2;
    loff[i] = (wr * RS + wc * PS + cq) * 8;
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
    p.ih0 = PH * p.tr * S - g.pt;
    p.iw0 = kPatchW * p.tc * S - g.pl;
    p.base = ((p.n * g.H + p.ih0) * g.W + p.iw0) * K * 2;
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
  u32x4 wreg[LI];  // window pieces of one chunk
  auto load_chunk = [&](const Offsets& o, int ch) {
#pragma unroll
    for (int i = 0; i < LI; ++i) wreg[i] = __builtin_amdgcn_raw_buffer_load_b128(xr, (int)o.v[i], CC * 2 * ch, 0);
  };

  // The filters' loads first, then the first chunk of the wavefront's first unit (fixed; the rest are handed out
  // by the counter): all in flight while the pointwise filter is transposed.
  Stage stage;
  stage.fetch(pw_w, tid);
  const h8 dwv = *reinterpret_cast<const h8*>(dw_w + 8 * (tid < 9 * K / 8 ? tid : 0));
  const half_t pwb = (pw_b ? pw_b : pw_w)[tid < N ? tid : 0];
  const half_t dwb = (dw_b ? dw_b : pw_w)[tid < K ? tid : 0];
  if (tid == 0) next_unit = kWaves;
  int cur = u0 + __builtin_amdgcn_readfirstlane(tid / 64);
  Place pc = place_of(cur < u1 ? cur : u0);
  Offsets oc = offsets_of(pc, cur < u1);
  load_chunk(oc, 0);
  stage.store(wl, tid);
  if (tid < 9 * K / 8) *reinterpret_cast<h8*>(dww_l + 8 * tid) = dwv;
  if (tid < N) pwb_l[rho(tid)] = pw_b ? (float)pwb : 0.f;
  if (tid < K) dwb_l[tid] = dw_b ? (float)dwb : 0.f;
  __syncthreads();

  const ActClamp dw_clamp = make_act(dw_act), pw_clamp = make_act(pw_act);
  const float dw_lo = dw_clamp.on ? 0.f : -INFINITY;
  // where this lane's taps start in a window: pixel (li / 8, li % 8) * S of slab 0, piece q
  const half_t* const tap0 = win + ((li / 8) * S * RS + (li % 8) * S * PS + q) * 8;
  const half_t* const w_base = wl + li * LD + 8 * q;

  while (cur < u1) {
    int ticket = 0;
    if (lane == 0) ticket = atomicAdd(&next_unit, 1);
    // depthwise layer, chunk by chunk: the chunk in the registers goes to LDS, the next one is requested, and the
    // operands of the chunk's k-steps are formed for both slabs.  The clamp is a median of three; that
    // instruction drops a NaN, so NaNs are looked for on the side and a wavefront that holds one repeats the
    // layer with the exact form.
    h8 a[SL][KS];
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
        for (int sc = 0; sc < SPC; ++sc) {
          const int s = SPC * ch + sc;  // k-step: channels 32 s + 8 q ... + 7
          const f32x4 b0 = *reinterpret_cast<const f32x4*>(dwb_l + 32 * s + 8 * q);
          const f32x4 b1 = *reinterpret_cast<const f32x4*>(dwb_l + 32 * s + 8 * q + 4);
#pragma unroll
          for (int sl = 0; sl < SL; ++sl) {
            float acc[8] = {b0[0], b0[1], b0[2], b0[3], b1[0], b1[1], b1[2], b1[3]};
            // (a loop over the window's rows that is not unrolled: unrolled, the compiler reads all nine taps of
            // both operands ahead and runs out of registers)
#pragma unroll 1
            for (int kh = 0; kh < 3; ++kh) {
#pragma unroll
              for (int kw = 0; kw < 3; ++kw) {
                const h8 xv = *reinterpret_cast<const h8*>(tap0 + ((2 * sl * S + kh) * RS + kw * PS + 4 * sc) * 8);
                const h8 wv = *reinterpret_cast<const h8*>(dww_l + (3 * kh + kw) * K + 32 * s + 8 * q);
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[e] = fmaf((float)xv[e], (float)wv[e], acc[e]);
              }
            }
            h8 o;
            if constexpr (decltype(exact)::value) {
#pragma unroll
              for (int e = 0; e < 8; ++e) o[e] = (half_t)apply_act(acc[e], dw_clamp);
            } else {
#pragma unroll
              for (int e = 0; e < 8; e += 2) nan |= __builtin_amdgcn_ballot_w64(__builtin_isunordered(acc[e], acc[e + 1]));
#pragma unroll
              for (int e = 0; e < 8; ++e) o[e] = (half_t)__builtin_amdgcn_fmed3f(acc[e], dw_lo, dw_clamp.hi);
            }
            a[sl][s] = o;
          }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
      }
      return nan;
    };
    if (depthwise(std::false_type{}) != 0) depthwise(std::true_type{});

    // the first chunk of the next unit's window is requested before the MFMAs of this one
    const int nxt = u0 + __builtin_amdgcn_readfirstlane(ticket);
    const Place pn = place_of(nxt < u1 ? nxt : cur);
    const Offsets on = offsets_of(pn, nxt < u1);
    load_chunk(on, 0);

    // pointwise layer, 128 output channels per pass over the operands and one k-step's filter fragments at a time
    // (the scheduling barriers keep the compiler from gathering all the reads in front, which does not fit the
    // registers); the accumulators start from the bias
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
      f32x4 acc[SL][NBP];
#pragma unroll
      for (int j = 0; j < NBP; ++j) {
        const f32x4 b = *reinterpret_cast<const f32x4*>(pwb_l + 16 * (NBP * p + j) + 4 * q);
#pragma unroll
        for (int sl = 0; sl < SL; ++sl) acc[sl][j] = b;
      }
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        h8 fw[NBP];
#pragma unroll
        for (int j = 0; j < NBP; ++j) fw[j] = *reinterpret_cast<const h8*>(w_base + 16 * (NBP * p + j) * LD + 32 * s);
#pragma unroll
        for (int j = 0; j < NBP; ++j)
#pragma unroll
          for (int sl = 0; sl < SL; ++sl)
            acc[sl][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fw[j], a[sl][s], acc[sl][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
      // epilogue: activation, and one 16-byte store per lane, slab and 32 channels
      auto emit = [&](const f32x4 (&acc)[NBP], int slab) {
        const int oh = PH * pc.tr + 2 * slab + li / 8, ow = kPatchW * pc.tc + li % 8;
        half_t* const yp = y + ((size_t)(pc.n * g.OH + oh) * g.OW + ow) * N + 16 * NBP * p + 8 * q;
        h8 o[NBP / 2];
        activate_and_pack(acc, pw_clamp, o);
        if (oh < g.OH && ow < g.OW) {
#pragma unroll
          for (int m = 0; m < NBP / 2; ++m) *reinterpret_cast<h8*>(yp + 32 * m) = o[m];
        }
      };
#pragma unroll
      for (int sl = 0; sl < SL; ++sl) emit(acc[sl], sl);
    }
    cur = nxt;
    pc = pn;
    oc = on;
  }
}

template <int K, int N, int S>
int launch_cfg(const half_t* x, const half_t* dw_w, const half_t* dw_b, const half_t* pw_w, const half_t* pw_b,
               half_t* y, const WindowBlockGeom16& g, int units, int dw_act, int pw_act, hipStream_t stream) {
  using WL = WindowLayout16<S, chunk_channels<K, S>(), patch_rows<K, N, S>()>;
  constexpr size_t lds_bytes = (size_t)N * filter_row_halfs(K) * 2 + N * 4 + 9 * K * 2 + K * 4 + (size_t)kWaves * WL::kHalfs * 2;
  static_assert(lds_bytes + 64 <= 160 * 1024, "LDS budget per workgroup");
  auto kern = separable_window_f16_kernel<K, N, S>;
  static std::atomic<uint64_t> lds_allowed{0};
  if (allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds_bytes, lds_allowed) != TFX_OK) return TFX_ERR_LAUNCH;
  // as many workgroups as are resident at once: each stages the filters once
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

// Blocks 1 - 4 (channels -> filters, stride) of the full-width network, many output pixels,
// 16-byte aligned operands, an input below 2^31 bytes.
bool separable_stream_f16_supported(int batch, int h, int w, int c, int n, int stride, int oh, int ow, const void* x,
                                    const void* dw_w, const void* dw_b, const void* pw_w, const void* pw_b,
                                    const void* y) {
  const bool shape = (c == 128 && n == 128 && stride == 1) || (c == 64 && n == 128 && stride == 2) ||
                     (c == 32 && n == 64 && stride == 1) || (c == 128 && n == 256 && stride == 2);
  const void* ptrs[] = {x, dw_w, dw_b, pw_w, pw_b, y};
  bool aligned = true;
  for (const void* p : ptrs) aligned = aligned && reinterpret_cast<uintptr_t>(p) % 16 == 0;
  const long long m = (long long)batch * oh * ow, x_bytes = (long long)batch * h * w * c * 2;
  // least output pixels from which the one launch beats the two kernels (measured on the network, per block)
  const long long least = n == 256 ? 6272 : 16384;
  return shape && aligned && m >= least && m <= 0x3fffffffLL && x_bytes < (1ll << 31);
}

int launch_separable_stream_f16(const uint16_t* x16, const uint16_t* dw_w16, const uint16_t* dw_b16, const uint16_t* pw_w16,
                                const uint16_t* pw_b16, uint16_t* y16, int batch, int h, int w, int c, int n, int oh,
                                int ow, int stride, int pt, int pl, int dw_act, int pw_act, hipStream_t stream) {
  const half_t* x = reinterpret_cast<const half_t*>(x16);
  const half_t* dw_w = reinterpret_cast<const half_t*>(dw_w16);
  const half_t* dw_b = reinterpret_cast<const half_t*>(dw_b16);
  const half_t* pw_w = reinterpret_cast<const half_t*>(pw_w16);
  const half_t* pw_b = reinterpret_cast<const half_t*>(pw_b16);
  half_t* y = reinterpret_cast<half_t*>(y16);
  const int ph = (c == 128 && n == 256 && stride == 2) ? patch_rows<128, 256, 2>() : patch_rows<32, 64, 1>();
  const WindowBlockGeom16 g{h, w, oh, ow, pt, pl, (ow + kPatchW - 1) / kPatchW, (oh + ph - 1) / ph,
                            (unsigned)((long long)batch * h * w * c * 2)};
  const long long units = (long long)batch * g.tiles_c * g.tiles_r;
  if (units > 0x3fffffffLL) return TFX_ERR_UNSUPPORTED;
#define TFX_WINDOW_BLOCK16(C, NN, SS) \
  if (c == C && n == NN && stride == SS) \
    return launch_cfg<C, NN, SS>(x, dw_w, dw_b, pw_w, pw_b, y, g, (int)units, dw_act, pw_act, stream);
  TFX_WINDOW_BLOCK16(128, 128, 1)
  TFX_WINDOW_BLOCK16(64, 128, 2)
  TFX_WINDOW_BLOCK16(32, 64, 1)
  TFX_WINDOW_BLOCK16(128, 256, 2)
#undef TFX_WINDOW_BLOCK16
  return TFX_ERR_UNSUPPORTED;
}

}  // namespace tfx
