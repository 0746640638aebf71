// Pointwise (1x1) conv2d on 16-bit float storage with a filter too large for one workgroup's LDS, or too few rows
// for the kernel that keeps the whole filter there:
//   y[M,N] = half(act(x[M,K] * w[K,N] + bias)),  K = 64, 128, 256 or 512, N = 128 ... 2048, M in the thousands
// (Section 4.1 storage format; the pointwise layers of the 28 x 28 ... 7 x 7 maps of the Section 3.9 network at
// large batch, and of its larger maps at batch 1 to 5).  At fp16 rate the matrix cores need 3 us for such a layer
// and a tiled GEMM spends its time around them: slices of both operands through LDS, two barriers per slice, 16
// slices per tile.  Here a workgroup keeps a column slab of the filter -- all K rows of NS = 128 columns, up to
// 133 KB -- in LDS (stream_f16.h: transposed once, rows in the order that leaves a lane with 8 consecutive output
// channels), and each of its 8 wavefronts takes units of 16 SL rows of x against it: a lane loads its own
// v_mfma_f32_16x16x32_f16 operands (its rows, 8 consecutive k per 16-byte load) straight from global memory, D
// k-steps ahead of their use and across the end of a unit, reads each filter fragment from LDS once for the SL
// slabs, and stores its outputs as 16-byte pieces.  No barrier after the filter is in place.  The N / NS
// workgroups that take the same rows against different slabs run on one XCD, so x comes from memory once and from
// that XCD's L2 afterwards.  What bounds it is the path from L2: 256 workgroups fetch a slab each and every row of
// x N / NS times (with K = 1024 only 64 columns fit, x would be fetched N / 64 times, and the tiled GEMM is faster).
#include "stream_f16.h"

namespace tfx {
namespace {

using namespace f16s;

constexpr int kThreads = 512, kWaves = kThreads / 64, kGrid = 256, kXcds = 8;

template <int K, int NS, int SL, int D>
__global__ __launch_bounds__(kThreads) void pointwise_slab_f16_kernel(const half_t* __restrict__ x,
                                                                      const half_t* __restrict__ w,
                                                                      const half_t* __restrict__ bias,
                                                                      half_t* __restrict__ y, int M, int N, int units,
                                                                      int act) {
  using Stage = FilterStage<K, NS, kThreads>;
  constexpr int KS = K / 32, NB = NS / 16, LD = Stage::LD, ROWS = 16 * SL;
  static_assert(K % 32 == 0 && NS % 32 == 0 && NS <= kThreads && KS % D == 0 && D <= KS && D >= 2, "shape");
  extern __shared__ __align__(16) half_t wl[];  // the slab, [NS][LD], then its bias as NS floats in the same row order
  float* const bias_l = reinterpret_cast<float*>(wl + NS * LD);

  const int tid = threadIdx.x;
  const int lane = tid % 64, li = lane % 16, q = lane / 16, wave = __builtin_amdgcn_readfirstlane(tid / 64);
  // workgroup -> (slab, part of the rows): workgroups are dealt to the 8 XCDs round robin; the `slabs` workgroups of
  // one part are neighbours inside an XCD
  const int slabs = N / NS, parts = kGrid / slabs;
  const int xcd = blockIdx.x % kXcds, in_xcd = blockIdx.x / kXcds;
  const int n0 = NS * (in_xcd % slabs), part = xcd + kXcds * (in_xcd / slabs);
  const int u0 = (int)((long long)units * part / parts), u1 = (int)((long long)units * (part + 1) / parts);

  // operands in flight: ring slot s % D holds k-step s of the unit being multiplied (or, once that step is done,
  // step s + D of it, or step s + D - KS of the wavefront's next unit)
  h8 a[SL][D];
  const half_t* xp[SL];
  auto locate = [&](int unit) {  // rows past M repeat the last one: loaded, never stored
#pragma unroll
    for (int sl = 0; sl < SL; ++sl) {
      const int row = unit * ROWS + 16 * sl + li;
      xp[sl] = x + (size_t)(row < M ? row : M - 1) * K + 8 * q;
    }
  };
  auto load_step = [&](int s) {
#pragma unroll
    for (int sl = 0; sl < SL; ++sl) a[sl][s % D] = *reinterpret_cast<const h8*>(xp[sl] + 32 * s);
  };

  // the slab's loads first, then the first operands of the wavefront's first unit
  Stage stage;
  stage.fetch(w + n0, tid, N);
  const float bias_c = tid < NS && bias ? (float)bias[n0 + tid] : 0.f;
  int cur = u0 + wave;
  locate(cur < u1 ? cur : u0);
  constexpr int PRE = 2;  // both kinds of loads share the path from L2: only the first k-steps go in front of the transpose
#pragma unroll
  for (int s = 0; s < PRE; ++s) load_step(s);
  stage.store(wl, tid);
#pragma unroll
  for (int s = PRE; s < D; ++s) load_step(s);
  if (tid < NS) bias_l[rho(tid)] = bias_c;
  const ActClamp clamp = make_act(act);
  const half_t* const w_base = wl + li * LD + 8 * q;
  __syncthreads();

  while (cur < u1) {
    const int nxt = cur + kWaves;
    f32x4 acc[SL][NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      const f32x4 b = *reinterpret_cast<const f32x4*>(bias_l + 16 * j + 4 * q);
#pragma unroll
      for (int sl = 0; sl < SL; ++sl) acc[sl][j] = b;
    }
    // filter fragments are read one k-step ahead (the scheduling barriers keep the compiler from gathering the
    // reads of the whole unit in front of it, which spills, or from moving them back to where they are used)
    h8 fw[2][NB];
    auto read_step = [&](int s, h8 (&f)[NB]) {
#pragma unroll
      for (int j = 0; j < NB; ++j) f[j] = *reinterpret_cast<const h8*>(w_base + 16 * j * LD + 32 * s);
    };
    read_step(0, fw[0]);
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      if (s + 1 < KS) read_step(s + 1, fw[(s + 1) & 1]);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int j = 0; j < NB; ++j)
#pragma unroll
        for (int sl = 0; sl < SL; ++sl)
          acc[sl][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fw[s & 1][j], a[sl][s % D], acc[sl][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      // the slot is free: k-step s + D of this unit, or the first steps of the next one (past the wavefront's last
      // unit: of this unit again, loaded and dropped -- no branch around a load)
      if (s + D == KS) locate(nxt < u1 ? nxt : cur);
      load_step(s + D < KS ? s + D : s + D - KS);
    }
    // Epilogue: activation, and one 16-byte store per lane, slab and 32 channels
#pragma unroll
    for (int sl = 0; sl < SL; ++sl) {
      const int row = cur * ROWS + 16 * sl + li;
      h8 o[NB / 2];
      activate_and_pack(acc[sl], clamp, o);
      if (row < M) {
        half_t* const yp = y + (size_t)row * N + n0 + 8 * q;
#pragma unroll
        for (int m = 0; m < NB / 2; ++m) *reinterpret_cast<h8*>(yp + 32 * m) = o[m];
      }
    }
    cur = nxt;
  }
}

template <int K, int NS, int SL, int D>
int launch_slab(const half_t* x, const half_t* w, const half_t* bias, half_t* y, int m, int n, int act,
                hipStream_t stream) {
  constexpr size_t lds_bytes = (size_t)NS * filter_row_halfs(K) * sizeof(half_t) + NS * sizeof(float);
  static_assert(lds_bytes + 64 <= 160 * 1024, "LDS budget per workgroup");
  auto kern = pointwise_slab_f16_kernel<K, NS, SL, D>;
  static std::atomic<uint64_t> lds_allowed{0};
  if (allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds_bytes, lds_allowed) != TFX_OK) return TFX_ERR_LAUNCH;
  const int units = (m + 16 * SL - 1) / (16 * SL);
  hipLaunchKernelGGL(kern, dim3(kGrid), dim3(kThreads), lds_bytes, stream, x, w, bias, y, m, n, units, act);
  return check_launch();
}

constexpr int kSlabColumns = 128;

}  // namespace

bool pointwise_slab_f16_supported(int m, int k, int n, const void* x, const void* w, const void* y) {
  if (k != 64 && k != 128 && k != 256 && k != 512) return false;
  const int slabs = n % kSlabColumns == 0 ? n / kSlabColumns : 0;
  const bool shape = slabs == 1 || slabs == 2 || slabs == 4 || slabs == 8 || slabs == 16;
  const bool aligned = reinterpret_cast<uintptr_t>(x) % 16 == 0 && reinterpret_cast<uintptr_t>(w) % 16 == 0 &&
                       reinterpret_cast<uintptr_t>(y) % 16 == 0;
  return shape && aligned && m >= 1536 && (long long)m * (k > n ? k : n) < (1ll << 31);
}

int launch_pointwise_slab_f16(const uint16_t* x16, const uint16_t* w16, const uint16_t* bias16, uint16_t* y16, int m,
                              int k, int n, int act, hipStream_t stream) {
  const half_t* x = reinterpret_cast<const half_t*>(x16);
  const half_t* w = reinterpret_cast<const half_t*>(w16);
  const half_t* bias = reinterpret_cast<const half_t*>(bias16);
  half_t* y = reinterpret_cast<half_t*>(y16);
  if (k == 64) return launch_slab<64, kSlabColumns, 2, 2>(x, w, bias, y, m, n, act, stream);
  if (k == 128) return launch_slab<128, kSlabColumns, 2, 4>(x, w, bias, y, m, n, act, stream);
  if (k == 256) return launch_slab<256, kSlabColumns, 2, 8>(x, w, bias, y, m, n, act, stream);
  if (k == 512) return launch_slab<512, kSlabColumns, 2, 8>(x, w, bias, y, m, n, act, stream);
  return TFX_ERR_UNSUPPORTED;
}

}  // namespace tfx
