// Pointwise (1x1) conv2d with a thin filter on 16-bit float storage for gfx950:
//   y[M,N] = half(act(x[M,K] * w[K,N] + bias)),  K*N small, M very large (Section 4.1 storage format,
//   the early pointwise layers of the Section 3.9 network at large batch).
// At 2 bytes per element these layers move one byte per 1.5 ... 6 multiply-adds and are bound by
// HBM, so the filter is the stationary operand: a workgroup transposes all of w into LDS once
// (stream_f16.h: K-contiguous rows as the matrix cores want them, padded against bank conflicts, in a row
// order that leaves a lane with 8 consecutive output channels) and its 8 wavefronts then stream 32-row
// units of x: a lane loads its own v_mfma_f32_16x16x32_f16 operand (its row, 8 consecutive k per 16-byte
// load) straight from global memory, one unit ahead of the MFMAs that use it, multiplies against the filter
// fragments from LDS (each fragment read serves two 16-row slabs) and stores its outputs as 16-byte pieces.
// Units are handed out by a counter in LDS.
#include "stream_f16.h"

namespace tfx {
namespace {

using namespace f16s;

constexpr int kThreads = 512, kWaves = kThreads / 64;

template <int K, int N>
__global__ __launch_bounds__(kThreads) void pointwise_stream_f16_kernel(const half_t* __restrict__ x,
                                                                        const half_t* __restrict__ w,
                                                                        const half_t* __restrict__ bias,
                                                                        half_t* __restrict__ y, int M, int units,
                                                                        int act) {
  using Stage = FilterStage<K, N, kThreads>;
  constexpr int KS = K / 32, NB = N / 16, LD = Stage::LD;
  constexpr int NBP = NB < 8 ? NB : 8, PASSES = NB / NBP;  // 16-channel blocks per pass over the unit
  static_assert(K % 32 == 0 && N % 32 == 0 && N <= kThreads, "filter shape");
  extern __shared__ __align__(16) half_t wl[];  // the filter, [N][LD], then the bias as N floats in the same row order
  float* const bias_l = reinterpret_cast<float*>(wl + N * LD);
  __shared__ int next_unit;

  const int tid = threadIdx.x;
  const int lane = tid % 64, li = lane % 16, q = lane / 16;
  const int u0 = (int)((long long)units * blockIdx.x / gridDim.x);
  const int u1 = (int)((long long)units * (blockIdx.x + 1) / gridDim.x);

  // A unit's operands: this lane's two rows (li and li + 16 of the unit's 32), k-group q of every 32 k.
  h8 a0[KS], a1[KS];
  const half_t *xp0, *xp1;
  auto locate = [&](int unit) {  // rows past M repeat the last one: loaded, never stored
    const int row0 = unit * 32 + li, row1 = row0 + 16;
    xp0 = x + (size_t)(row0 < M ? row0 : M - 1) * K + 8 * q;
    xp1 = x + (size_t)(row1 < M ? row1 : M - 1) * K + 8 * q;
  };
  auto load_step = [&](int s) {
    a0[s] = *reinterpret_cast<const h8*>(xp0 + 32 * s);
    a1[s] = *reinterpret_cast<const h8*>(xp1 + 32 * s);
  };

  // The filter's loads first, then the operands of the wavefront's first unit (fixed; the rest are handed out by
  // a counter in LDS): all of them are in flight while the filter is transposed.
  Stage stage;
  stage.fetch(w, tid);
  const float bias_c = tid < N && bias ? (float)bias[tid] : 0.f;
  int cur = u0 + __builtin_amdgcn_readfirstlane(tid / 64);
  if (tid == 0) next_unit = kWaves;
  locate(cur < u1 ? cur : u0);
#pragma unroll
  for (int s = 0; s < KS; ++s) load_step(s);
  stage.store(wl, tid);
  if (tid < N) bias_l[rho(tid)] = bias_c;
  const ActClamp clamp = make_act(act);
  const half_t* const w_base = wl + li * LD + 8 * q;
  __syncthreads();
  auto draw = [&]() {
    int ticket = 0;
    if (lane == 0) ticket = atomicAdd(&next_unit, 1);
    return ticket;
  };

  // Per pass: the MFMAs of unit `cur`, whose operands are in the registers; the registers of a k-step are
  // refilled with the same step of unit `nxt` as soon as its last MFMAs have been issued, so a load has the time
  // of a whole pass to arrive (a second unit in flight per wavefront was measured and is no faster).  The
  // accumulators start from the bias.
  int nxt = u0 + __builtin_amdgcn_readfirstlane(draw());
  while (cur < u1) {
    const int ticket = draw();  // the unit after `nxt`; its number is not needed before the end of the pass
    locate(nxt < u1 ? nxt : cur);
    // step t = KS p + s: k-step s of column pass p; its filter fragments are read from LDS one step ahead (the
    // scheduling barriers keep the compiler from gathering all the reads of a pass in front of it, which spills,
    // or from moving them back to where their values are used)
    constexpr int STEPS = PASSES * KS;
    h8 fw[2][NBP];
    auto read_step = [&](int t, h8 (&f)[NBP]) {
#pragma unroll
      for (int j = 0; j < NBP; ++j)
        f[j] = *reinterpret_cast<const h8*>(w_base + 16 * (NBP * (t / KS) + j) * LD + 32 * (t % KS));
    };
    read_step(0, fw[0]);
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
      f32x4 acc0[NBP], acc1[NBP];
#pragma unroll
      for (int j = 0; j < NBP; ++j) acc0[j] = acc1[j] = *reinterpret_cast<const f32x4*>(bias_l + 16 * (NBP * p + j) + 4 * q);
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        const int t = KS * p + s;
        if (t + 1 < STEPS) read_step(t + 1, fw[(t + 1) & 1]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < NBP; ++j) {
          acc0[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fw[t & 1][j], a0[s], acc0[j], 0, 0, 0);
          acc1[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fw[t & 1][j], a1[s], acc1[j], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (p + 1 == PASSES) load_step(s);
      }
      // Epilogue: activation, and one 16-byte store per lane, slab and 32 channels (a row's 4 lanes write 64
      // consecutive bytes).
      auto emit = [&](const f32x4 (&acc)[NBP], int slab) {
        const int row = cur * 32 + 16 * slab + li;
        h8 o[NBP / 2];
        activate_and_pack(acc, clamp, o);
        if (row < M) {
          half_t* const yp = y + (size_t)row * N + 16 * NBP * p + 8 * q;
#pragma unroll
          for (int m = 0; m < NBP / 2; ++m) *reinterpret_cast<h8*>(yp + 32 * m) = o[m];
        }
      };
      emit(acc0, 0);
      emit(acc1, 1);
    }
    cur = nxt;
    nxt = u0 + __builtin_amdgcn_readfirstlane(ticket);
  }
}

template <int K, int N>
int launch_stream_f16(const half_t* x, const half_t* w, const half_t* bias, half_t* y, int m, int act,
                      hipStream_t stream) {
  constexpr size_t lds_bytes = (size_t)N * filter_row_halfs(K) * sizeof(half_t) + N * sizeof(float);
  static_assert(lds_bytes + 64 <= 160 * 1024, "LDS budget per workgroup");
  auto kern = pointwise_stream_f16_kernel<K, N>;
  static std::atomic<uint64_t> lds_allowed{0};
  if (allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds_bytes, lds_allowed) != TFX_OK) return TFX_ERR_LAUNCH;
  // as many workgroups as are resident at once (one or two per CU, by registers and LDS): each transposes the
  // filter once
  static std::atomic<int> resident{0};
  int per_cu = resident.load(std::memory_order_relaxed);
  if (per_cu == 0) {
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, kThreads, lds_bytes) != hipSuccess || per_cu < 1)
      per_cu = 1;
    if (per_cu > 2) per_cu = 2;
    resident.store(per_cu, std::memory_order_relaxed);
  }
  const int units = (m + 31) / 32;
  int blocks = 256 * per_cu;
  if (blocks > (units + kWaves - 1) / kWaves) blocks = (units + kWaves - 1) / kWaves;
  hipLaunchKernelGGL(kern, dim3(blocks), dim3(kThreads), lds_bytes, stream, x, w, bias, y, m, units, act);
  return check_launch();
}

}  // namespace

bool pointwise_stream_f16_supported(int m, int k, int n, const void* x, const void* w, const void* y) {
  const bool shape = (k == 32 && n == 64) || (k == 64 && n == 128) || (k == 128 && n == 128) || (k == 128 && n == 256);
  const bool aligned = reinterpret_cast<uintptr_t>(x) % 16 == 0 && reinterpret_cast<uintptr_t>(w) % 16 == 0 &&
                       reinterpret_cast<uintptr_t>(y) % 16 == 0;
  return shape && aligned && m >= 16384;
}

int launch_pointwise_stream_f16(const uint16_t* x16, const uint16_t* w16, const uint16_t* bias16, uint16_t* y16, int m,
                                int k, int n, int act, hipStream_t stream) {
  const half_t* x = reinterpret_cast<const half_t*>(x16);
  const half_t* w = reinterpret_cast<const half_t*>(w16);
  const half_t* bias = reinterpret_cast<const half_t*>(bias16);
  half_t* y = reinterpret_cast<half_t*>(y16);
  if (k == 32 && n == 64) return launch_stream_f16<32, 64>(x, w, bias, y, m, act, stream);
  if (k == 64 && n == 128) return launch_stream_f16<64, 128>(x, w, bias, y, m, act, stream);
  if (k == 128 && n == 128) return launch_stream_f16<128, 128>(x, w, bias, y, m, act, stream);
  if (k == 128 && n == 256) return launch_stream_f16<128, 256>(x, w, bias, y, m, act, stream);
  return TFX_ERR_UNSUPPORTED;
}

}  // namespace tfx
