// Pointwise (1x1) conv2d for thin filters on gfx950: y[M,N] = act(x[M,K] * w[K,N] + bias), K*N small.
//
// MobileNet's early pointwise layers have K, N <= 256 and very large M = batch*H*W, so each
// output needs few multiply-adds per byte and the layer runs close to the HBM roofline.  The
// filter is therefore the stationary operand: a workgroup loads all of w into LDS once and its
// wavefronts then stream 32-row slabs of x independently -- a lane loads its own MFMA A-operand
// values (row l%32, 4 consecutive k per 128-bit load) straight from global memory into
// registers, multiplies against w from LDS with v_mfma_f32_32x32x2_f32 and writes 32 x N outputs
// with the bias + activation epilogue.  There is no barrier after the filter load, so the
// wavefronts of a CU drift apart and loads, MFMAs and stores of different slabs overlap.
#include "tfx_internal.h"

namespace tfx {

typedef float floatx16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int kThreads = 512;  // 8 wavefronts (two per SIMD) share one copy of the filter

// KG = K / 8 (k-groups), NB = N / 32 (32-column blocks), TN = column blocks accumulated at once.
template <int KG, int NB>
__global__ __launch_bounds__(kThreads) void pointwise_stream_kernel(const float* __restrict__ x,
                                                                    const float* __restrict__ w,
                                                                    const float* __restrict__ bias,
                                                                    float* __restrict__ y, int M, int slabs, int act) {
  constexpr int K = KG * 8, N = NB * 32;
  constexpr int TN = NB < 2 ? NB : 2;  // two accumulators live at a time: fewer registers, measured fastest
  constexpr int PASSES = NB / TN;
  static_assert(NB % TN == 0, "column blocks");
  static_assert((K * N / 4) % kThreads == 0, "filter staging");
  extern __shared__ __align__(16) float wl[];  // [K][N]

  const int tid = threadIdx.x;
  {
    // stage the filter: all of a thread's loads are issued before the first LDS write
    constexpr int PER = K * N / 4 / kThreads;
    float4 t[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) t[i] = reinterpret_cast<const float4*>(w)[tid + i * kThreads];
#pragma unroll
    for (int i = 0; i < PER; ++i) reinterpret_cast<float4*>(wl)[tid + i * kThreads] = t[i];
  }
  __syncthreads();

  const int lane = tid % 64, li = lane % 32, h = lane / 32;
  constexpr int waves = kThreads / 64;
  const ActClamp clamp = make_act(act);
  // a workgroup owns a contiguous range of 32-row slabs; its wavefronts take them round-robin
  const int s0 = (int)((long long)slabs * blockIdx.x / gridDim.x);
  const int s1 = (int)((long long)slabs * (blockIdx.x + 1) / gridDim.x);
  for (int slab = s0 + tid / 64; slab < s1; slab += waves) {
    // A operand: this lane's row, k = 8g + 4h .. + 3 for every k-group.  Rows past the end are
    // clamped (loaded but never stored) so that the loads need no branches.
    int row = slab * 32 + li;
    row = row < M ? row : M - 1;
    float4 a[KG];
    const float* xp = x + (size_t)row * K + 4 * h;
#pragma unroll
    for (int g = 0; g < KG; ++g) a[g] = *reinterpret_cast<const float4*>(xp + 8 * g);

#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
      floatx16 acc[TN];
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
#pragma unroll
      for (int g = 0; g < KG; ++g) {
        const float av[4] = {a[g].x, a[g].y, a[g].z, a[g].w};
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          const float* wr = wl + (8 * g + 4 * h + s) * N + p * TN * 32 + li;
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[s], wr[32 * j], acc[j], 0, 0, 0);
        }
        // keep the LDS reads of later k-groups from being hoisted (they would spill registers)
        __builtin_amdgcn_sched_barrier(0);
      }
      // epilogue: register v of lane l holds row 8*(v/4) + 4*h + v%4, column l%32 of each block
      const int r0 = slab * 32 + 4 * h;
      const bool full = slab * 32 + 32 <= M;
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int col = (p * TN + j) * 32 + li;
        const float bv = bias ? bias[col] : 0.f;
        float* yp = y + (size_t)r0 * N + col;
        if (full) {
#pragma unroll
          for (int v = 0; v < 16; ++v) yp[(size_t)(8 * (v / 4) + (v % 4)) * N] = apply_act(acc[j][v] + bv, clamp);
        } else {
#pragma unroll
          for (int v = 0; v < 16; ++v)
            if (r0 + 8 * (v / 4) + (v % 4) < M) yp[(size_t)(8 * (v / 4) + (v % 4)) * N] = apply_act(acc[j][v] + bv, clamp);
        }
      }
    }
  }
}

template <int KG, int NB>
int launch_stream(const float* x, const float* w, const float* bias, float* y, int m, int act, hipStream_t stream) {
  constexpr size_t lds_bytes = (size_t)KG * 8 * NB * 32 * sizeof(float);
  static_assert(lds_bytes <= 128 * 1024, "filter must fit in LDS");
  auto kern = pointwise_stream_kernel<KG, NB>;
  static bool attr_set = false;
  if (!attr_set && lds_bytes > 64 * 1024) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)lds_bytes) != hipSuccess)
      return TFX_ERR_LAUNCH;
    attr_set = true;
  }
  const int slabs = (m + 31) / 32;
  int blocks = (slabs + 7) / 8;
  if (blocks > 256) blocks = 256;  // one workgroup per CU
  hipLaunchKernelGGL(kern, dim3(blocks), dim3(kThreads), lds_bytes, stream, x, w, bias, y, m, slabs, act);
  return check_launch();
}

}  // namespace

bool pointwise_stream_supported(int m, int k, int n, const void* x, const void* w, const void* y) {
  const bool shape = (k == 32 && n == 64) || (k == 64 && n == 128) || (k == 128 && n == 128) || (k == 128 && n == 256);
  const bool aligned = reinterpret_cast<uintptr_t>(x) % 16 == 0 && reinterpret_cast<uintptr_t>(w) % 16 == 0 &&
                       reinterpret_cast<uintptr_t>(y) % 4 == 0;
  // worthwhile once every one of the 256 CUs gets a full workgroup of 8 slabs (measured: below that the tiled GEMM wins)
  return shape && aligned && m >= 65536;
}

int launch_pointwise_stream(const float* x, const float* w, const float* bias, float* y, int m, int k, int n, int act,
                            hipStream_t stream) {
  if (k == 32 && n == 64) return launch_stream<4, 2>(x, w, bias, y, m, act, stream);
  if (k == 64 && n == 128) return launch_stream<8, 4>(x, w, bias, y, m, act, stream);
  if (k == 128 && n == 128) return launch_stream<16, 4>(x, w, bias, y, m, act, stream);
  if (k == 128 && n == 256) return launch_stream<16, 8>(x, w, bias, y, m, act, stream);
  return TFX_ERR_UNSUPPORTED;
}

}  // namespace tfx
