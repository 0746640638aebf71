// Pointwise (1x1) conv2d for thin filters on gfx950: y[M,N] = act(x[M,K] * w[K,N] + bias), K*N small.
//
// MobileNet's early pointwise layers have K, N <= 256 and very large M = batch*H*W, so each
// output needs few multiply-adds per byte and the layer runs close to the HBM roofline.  The
// filter is therefore the stationary operand: a workgroup loads all of w into LDS once and its
// wavefronts then stream 16-row slabs of x independently -- a lane loads its own MFMA operand
// values (its row, 4 consecutive k per 128-bit load) straight from global memory into registers,
// multiplies against w from LDS with v_mfma_f32_16x16x4_f32 and writes 16 x N outputs with the
// bias + activation epilogue.  There is no barrier after the filter load, so the wavefronts of a
// CU drift apart and loads, MFMAs and stores of different slabs overlap.
#include "tfx_internal.h"

namespace tfx {
namespace {

constexpr int kThreads = 512;  // 8 wavefronts share one copy of the filter

typedef float floatx4 __attribute__((ext_vector_type(4)));

// The filter is the MFMA A operand (lane l: column n = l % 16 of a 16-column block, k = l / 16) and
// the activations the B operand (lane l: row m = l % 16 of the slab, k = l / 16), so D[i = n][j = m]
// leaves every lane with 4 consecutive output columns of its row per 16-column block: 128-bit
// stores.  Within a group of 16 consecutive k, lane quarter q = l / 16 takes k = 16g + 4q + s in
// step s, i.e. one 128-bit load of its row per group.  LDS rows are padded by 4 floats so that the
// four k rows read by one instruction fall into different banks.  Wavefronts of a workgroup take
// the workgroup's slabs first come, first served (LDS counter).
template <int K, int N>
__global__ __launch_bounds__(kThreads) void pointwise_stream16_kernel(const float* __restrict__ x,
                                                                      const float* __restrict__ w,
                                                                      const float* __restrict__ bias,
                                                                      float* __restrict__ y, int M, int slabs, int act) {
  constexpr int KG = K / 16, NB = N / 16, LD = N + 4;
  constexpr int NBP = NB < 8 ? NB : 8;  // 16-column blocks per pass
  static_assert((K * N / 4) % kThreads == 0, "filter staging");
  extern __shared__ __align__(16) float wl[];  // [K][N + 4]
  __shared__ int next_slab;                    // wavefronts of the workgroup take slabs first come, first served

  const int tid = threadIdx.x;
  if (tid == 0) next_slab = 0;
  {
    constexpr int PER = K * N / 4 / kThreads;
    float4 t[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) t[i] = reinterpret_cast<const float4*>(w)[tid + i * kThreads];
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int e = tid + i * kThreads;  // float4 index: row e / (N/4), column quad e % (N/4)
      *reinterpret_cast<float4*>(wl + (e / (N / 4)) * LD + 4 * (e % (N / 4))) = t[i];
    }
  }
  __syncthreads();

  const int lane = tid % 64, li = lane % 16, q = lane / 16;
  constexpr int waves = kThreads / 64;
  const ActClamp clamp = make_act(act);
  const int s0 = (int)((long long)slabs * blockIdx.x / gridDim.x);
  const int s1 = (int)((long long)slabs * (blockIdx.x + 1) / gridDim.x);
  (void)waves;
  for (;;) {
    int ticket = 0;
    if (lane == 0) ticket = atomicAdd(&next_slab, 1);
    const int slab = s0 + __builtin_amdgcn_readfirstlane(ticket);
    if (slab >= s1) break;
    const int row = slab * 16 + li;
    const int rowc = row < M ? row : M - 1;  // clamped: loaded, never stored
    float4 a[KG];
    const float* xp = x + (size_t)rowc * K + 4 * q;
#pragma unroll
    for (int g = 0; g < KG; ++g) a[g] = *reinterpret_cast<const float4*>(xp + 16 * g);

#pragma unroll
    for (int p = 0; p < NB / NBP; ++p) {  // column passes of at most 128 columns keep the accumulators few
      floatx4 acc[NBP];
#pragma unroll
      for (int j = 0; j < NBP; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[j][v] = 0.f;
#pragma unroll
      for (int g = 0; g < KG; ++g) {
        const float av[4] = {a[g].x, a[g].y, a[g].z, a[g].w};
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          const float* wr = wl + (16 * g + 4 * q + s) * LD + 16 * NBP * p + li;
#pragma unroll
          for (int j = 0; j < NBP; ++j)
            acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(wr[16 * j], av[s], acc[j], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);  // keep later groups' LDS reads from being hoisted
      }
      if (row < M) {
        float* yp = y + (size_t)row * N + 16 * NBP * p + 4 * q;
#pragma unroll
        for (int j = 0; j < NBP; ++j) {
          float4 bv = make_float4(0.f, 0.f, 0.f, 0.f);
          if (bias) bv = *reinterpret_cast<const float4*>(bias + 16 * NBP * p + 16 * j + 4 * q);
          float4 o;
          o.x = apply_act(acc[j][0] + bv.x, clamp);
          o.y = apply_act(acc[j][1] + bv.y, clamp);
          o.z = apply_act(acc[j][2] + bv.z, clamp);
          o.w = apply_act(acc[j][3] + bv.w, clamp);
          *reinterpret_cast<float4*>(yp + 16 * j) = o;
        }
      }
    }
  }
}

template <int K, int N>
int launch_stream16(const float* x, const float* w, const float* bias, float* y, int m, int act, hipStream_t stream) {
  constexpr size_t lds_bytes = (size_t)K * (N + 4) * sizeof(float);
  static_assert(lds_bytes <= 160 * 1024, "filter must fit in LDS");
  auto kern = pointwise_stream16_kernel<K, N>;
  static std::atomic<uint64_t> lds_allowed{0};
  if (allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds_bytes, lds_allowed) != TFX_OK) return TFX_ERR_LAUNCH;
  const int slabs = (m + 15) / 16;
  // as many workgroups as fit on the chip at once (two per CU when the filter takes <= 80 KB of LDS)
  int blocks = lds_bytes <= 80 * 1024 ? 512 : 256;
  if (blocks > (slabs + 7) / 8) blocks = (slabs + 7) / 8;
  hipLaunchKernelGGL(kern, dim3(blocks), dim3(kThreads), lds_bytes, stream, x, w, bias, y, m, slabs, act);
  return check_launch();
}

}  // namespace

bool pointwise_stream_supported(int m, int k, int n, const void* x, const void* w, const void* bias, const void* y) {
  const bool shape = (k == 32 && n == 64) || (k == 64 && n == 128) || (k == 128 && n == 128) || (k == 128 && n == 256);
  const bool aligned = reinterpret_cast<uintptr_t>(x) % 16 == 0 && reinterpret_cast<uintptr_t>(w) % 16 == 0 &&
                       reinterpret_cast<uintptr_t>(y) % 16 == 0 && reinterpret_cast<uintptr_t>(bias) % 16 == 0;  // a null bias passes
  // worthwhile once every one of the 256 CUs gets a full workgroup of 8 slabs (measured: below that the tiled GEMM wins)
  return shape && aligned && m >= 16384;
}

int launch_pointwise_stream(const float* x, const float* w, const float* bias, float* y, int m, int k, int n, int act,
                            hipStream_t stream) {
  if (k == 32 && n == 64) return launch_stream16<32, 64>(x, w, bias, y, m, act, stream);
  if (k == 64 && n == 128) return launch_stream16<64, 128>(x, w, bias, y, m, act, stream);
  if (k == 128 && n == 128) return launch_stream16<128, 128>(x, w, bias, y, m, act, stream);
  if (k == 128 && n == 256) return launch_stream16<128, 256>(x, w, bias, y, m, act, stream);
  return TFX_ERR_UNSUPPORTED;
}

}  // namespace tfx
