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

// Value held by the lane 8 places away within the lane's group of 16 (l % 16 <-> (l % 16) ^ 8): DPP row rotate by 8.
__device__ __forceinline__ float swap8(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x128, 0xf, 0xf, false));
}

// Bias + activation + store of NBLK 16-column blocks (NBLK even) of one 16-row slab.  After the MFMAs lane
// (li = l % 16, q = l / 16) holds columns 16j + 4q .. + 3 of row li for every block j; stored like that, an
// instruction would write 64-byte pieces of 16 rows (measured: half-line pieces cost 12 us of 72 on the
// 32 -> 64 layer).  Lanes li and li ^ 8 therefore trade blocks 2h + 1 / 2h first, so that the lanes with
// li < 8 hold block 2h of rows li and li + 8 and the others block 2h + 1 of rows li - 8 and li: two store
// instructions per block pair, each writing whole 128-byte lines of 8 rows.  bv[h]: bias of the lane's 4
// columns 32h + (li < 8 ? 0 : 16) + 4q .. + 3; yc: y + first column of block 0.
template <int NBLK>
__device__ __forceinline__ void store_slab(const floatx4 (&acc)[NBLK], const float4 (&bv)[NBLK / 2], float* yc, int n,
                                           int row0, int M, int li, int q, const ActClamp& clamp) {
  static_assert(NBLK % 2 == 0, "blocks are stored in pairs");
  const bool lo = li < 8;
  const int ra = row0 + (li & 7), rb = ra + 8;
#pragma unroll
  for (int h = 0; h < NBLK / 2; ++h) {
    float got[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) got[v] = swap8(lo ? acc[2 * h + 1][v] : acc[2 * h][v]);
    float4 oa, ob;
    oa.x = apply_act((lo ? acc[2 * h][0] : got[0]) + bv[h].x, clamp);
    oa.y = apply_act((lo ? acc[2 * h][1] : got[1]) + bv[h].y, clamp);
    oa.z = apply_act((lo ? acc[2 * h][2] : got[2]) + bv[h].z, clamp);
    oa.w = apply_act((lo ? acc[2 * h][3] : got[3]) + bv[h].w, clamp);
    ob.x = apply_act((lo ? got[0] : acc[2 * h + 1][0]) + bv[h].x, clamp);
    ob.y = apply_act((lo ? got[1] : acc[2 * h + 1][1]) + bv[h].y, clamp);
    ob.z = apply_act((lo ? got[2] : acc[2 * h + 1][2]) + bv[h].z, clamp);
    ob.w = apply_act((lo ? got[3] : acc[2 * h + 1][3]) + bv[h].w, clamp);
    const int col = 32 * h + (lo ? 0 : 16) + 4 * q;
    if (ra < M) *reinterpret_cast<float4*>(yc + (size_t)ra * n + col) = oa;
    if (rb < M) *reinterpret_cast<float4*>(yc + (size_t)rb * n + col) = ob;
  }
}

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
      float4 bv[NBP / 2];
#pragma unroll
      for (int h = 0; h < NBP / 2; ++h)
        bv[h] = bias ? *reinterpret_cast<const float4*>(bias + 16 * NBP * p + 32 * h + (li < 8 ? 0 : 16) + 4 * q)
                     : make_float4(0.f, 0.f, 0.f, 0.f);
      store_slab<NBP>(acc, bv, y + 16 * NBP * p, N, slab * 16, M, li, q, clamp);
    }
  }
}

// K = 32, N = 64 (MobileNet's first pointwise layer: 10.6 multiply-adds per byte, far below the ridge).
// The whole filter is 32 registers per lane in the operand layout above (k = 16g + 4q + s, n = 16j + l % 16),
// so it is loaded once per wavefront and the slab loop touches neither LDS nor a work counter: wavefront
// number v of the grid takes slabs v, v + V, v + 2V, ... (all wavefronts advance along one front through x and
// y) and fetches its next slab before multiplying the current one.
constexpr int kThinThreads = 256;
__global__ __launch_bounds__(kThinThreads) void pointwise_k32n64_kernel(const float* __restrict__ x,
                                                                         const float* __restrict__ w,
                                                                         const float* __restrict__ bias,
                                                                         float* __restrict__ y, int M, int slabs, int act) {
  constexpr int K = 32, N = 64, KG = 2, NB = 4;
  const int lane = threadIdx.x % 64, li = lane % 16, q = lane / 16;
  const int waves = gridDim.x * (kThinThreads / 64);
  int slab = blockIdx.x * (kThinThreads / 64) + threadIdx.x / 64;
  if (slab >= slabs) return;

  float wr[KG][4][NB];
#pragma unroll
  for (int g = 0; g < KG; ++g)
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
      for (int j = 0; j < NB; ++j) wr[g][s][j] = w[(16 * g + 4 * q + s) * N + 16 * j + li];
  float4 bv[NB / 2];  // bias of the columns this lane stores (see store_slab)
#pragma unroll
  for (int h = 0; h < NB / 2; ++h)
    bv[h] = bias ? *reinterpret_cast<const float4*>(bias + 32 * h + (li < 8 ? 0 : 16) + 4 * q)
                 : make_float4(0.f, 0.f, 0.f, 0.f);
  const ActClamp clamp = make_act(act);

  // a lane's operand values of one slab: its row (clamped: loaded, never stored), k = 16g + 4q .. + 3
  auto slab_ptr = [&](int sl) {
    const int row = sl * 16 + li;
    return reinterpret_cast<const float4*>(x + (size_t)(row < M ? row : M - 1) * K + 4 * q);
  };
  const float4* xp = slab_ptr(slab);
  float4 a0 = xp[0], a1 = xp[4], n0, n1;
  for (;;) {
    const int next = slab + waves;
    xp = slab_ptr(next < slabs ? next : slab);  // the last round re-reads its own slab (in cache) instead of branching
    n0 = xp[0];
    n1 = xp[4];
    const float4 a[KG] = {a0, a1};
    floatx4 acc[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) acc[j][v] = 0.f;
#pragma unroll
    for (int g = 0; g < KG; ++g) {
      const float av[4] = {a[g].x, a[g].y, a[g].z, a[g].w};
#pragma unroll
      for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int j = 0; j < NB; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(wr[g][s][j], av[s], acc[j], 0, 0, 0);
    }
    store_slab<NB>(acc, bv, y, N, slab * 16, M, li, q, clamp);
    if (next >= slabs) break;
    slab = next;
    a0 = n0;
    a1 = n1;
  }
}

int launch_k32n64(const float* x, const float* w, const float* bias, float* y, int m, int act, hipStream_t stream) {
  const int slabs = (m + 15) / 16;
  // 4 workgroups of 4 wavefronts per CU, all resident at once
  int blocks = 256 * 4;
  if (blocks > (slabs + 3) / 4) blocks = (slabs + 3) / 4;
  hipLaunchKernelGGL(pointwise_k32n64_kernel, dim3(blocks), dim3(kThinThreads), 0, stream, x, w, bias, y, m, slabs, act);
  return check_launch();
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
  if (k == 32 && n == 64) return launch_k32n64(x, w, bias, y, m, act, stream);
  if (k == 64 && n == 128) return launch_stream16<64, 128>(x, w, bias, y, m, act, stream);
  if (k == 128 && n == 128) return launch_stream16<128, 128>(x, w, bias, y, m, act, stream);
  if (k == 128 && n == 256) return launch_stream16<128, 256>(x, w, bias, y, m, act, stream);
  return TFX_ERR_UNSUPPORTED;
}

}  // namespace tfx
