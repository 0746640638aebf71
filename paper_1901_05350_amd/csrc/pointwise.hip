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

#include <type_traits>

namespace tfx {
namespace {

constexpr int kThreads = 512;  // 8 wavefronts share one copy of the filter


template <int KG>
__device__ __forceinline__ void fetch_slab(const float4* __restrict__ xp, float4 (&a)[KG]) {
#pragma unroll
  for (int g = 0; g < KG; ++g) a[g] = xp[4 * g];
}

// The filter is the MFMA A operand (lane l: column n = l % 16 of a 16-column block, k = l / 16) and
// the activations the B operand (lane l: row m = l % 16 of the slab, k = l / 16), so D[i = n][j = m]
// leaves every lane with 4 consecutive output columns of its row per 16-column block: 128-bit
// stores.  Within a group of 16 consecutive k, lane quarter q = l / 16 takes k = 16g + 4q + s in
// step s, i.e. one 128-bit load of its row per group.  LDS rows are padded by 4 floats so that the
// four k rows read by one instruction fall into different banks.  Wavefronts of a workgroup take
// the workgroup's slabs first come, first served (LDS counter).
// The accumulators start from the bias (kept in LDS behind the filter).  Cutting the slabs left over after a
// workgroup's last full round of 8 into column parts, so that the last round is short for everybody, was measured
// and gained nothing: the workgroups end 15 us apart anyway, in the order in which memory served their first slabs.
template <int K, int N>
__global__ __launch_bounds__(kThreads) void pointwise_stream16_kernel(const float* __restrict__ x,
                                                                      const float* __restrict__ w,
                                                                      const float* __restrict__ bias,
                                                                      float* __restrict__ y, int M, int slabs, int act) {
  constexpr int KG = K / 16, NB = N / 16, LD = N + 4;
  constexpr int NBP = NB < 8 ? NB : 8;  // 16-column blocks per pass
  static_assert((K * N / 4) % kThreads == 0 && N <= kThreads && NB % 2 == 0, "filter staging");
  extern __shared__ __align__(16) float wl[];  // [K][N + 4], then the bias (N floats; zeros without one)
  float* const bias_l = wl + K * LD;
  __shared__ int next_slab;                    // wavefronts of the workgroup take slabs first come, first served

  const int tid = threadIdx.x;
  if (tid == 0) next_slab = 0;
  {
    constexpr int PER = K * N / 4 / kThreads;
    float4 t[PER];
#pragma unroll
    for (int i = 0; i < PER; ++i) t[i] = reinterpret_cast<const float4*>(w)[tid + i * kThreads];
    const float bias_c = (bias ? bias : w)[tid < N ? tid : 0];
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int e = tid + i * kThreads;  // float4 index: row e / (N/4), column quad e % (N/4)
      *reinterpret_cast<float4*>(wl + (e / (N / 4)) * LD + 4 * (e % (N / 4))) = t[i];
    }
    if (tid < N) bias_l[tid] = bias ? bias_c : 0.f;
  }
  __syncthreads();

  const int lane = tid % 64, li = lane % 16, q = lane / 16;
  const ActClamp clamp = make_act(act);
  const int s0 = (int)((long long)slabs * blockIdx.x / gridDim.x);
  const int s1 = (int)((long long)slabs * (blockIdx.x + 1) / gridDim.x);
  // W blocks of 16 columns, starting at block jb, of one slab whose operand values are in a[]
  auto columns = [&](auto wc, const float4 (&a)[KG], int slab, int jb) {
    constexpr int W = decltype(wc)::value;
    floatx4 acc[W];
#pragma unroll
    for (int j = 0; j < W; ++j) acc[j] = *reinterpret_cast<const floatx4*>(bias_l + 16 * (jb + j) + 4 * q);
#pragma unroll
    for (int g = 0; g < KG; ++g) {
      const float av[4] = {a[g].x, a[g].y, a[g].z, a[g].w};
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const float* wr = wl + (16 * g + 4 * q + s) * LD + 16 * jb + li;
#pragma unroll
        for (int j = 0; j < W; ++j)
          acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(wr[16 * j], av[s], acc[j], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);  // keep later groups' LDS reads from being hoisted
    }
    store_slab_biased<W, true>(acc, y + 16 * jb, N, slab * 16, M, li, q, clamp);
  };

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
    for (int p = 0; p < NB / NBP; ++p)  // column passes of at most 128 columns keep the accumulators few
      columns(std::integral_constant<int, NBP>{}, a, slab, NBP * p);
  }
}

// Filter in registers.  In the operand layout above a lane needs K/16 x 4 x NW/16 filter values for NW
// output columns: 32 registers for K = 32 with NW = 64, K/2 registers with NW = 32.  A wavefront therefore
// owns one group of NW columns for the whole launch, loads its part of the filter once and then walks
// over slabs without touching LDS or a work counter: the N/NW wavefronts that share a slab are neighbours
// in one workgroup (x comes from HBM once and from L1 for the others), wavefront group v of the grid takes
// slabs v, v + V, v + 2V, ... (the whole grid advances along one front through x and y), and a wavefront
// fetches its next slab before multiplying the current one.
constexpr int kThinThreads = 256;
template <int K, int N, int NW>
__global__ __launch_bounds__(kThinThreads) void pointwise_regfilter_kernel(const float* __restrict__ x,
                                                                            const float* __restrict__ w,
                                                                            const float* __restrict__ bias,
                                                                            float* __restrict__ y, int M, int slabs,
                                                                            int act) {
  constexpr int KG = K / 16, NB = NW / 16, CG = N / NW, WPB = kThinThreads / 64;
  static_assert(N % NW == 0 && WPB % CG == 0 && NB % 2 == 0, "column groups share a workgroup");
  const int lane = threadIdx.x % 64, li = lane % 16, q = lane / 16;
  const int gw = blockIdx.x * WPB + threadIdx.x / 64;
  const int col0 = (gw % CG) * NW;          // this wavefront's columns
  const int stride = gridDim.x * WPB / CG;  // slabs between two slabs of one wavefront
  const int group = gw / CG;  // wavefronts of one group share their slabs
  if (group >= slabs) return;

  float wr[KG][4][NB];
#pragma unroll
  for (int g = 0; g < KG; ++g)
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
      for (int j = 0; j < NB; ++j) wr[g][s][j] = w[(16 * g + 4 * q + s) * N + col0 + 16 * j + li];
  float4 bv[NB / 2];  // bias of the columns this lane stores (see store_slab)
#pragma unroll
  for (int h = 0; h < NB / 2; ++h)
    bv[h] = bias ? *reinterpret_cast<const float4*>(bias + col0 + 32 * h + (li < 8 ? 0 : 16) + 4 * q)
                 : make_float4(0.f, 0.f, 0.f, 0.f);
  const ActClamp clamp = make_act(act);

  // a lane's operand values of one slab: its row (clamped: loaded, never stored), k = 16g + 4q .. + 3
  auto slab_ptr = [&](int sl) {
    const int row = sl * 16 + li;
    return reinterpret_cast<const float4*>(x + (size_t)(row < M ? row : M - 1) * K + 4 * q);
  };
  auto multiply = [&](const float4 (&a)[KG], floatx4 (&acc)[NB]) {
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
  };

  const int full = M / 16;  // slabs with all 16 rows
  float4 a[KG], an[KG];  // the slab being multiplied and the next one, in flight meanwhile
  floatx4 acc[NB];
  if (group < full) {
    int slab = group;
    fetch_slab<KG>(slab_ptr(slab), a);
    // Wait for the first slab here (vmcnt(0)), not at the loop head: a wait at the loop head would also run on
    // every later round, where it could only be met by waiting for the previous round's stores as well.
    __builtin_amdgcn_s_waitcnt(0x0F70);
    // One basic block per round, fenced for the instruction scheduler: loads of the next slab, then the MFMAs and
    // stores of this one, then the hand-over (the only place that waits for the loads).  Left to itself the
    // compiler sinks the loads to their first use, which turns the prefetch into a stall per round.
    for (;;) {
      const int next = slab + stride;
      const bool more = next < full;
      fetch_slab<KG>(slab_ptr(more ? next : slab), an);  // the last round re-reads its own slab (in cache)
      __builtin_amdgcn_sched_barrier(0);
      multiply(a, acc);
      store_slab<NB, false>(acc, bv, y + col0, N, slab * 16, M, li, q, clamp);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int g = 0; g < KG; ++g) a[g] = an[g];
      slab = next;
      if (!more) break;
    }
  }
  // the ragged last slab (M % 16 rows), by the group whose turn it is
  if (full < slabs && full % stride == group) {
    fetch_slab<KG>(slab_ptr(full), a);
    multiply(a, acc);
    store_slab<NB, true>(acc, bv, y + col0, N, full * 16, M, li, q, clamp);
  }
}

template <int K, int N, int NW>
int launch_regfilter(const float* x, const float* w, const float* bias, float* y, int m, int act, hipStream_t stream) {
  const int slabs = (m + 15) / 16;
  constexpr int CG = N / NW, WPB = kThinThreads / 64;
  // as many workgroups as are resident at once (slabs are dealt out statically, so a workgroup that had to
  // wait for a free slot would finish last); the count depends only on the kernel's registers
  static std::atomic<int> per_cu{0};
  int resident = per_cu.load(std::memory_order_relaxed);
  if (resident == 0) {
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&resident, pointwise_regfilter_kernel<K, N, NW>, kThinThreads, 0) !=
            hipSuccess || resident < 1)
      return TFX_ERR_LAUNCH;
    per_cu.store(resident, std::memory_order_relaxed);
  }
  int cus = 0;
  {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
      return TFX_ERR_LAUNCH;
  }
  long long blocks = (long long)cus * resident;
  const long long needed = ((long long)slabs * CG + WPB - 1) / WPB;
  if (blocks > needed) blocks = needed;
  hipLaunchKernelGGL((pointwise_regfilter_kernel<K, N, NW>), dim3((unsigned)blocks), dim3(kThinThreads), 0, stream, x, w,
                     bias, y, m, slabs, act);
  return check_launch();
}

template <int K, int N>
int launch_stream16(const float* x, const float* w, const float* bias, float* y, int m, int act, hipStream_t stream) {
  constexpr size_t lds_bytes = ((size_t)K * (N + 4) + N) * sizeof(float);
  static_assert(lds_bytes + 64 <= 160 * 1024, "filter must fit in LDS");
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
  // worthwhile once every one of the 256 CUs gets a full workgroup of 8 slabs (measured: below that the tiled GEMM
  // wins); the 128 KB filter leaves one workgroup per CU and needs 4 times as many rows to pay
  return shape && aligned && m >= (k == 128 && n == 256 ? 65536 : 16384);
}

int launch_pointwise_stream(const float* x, const float* w, const float* bias, float* y, int m, int k, int n, int act,
                            hipStream_t stream) {
  if (k == 32 && n == 64) return launch_regfilter<32, 64, 64>(x, w, bias, y, m, act, stream);
  if (k == 64 && n == 128) return launch_stream16<64, 128>(x, w, bias, y, m, act, stream);
  if (k == 128 && n == 128) return launch_stream16<128, 128>(x, w, bias, y, m, act, stream);
  if (k == 128 && n == 256) return launch_stream16<128, 256>(x, w, bias, y, m, act, stream);
  return TFX_ERR_UNSUPPORTED;
}

}  // namespace tfx
