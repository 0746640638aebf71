// Pointwise (1x1) conv2d with a thin filter on 16-bit float storage for gfx950:
//   y[M,N] = half(act(x[M,K] * w[K,N] + bias)),  K*N small, M very large (Section 4.1 storage format,
//   the early pointwise layers of the Section 3.9 network at large batch).
// At 2 bytes per element these layers move one byte per 1.5 ... 6 multiply-adds and are bound by
// HBM, so the filter is the stationary operand: a workgroup transposes all of w into LDS once
// ([N][K + 8] halfs, K-contiguous rows as the matrix cores want them) and its 8 wavefronts then
// stream 32-row units of x: a lane loads its own v_mfma_f32_16x16x32_f16 operand (its row, 8
// consecutive k per 16-byte load) straight from global memory, multiplies against the filter
// fragments from LDS (each fragment read serves two 16-row slabs) and writes its outputs through a
// private LDS strip so that they leave as whole 128-byte lines.  Units are handed out by a counter in LDS.
#include "tfx_internal.h"

namespace tfx {
namespace {

typedef _Float16 half_t;
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 512;

template <int K, int N>
__global__ __launch_bounds__(kThreads) void pointwise_stream_f16_kernel(const half_t* __restrict__ x,
                                                                        const half_t* __restrict__ w,
                                                                        const half_t* __restrict__ bias,
                                                                        half_t* __restrict__ y, int M, int units,
                                                                        int act) {
  constexpr int KS = K / 32, NB = N / 16, LD = K + 8;
  constexpr int NBP = NB < 8 ? NB : 8;  // 16-channel blocks per pass
  static_assert(K % 32 == 0 && N % 16 == 0, "filter shape");
  extern __shared__ __align__(16) half_t wl[];  // [N][K + 8], then 8 wavefront-private output strips
  half_t* const stage = wl + N * LD;
  __shared__ int next_unit;

  const int tid = threadIdx.x;
  if (tid == 0) next_unit = 0;
  {
    // Filter transpose, once per workgroup: block u covers k-rows 4 kq ... + 3 of columns 8 nb ... + 7
    // (kq = u % (K/4) so that the lanes of a wavefront write consecutive 8-byte pieces of one LDS row);
    // four 16-byte loads, a 4 x 8 transpose in registers, eight 8-byte LDS writes.
    constexpr int BLOCKS = (K / 4) * (N / 8), PER = (BLOCKS + kThreads - 1) / kThreads;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int u = tid + i * kThreads;
      if (u < BLOCKS) {
        const int kq = u % (K / 4), nb = u / (K / 4);
        h8 r[4];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) r[kk] = *reinterpret_cast<const h8*>(w + (size_t)(4 * kq + kk) * N + 8 * nb);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const h4 o = {r[0][j], r[1][j], r[2][j], r[3][j]};
          *reinterpret_cast<h4*>(wl + (8 * nb + j) * LD + 4 * kq) = o;
        }
      }
    }
  }
  __syncthreads();

  const int lane = tid % 64, li = lane % 16, q = lane / 16;
  const ActClamp clamp = make_act(act);
  const int u0 = (int)((long long)units * blockIdx.x / gridDim.x);
  const int u1 = (int)((long long)units * (blockIdx.x + 1) / gridDim.x);
  for (;;) {
    int ticket = 0;
    if (lane == 0) ticket = atomicAdd(&next_unit, 1);
    const int unit = u0 + __builtin_amdgcn_readfirstlane(ticket);
    if (unit >= u1) break;
    const int row0 = unit * 32 + li, row1 = row0 + 16;
    const int r0c = row0 < M ? row0 : M - 1, r1c = row1 < M ? row1 : M - 1;  // clamped: loaded, never stored
    h8 a0[KS], a1[KS];
    const half_t* xp0 = x + (size_t)r0c * K + 8 * q;
    const half_t* xp1 = x + (size_t)r1c * K + 8 * q;
#pragma unroll
    for (int s = 0; s < KS; ++s) a0[s] = *reinterpret_cast<const h8*>(xp0 + 32 * s);
#pragma unroll
    for (int s = 0; s < KS; ++s) a1[s] = *reinterpret_cast<const h8*>(xp1 + 32 * s);

#pragma unroll
    for (int p = 0; p < NB / NBP; ++p) {
      f32x4 acc0[NBP], acc1[NBP];
#pragma unroll
      for (int j = 0; j < NBP; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc0[j][v] = acc1[j][v] = 0.f;
#pragma unroll
      for (int s = 0; s < KS; ++s) {
#pragma unroll
        for (int j = 0; j < NBP; ++j) {
          const h8 wf = *reinterpret_cast<const h8*>(wl + (16 * (NBP * p + j) + li) * LD + 32 * s + 8 * q);
          acc0[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wf, a0[s], acc0[j], 0, 0, 0);
          acc1[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wf, a1[s], acc1[j], 0, 0, 0);
        }
      }
      // Epilogue through a wavefront-private LDS strip: a lane's 4 consecutive channels (8 bytes) per block
      // are written to [16 rows][PW + 8], read back as 16 bytes per lane along a row and stored as whole
      // 128-byte lines (8-byte stores scattered over 16 rows cost more than the rest of the kernel).
      constexpr int PW = 16 * NBP, LS = PW + 8;            // columns per pass, strip row stride
      constexpr int LPR = PW / 8, RPI = 64 / LPR;          // lanes per row, rows per store instruction
      half_t* strip = stage + (tid / 64) * 16 * LS;
      auto emit = [&](const f32x4 (&acc)[NBP], int slab) {
#pragma unroll
        for (int j = 0; j < NBP; ++j) {
          const int col = 16 * j + 4 * q;
          float bv[4] = {0.f, 0.f, 0.f, 0.f};
          if (bias) {
#pragma unroll
            for (int e = 0; e < 4; ++e) bv[e] = (float)bias[PW * p + col + e];
          }
          h4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = (half_t)apply_act(acc[j][e] + bv[e], clamp);
          *reinterpret_cast<h4*>(strip + li * LS + col) = o;
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int r0 = 0; r0 < 16; r0 += RPI) {
          const int r = r0 + lane / LPR, c = 8 * (lane % LPR);
          const h8 v = *reinterpret_cast<const h8*>(strip + r * LS + c);
          const int row = unit * 32 + 16 * slab + r;
          if (row < M) *reinterpret_cast<h8*>(y + (size_t)row * N + PW * p + c) = v;
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
      };
      emit(acc0, 0);
      emit(acc1, 1);
    }
  }
}

template <int K, int N>
int launch_stream_f16(const half_t* x, const half_t* w, const half_t* bias, half_t* y, int m, int act,
                      hipStream_t stream) {
  constexpr int NBP = N / 16 < 8 ? N / 16 : 8;
  constexpr size_t lds_bytes = ((size_t)N * (K + 8) + 8 * 16 * (16 * NBP + 8)) * sizeof(half_t);
  static_assert(lds_bytes <= 160 * 1024, "LDS budget per workgroup");
  auto kern = pointwise_stream_f16_kernel<K, N>;
  static std::atomic<uint64_t> lds_allowed{0};
  if (allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds_bytes, lds_allowed) != TFX_OK) return TFX_ERR_LAUNCH;
  const int units = (m + 31) / 32;
  int blocks = lds_bytes <= 80 * 1024 ? 512 : 256;  // two workgroups per CU when the filter and strips allow
  if (blocks > (units + 7) / 8) blocks = (units + 7) / 8;
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
