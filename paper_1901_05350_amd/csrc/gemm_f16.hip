// batchMatMul on 16-bit float storage for gfx950 (Section 4.1: the same matMul renders to a 32-bit
// or a 16-bit floating point texture; Listing 2 defines the product).
//   C[b] = half( act( op(A[b]) * op(B[b]) + bias[col] ) ),  operands, bias and result IEEE binary16,
// products accumulated in fp32 on the matrix cores (v_mfma_f32_32x32x16_f16: 32x32 outputs, 16 k
// per instruction, 8 consecutive k per lane and operand).
//
// A workgroup of 4 wavefronts (2 x 2) computes a (64 TM) x (64 TN) tile; k-slices of 64 halfs are
// double-buffered in LDS as K-contiguous rows of 144 bytes (128 + 16 padding: the 16-byte fragment
// reads of 32 consecutive rows fall on distinct banks), the next slice's global loads are issued
// before the current slice's MFMAs.  The MFMA is issued with the operands swapped (B's fragment
// first), so a lane's accumulator registers hold 4 consecutive output columns of one row and the
// epilogue stores 8 bytes at a time.
#include "tfx_internal.h"

namespace tfx {
namespace {

typedef _Float16 half_t;
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kBK = 64;       // halfs per k-slice
constexpr int kLd = kBK + 8;  // LDS row stride in halfs
constexpr int kNT = 256;      // threads per workgroup
constexpr int kXcds = 8;

// ---- global -> register loaders for one ROWS x 64 slice of an operand -------------------------
// VEC: the operand is K-contiguous in memory, K % 8 == 0 and 16-byte aligned: 16-byte loads,
// slot s = tid + 256 i covers row s / 8, halfs 8 (s % 8) ... + 7.
template <int ROWS>
__device__ __forceinline__ void load_vec(const half_t* __restrict__ g, int ld, int rows, int K, int row0, int k0,
                                         int tid, h8 (&r)[ROWS * 8 / kNT]) {
  const h8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
  for (int i = 0; i < ROWS * 8 / kNT; ++i) {
    const int s = tid + i * kNT;
    const int row = row0 + s / 8, k = k0 + 8 * (s % 8);
    r[i] = (row < rows && k < K) ? *reinterpret_cast<const h8*>(g + (size_t)row * ld + k) : zero;
  }
}
template <int ROWS>
__device__ __forceinline__ void store_vec(half_t* lds, int tid, const h8 (&r)[ROWS * 8 / kNT]) {
#pragma unroll
  for (int i = 0; i < ROWS * 8 / kNT; ++i) {
    const int s = tid + i * kNT;
    *reinterpret_cast<h8*>(lds + (s / 8) * kLd + 8 * (s % 8)) = r[i];
  }
}

// Scalar: any layout, any K, any alignment.  kc: K is the contiguous dimension in memory
// (element (row, k) at row * ld + k), else the row index is (element at k * ld + row).
// Consecutive threads walk along the contiguous dimension.
template <int ROWS>
__device__ __forceinline__ void load_scalar(const half_t* __restrict__ g, bool kc, int ld, int rows, int K, int row0,
                                            int k0, int tid, half_t (&r)[ROWS * kBK / kNT]) {
#pragma unroll
  for (int i = 0; i < ROWS * kBK / kNT; ++i) {
    const int e = tid + i * kNT;
    const int row = row0 + (kc ? e / kBK : e % ROWS), k = k0 + (kc ? e % kBK : e / ROWS);
    const size_t idx = kc ? (size_t)row * ld + k : (size_t)k * ld + row;
    r[i] = (row < rows && k < K) ? g[idx] : (half_t)0;
  }
}
template <int ROWS>
__device__ __forceinline__ void store_scalar(half_t* lds, bool kc, int tid, const half_t (&r)[ROWS * kBK / kNT]) {
#pragma unroll
  for (int i = 0; i < ROWS * kBK / kNT; ++i) {
    const int e = tid + i * kNT;
    const int row = kc ? e / kBK : e % ROWS, k = kc ? e % kBK : e / ROWS;
    lds[row * kLd + k] = r[i];
  }
}

template <int ROWS, bool VEC>
struct Regs {
  h8 v[VEC ? ROWS * 8 / kNT : 1];
  half_t s[VEC ? 1 : ROWS * kBK / kNT];
};

template <int TM, int TN, bool VEC>
__global__ __launch_bounds__(kNT) void gemm_f16_kernel(const half_t* __restrict__ A, const half_t* __restrict__ B,
                                                       half_t* __restrict__ C, const half_t* __restrict__ bias, int M,
                                                       int N, int K, int a_kc, int b_kc, int tiles_m, int tiles_n,
                                                       int total_blocks, long long strideA, long long strideB,
                                                       long long strideC, int act, int m_fastest, int c_vec) {
  constexpr int BM = 64 * TM, BN = 64 * TN;
  constexpr int WM = 32 * TM, WN = 32 * TN;
  constexpr int kTileA = BM * kLd, kTileB = BN * kLd;  // halfs per LDS buffer
  extern __shared__ __align__(16) half_t smem_h[];
  half_t* const lds_a = smem_h;  // two A buffers, then two B buffers
  half_t* const lds_b = smem_h + 2 * kTileA;

  // Hardware block id x lands on XCD x % 8: give each XCD (own L2) a contiguous range of tiles.
  const int bid = blockIdx.x;
  const int q = total_blocks / kXcds, rem = total_blocks % kXcds;
  const int xcd = bid % kXcds;
  const int vid = xcd * q + (xcd < rem ? xcd : rem) + bid / kXcds;
  const int tiles = tiles_m * tiles_n;
  const int batch = vid / tiles;
  const int t = vid % tiles;
  const int tile_m = m_fastest ? t % tiles_m : t / tiles_n;
  const int tile_n = m_fastest ? t / tiles_m : t % tiles_n;

  const int lda = a_kc ? K : M, ldb = b_kc ? K : N;
  A += (size_t)batch * strideA;
  B += (size_t)batch * strideB;
  C += (size_t)batch * strideC;

  const int tid = threadIdx.x;
  const int wave = tid / 64, lane = tid % 64;
  const int wm0 = (wave / 2) * WM, wn0 = (wave % 2) * WN;
  const int li = lane % 32, hh = lane / 32;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  Regs<BM, VEC> ra;
  Regs<BN, VEC> rb;
  auto load = [&](int k0) {
    if constexpr (VEC) {
      load_vec<BM>(A, lda, M, K, m0, k0, tid, ra.v);
      load_vec<BN>(B, ldb, N, K, n0, k0, tid, rb.v);
    } else {
      load_scalar<BM>(A, a_kc != 0, lda, M, K, m0, k0, tid, ra.s);
      load_scalar<BN>(B, b_kc != 0, ldb, N, K, n0, k0, tid, rb.s);
    }
  };
  auto store = [&](int buf) {
    if constexpr (VEC) {
      store_vec<BM>(lds_a + buf * kTileA, tid, ra.v);
      store_vec<BN>(lds_b + buf * kTileB, tid, rb.v);
    } else {
      store_scalar<BM>(lds_a + buf * kTileA, a_kc != 0, tid, ra.s);
      store_scalar<BN>(lds_b + buf * kTileB, b_kc != 0, tid, rb.s);
    }
  };

  const int nk = (K + kBK - 1) / kBK;
  load(0);
  store(0);
  __syncthreads();

  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) load((kt + 1) * kBK);
    const half_t* la = lds_a + cur * kTileA + (wm0 + li) * kLd + 8 * hh;
    const half_t* lb = lds_b + cur * kTileB + (wn0 + li) * kLd + 8 * hh;
    h8 fa[2][TM], fb[2][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[0][i] = *reinterpret_cast<const h8*>(la + 32 * i * kLd);
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[0][j] = *reinterpret_cast<const h8*>(lb + 32 * j * kLd);
#pragma unroll
    for (int s = 0; s < kBK / 16; ++s) {
      if (s + 1 < kBK / 16) {
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[(s + 1) & 1][i] = *reinterpret_cast<const h8*>(la + 32 * i * kLd + 16 * (s + 1));
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[(s + 1) & 1][j] = *reinterpret_cast<const h8*>(lb + 32 * j * kLd + 16 * (s + 1));
      }
      __builtin_amdgcn_sched_barrier(0);  // keep those LDS reads ahead of this step's MFMAs
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fb[s & 1][j], fa[s & 1][i], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) store(cur ^ 1);
    __syncthreads();
  }

  // Epilogue.  acc[i][j][v] is the output at row m0 + wm0 + 32 i + li, column
  // n0 + wn0 + 32 j + 8 (v / 4) + 4 hh + v % 4: four consecutive columns per register quad.
  const ActClamp clamp = make_act(act);
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int row = m0 + wm0 + 32 * i + li;
    if (row >= M) continue;
    half_t* crow = C + (size_t)row * N;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int col = n0 + wn0 + 32 * j + 8 * g + 4 * hh;
        if (col >= N) continue;
        float o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float bv = (bias != nullptr && col + e < N) ? (float)bias[col + e] : 0.f;
          o[e] = apply_act(acc[i][j][4 * g + e] + bv, clamp);
        }
        if (c_vec && col + 3 < N) {
          h4 pk = {(half_t)o[0], (half_t)o[1], (half_t)o[2], (half_t)o[3]};
          *reinterpret_cast<h4*>(crow + col) = pk;
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (col + e < N) crow[col + e] = (half_t)o[e];
        }
      }
    }
  }
}

template <int TM, int TN, bool VEC>
int launch_cfg(const half_t* a, const half_t* b, half_t* c, const half_t* bias, int batch, int m, int n, int k,
               bool a_kc, bool b_kc, int act, hipStream_t stream) {
  constexpr int BM = 64 * TM, BN = 64 * TN;
  constexpr size_t lds_bytes = 2 * (size_t)(BM + BN) * kLd * sizeof(half_t);
  static_assert(lds_bytes <= 160 * 1024, "LDS budget per workgroup");
  auto kern = gemm_f16_kernel<TM, TN, VEC>;
  static bool attr_set = false;
  if (!attr_set && lds_bytes > 64 * 1024) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)lds_bytes) != hipSuccess)
      return TFX_ERR_LAUNCH;
    attr_set = true;
  }
  const int tiles_m = (m + BM - 1) / BM, tiles_n = (n + BN - 1) / BN;
  const long long total = (long long)batch * tiles_m * tiles_n;
  if (total > 0x7fffffffLL) return TFX_ERR_UNSUPPORTED;
  // 8-byte stores need every row of C to start 8-byte aligned
  const int c_vec = (n % 4 == 0 && reinterpret_cast<uintptr_t>(c) % 8 == 0) ? 1 : 0;
  hipLaunchKernelGGL(kern, dim3((unsigned)total), dim3(kNT), lds_bytes, stream, a, b, c, bias, m, n, k, a_kc ? 1 : 0,
                     b_kc ? 1 : 0, tiles_m, tiles_n, (int)total, (long long)m * k, (long long)n * k,
                     (long long)m * n, act, n > m ? 1 : 0, c_vec);
  return check_launch();
}

}  // namespace

int launch_gemm_f16(const uint16_t* a16, const uint16_t* b16, uint16_t* c16, const uint16_t* bias16, int batch, int m,
                    int n, int k, bool a_kc, bool b_kc, int act, hipStream_t stream) {
  const half_t* a = reinterpret_cast<const half_t*>(a16);
  const half_t* b = reinterpret_cast<const half_t*>(b16);
  half_t* c = reinterpret_cast<half_t*>(c16);
  const half_t* bias = reinterpret_cast<const half_t*>(bias16);
  // 16-byte loads: both operands K-contiguous, K a multiple of 8 (then every row and every batch
  // starts 16-byte aligned if the base pointers do)
  const bool vec = a_kc && b_kc && k % 8 == 0 && reinterpret_cast<uintptr_t>(a) % 16 == 0 &&
                   reinterpret_cast<uintptr_t>(b) % 16 == 0;
  const long long t128 = (long long)batch * ((m + 127) / 128) * ((n + 127) / 128);
  const long long t256 = (long long)batch * ((m + 255) / 256) * ((n + 127) / 128);
  if (vec) {
    if (t256 >= 512) return launch_cfg<4, 2, true>(a, b, c, bias, batch, m, n, k, a_kc, b_kc, act, stream);
    if (t128 >= 256) return launch_cfg<2, 2, true>(a, b, c, bias, batch, m, n, k, a_kc, b_kc, act, stream);
    return launch_cfg<1, 1, true>(a, b, c, bias, batch, m, n, k, a_kc, b_kc, act, stream);
  }
  if (t128 >= 256) return launch_cfg<2, 2, false>(a, b, c, bias, batch, m, n, k, a_kc, b_kc, act, stream);
  return launch_cfg<1, 1, false>(a, b, c, bias, batch, m, n, k, a_kc, b_kc, act, stream);
}

}  // namespace tfx
