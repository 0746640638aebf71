// fp32 MFMA GEMM for gfx950: C[b] = act(op(A[b]) * op(B[b]) + bias).
//
// This one kernel family serves matMul / batchMatMul (Section 4.1, Listing 2 of the
// TensorFlow.js paper defines the op: one dot product per output value) and the 1x1
// "pointwise" conv2d, which is the same contraction with M = N*H*W, K = inC, N = outC.
// The paper's shader computes one output per fragment with no data sharing; here a
// workgroup computes a tile, stages A and B k-slices through LDS and feeds the matrix cores
// (64-wide wavefronts): v_mfma_f32_32x32x2_f32 in the tiled kernel for medium and large
// problems, v_mfma_f32_16x16x4_f32 in the 16-row kernel for small M x N.
//
// Layout of one MFMA 32x32x2 (wave64), used below:
//   A operand: lane l holds A[i = l % 32][k = l / 32]
//   B operand: lane l holds B[k = l / 32][j = l % 32]
//   D result : register v of lane l holds D[i = 8*(v/4) + 4*(l/32) + v%4][j = l % 32]
// The contraction index may be permuted freely as long as A and B agree, so within a
// group of 8 consecutive k a lane with h = l/32 takes k = 8g + 4h + s in step s = 0..3.
// That makes a lane's four steps one contiguous float4 in a K-contiguous LDS tile.
#include "tfx_internal.h"

#include <type_traits>

namespace tfx {

typedef float floatx16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int kXcds = 8;  // workgroups are dealt round-robin to the 8 XCDs, each with its own L2

// LDS tile of one operand.  KC = true : stored [ROWS][BK + 4]  (k contiguous, padded rows)
//                           KC = false: stored [BK][ROWS]      (row index contiguous)
template <int ROWS, int BK, bool KC>
struct Tile {
  static constexpr int kStride = KC ? (BK + 4) : ROWS;
  static constexpr int kFloats = KC ? ROWS * (BK + 4) : BK * ROWS;
  static constexpr int kSlots = ROWS * BK / 4;  // float4 slots per tile
};

// Global -> registers for one operand tile.  Slot s of the tile is one float4:
//   KC : row r = s / (BK/4), k = 4 * (s % (BK/4))       -> g[(row0 + r) * ld + k0 + k .. +3]
//   !KC: k = s / (ROWS/4),   r = 4 * (s % (ROWS/4))     -> g[(k0 + k) * ld + row0 + r .. +3]
// Out-of-range elements read as zero, so ragged M, N and K tails add nothing.
template <int ROWS, int BK, bool KC, bool VEC, int NT, int NSLOT>
__device__ __forceinline__ void load_tile(const float* __restrict__ g, int ld, int rows_total, int k_total, int row0,
                                          int k0, int tid, float4 (&reg)[NSLOT]) {
#pragma unroll
  for (int it = 0; it < NSLOT; ++it) {
    const int s = tid + it * NT;
    int r, k;
    if (KC) {
      r = s / (BK / 4);
      k = 4 * (s % (BK / 4));
    } else {
      k = s / (ROWS / 4);
      r = 4 * (s % (ROWS / 4));
    }
    const int gr = row0 + r, gk = k0 + k;
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (KC) {
      if (gr < rows_total) {
        const float* p = g + (size_t)gr * ld + gk;
        if (VEC) {
          if (gk < k_total) v = *reinterpret_cast<const float4*>(p);
        } else {
          if (gk + 0 < k_total) v.x = p[0];
          if (gk + 1 < k_total) v.y = p[1];
          if (gk + 2 < k_total) v.z = p[2];
          if (gk + 3 < k_total) v.w = p[3];
        }
      }
    } else {
      if (gk < k_total) {
        const float* p = g + (size_t)gk * ld + gr;
        if (VEC) {
          if (gr < rows_total) v = *reinterpret_cast<const float4*>(p);
        } else {
          if (gr + 0 < rows_total) v.x = p[0];
          if (gr + 1 < rows_total) v.y = p[1];
          if (gr + 2 < rows_total) v.z = p[2];
          if (gr + 3 < rows_total) v.w = p[3];
        }
      }
    }
    reg[it] = v;
  }
}

// Branch-free variant for k-slices that lie entirely inside K (vector loads only).  A thread's slots keep a
// pointer each, set up once: rows past the end of the operand are clamped to a valid row instead of masked --
// they only feed output rows / columns that are never stored -- so a k-slice is NSLOT unconditional loads and
// no other vector instruction (on this chip every vector-ALU instruction takes issue time away from the
// matrix cores: the masked loader's compares, zero fills and branches cost ~10% of the main loop).
template <int ROWS, int BK, bool KC, int NT, int NSLOT>
__device__ __forceinline__ void slot_pointers(const float* __restrict__ g, int ld, int rows_total, int row0, int tid,
                                              const float* (&ptr)[NSLOT]) {
#pragma unroll
  for (int it = 0; it < NSLOT; ++it) {
    const int s = tid + it * NT;
    if (KC) {
      const int gr = min(row0 + s / (BK / 4), rows_total - 1);
      ptr[it] = g + (size_t)gr * ld + 4 * (s % (BK / 4));
    } else {
      int gr = row0 + 4 * (s % (ROWS / 4));  // 4 consecutive rows, all inside or all outside (rows_total % 4 == 0)
      if (gr >= rows_total) gr = 0;
      ptr[it] = g + (size_t)(s / (ROWS / 4)) * ld + gr;
    }
  }
}
template <int NSLOT>
__device__ __forceinline__ void load_tile_full(const float* (&ptr)[NSLOT], size_t k_offset, float4 (&reg)[NSLOT]) {
#pragma unroll
  for (int it = 0; it < NSLOT; ++it) reg[it] = *reinterpret_cast<const float4*>(ptr[it] + k_offset);
}

template <int ROWS, int BK, bool KC, int NT, int NSLOT>
__device__ __forceinline__ void store_tile(float* __restrict__ lds, int tid, const float4 (&reg)[NSLOT]) {
  using T = Tile<ROWS, BK, KC>;
#pragma unroll
  for (int it = 0; it < NSLOT; ++it) {
    const int s = tid + it * NT;
    int off;
    if (KC) {
      off = (s / (BK / 4)) * T::kStride + 4 * (s % (BK / 4));
    } else {
      off = (s / (ROWS / 4)) * T::kStride + 4 * (s % (ROWS / 4));
    }
    *reinterpret_cast<float4*>(lds + off) = reg[it];
  }
}

// Implicit-GEMM view of a convolution input (NHWC): GEMM row = output pixel (n, oh, ow), GEMM
// column k = (kh, kw, c) with c fastest, so A[row][k] = x[n, oh*sh - pt + kh, ow*sw - pl + kw, c]
// (zero outside the image) and B = the HWIO filter seen as [fh*fw*Ci, Co].
struct ConvA {
  const float* x;
  int H, W, Ci, OH, OW, fw, sh, sw, pt, pl;
};

// What a thread needs to know about the output pixel of one of its A-tile slots.
struct ConvRow {
  int ih0, iw0;      // input coordinates of filter tap (0, 0)
  long long base;    // element offset of image n, or -1 if the row is past M
};

template <int BM, int BK, int NT, int NSLOT>
__device__ __forceinline__ void conv_rows(const ConvA& cv, int M, int m0, int tid, ConvRow (&rows)[NSLOT]) {
#pragma unroll
  for (int it = 0; it < NSLOT; ++it) {
    const int r = m0 + (tid + it * NT) / (BK / 4);
    const int ow = r % cv.OW;
    const int t = r / cv.OW;
    const int oh = t % cv.OH;
    const int n = t / cv.OH;
    rows[it].ih0 = oh * cv.sh - cv.pt;
    rows[it].iw0 = ow * cv.sw - cv.pl;
    rows[it].base = r < M ? (long long)n * cv.H * cv.W * cv.Ci : -1;
  }
}

// A-tile loader of the implicit GEMM.  All slots of a thread share the same k offset (NT is a
// multiple of BK/4), so (kh, kw, c) is decoded once per thread per k-slice.  With VEC, Ci % 4 == 0
// and a float4 never crosses a filter tap; otherwise each of the 4 elements is decoded on its own.
template <int BM, int BK, bool VEC, int NT, int NSLOT>
__device__ __forceinline__ void load_tile_conv(const ConvA& cv, int K, int k0, int tid, const ConvRow (&rows)[NSLOT],
                                               float4 (&reg)[NSLOT]) {
  static_assert(NT % (BK / 4) == 0, "k offset must be the same for all slots of a thread");
  const int gk = k0 + 4 * (tid % (BK / 4));
  int kh[4], kw[4], c[4];
#pragma unroll
  for (int e = 0; e < (VEC ? 1 : 4); ++e) {
    const int k = gk + e;
    c[e] = k % cv.Ci;
    const int t = k / cv.Ci;
    kw[e] = t % cv.fw;
    kh[e] = t / cv.fw;
  }
#pragma unroll
  for (int it = 0; it < NSLOT; ++it) {
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (rows[it].base >= 0) {
      if (VEC) {
        const int ih = rows[it].ih0 + kh[0], iw = rows[it].iw0 + kw[0];
        if (gk < K && ih >= 0 && ih < cv.H && iw >= 0 && iw < cv.W)
          v = *reinterpret_cast<const float4*>(cv.x + rows[it].base + ((long long)ih * cv.W + iw) * cv.Ci + c[0]);
      } else {
        float e4[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int ih = rows[it].ih0 + kh[e], iw = rows[it].iw0 + kw[e];
          if (gk + e < K && ih >= 0 && ih < cv.H && iw >= 0 && iw < cv.W)
            e4[e] = cv.x[rows[it].base + ((long long)ih * cv.W + iw) * cv.Ci + c[e]];
        }
        v = make_float4(e4[0], e4[1], e4[2], e4[3]);
      }
    }
    reg[it] = v;
  }
}

// Lean A-tile loader of the implicit GEMM for Ci % BK == 0 (vector loads, at most 32 filter taps): a k-slice
// then lies inside one filter tap, so the tap (kh, kw) and the channel offset are the same for the whole
// workgroup and live in scalar registers.  A slot keeps, from set-up, the address of its pixel's tap (0, 0) and
// one validity bit per tap; per k-slice it adds the slice's uniform offset and, for a tap outside the image,
// reads a zero quad instead: 5 vector-ALU instructions per slot where the general loader spends ~100 on
// decoding and range checks (which take their issue time from the matrix cores).
__device__ __align__(16) float kZeroQuad[4] = {0.f, 0.f, 0.f, 0.f};  // never written (not const: same address space as x)

template <int BM, int BK, int NT, int NSLOT>
__device__ __forceinline__ void conv_lean_rows(const ConvA& cv, int M, int K, int m0, int tid, const float* (&p0)[NSLOT],
                                               unsigned (&ok)[NSLOT]) {
  const int fh = K / (cv.fw * cv.Ci);
#pragma unroll
  for (int it = 0; it < NSLOT; ++it) {
    const int r = min(m0 + (tid + it * NT) / (BK / 4), M - 1);  // rows past M repeat the last row (never stored)
    const int ow = r % cv.OW;
    const int t = r / cv.OW;
    const int oh = t % cv.OH;
    const int n = t / cv.OH;
    const int ih0 = oh * cv.sh - cv.pt, iw0 = ow * cv.sw - cv.pl;
    // address of tap (0, 0), channel 4 * (tid % (BK/4)); outside the image for border pixels, where only the taps
    // whose bit is set are ever dereferenced
    const long long e = (((long long)n * cv.H + ih0) * cv.W + iw0) * cv.Ci + 4 * (tid % (BK / 4));
    p0[it] = cv.x + e;
    unsigned bits = 0;
    for (int kh = 0; kh < fh; ++kh)
      for (int kw = 0; kw < cv.fw; ++kw)
        if (ih0 + kh >= 0 && ih0 + kh < cv.H && iw0 + kw >= 0 && iw0 + kw < cv.W) bits |= 1u << (kh * cv.fw + kw);
    ok[it] = bits;
  }
}

template <int NSLOT>
__device__ __forceinline__ void load_tile_conv_lean(const float* (&p0)[NSLOT], const unsigned (&ok)[NSLOT], int tap,
                                                    long long slice_offset, float4 (&reg)[NSLOT]) {
  const unsigned bit = 1u << tap;
#pragma unroll
  for (int it = 0; it < NSLOT; ++it) {
    const float* p = (ok[it] & bit) ? p0[it] + slice_offset : kZeroQuad;
    const floatx4 v = *reinterpret_cast<const floatx4*>(p);  // as a vector: a struct copy from a selected pointer stays in memory
    reg[it] = make_float4(v[0], v[1], v[2], v[3]);
  }
}

// MFMA operand of one 32-row sub-tile for k-group g: four steps' values for this lane.
template <int ROWS, int BK, bool KC>
__device__ __forceinline__ float4 read_frag(const float* __restrict__ lds, int row, int g, int h) {
  using T = Tile<ROWS, BK, KC>;
  if (KC) {
    return *reinterpret_cast<const float4*>(lds + row * T::kStride + 8 * g + 4 * h);
  } else {
    const float* p = lds + (8 * g + 4 * h) * T::kStride + row;
    return make_float4(p[0], p[T::kStride], p[2 * T::kStride], p[3 * T::kStride]);
  }
}

__device__ __forceinline__ float f4_get(const float4& v, int s) {
  return s == 0 ? v.x : (s == 1 ? v.y : (s == 2 ? v.z : v.w));
}

// Tiled kernel for medium and large problems: BM x BN tile, BK-deep k-slices double-buffered in LDS
// (one barrier per slice), WAVES_M x WAVES_N wavefronts each owning a (BM/WAVES_M) x (BN/WAVES_N) sub-tile.
// CONV: the A operand is the implicit im2col view `cv` of a convolution input instead of a matrix.
template <int BM, int BN, int BK, int WAVES_M, int WAVES_N, bool A_KC, bool B_KC, bool VEC, bool CONV, bool LEAN>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void gemm_mfma_kernel(
    const float* __restrict__ A, const float* __restrict__ B, float* __restrict__ C, const float* __restrict__ bias,
    int M, int N, int K, int tiles_m, int tiles_n, int total_blocks, long long strideA, long long strideB,
    long long strideC, int act, int m_fastest, ConvA cv) {
  static_assert(!CONV || A_KC, "the im2col view is K-contiguous");
  static_assert(!LEAN || (CONV && VEC), "the lean loader is the vector form of the convolution loader");
  constexpr int NT = 64 * WAVES_M * WAVES_N;
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int GROUPS = BK / 8;  // k-groups of 8 per tile
  static_assert(WM % 32 == 0 && WN % 32 == 0 && BK % 8 == 0, "tile shape");
  using TA = Tile<BM, BK, A_KC>;
  using TB = Tile<BN, BK, B_KC>;
  static_assert(TA::kSlots % NT == 0 && TB::kSlots % NT == 0, "loader shape");
  constexpr int SA = TA::kSlots / NT, SB = TB::kSlots / NT;

  extern __shared__ __align__(16) float smem[];
  float* const lds_a = smem;                    // two A buffers, then two B buffers
  float* const lds_b = smem + 2 * TA::kFloats;

  // XCD-aware block order: hardware block id x lands on XCD x % 8.  Give each XCD a contiguous
  // range of logical tiles (same batch, neighbouring tiles) so that its L2 sees each A / B panel once.
  // Within a batch, consecutive tiles walk along M when B is the larger operand (every XCD then owns
  // a column slice of B and only the smaller A is fetched by several L2s), along N otherwise.
  const int bid = blockIdx.x;
  const int q = total_blocks / kXcds, rem = total_blocks % kXcds;
  const int xcd = bid % kXcds;
  const int vid = xcd * q + (xcd < rem ? xcd : rem) + bid / kXcds;
  const int tiles = tiles_m * tiles_n;
  const int batch = vid / tiles;
  const int t = vid % tiles;
  const int tile_m = m_fastest ? t % tiles_m : t / tiles_n;
  const int tile_n = m_fastest ? t / tiles_m : t % tiles_n;

  const int lda = A_KC ? K : M;
  const int ldb = B_KC ? K : N;
  A += (size_t)batch * strideA;
  B += (size_t)batch * strideB;
  C += (size_t)batch * strideC;

  const int tid = threadIdx.x;
  const int wave = tid / 64, lane = tid % 64;
  const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;
  const int li = lane % 32, h = lane / 32;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // bias for this lane's output columns, fetched now so that its latency hides under the main loop
  float bv[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int col = n0 + wn0 + 32 * j + li;
    bv[j] = (bias != nullptr && col < N) ? bias[col] : 0.f;
  }

  float4 ra[SA], rb[SB];
  const int nk = (K + BK - 1) / BK;
  ConvRow crow[CONV && !LEAN ? SA : 1];
  if constexpr (CONV && !LEAN) conv_rows<BM, BK, NT, SA>(cv, M, m0, tid, crow);
  const float* cp0[SA];  // lean loader only
  unsigned cok[SA];
  // filter tap (kh, kw), its index and the channel offset of the next slice load_a is asked for (slices are
  // requested in order 0, 1, 2, ...); uniform across the workgroup
  int tap_c0 = 0, tap_kh = 0, tap_kw = 0, tap_idx = 0;
  if constexpr (LEAN) conv_lean_rows<BM, BK, NT, SA>(cv, M, K, m0, tid, cp0, cok);
  // k-slices that lie entirely inside K take the branch-free loaders (vector layouts only)
  constexpr bool FAST_A = VEC && !CONV, FAST_B = VEC;
  const int nk_full = K / BK;
  const float* pa[SA];
  const float* pb[SB];
  if constexpr (FAST_A) slot_pointers<BM, BK, A_KC, NT, SA>(A, lda, M, m0, tid, pa);
  if constexpr (FAST_B) slot_pointers<BN, BK, B_KC, NT, SB>(B, ldb, N, n0, tid, pb);
  const size_t step_a = A_KC ? (size_t)BK : (size_t)BK * lda, step_b = B_KC ? (size_t)BK : (size_t)BK * ldb;
  // FULL: k-slice kt is known to lie inside K
  auto load_a = [&](int kt, auto full) {
    if constexpr (LEAN) {
      load_tile_conv_lean<SA>(cp0, cok, tap_idx, ((long long)tap_kh * cv.W + tap_kw) * cv.Ci + tap_c0, ra);
      tap_c0 += BK;
      if (tap_c0 >= cv.Ci) {
        tap_c0 = 0;
        ++tap_idx;
        if (++tap_kw == cv.fw) {
          tap_kw = 0;
          ++tap_kh;
        }
      }
    } else if constexpr (CONV) load_tile_conv<BM, BK, VEC, NT, SA>(cv, K, kt * BK, tid, crow, ra);
    else if constexpr (FAST_A && decltype(full)::value) load_tile_full<SA>(pa, kt * step_a, ra);
    else load_tile<BM, BK, A_KC, VEC, NT, SA>(A, lda, M, K, m0, kt * BK, tid, ra);
  };
  auto load_b = [&](int kt, auto full) {
    if constexpr (FAST_B && decltype(full)::value) load_tile_full<SB>(pb, kt * step_b, rb);
    else load_tile<BN, BK, B_KC, VEC, NT, SB>(B, ldb, N, K, n0, kt * BK, tid, rb);
  };
  load_a(0, std::false_type{});
  load_b(0, std::false_type{});
  store_tile<BM, BK, A_KC, NT, SA>(lds_a, tid, ra);
  store_tile<BN, BK, B_KC, NT, SB>(lds_b, tid, rb);
  __syncthreads();

  // One k-slice: fetch slice kt + 1 into registers, multiply slice kt from LDS, hand the registers to the other
  // LDS buffer.  NEXT_FULL: slice kt + 1 exists and lies inside K.
  auto k_slice = [&](int kt, auto next_full) {
    constexpr bool NEXT_FULL = decltype(next_full)::value;
    const int cur = kt & 1, nxt = cur ^ 1;
    if (NEXT_FULL || kt + 1 < nk) {
      load_a(kt + 1, next_full);
      load_b(kt + 1, next_full);
    }
    const float* la = lds_a + cur * TA::kFloats;
    const float* lb = lds_b + cur * TB::kFloats;
    // fragments of k-group gg+1 are fetched from LDS before the MFMAs of group gg are issued
    __builtin_amdgcn_s_setprio(1);  // MFMA phase: do not let the co-resident workgroup's wave cut in
    float4 fa[2][TM], fb[2][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[0][i] = read_frag<BM, BK, A_KC>(la, wm0 + 32 * i + li, 0, h);
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[0][j] = read_frag<BN, BK, B_KC>(lb, wn0 + 32 * j + li, 0, h);
#pragma unroll
    for (int gg = 0; gg < GROUPS; ++gg) {
      const int g = gg;
      if (gg + 1 < GROUPS) {
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[(gg + 1) & 1][i] = read_frag<BM, BK, A_KC>(la, wm0 + 32 * i + li, g + 1, h);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[(gg + 1) & 1][j] = read_frag<BN, BK, B_KC>(lb, wn0 + 32 * j + li, g + 1, h);
      }
      __builtin_amdgcn_sched_barrier(0);  // keep those LDS reads ahead of this group's MFMAs
#pragma unroll
      for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(f4_get(fa[gg & 1][i], s), f4_get(fb[gg & 1][j], s), acc[i][j],
                                                             0, 0, 0);
    }
    __builtin_amdgcn_s_setprio(0);
    if (NEXT_FULL || kt + 1 < nk) {
      store_tile<BM, BK, A_KC, NT, SA>(lds_a + nxt * TA::kFloats, tid, ra);
      store_tile<BN, BK, B_KC, NT, SB>(lds_b + nxt * TB::kFloats, tid, rb);
    }
    __syncthreads();
  };
  int kt = 0;
  for (; kt + 1 < nk_full; ++kt) k_slice(kt, std::true_type{});
  for (; kt < nk; ++kt) k_slice(kt, std::false_type{});
  const ActClamp clamp = make_act(act);
  // Epilogue: bias[col] then activation, one dword per lane per register (two 128-byte rows per store).
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int col = n0 + wn0 + 32 * j + li;
    if (col >= N) continue;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = m0 + wm0 + 32 * i + 8 * (v / 4) + 4 * h + (v % 4);
        if (row < M) C[(size_t)row * N + col] = apply_act(acc[i][j][v] + bv[j], clamp);
      }
    }
  }
}

template <int BM, int BN, int BK, int WAVES_M, int WAVES_N, bool A_KC, bool B_KC, bool VEC, bool CONV = false,
          bool LEAN = false>
int launch_cfg(const float* a, const float* b, float* c, const float* bias, int batch, int m, int n, int k, int act,
               hipStream_t stream, const ConvA& cv = ConvA{}) {
  using TA = Tile<BM, BK, A_KC>;
  using TB = Tile<BN, BK, B_KC>;
  constexpr size_t lds_bytes = 2 * (TA::kFloats + TB::kFloats) * sizeof(float);
  static_assert(lds_bytes <= 160 * 1024, "LDS budget per workgroup");
  auto kern = gemm_mfma_kernel<BM, BN, BK, WAVES_M, WAVES_N, A_KC, B_KC, VEC, CONV, LEAN>;
  static std::atomic<uint64_t> lds_allowed{0};
  if (allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds_bytes, lds_allowed) != TFX_OK) return TFX_ERR_LAUNCH;
  const int tiles_m = (m + BM - 1) / BM, tiles_n = (n + BN - 1) / BN;
  const long long total = (long long)batch * tiles_m * tiles_n;
  if (total > 0x7fffffffLL) return TFX_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(kern, dim3((unsigned)total), dim3(64 * WAVES_M * WAVES_N), lds_bytes, stream, a, b, c,
                     bias, m, n, k, tiles_m, tiles_n, (int)total, (long long)m * k, (long long)n * k, (long long)m * n,
                     act, n > m ? 1 : 0, cv);
  return check_launch();
}

template <int BM, int BN, int BK, int WAVES_M, int WAVES_N>
int launch_layout(const float* a, const float* b, float* c, const float* bias, int batch, int m, int n, int k,
                  bool a_kc, bool b_kc, bool vec, int act, hipStream_t stream) {
#define TFX_GEMM_CASE(AK, BKC, V)                                                                              \
  if (a_kc == AK && b_kc == BKC && vec == V)                                                                   \
    return launch_cfg<BM, BN, BK, WAVES_M, WAVES_N, AK, BKC, V>(a, b, c, bias, batch, m, n, k, act, stream);
  TFX_GEMM_CASE(true, true, true)
  TFX_GEMM_CASE(true, false, true)
  TFX_GEMM_CASE(false, true, true)
  TFX_GEMM_CASE(false, false, true)
  TFX_GEMM_CASE(true, true, false)
  TFX_GEMM_CASE(true, false, false)
  TFX_GEMM_CASE(false, true, false)
  TFX_GEMM_CASE(false, false, false)
#undef TFX_GEMM_CASE
  return TFX_ERR_ARG;
}

// ---------------------------------------------------------------------------------------------
// Small-M variant: 16 x (16*TN) output tile with v_mfma_f32_16x16x4_f32.
// MobileNet's 14x14 and 7x7 pointwise layers have M = 196 or 49: with 32 x 32 tiles only 64-112
// workgroups exist and each needs >= 1.7 us of matrix-core time on its CU.  A 16-row tile doubles or
// quadruples the number of workgroups (and wastes fewer padded rows: 208 instead of 224 for M = 196).
// One BK-deep tile (single LDS stage) is split over WAVES_K wavefronts; the partial tiles are added
// through LDS by 256*TN threads, which also apply the epilogue.
// Layout of one MFMA 16x16x4 (wave64): A: lane l holds A[i = l % 16][k = l / 16]; B: lane l holds
// B[k = l / 16][j = l % 16]; D: register v of lane l holds D[i = 4 * (l / 16) + v][j = l % 16].
// Within a group of 16 consecutive k, lane quarter q = l / 16 takes k = 16g + 4q + s in step s.

template <int ROWS, int BK, bool KC>
__device__ __forceinline__ float4 read_frag16(const float* __restrict__ lds, int row, int g, int q) {
  using T = Tile<ROWS, BK, KC>;
  if (KC) {
    return *reinterpret_cast<const float4*>(lds + row * T::kStride + 16 * g + 4 * q);
  } else {
    const float* p = lds + (16 * g + 4 * q) * T::kStride + row;
    return make_float4(p[0], p[T::kStride], p[2 * T::kStride], p[3 * T::kStride]);
  }
}

template <int TN, int BK, int WAVES_K, bool A_KC, bool B_KC, bool VEC>
__global__ __launch_bounds__(64 * WAVES_K) void gemm_m16_kernel(
    const float* __restrict__ A, const float* __restrict__ B, float* __restrict__ C, const float* __restrict__ bias,
    int M, int N, int K, int tiles_m, int tiles_n, int total_blocks, long long strideA, long long strideB,
    long long strideC, int act, int m_fastest) {
  constexpr int BM = 16, BN = 16 * TN;
  constexpr int NT = 64 * WAVES_K;
  constexpr int GROUPS = BK / 16 / WAVES_K;  // k-groups of 16 per wavefront per tile
  constexpr int NACC = 4 / TN;                // accumulator chains per column tile (4 chains in all)
  static_assert(BK % (16 * WAVES_K) == 0 && (TN == 1 || TN == 2), "tile shape");
  using TA = Tile<BM, BK, A_KC>;
  using TB = Tile<BN, BK, B_KC>;
  static_assert(TA::kSlots % NT == 0 && TB::kSlots % NT == 0, "loader shape");
  constexpr int SA = TA::kSlots / NT, SB = TB::kSlots / NT;
  static_assert(WAVES_K * 256 * TN <= TA::kFloats + TB::kFloats, "split-K reduction reuses the tile buffers");
  static_assert(256 * TN <= NT, "epilogue threads");

  extern __shared__ __align__(16) float smem[];
  float* const lds_a = smem;
  float* const lds_b = smem + TA::kFloats;

  const int bid = blockIdx.x;
  const int q8 = total_blocks / kXcds, rem = total_blocks % kXcds;
  const int xcd = bid % kXcds;
  const int vid = xcd * q8 + (xcd < rem ? xcd : rem) + bid / kXcds;
  const int tiles = tiles_m * tiles_n;
  const int batch = vid / tiles;
  const int t = vid % tiles;
  const int tile_m = m_fastest ? t % tiles_m : t / tiles_n;
  const int tile_n = m_fastest ? t / tiles_m : t % tiles_n;

  const int lda = A_KC ? K : M;
  const int ldb = B_KC ? K : N;
  A += (size_t)batch * strideA;
  B += (size_t)batch * strideB;
  C += (size_t)batch * strideC;

  const int tid = threadIdx.x;
  const int wk = tid / 64, lane = tid % 64;
  const int li = lane % 16, q = lane / 16;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  // epilogue thread e < 256*TN owns output element (row, col) = the value of register v of lane l of
  // column tile j with e = (j*4 + v)*64 + l; fetch its bias now
  const int ej = tid / 256, ev = (tid / 64) % 4, el = tid % 64;
  const int erow = m0 + 4 * (el / 16) + ev, ecol = n0 + 16 * ej + el % 16;
  float ebias = 0.f;
  if (tid < 256 * TN && bias != nullptr && ecol < N) ebias = bias[ecol];

  floatx4 acc[NACC][TN];
#pragma unroll
  for (int c = 0; c < NACC; ++c)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) acc[c][j][v] = 0.f;

  float4 ra[SA], rb[SB];
  const int nk = (K + BK - 1) / BK;
  load_tile<BM, BK, A_KC, VEC, NT, SA>(A, lda, M, K, m0, 0, tid, ra);
  load_tile<BN, BK, B_KC, VEC, NT, SB>(B, ldb, N, K, n0, 0, tid, rb);
  for (int kt = 0; kt < nk; ++kt) {
    if (kt > 0) __syncthreads();  // everyone has finished reading the previous tile
    store_tile<BM, BK, A_KC, NT, SA>(lds_a, tid, ra);
    store_tile<BN, BK, B_KC, NT, SB>(lds_b, tid, rb);
    __syncthreads();
    if (kt + 1 < nk) {
      load_tile<BM, BK, A_KC, VEC, NT, SA>(A, lda, M, K, m0, (kt + 1) * BK, tid, ra);
      load_tile<BN, BK, B_KC, VEC, NT, SB>(B, ldb, N, K, n0, (kt + 1) * BK, tid, rb);
    }
#pragma unroll
    for (int gg = 0; gg < GROUPS; ++gg) {
      const int g = wk * GROUPS + gg;
      if (kt * BK + 16 * g >= K) break;  // k-groups past the end of K hold zeros
      const float4 fa = read_frag16<BM, BK, A_KC>(lds_a, li, g, q);
      float4 fb[TN];
#pragma unroll
      for (int j = 0; j < TN; ++j) fb[j] = read_frag16<BN, BK, B_KC>(lds_b, 16 * j + li, g, q);
#pragma unroll
      for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[s % NACC][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(f4_get(fa, s), f4_get(fb[j], s), acc[s % NACC][j], 0, 0, 0);
    }
  }
#pragma unroll
  for (int c = 1; c < NACC; ++c)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) acc[0][j][v] += acc[c][j][v];

  // add the WAVES_K partial tiles through LDS: layout [wk][j][v][lane]
  __syncthreads();
  float* red = smem;
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int v = 0; v < 4; ++v) red[(wk * TN * 4 + j * 4 + v) * 64 + lane] = acc[0][j][v];
  __syncthreads();
  if (tid < 256 * TN) {
    float sum = ebias;
#pragma unroll
    for (int w = 0; w < WAVES_K; ++w) sum += red[w * TN * 256 + tid];
    if (erow < M && ecol < N) C[(size_t)erow * N + ecol] = apply_act(sum, make_act(act));
  }
}

template <int TN, int BK, int WAVES_K, bool A_KC, bool B_KC, bool VEC>
int launch_m16_cfg(const float* a, const float* b, float* c, const float* bias, int batch, int m, int n, int k, int act,
                   hipStream_t stream) {
  using TA = Tile<16, BK, A_KC>;
  using TB = Tile<16 * TN, BK, B_KC>;
  constexpr size_t lds_bytes = (TA::kFloats + TB::kFloats) * sizeof(float);
  static_assert(lds_bytes <= 160 * 1024, "LDS budget per workgroup");
  auto kern = gemm_m16_kernel<TN, BK, WAVES_K, A_KC, B_KC, VEC>;
  static std::atomic<uint64_t> lds_allowed{0};
  if (allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds_bytes, lds_allowed) != TFX_OK) return TFX_ERR_LAUNCH;
  const int tiles_m = (m + 15) / 16, tiles_n = (n + 16 * TN - 1) / (16 * TN);
  const long long total = (long long)batch * tiles_m * tiles_n;
  if (total > 0x7fffffffLL) return TFX_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(kern, dim3((unsigned)total), dim3(64 * WAVES_K), lds_bytes, stream, a, b, c, bias, m, n, k,
                     tiles_m, tiles_n, (int)total, (long long)m * k, (long long)n * k, (long long)m * n, act,
                     n > m ? 1 : 0);
  return check_launch();
}

// 16-row tiles without operand staging, for A stored [M,K], B stored [K,N] (the pointwise-conv layout) and
// K = 64 ... 1024 (a multiple of 16 per wavefront): the WAVES_K wavefronts of a workgroup split K into chunks of 16 ... 128, and every
// wavefront loads the MFMA operands of its chunk straight into registers -- its row of A as 128-bit loads (4
// consecutive k, the contraction order permuted inside groups of 16 as in the other kernels) and, for the same
// k, TN adjacent columns of B as one load (TN = 2: 16 lanes read 128 contiguous bytes of a row of B; output
// column 2c + j of the 32-column tile is then column c of MFMA column block j).  All loads of a wavefront are
// issued before its first MFMA; there is no LDS fill and no barrier before the split-K reduction, which takes
// 0.4-0.7 us off kernels that last 4-6 us (the batch-1 network's 56x56 ... 7x7 pointwise layers).
// CONV: A is the implicit-GEMM view of a convolution input with Ci = CHUNK channels and WAVES_K filter taps, one
// tap per wavefront (K = taps x Ci): a lane's A operand is 4 consecutive channels of its output pixel's input
// pixel under that tap, or zeros if the tap falls outside the image.
template <int CHUNK, int WAVES_K, int TN, bool CONV = false>
__global__ __launch_bounds__(64 * WAVES_K) void gemm_m16_direct_kernel(const float* __restrict__ A,
                                                                       const float* __restrict__ B, float* __restrict__ C,
                                                                       const float* __restrict__ bias, int M, int N, int K,
                                                                       int tiles_m, int tiles_n, int total_blocks, int act,
                                                                       int m_fastest, ConvA cv) {
  constexpr int G = CHUNK / 16;  // k-groups of 16 per wavefront
  static_assert(CHUNK % 16 == 0 && CHUNK <= 128 && (TN == 1 || TN == 2) && 64 * WAVES_K >= 256, "shape");
  __shared__ float red[WAVES_K * TN * 4 * 64];  // split-K partials: [wavefront][column block j][register v][lane]

  const int bid = blockIdx.x;
  const int q8 = total_blocks / kXcds, rem = total_blocks % kXcds;
  const int xcd = bid % kXcds;
  const int vid = xcd * q8 + (xcd < rem ? xcd : rem) + bid / kXcds;
  const int tile_m = m_fastest ? vid % tiles_m : vid / tiles_n;
  const int tile_n = m_fastest ? vid / tiles_m : vid % tiles_n;
  const int tid = threadIdx.x, wk = tid / 64, lane = tid % 64, li = lane % 16, q = lane / 16;
  const int m0 = tile_m * 16, n0 = tile_n * 16 * TN;

  // operand addresses: rows / columns past the matrix are clamped (they only feed outputs that are not stored)
  const int arow = min(m0 + li, M - 1);
  const int bcol = min(n0 + TN * li, N - TN);
  const float* ap;
  bool inside = true;
  if constexpr (CONV) {
    const int ow = arow % cv.OW;
    const int t = arow / cv.OW;
    const int oh = t % cv.OH;
    const int n = t / cv.OH;
    const int ih = oh * cv.sh - cv.pt + wk / cv.fw, iw = ow * cv.sw - cv.pl + wk % cv.fw;
    inside = ih >= 0 && ih < cv.H && iw >= 0 && iw < cv.W;
    // outside the image: load from the (valid) clamped pixel, zero the values below
    const int ihc = min(max(ih, 0), cv.H - 1), iwc = min(max(iw, 0), cv.W - 1);
    ap = cv.x + (((size_t)n * cv.H + ihc) * cv.W + iwc) * CHUNK + 4 * q;
  } else {
    ap = A + (size_t)arow * K + wk * CHUNK + 4 * q;
  }
  const float* bp = B + (size_t)(wk * CHUNK + 4 * q) * N + bcol;
  float4 a[G];
  float b[G][4][TN];
#pragma unroll
  for (int g = 0; g < G; ++g) a[g] = *reinterpret_cast<const float4*>(ap + 16 * g);
  if constexpr (CONV) {
#pragma unroll
    for (int g = 0; g < G; ++g)
      if (!inside) a[g] = make_float4(0.f, 0.f, 0.f, 0.f);
  }
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const float* p = bp + (size_t)(16 * g + s) * N;
      if constexpr (TN == 2) {
        const float2 t = *reinterpret_cast<const float2*>(p);
        b[g][s][0] = t.x;
        b[g][s][1] = t.y;
      } else {
        b[g][s][0] = *p;
      }
    }

  // epilogue thread e < 256 owns register v = e / 64 of lane l = e % 64: row 4 (l / 16) + v, columns
  // TN (l % 16) ... + TN - 1; fetch its bias now
  const int ev = tid / 64, el = tid % 64;
  const int erow = m0 + 4 * (el / 16) + ev, ecol = n0 + TN * (el % 16);
  float ebias[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) ebias[j] = (tid < 256 && bias != nullptr && ecol + j < N) ? bias[ecol + j] : 0.f;

  floatx4 acc[2][TN];  // [chain][column block]
#pragma unroll
  for (int c = 0; c < 2; ++c)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) acc[c][j][v] = 0.f;
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[s & 1][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(f4_get(a[g], s), b[g][s][j], acc[s & 1][j], 0, 0, 0);
#pragma unroll
  for (int j = 0; j < TN; ++j)
#pragma unroll
    for (int v = 0; v < 4; ++v) red[((wk * TN + j) * 4 + v) * 64 + lane] = acc[0][j][v] + acc[1][j][v];
  __syncthreads();
  if (tid < 256 && erow < M) {
    const ActClamp clamp = make_act(act);
    float o[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      float sum = ebias[j];
#pragma unroll
      for (int w = 0; w < WAVES_K; ++w) sum += red[((w * TN + j) * 4 + ev) * 64 + el];
      o[j] = apply_act(sum, clamp);
    }
    float* cp = C + (size_t)erow * N + ecol;
    if constexpr (TN == 2) {
      if (ecol + 1 < N) *reinterpret_cast<float2*>(cp) = make_float2(o[0], o[1]);
    } else {
      if (ecol < N) *cp = o[0];
    }
  }
}

// K one of the supported depths in 64 ... 1024, N even, 16-byte aligned A (K % 4 == 0 holds), 8-byte aligned B, C and bias.
bool m16_direct_supported(const float* a, const float* b, const float* c, const float* bias, int batch, int n, int k,
                          bool a_kc, bool b_kc) {
  const bool aligned = reinterpret_cast<uintptr_t>(a) % 16 == 0 && reinterpret_cast<uintptr_t>(b) % 8 == 0 &&
                       reinterpret_cast<uintptr_t>(c) % 8 == 0 && reinterpret_cast<uintptr_t>(bias) % 8 == 0;
  return batch == 1 && a_kc && !b_kc && aligned && n % 2 == 0 && n >= 2 &&
         (k == 64 || k == 96 || k == 128 || k == 192 || k == 256 || k == 384 || k == 512 || k == 768 || k == 1024);
}

template <int TN>
int launch_m16_direct(const float* a, const float* b, float* c, const float* bias, int m, int n, int k, int act,
                      hipStream_t stream) {
  const int tiles_m = (m + 15) / 16, tiles_n = (n + 16 * TN - 1) / (16 * TN);
  const long long total = (long long)tiles_m * tiles_n;
  if (total > 0x7fffffffLL) return TFX_ERR_UNSUPPORTED;
#define TFX_DIRECT(CHUNK, WK)                                                                                      \
  hipLaunchKernelGGL((gemm_m16_direct_kernel<CHUNK, WK, TN>), dim3((unsigned)total), dim3(64 * WK), 0, stream, a, b, c, \
                     bias, m, n, k, tiles_m, tiles_n, (int)total, act, n > m ? 1 : 0, ConvA{})
  // K = chunk x wavefronts (the channel counts of the MobileNet family at widths 0.5, 0.75 and 1)
  if (k == 64) TFX_DIRECT(16, 4);
  else if (k == 96) TFX_DIRECT(16, 6);
  else if (k == 128) TFX_DIRECT(16, 8);
  else if (k == 192) TFX_DIRECT(32, 6);
  else if (k == 256) TFX_DIRECT(32, 8);
  else if (k == 384) TFX_DIRECT(48, 8);
  else if (k == 512) TFX_DIRECT(64, 8);
  else if (k == 768) TFX_DIRECT(96, 8);
  else TFX_DIRECT(128, 8);
#undef TFX_DIRECT
  return check_launch();
}

template <int TN, int BK, int WAVES_K>
int launch_m16_layout(const float* a, const float* b, float* c, const float* bias, int batch, int m, int n, int k,
                      bool a_kc, bool b_kc, bool vec, int act, hipStream_t stream) {
#define TFX_GEMM_CASE(AK, BKC, V)                                                                  \
  if (a_kc == AK && b_kc == BKC && vec == V)                                                       \
    return launch_m16_cfg<TN, BK, WAVES_K, AK, BKC, V>(a, b, c, bias, batch, m, n, k, act, stream);
  TFX_GEMM_CASE(true, true, true)
  TFX_GEMM_CASE(true, false, true)
  TFX_GEMM_CASE(false, true, true)
  TFX_GEMM_CASE(false, false, true)
  TFX_GEMM_CASE(true, true, false)
  TFX_GEMM_CASE(true, false, false)
  TFX_GEMM_CASE(false, true, false)
  TFX_GEMM_CASE(false, false, false)
#undef TFX_GEMM_CASE
  return TFX_ERR_ARG;
}

// Fraction of a tiling's multiply-adds that land inside the m x n output (the rest is padding).
double tile_efficiency(long long m, long long n, int bm, int bn) {
  const long long tm = (m + bm - 1) / bm, tn = (n + bn - 1) / bn;
  return (double)m * (double)n / ((double)tm * bm * (double)tn * bn);
}

// 128 x 128 tiles when there is one per CU, they are not mostly padding (e.g. n = 64 would waste half
// of every tile) and they fill the chip's 512 resident slots (two workgroups per CU) evenly: with 392
// tiles, 120 CUs would run one workgroup while 136 run two, and the kernel lasts as long as the pairs.
// 64 x 64 tiles are ~20% less efficient per tile but balance almost perfectly (measured crossover).
bool prefer_128(int batch, long long m, long long n) {
  const long long blocks128 = (long long)batch * ((m + 127) / 128) * ((n + 127) / 128);
  if (blocks128 < 256) return false;
  if (tile_efficiency(m, n, 128, 128) < 0.8 * tile_efficiency(m, n, 64, 64)) return false;
  const long long slots = 512;
  const double imbalance = (double)((blocks128 + slots - 1) / slots * slots) / (double)blocks128;
  return imbalance <= 1.2;
}

}  // namespace

int launch_gemm(const float* a, const float* b, float* c, const float* bias, int batch, int m, int n, int k, bool a_kc,
                bool b_kc, int act, hipStream_t stream) {
  // float4 global loads need 16-byte aligned rows: base pointers aligned and the contiguous
  // extent of each operand a multiple of 4 (which also keeps every batch slice aligned).
  const int a_inner = a_kc ? k : m, b_inner = b_kc ? k : n;
  const bool vec = (reinterpret_cast<uintptr_t>(a) % 16 == 0) && (reinterpret_cast<uintptr_t>(b) % 16 == 0) &&
                   (a_inner % 4 == 0) && (b_inner % 4 == 0);
  // Tile choice.  Large problems: 128 x 128 tiles (best reuse).  Medium: 64 x 64.
  const long long blocks64 = (long long)batch * ((m + 63) / 64) * ((n + 63) / 64);
  if (prefer_128(batch, m, n))
    return launch_layout<128, 128, 32, 2, 2>(a, b, c, bias, batch, m, n, k, a_kc, b_kc, vec, act, stream);
  if (blocks64 >= 192 || k <= 32)
    return launch_layout<64, 64, 32, 2, 2>(a, b, c, bias, batch, m, n, k, a_kc, b_kc, vec, act, stream);
  // Small M x N (too few 64 x 64 tiles for the 256 CUs): 16-row tiles, 16 x 32 or, when even those are
  // few, 16 x 16, so that every CU gets a workgroup; the tile depth covers K in one step when K <= 512.
  // These problems are bound by memory latency and by the matrix-core time of a single tile, not by
  // throughput (measured on the MobileNet 28x28 .. 7x7 pointwise layers: 3.8-6.1 us each).
  const long long blocks16x32 = (long long)batch * ((m + 15) / 16) * ((n + 31) / 32);
  const bool wide = blocks16x32 >= 160;
  // (with more tiles than the chip holds at once and K = 1024 the staged kernel's 128-deep tiles overlap better:
  // M = 392, 1024 -> 1024: 18.6 us against 26.0)
  if (m16_direct_supported(a, b, c, bias, batch, n, k, a_kc, b_kc) && (blocks16x32 <= 512 || k <= 512))
    return wide ? launch_m16_direct<2>(a, b, c, bias, m, n, k, act, stream)
                : launch_m16_direct<1>(a, b, c, bias, m, n, k, act, stream);
  // more tiles than fit on the chip at once (one 512-deep tile per CU): 128-deep tiles, so that several
  // workgroups share a CU and one's loads overlap another's MFMAs (M = 392, 512 -> 1024: 15.8 -> 11.2 us)
  const int kcap = blocks16x32 > 512 ? 128 : 1 << 30;
  if (k <= 128 || kcap <= 128)
    return wide ? launch_m16_layout<2, 128, 8>(a, b, c, bias, batch, m, n, k, a_kc, b_kc, vec, act, stream)
                : launch_m16_layout<1, 128, 8>(a, b, c, bias, batch, m, n, k, a_kc, b_kc, vec, act, stream);
  if (k <= 256 || kcap <= 256)
    return wide ? launch_m16_layout<2, 256, 8>(a, b, c, bias, batch, m, n, k, a_kc, b_kc, vec, act, stream)
                : launch_m16_layout<1, 256, 8>(a, b, c, bias, batch, m, n, k, a_kc, b_kc, vec, act, stream);
  return wide ? launch_m16_layout<2, 512, 8>(a, b, c, bias, batch, m, n, k, a_kc, b_kc, vec, act, stream)
              : launch_m16_layout<1, 512, 8>(a, b, c, bias, batch, m, n, k, a_kc, b_kc, vec, act, stream);
}

// 3x3 convolution of a small feature map (few 16 x 32 output tiles) with 16 / 32 / 64 / 128 input channels: one
// filter tap per wavefront, operands straight from memory (gemm_m16_direct_kernel<..., CONV>).
template <int CI>
int launch_conv3x3_direct(const ConvA& cv, const float* w, const float* bias, float* y, int m, int co, int act,
                          hipStream_t stream) {
  const int tiles_m = (m + 15) / 16, tiles_n = (co + 31) / 32;
  const int total = tiles_m * tiles_n;
  hipLaunchKernelGGL((gemm_m16_direct_kernel<CI, 9, 2, true>), dim3((unsigned)total), dim3(64 * 9), 0, stream, nullptr, w, y,
                     bias, m, co, 9 * CI, tiles_m, tiles_n, total, act, co > m ? 1 : 0, cv);
  return check_launch();
}

int launch_conv2d_gemm(const float* x, const float* w, const float* bias, float* y, int n, int h, int wd, int ci, int fh,
                       int fw, int co, int oh, int ow, int sh, int sw, int pt, int pl, int act, hipStream_t stream) {
  const long long m = (long long)n * oh * ow, k = (long long)fh * fw * ci;
  if (m > 0x7fffffffLL || k > 0x7fffffffLL) return TFX_ERR_UNSUPPORTED;
  const ConvA cv{x, h, wd, ci, oh, ow, fw, sh, sw, pt, pl};
  const bool vec = reinterpret_cast<uintptr_t>(x) % 16 == 0 && reinterpret_cast<uintptr_t>(w) % 16 == 0 &&
                   ci % 4 == 0 && co % 4 == 0;
  // small maps (at most 512 tiles of 16 x 32: the tiled kernel would leave most CUs idle and run its 9 Ci / 32 k-slices
  // one after the other on the rest)
  const long long tiles16x32 = ((m + 15) / 16) * ((co + 31) / 32);
  if (vec && fh == 3 && fw == 3 && tiles16x32 <= 512 && reinterpret_cast<uintptr_t>(y) % 8 == 0 &&
      reinterpret_cast<uintptr_t>(bias) % 8 == 0) {
    if (ci == 16) return launch_conv3x3_direct<16>(cv, w, bias, y, (int)m, co, act, stream);
    if (ci == 32) return launch_conv3x3_direct<32>(cv, w, bias, y, (int)m, co, act, stream);
    if (ci == 64) return launch_conv3x3_direct<64>(cv, w, bias, y, (int)m, co, act, stream);
    if (ci == 128) return launch_conv3x3_direct<128>(cv, w, bias, y, (int)m, co, act, stream);
  }
  // k-slices of 32 inside one filter tap, one validity bit per tap: the lean loader
  const bool lean = vec && ci % 32 == 0 && fh * fw <= 32;
  if (lean)
    return prefer_128(1, m, co)
               ? launch_cfg<128, 128, 32, 2, 2, true, false, true, true, true>(nullptr, w, y, bias, 1, (int)m, co, (int)k, act, stream, cv)
               : launch_cfg<64, 64, 32, 2, 2, true, false, true, true, true>(nullptr, w, y, bias, 1, (int)m, co, (int)k, act, stream, cv);
  if (prefer_128(1, m, co)) {
    return vec ? launch_cfg<128, 128, 32, 2, 2, true, false, true, true>(nullptr, w, y, bias, 1, (int)m, co, (int)k, act, stream, cv)
               : launch_cfg<128, 128, 32, 2, 2, true, false, false, true>(nullptr, w, y, bias, 1, (int)m, co, (int)k, act, stream, cv);
  }
  return vec ? launch_cfg<64, 64, 32, 2, 2, true, false, true, true>(nullptr, w, y, bias, 1, (int)m, co, (int)k, act, stream, cv)
             : launch_cfg<64, 64, 32, 2, 2, true, false, false, true>(nullptr, w, y, bias, 1, (int)m, co, (int)k, act, stream, cv);
}

}  // namespace tfx
