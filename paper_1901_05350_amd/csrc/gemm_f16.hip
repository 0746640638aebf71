// batchMatMul on 16-bit float storage for gfx950 (Section 4.1: the same matMul renders to a 32-bit
// or a 16-bit floating point texture; Listing 2 defines the product).
//   C[b] = half( act( op(A[b]) * op(B[b]) + bias[col] ) ),  operands, bias and result IEEE binary16,
// products accumulated in fp32 on the matrix cores (v_mfma_f32_32x32x16_f16: 32x32 outputs, 16 k
// per instruction, 8 consecutive k per lane and operand).
//
// A workgroup of WAVES_M x WAVES_N wavefronts computes a (32 TM WAVES_M) x (32 TN WAVES_N) tile;
// k-slices of 64 halfs are double-buffered in LDS as K-contiguous rows of 144 bytes (128 + 16
// padding: the 16-byte fragment reads of 32 consecutive rows fall on distinct banks).  The MFMA is
// issued with the operands swapped (B's fragment first), so a lane's accumulator registers hold 4
// consecutive output columns of one row and the epilogue stores 8 bytes at a time.
// Two kernels: a software-pipelined one for K-contiguous, 16-byte aligned operands (A stored
// [M,K], B stored [N,K]) and a general one with an element-wise loader for everything else.
#include "tfx_internal.h"

#include <type_traits>

namespace tfx {
namespace {

typedef _Float16 half_t;
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kBK = 64;       // halfs per k-slice
constexpr int kLd = kBK + 8;  // LDS row stride in halfs
constexpr int kXcds = 8;

// ---- element-wise global -> register loader for one ROWS x 64 slice of an operand ----------------
// Any layout, any K, any alignment.  kc: K is the contiguous dimension in memory
// (element (row, k) at row * ld + k), else the row index is (element at k * ld + row).
// Consecutive threads walk along the contiguous dimension.
template <int ROWS, int NT>
__device__ __forceinline__ void load_scalar(const half_t* __restrict__ g, bool kc, int ld, int rows, int K, int row0,
                                            int k0, int tid, half_t (&r)[ROWS * kBK / NT]) {
#pragma unroll
  for (int i = 0; i < ROWS * kBK / NT; ++i) {
    const int e = tid + i * NT;
    const int row = row0 + (kc ? e / kBK : e % ROWS), k = k0 + (kc ? e % kBK : e / ROWS);
    const size_t idx = kc ? (size_t)row * ld + k : (size_t)k * ld + row;
    r[i] = (row < rows && k < K) ? g[idx] : (half_t)0;
  }
}
template <int ROWS, int NT>
__device__ __forceinline__ void store_scalar(half_t* lds, bool kc, int tid, const half_t (&r)[ROWS * kBK / NT]) {
#pragma unroll
  for (int i = 0; i < ROWS * kBK / NT; ++i) {
    const int e = tid + i * NT;
    const int row = kc ? e / kBK : e % ROWS, k = kc ? e % kBK : e / ROWS;
    lds[row * kLd + k] = r[i];
  }
}

// General kernel: operands of any layout and alignment through the element-wise loader; the slice
// kt+1 is fetched into registers before the MFMAs of slice kt and written to LDS after them.
template <int WAVES_M, int WAVES_N, int TM, int TN>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void gemm_f16_kernel(
    const half_t* __restrict__ A, const half_t* __restrict__ B, half_t* __restrict__ C, const half_t* __restrict__ bias,
    int M, int N, int K, int a_kc, int b_kc, int tiles_m, int tiles_n, int total_blocks, long long strideA,
    long long strideB, long long strideC, int act, int group_m, int c_vec) {
  constexpr int kNT = 64 * WAVES_M * WAVES_N;
  constexpr int WM = 32 * TM, WN = 32 * TN;
  constexpr int BM = WM * WAVES_M, BN = WN * WAVES_N;
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
  // within a batch, tiles are walked in bands of group_m tile rows, column by column, so that the
  // tiles an XCD works on at the same time form a compact block (few distinct A and B panels)
  const int band = t / (group_m * tiles_n);
  const int band_rows = min(group_m, tiles_m - band * group_m);
  const int tb = t - band * group_m * tiles_n;
  const int tile_m = band * group_m + tb % band_rows;
  const int tile_n = tb / band_rows;

  const int lda = a_kc ? K : M, ldb = b_kc ? K : N;
  A += (size_t)batch * strideA;
  B += (size_t)batch * strideB;
  C += (size_t)batch * strideC;

  const int tid = threadIdx.x;
  const int wave = tid / 64, lane = tid % 64;
  const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;
  const int li = lane % 32, hh = lane / 32;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  half_t ra[BM * kBK / kNT], rb[BN * kBK / kNT];
  auto load = [&](int k0) {
    load_scalar<BM, kNT>(A, a_kc != 0, lda, M, K, m0, k0, tid, ra);
    load_scalar<BN, kNT>(B, b_kc != 0, ldb, N, K, n0, k0, tid, rb);
  };
  auto store = [&](int buf) {
    store_scalar<BM, kNT>(lds_a + buf * kTileA, a_kc != 0, tid, ra);
    store_scalar<BN, kNT>(lds_b + buf * kTileB, b_kc != 0, tid, rb);
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

// Software-pipelined variant for K-contiguous, 16-byte aligned operands.  The vector memory
// path delivers 64 bytes per clock to a CU, so a k-slice's global loads take a large part of the
// slice's MFMA time and must be spread evenly through it; the same holds for the LDS writes.
// Iteration kt (slice kt in LDS buffer kt & 1):
// after every few MFMAs one 16-byte slot of slice kt+1 (loaded a whole iteration earlier) moves from
// its registers to the other LDS buffer and the same registers are refilled with that slot of slice
// kt+2; one barrier per slice.
template <int WAVES_M, int WAVES_N, int TM, int TN, bool B_KC>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void gemm_f16_pipe_kernel(
    const half_t* __restrict__ A, const half_t* __restrict__ B, half_t* __restrict__ C, const half_t* __restrict__ bias,
    int M, int N, int K, int tiles_m, int tiles_n, int total_blocks, long long strideA, long long strideB,
    long long strideC, int act, int group_m, int c_vec) {
  constexpr int kNT = 64 * WAVES_M * WAVES_N;
  constexpr int WM = 32 * TM, WN = 32 * TN;
  constexpr int BM = WM * WAVES_M, BN = WN * WAVES_N;
  constexpr int kTileA = BM * kLd, kTileB = BN * kLd;
  constexpr int SA = BM * 8 / kNT, SB = BN * 8 / kNT, SLOTS = SA + SB;  // 16-byte slots per thread and slice
  constexpr int STEPS = kBK / 16, MF = TM * TN;  // k-steps per slice, MFMAs per step
  static_assert(BM * 8 % kNT == 0 && BN * 8 % kNT == 0, "loader shape");
  static_assert(B_KC || (SB == 4 && kNT / 16 == BN / 8), "the [K,N] loader moves 4 k-rows x 8 columns per thread");
  extern __shared__ __align__(16) half_t smem_h[];
  half_t* const lds_a = smem_h;
  half_t* const lds_b = smem_h + 2 * kTileA;

  const int bid = blockIdx.x;
  const int q = total_blocks / kXcds, rem = total_blocks % kXcds;
  const int xcd = bid % kXcds;
  const int vid = xcd * q + (xcd < rem ? xcd : rem) + bid / kXcds;
  const int tiles = tiles_m * tiles_n;
  const int batch = vid / tiles;
  const int t = vid % tiles;
  const int band = t / (group_m * tiles_n);
  const int band_rows = min(group_m, tiles_m - band * group_m);
  const int tb = t - band * group_m * tiles_n;
  const int tile_m = band * group_m + tb % band_rows;
  const int tile_n = tb / band_rows;

  A += (size_t)batch * strideA;
  B += (size_t)batch * strideB;
  C += (size_t)batch * strideC;

  const int tid = threadIdx.x;
  const int wave = tid / 64, lane = tid % 64;
  const int wm0 = (wave / WAVES_N) * WM, wn0 = (wave % WAVES_N) * WN;
  const int li = lane % 32, hh = lane / 32;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // slot w of a slice: w < SA is A's slot w, else B's slot w - SA; slot i of an operand covers
  // tile row (tid + i * kNT) / 8, halfs 8 * ((tid + i * kNT) % 8) ... + 7.  Rows past the matrix
  // are clamped to its last row (they only feed outputs that are never stored) and k-slices are
  // clamped to the last one, so every load is unconditional and in bounds; halfs past K are zeroed
  // with a mask.  The loop body therefore has no branch.
  const int srow = tid / 8, scol = 8 * (tid % 8);
  constexpr int kRowStep = kNT / 8;
  typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
  //
  // B stored [K,N] (!B_KC, N % 8 == 0): thread (kq = tid % 16, nb = tid / 16) loads k-rows 4 kq ... + 3 of
  // columns 8 nb ... + 7 as four 16-byte slots (16 lanes with consecutive kq: the 8-byte LDS writes of
  // one row are contiguous), transposes the 4 x 8 block in registers and writes, for each of the 8
  // columns, 4 consecutive k to the K-contiguous LDS row of that column.  The block is written when
  // its first slot comes up in the schedule, its slots are refilled one by one.
  u32x4 reg[SLOTS];
  unsigned boff[SLOTS];  // byte offset of the slot at k0 = 0 from its operand's base (operands hold < 2^31 elements)
  const int kq = tid % 16, nb = tid / 16;
  const unsigned bcol = n0 + 8 * nb < N ? (unsigned)(n0 + 8 * nb) : 0u;  // past N: any valid column block
#pragma unroll
  for (int w = 0; w < SLOTS; ++w) {
    const bool is_a = w < SA;
    const int i = is_a ? w : w - SA;
    if (is_a || B_KC) {
      const int row = min((is_a ? m0 : n0) + srow + i * kRowStep, (is_a ? M : N) - 1);
      boff[w] = 2u * ((unsigned)row * (unsigned)K + (unsigned)scol);
    } else {
      boff[w] = 2u * ((unsigned)(4 * kq + i) * (unsigned)N + bcol);
    }
  }
  const int nk = (K + kBK - 1) / kBK;
  const int k_last = (nk - 1) * kBK;
  // FULL: the slice starting at k0 lies inside K.  Then a load is the operand's base advanced by the slice
  // (uniform, scalar registers) plus the slot's constant 32-bit offset, and a store needs no mask: no vector
  // ALU instruction per slot (each one would take issue time from the matrix cores).
  auto load_slot = [&](int w, int k0, auto full) {
    const char* g = reinterpret_cast<const char*>(w < SA ? A : B);
    if (w < SA || B_KC) {
      if constexpr (decltype(full)::value) {
        reg[w] = *reinterpret_cast<const u32x4*>(g + 2 * (size_t)k0 + boff[w]);
      } else {
        // past K: the start of the slot's row (a valid address), zeroed when stored
        const unsigned off = k0 + scol < K ? boff[w] + 2u * (unsigned)k0 : boff[w] - 2u * (unsigned)scol;
        reg[w] = *reinterpret_cast<const u32x4*>(g + off);
      }
    } else {
      if constexpr (decltype(full)::value) {
        reg[w] = *reinterpret_cast<const u32x4*>(g + 2 * (size_t)k0 * (size_t)N + boff[w]);
      } else {
        const int k = k0 + 4 * kq + (w - SA);
        const unsigned off = k < K ? boff[w] + 2u * (unsigned)k0 * (unsigned)N : 2u * bcol;  // past K: row 0
        reg[w] = *reinterpret_cast<const u32x4*>(g + off);
      }
    }
  };
  // k0: first k of the slice the registers hold; the zeroing of halfs past K happens here, when the
  // registers are consumed, so that nothing waits on a load right after issuing it
  auto store_slot = [&](int w, int buf, int k0, auto full) {
    constexpr bool FULL = decltype(full)::value;
    if (w < SA || B_KC) {
      const bool is_a = w < SA;
      const int i = is_a ? w : w - SA;
      half_t* l = is_a ? lds_a + buf * kTileA : lds_b + buf * kTileB;
      const unsigned mask = (FULL || k0 + scol < K) ? 0xffffffffu : 0u;
      *reinterpret_cast<u32x4*>(l + (srow + i * kRowStep) * kLd + scol) = FULL ? reg[w] : reg[w] & mask;
    } else if (w == SA) {
      h8 r[4];
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const unsigned mask = (FULL || k0 + 4 * kq + kk < K) ? 0xffffffffu : 0u;
        r[kk] = __builtin_bit_cast(h8, FULL ? reg[SA + kk] : reg[SA + kk] & mask);
      }
      half_t* l = lds_b + buf * kTileB + (8 * nb) * kLd + 4 * kq;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const h4 o = {r[0][i], r[1][i], r[2][i], r[3][i]};
        *reinterpret_cast<h4*>(l + i * kLd) = o;
      }
    }
  };
  constexpr std::false_type kMasked{};

#pragma unroll
  for (int w = 0; w < SLOTS; ++w) load_slot(w, 0, kMasked);
#pragma unroll
  for (int w = 0; w < SLOTS; ++w) store_slot(w, 0, 0, kMasked);
#pragma unroll
  for (int w = 0; w < SLOTS; ++w) load_slot(w, min(kBK, k_last), kMasked);
  __syncthreads();

  // One k-slice.  FULL: slices kt + 1 (stored) and kt + 2 (fetched) both lie inside K.
  auto k_slice = [&](int kt, auto full) {
    const int cur = kt & 1;
    // the last two iterations refetch the last slice (unused)
    const int k_next = decltype(full)::value ? (kt + 2) * kBK : min((kt + 2) * kBK, k_last);
    const half_t* la = lds_a + cur * kTileA + (wm0 + li) * kLd + 8 * hh;
    const half_t* lb = lds_b + cur * kTileB + (wn0 + li) * kLd + 8 * hh;
    h8 fa[2][TM], fb[2][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[0][i] = *reinterpret_cast<const h8*>(la + 32 * i * kLd);
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[0][j] = *reinterpret_cast<const h8*>(lb + 32 * j * kLd);
#pragma unroll
    for (int s = 0; s < STEPS; ++s) {
      if (s + 1 < STEPS) {
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[(s + 1) & 1][i] = *reinterpret_cast<const h8*>(la + 32 * i * kLd + 16 * (s + 1));
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[(s + 1) & 1][j] = *reinterpret_cast<const h8*>(lb + 32 * j * kLd + 16 * (s + 1));
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fb[s & 1][j], fa[s & 1][i], acc[i][j], 0, 0, 0);
          // memory instructions due after this MFMA: slots [p * SLOTS / ALL, (p + 1) * SLOTS / ALL) of the slice.
          // A slot's registers (slice kt+1, loaded one iteration ago) go to the other LDS buffer and are
          // refilled at once with the same slot of slice kt+2.
          constexpr int ALL = STEPS * MF;
          const int p = s * MF + i * TN + j;
#pragma unroll
          for (int w = p * SLOTS / ALL; w < (p + 1) * SLOTS / ALL; ++w) {
            store_slot(w, cur ^ 1, (kt + 1) * kBK, full);
            load_slot(w, k_next, full);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    __syncthreads();
  };
  int kt = 0;
  for (; (kt + 3) * kBK <= K; ++kt) k_slice(kt, std::true_type{});
  for (; kt < nk; ++kt) k_slice(kt, kMasked);

  const ActClamp clamp = make_act(act);
  if (c_vec == 2) {
    // Staged epilogue (N % 8 == 0, C 16-byte aligned): every wavefront converts its WM x WN block to
    // binary16 in a private LDS region (all k-slice buffers are free after the loop's last barrier),
    // then reads it back row-wise and stores 16 bytes per lane, whole 128-byte lines per row.
    constexpr int kLs = WN + 8;  // staging row stride in halfs
    static_assert((size_t)WAVES_M * WAVES_N * WM * kLs <= 2 * (size_t)(BM + BN) * kLd, "staging fits in the slice buffers");
    half_t* stage = smem_h + wave * WM * kLs;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int cl = 32 * j + 8 * g + 4 * hh;  // column inside the wave's block
        const int col = n0 + wn0 + cl;
        float bv[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) bv[e] = (bias != nullptr && col + e < N) ? (float)bias[col + e] : 0.f;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
          h4 pk;
#pragma unroll
          for (int e = 0; e < 4; ++e) pk[e] = (half_t)apply_act(acc[i][j][4 * g + e] + bv[e], clamp);
          *reinterpret_cast<h4*>(stage + (32 * i + li) * kLs + cl) = pk;
        }
      }
    }
    constexpr int kLanesPerRow = WN / 8, kRowsPerStep = 64 / kLanesPerRow;
    const int rr = lane / kLanesPerRow, cc = 8 * (lane % kLanesPerRow);
    const int col = n0 + wn0 + cc;
#pragma unroll
    for (int r0 = 0; r0 < WM; r0 += kRowsPerStep) {
      const int row = m0 + wm0 + r0 + rr;
      const h8 v = *reinterpret_cast<const h8*>(stage + (r0 + rr) * kLs + cc);
      if (row < M && col < N) *reinterpret_cast<h8*>(C + (size_t)row * N + col) = v;
    }
    return;
  }
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

template <int WAVES_M, int WAVES_N, int TM, int TN, bool B_KC = true>
int launch_pipe(const half_t* a, const half_t* b, half_t* c, const half_t* bias, int batch, int m, int n, int k,
                bool, bool, int act, hipStream_t stream, int group_m = 4) {
  constexpr int BM = 32 * TM * WAVES_M, BN = 32 * TN * WAVES_N, NT = 64 * WAVES_M * WAVES_N;
  constexpr size_t lds_bytes = 2 * (size_t)(BM + BN) * kLd * sizeof(half_t);
  static_assert(lds_bytes <= 160 * 1024, "LDS budget per workgroup");
  auto kern = gemm_f16_pipe_kernel<WAVES_M, WAVES_N, TM, TN, B_KC>;
  static std::atomic<uint64_t> lds_allowed{0};
  if (allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds_bytes, lds_allowed) != TFX_OK) return TFX_ERR_LAUNCH;
  const int tiles_m = (m + BM - 1) / BM, tiles_n = (n + BN - 1) / BN;
  const long long total = (long long)batch * tiles_m * tiles_n;
  if (total > 0x7fffffffLL) return TFX_ERR_UNSUPPORTED;
  // 2: staged 16-byte stores (every row of C starts 16-byte aligned), 1: direct 8-byte stores, 0: element stores
  const int c_vec = (n % 8 == 0 && reinterpret_cast<uintptr_t>(c) % 16 == 0) ? 2
                    : (n % 4 == 0 && reinterpret_cast<uintptr_t>(c) % 8 == 0) ? 1 : 0;
  hipLaunchKernelGGL(kern, dim3((unsigned)total), dim3(NT), lds_bytes, stream, a, b, c, bias, m, n, k, tiles_m, tiles_n,
                     (int)total, (long long)m * k, (long long)n * k, (long long)m * n, act, group_m, c_vec);
  return check_launch();
}

template <int WAVES_M, int WAVES_N, int TM, int TN>
int launch_cfg(const half_t* a, const half_t* b, half_t* c, const half_t* bias, int batch, int m, int n, int k,
               bool a_kc, bool b_kc, int act, hipStream_t stream, int group_m = 4) {
  constexpr int BM = 32 * TM * WAVES_M, BN = 32 * TN * WAVES_N, NT = 64 * WAVES_M * WAVES_N;
  constexpr size_t lds_bytes = 2 * (size_t)(BM + BN) * kLd * sizeof(half_t);
  static_assert(lds_bytes <= 160 * 1024, "LDS budget per workgroup");
  auto kern = gemm_f16_kernel<WAVES_M, WAVES_N, TM, TN>;
  static std::atomic<uint64_t> lds_allowed{0};
  if (allow_dynamic_lds(reinterpret_cast<const void*>(kern), lds_bytes, lds_allowed) != TFX_OK) return TFX_ERR_LAUNCH;
  const int tiles_m = (m + BM - 1) / BM, tiles_n = (n + BN - 1) / BN;
  const long long total = (long long)batch * tiles_m * tiles_n;
  if (total > 0x7fffffffLL) return TFX_ERR_UNSUPPORTED;
  // 8-byte stores need every row of C to start 8-byte aligned
  const int c_vec = (n % 4 == 0 && reinterpret_cast<uintptr_t>(c) % 8 == 0) ? 1 : 0;
  hipLaunchKernelGGL(kern, dim3((unsigned)total), dim3(NT), lds_bytes, stream, a, b, c, bias, m, n, k, a_kc ? 1 : 0,
                     b_kc ? 1 : 0, tiles_m, tiles_n, (int)total, (long long)m * k, (long long)n * k,
                     (long long)m * n, act, group_m, c_vec);
  return check_launch();
}

// Small M x N (the 28x28 ... 7x7 pointwise layers of a batch-1 MobileNet: 49 ... 3136 rows): too few
// 64 x 64 tiles for 256 CUs, and each tile is bound by memory latency, not by the matrix cores.
// 16 x 32 tiles (v_mfma_f32_16x16x32_f16), a tile as deep as K up to 512 so that the whole K panel is
// in flight in one memory round trip, the depth split over 8 wavefronts whose partial tiles are
// added through LDS by the 512 threads that also apply the epilogue.  A stored [M,K], B stored
// [K,N] (N % 8 == 0, K % 8 == 0, 16-byte aligned); B goes through the 4 x 8 register transpose
// of the pipelined kernel.
typedef float f32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(512) void gemm_f16_small_kernel(const half_t* __restrict__ A, const half_t* __restrict__ B,
                                                             half_t* __restrict__ C, const half_t* __restrict__ bias,
                                                             int M, int N, int K, int tiles_m, int tiles_n,
                                                             int total_blocks, long long strideA, long long strideB,
                                                             long long strideC, int act) {
  constexpr int BM = 16, BN = 32, BKS = 512, LD = BKS + 8, NT = 512, WAVES_K = 8;
  __shared__ __align__(16) half_t lds[(BM + BN) * LD];
  half_t* const lds_a = lds;
  half_t* const lds_b = lds + BM * LD;

  const int bid = blockIdx.x;
  const int q8 = total_blocks / kXcds, rem = total_blocks % kXcds;
  const int xcd = bid % kXcds;
  const int vid = xcd * q8 + (xcd < rem ? xcd : rem) + bid / kXcds;
  const int tiles = tiles_m * tiles_n;
  const int batch = vid / tiles;
  const int t = vid % tiles;
  const int tile_m = t % tiles_m, tile_n = t / tiles_m;  // consecutive workgroups share a column panel of B

  A += (size_t)batch * strideA;
  B += (size_t)batch * strideB;
  C += (size_t)batch * strideC;

  const int tid = threadIdx.x;
  const int wk = tid / 64, lane = tid % 64;
  const int li = lane % 16, q = lane / 16;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  // epilogue thread e owns the value of register v of lane l of column block j, e = (j * 4 + v) * 64 + l
  const int ej = tid / 256, ev = (tid / 64) % 4, el = tid % 64;
  const int erow = m0 + 4 * (el / 16) + ev, ecol = n0 + 16 * ej + el % 16;
  float ebias = 0.f;
  if (bias != nullptr && ecol < N) ebias = (float)bias[ecol];

  typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
  // A: 2 slots per thread, slot s = tid + 512 i: row s / 64, halfs 8 (s % 64) ... + 7
  // B: thread (kq = tid / 4, nb = tid % 4) owns k-rows 4 kq ... + 3 of columns 8 nb ... + 7
  u32x4 ra[2], rb[4];
  const int kq = tid / 4, nb = tid % 4;
  const unsigned bcol = n0 + 8 * nb < N ? (unsigned)(n0 + 8 * nb) : 0u;
  auto load = [&](int k0) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int s = tid + i * NT;
      const int row = min(m0 + s / 64, M - 1), k = k0 + 8 * (s % 64);
      ra[i] = *reinterpret_cast<const u32x4*>(A + (size_t)((unsigned)row * (unsigned)K + (k < K ? (unsigned)k : 0u)));
    }
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const int k = k0 + 4 * kq + kk;
      rb[kk] = *reinterpret_cast<const u32x4*>(B + (size_t)((k < K ? (unsigned)k : 0u) * (unsigned)N + bcol));
    }
  };
  auto store = [&](int k0) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int s = tid + i * NT;
      const unsigned mask = k0 + 8 * (s % 64) < K ? 0xffffffffu : 0u;
      *reinterpret_cast<u32x4*>(lds_a + (s / 64) * LD + 8 * (s % 64)) = ra[i] & mask;
    }
    h8 r[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const unsigned mask = k0 + 4 * kq + kk < K ? 0xffffffffu : 0u;
      r[kk] = __builtin_bit_cast(h8, rb[kk] & mask);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const h4 o = {r[0][i], r[1][i], r[2][i], r[3][i]};
      *reinterpret_cast<h4*>(lds_b + (8 * nb + i) * LD + 4 * kq) = o;
    }
  };

  f32x4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
  const int nk = (K + BKS - 1) / BKS;
  load(0);
  for (int kt = 0; kt < nk; ++kt) {
    if (kt > 0) __syncthreads();  // everyone has finished reading the previous slice
    store(kt * BKS);
    __syncthreads();
    if (kt + 1 < nk) load((kt + 1) * BKS);
#pragma unroll
    for (int s = 0; s < BKS / WAVES_K / 32; ++s) {
      const int kb = wk * (BKS / WAVES_K) + 32 * s;  // this wavefront's 32 k of the slice
      if (kt * BKS + kb >= K) break;                 // past the end of K: zeros
      const h8 fa = *reinterpret_cast<const h8*>(lds_a + li * LD + kb + 8 * q);
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const h8 fb = *reinterpret_cast<const h8*>(lds_b + (16 * j + li) * LD + kb + 8 * q);
        acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fa, fb, acc[j], 0, 0, 0);
      }
    }
  }

  // add the 8 partial tiles through LDS: layout [wk][j][v][lane]
  __syncthreads();
  float* red = reinterpret_cast<float*>(lds);
  static_assert(WAVES_K * 2 * 4 * 64 * sizeof(float) <= sizeof(lds), "reduction reuses the slice buffers");
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int v = 0; v < 4; ++v) red[(wk * 8 + j * 4 + v) * 64 + lane] = acc[j][v];
  __syncthreads();
  float sum = ebias;
#pragma unroll
  for (int w = 0; w < WAVES_K; ++w) sum += red[w * 512 + tid];
  if (erow < M && ecol < N) C[(size_t)erow * N + ecol] = (half_t)apply_act(sum, make_act(act));
}

int launch_small(const half_t* a, const half_t* b, half_t* c, const half_t* bias, int batch, int m, int n, int k,
                 int act, hipStream_t stream) {
  const int tiles_m = (m + 15) / 16, tiles_n = (n + 31) / 32;
  const long long total = (long long)batch * tiles_m * tiles_n;
  if (total > 0x7fffffffLL) return TFX_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(gemm_f16_small_kernel, dim3((unsigned)total), dim3(512), 0, stream, a, b, c, bias, m, n, k,
                     tiles_m, tiles_n, (int)total, (long long)m * k, (long long)n * k, (long long)m * n, act);
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
  const bool aligned = reinterpret_cast<uintptr_t>(a) % 16 == 0 && reinterpret_cast<uintptr_t>(b) % 16 == 0;
  const bool vec = a_kc && b_kc && k % 8 == 0 && aligned;
  // A [M,K] with B stored [K,N] (matMul without transposes, a pointwise convolution's filter): 16-byte
  // loads along N and a register transpose on the way into LDS
  const bool vec_kn = a_kc && !b_kc && k % 8 == 0 && n % 8 == 0 && aligned;
  auto tiles = [&](int bm, int bn) { return (long long)batch * ((m + bm - 1) / bm) * ((n + bn - 1) / bn); };
  // a tile shape is acceptable if it wastes at most 10% more of its area on padding than 128 x 128 tiles do
  auto fits = [&](int bm, int bn) {
    const double pad = (double)((m + bm - 1) / bm * bm) * ((n + bn - 1) / bn * bn);
    const double pad128 = (double)((m + 127) / 128 * 128) * ((n + 127) / 128 * 128);
    return pad <= 1.1 * pad128;
  };
  if (vec) {
    // 256 x 256 tiles (8 wavefronts) once they fill most of the 256 CUs, then 256 x 128 (8 wavefronts),
    // 128 x 128 (4 wavefronts, two workgroups per CU) for mid-size problems, 64 x 64 below that
    if (tiles(256, 256) >= 192 && fits(256, 256))
      return launch_pipe<2, 4, 4, 2>(a, b, c, bias, batch, m, n, k, true, true, act, stream);
    if (tiles(256, 128) >= 192 && fits(256, 128))
      return launch_pipe<4, 2, 2, 2>(a, b, c, bias, batch, m, n, k, true, true, act, stream);
    if (tiles(128, 128) >= 128) return launch_pipe<2, 2, 2, 2>(a, b, c, bias, batch, m, n, k, true, true, act, stream);
    return launch_pipe<2, 2, 1, 1>(a, b, c, bias, batch, m, n, k, true, true, act, stream);
  }
  if (batch == 1 && a_kc && !b_kc && pointwise_stream_f16_supported(m, k, n, a, b, c))
    return launch_pointwise_stream_f16(a16, b16, bias16, c16, m, k, n, act, stream);
  if (batch == 1 && a_kc && !b_kc && pointwise_slab_f16_supported(m, k, n, a, b, c))
    return launch_pointwise_slab_f16(a16, b16, bias16, c16, m, k, n, act, stream);
  if (vec_kn) {
    if (tiles(256, 256) >= 192 && fits(256, 256))
      return launch_pipe<2, 4, 4, 2, false>(a, b, c, bias, batch, m, n, k, true, false, act, stream);
    if (tiles(128, 128) >= 128) return launch_pipe<2, 2, 2, 2, false>(a, b, c, bias, batch, m, n, k, true, false, act, stream);
    if (tiles(64, 64) >= 128) return launch_pipe<2, 1, 1, 2, false>(a, b, c, bias, batch, m, n, k, true, false, act, stream);
    return launch_small(a, b, c, bias, batch, m, n, k, act, stream);
  }
  if (tiles(128, 128) >= 256) return launch_cfg<2, 2, 2, 2>(a, b, c, bias, batch, m, n, k, a_kc, b_kc, act, stream);
  return launch_cfg<2, 2, 1, 1>(a, b, c, bias, batch, m, n, k, a_kc, b_kc, act, stream);
}

}  // namespace tfx
