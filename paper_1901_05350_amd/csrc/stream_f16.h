// Pieces shared by the filter-stationary kernels on 16-bit float storage (pointwise_f16.hip, conv_stream_f16.hip):
// the filter's layout in LDS, its transpose from global memory, and the epilogue that turns accumulators into
// 16-byte pieces of output.  All of it is written for v_mfma_f32_16x16x32_f16 with the filter as the first operand:
// lane (li = lane % 16, q = lane / 16) supplies filter row li and k-group q, and receives rows 4 q ... 4 q + 3 of
// the 16-row output block in its four accumulator registers.
#pragma once
#include "tfx_internal.h"

namespace tfx {
namespace f16s {

typedef _Float16 half_t;
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Filter rows in LDS: K halfs (k-contiguous, as the matrix cores want them) plus the least padding, in 16-byte
// pieces, that makes the fragment read of 16 consecutive rows free of conflicts.
struct FilterRowPieces {
  int pieces;  // row stride in 16-byte pieces
  constexpr int operator()(int li, int q) const { return li * pieces + q; }
};
constexpr int filter_row_halfs(int K) {
  for (int pieces = K / 8 + 1;; ++pieces)
    if (conflict_free(FilterRowPieces{pieces})) return pieces * 8;
}

// Column c of the filter goes to LDS row rho(c) = 32 (c / 32) + 16 (c % 8 / 4) + 4 (c % 32 / 8) + c % 4.  With the
// MFMA's output layout a lane then owns channels 8 q ... 8 q + 7 of every 32 -- the first four in block 2 m, the
// rest in block 2 m + 1 -- and stores them as one 16-byte piece.
__device__ __forceinline__ constexpr int rho(int c) { return 32 * (c / 32) + 16 * (c % 8 / 4) + 4 * (c % 32 / 8) + c % 4; }

// The filter w[K][N] moves to LDS as [N rows in rho order][LD halfs] in two steps, so that the caller can put other
// loads between them: `fetch` issues every 16-byte load of the thread (block u covers k-rows 4 kq ... + 3 of
// columns 8 nb ... + 7; no branch: a thread
// without a block in the last pass over the blocks reads block 0 again -- behind a guarded load the compiler waits
// for every load still in flight; `row_halfs` is the length of w's rows where the N columns are a slab of a wider
// filter), `store` transposes each 4 x 8 block in registers and writes eight 8-byte pieces.
template <int K, int N, int NT>
struct FilterStage {
  static constexpr int BLOCKS = (K / 4) * (N / 8), PER = (BLOCKS + NT - 1) / NT, LD = filter_row_halfs(K);
  // Block u -> (column block nb, k-group kq).  The 8-byte LDS writes of a wavefront go to row rho(8 nb + j) at
  // half 4 kq.  A row is an odd multiple of 32 bytes long, so the rows of column blocks nb, nb + 1, nb + 2, nb + 3
  // (4 rows apart) start at the four multiples of 128 bytes modulo 512.  Where K allows it (64 k = 16 k-groups per
  // wavefront) the 64 blocks of a wavefront are therefore 4 neighbouring column blocks x 16 k-groups: 4 x 128
  // consecutive bytes, every bank once, and the loads still read 64 consecutive bytes of each row of w.
  // Otherwise: the column blocks of whole rows of w (several writes per bank; only small filters take this form).
  static constexpr bool kByGroups = K % 64 == 0 && N % 32 == 0;
  __device__ __forceinline__ static void place(int u, int* nb, int* kq) {
    if constexpr (kByGroups) {
      const int g = u / 64, l = u % 64;
      *nb = 4 * (g % (N / 32)) + l % 4;
      *kq = 16 * (g / (N / 32)) + l / 4;
    } else {
      *nb = u % (N / 8);
      *kq = u / (N / 8);
    }
  }
  h8 r[PER][4];
  __device__ __forceinline__ void fetch(const half_t* __restrict__ w, int tid, int row_halfs = N) {
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      int nb, kq;
      place(tid + i * NT < BLOCKS ? tid + i * NT : 0, &nb, &kq);
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) r[i][kk] = *reinterpret_cast<const h8*>(w + (size_t)(4 * kq + kk) * row_halfs + 8 * nb);
    }
  }
  __device__ __forceinline__ void store(half_t* wl, int tid) const {
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int u = tid + i * NT;
      int nb, kq;
      place(u, &nb, &kq);
      if (BLOCKS % NT == 0 || i + 1 < PER || u < BLOCKS) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const h4 o = {r[i][0][j], r[i][1][j], r[i][2][j], r[i][3][j]};
          *reinterpret_cast<h4*>(wl + rho(8 * nb + j) * LD + 4 * kq) = o;
        }
      }
    }
  }
};

// Bias in the accumulators' layout (block j, rows 4 q ... 4 q + 3 = channels 32 (j / 2) + 8 q + 4 (j % 2) ...):
// `fetch` issues the loads without a branch (with no bias they read `fallback`, any readable array of at least as
// many halfs, and the values are dropped), `get` converts them; nothing between the two waits for the loads.
template <int NB>
struct BiasRows {
  half_t raw[NB][4];
  __device__ __forceinline__ void fetch(const half_t* __restrict__ bias, const half_t* __restrict__ fallback, int q) {
    const half_t* const p = bias ? bias : fallback;
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) raw[j][e] = p[32 * (j / 2) + 8 * q + 4 * (j % 2) + e];
  }
  __device__ __forceinline__ void get(bool have, f32x4 (&bv)[NB]) const {
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) bv[j][e] = have ? (float)raw[j][e] : 0.f;
  }
};

// Activation and rounding of one 16-row slab: accumulator blocks 2 m and 2 m + 1 become the 8 halfs o[m].  The clamp
// is one median-of-three per value; that instruction, like max and min, drops a NaN, so NaNs are looked for on the
// side (a compare per pair of values, collected in scalar registers) and a wavefront that holds one takes the exact
// form, through which a NaN passes.
template <int NB>
__device__ __forceinline__ void activate_and_pack(const f32x4 (&acc)[NB], const ActClamp& clamp, h8 (&o)[NB / 2]) {
  const float lo = clamp.on ? 0.f : -INFINITY;
  unsigned long long nan = 0;
#pragma unroll
  for (int m = 0; m < NB / 2; ++m) {
    float v[8];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      v[e] = acc[2 * m][e];
      v[4 + e] = acc[2 * m + 1][e];
    }
#pragma unroll
    for (int e = 0; e < 8; e += 2) nan |= __builtin_amdgcn_ballot_w64(__builtin_isunordered(v[e], v[e + 1]));
#pragma unroll
    for (int e = 0; e < 8; ++e) o[m][e] = (half_t)__builtin_amdgcn_fmed3f(v[e], lo, clamp.hi);
  }
  if (nan != 0) {
#pragma unroll
    for (int m = 0; m < NB / 2; ++m)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        o[m][e] = (half_t)apply_act(acc[2 * m][e], clamp);
        o[m][4 + e] = (half_t)apply_act(acc[2 * m + 1][e], clamp);
      }
  }
}

}  // namespace f16s
}  // namespace tfx
