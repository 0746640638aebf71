// conv2d on 16-bit float storage as an implicit GEMM on the matrix cores (Section 4.1: 16-bit floating point
// textures; the NHWC index order of the conv2d sampler), for any filter size / stride / padding when the
// channel counts are multiples of 8:
//   y[M, Co] = half( act( A[M, K] * filter[K, Co] + bias ) ),  M = n * oh * ow,  K = fh * fw * Ci,
// where row m of A is the 3-D window of output pixel m, never materialised: 8 consecutive k are 8 consecutive
// channels of one input pixel under one filter tap (Ci % 8 == 0), i.e. one 16-byte load, or zeros where the
// tap falls outside the image.  Products are accumulated in fp32 (v_mfma_f32_32x32x16_f16), the result is
// rounded once.
//
// A workgroup of 2 x 2 wavefronts computes a 128 x 128 tile (64 columns when that pads the output channels
// less, 64 rows for small problems); k-slices of 64 halfs are double-buffered in LDS as K-contiguous rows of 144 bytes.  The slice kt + 1
// is fetched into registers before the MFMAs of slice kt and written to LDS after them.  A thread's four A slots share their k position (8 halfs at k0 + 8 (tid % 8)),
// so the tap and channel of that position are kept per thread and advanced by 64 per slice without a
// division; each slot keeps its pixel's window origin and one validity bit per tap.  The filter is stored
// [K, Co]: a thread loads 4 k-rows x 8 columns as four 16-byte loads, transposes the block in registers and
// writes 4 consecutive k per column to the K-contiguous LDS rows.
#include "tfx_internal.h"

namespace tfx {
namespace {

typedef _Float16 half_t;
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kBK = 64;       // halfs per k-slice
constexpr int kLd = kBK + 8;  // LDS row stride in halfs
constexpr int kXcds = 8;
constexpr int kNT = 256;
constexpr int kSlots = 4;  // 16-byte filter slots per thread and slice

struct ConvGeomF16 {
  const half_t* x;
  int H, W, Ci, OH, OW, fh, fw, taps, sh, sw, pt, pl;
};

// TM, TN: 32-row / 32-column MFMA blocks per wavefront (tile 64 TM x 64 TN).
// LEAN (Ci % 64 == 0, operands of fewer than 2^31 bytes): a k-slice lies inside one filter tap, the same for
// every thread, so tap and channel are scalar state, a slot's address is a uniform base plus a 32-bit offset,
// and no slice of the filter is ragged -- a fraction of the vector-ALU instructions of the general form.
template <int TM, int TN, bool LEAN>
__global__ __launch_bounds__(kNT) void conv_f16_gemm_kernel(ConvGeomF16 cv, const half_t* __restrict__ w,
                                                            const half_t* __restrict__ bias, half_t* __restrict__ y,
                                                            int M, int N, int K, int tiles_n, int total_blocks,
                                                            int wraps, int act, int c_vec) {
  constexpr int kBM = 64 * TM, kBN = 64 * TN, kTileA = kBM * kLd, kTileB = kBN * kLd;
  constexpr int kSlotsA = 2 * TM;  // 16-byte window slots per thread and slice
  extern __shared__ __align__(16) half_t smem_h[];
  half_t* const lds_a = smem_h;  // two A buffers, then two B buffers
  half_t* const lds_b = smem_h + 2 * kTileA;

  // hardware block id b lands on XCD b % 8: give each XCD (own L2) a contiguous range of tiles; the column
  // tiles of one row tile are neighbours, so the window rows they share are fetched once per XCD
  const int bid = blockIdx.x;
  const int q8 = total_blocks / kXcds, rem = total_blocks % kXcds;
  const int xcd = bid % kXcds;
  const int vid = xcd * q8 + (xcd < rem ? xcd : rem) + bid / kXcds;
  const int tile_m = vid / tiles_n, tile_n = vid % tiles_n;
  const int m0 = tile_m * kBM, n0 = tile_n * kBN;

  const int tid = threadIdx.x;
  const int wave = tid / 64, lane = tid % 64;
  const int wm0 = (wave / 2) * 32 * TM, wn0 = (wave % 2) * 32 * TN;
  const int li = lane % 32, hh = lane / 32;

  // A slots: tile row srow + 32 i, halfs scol ... scol + 7 of the slice.  Per slot: element offset of the
  // window origin (oh * sh - pt, ow * sw - pl), which may lie outside the image, and a validity bit per tap.
  const int srow = tid / 8, scol = 8 * (tid % 8);
  long long origin[kSlotsA];
  unsigned origin_b[kSlotsA];  // LEAN: byte offset of (window origin, channel scol), modulo 2^32
  unsigned tap_ok[kSlotsA];
#pragma unroll
  for (int i = 0; i < kSlotsA; ++i) {
    const int r = min(m0 + srow + 32 * i, M - 1);  // rows past M repeat the last one (never stored)
    const int ow = r % cv.OW;
    const int t = r / cv.OW;
    const int oh = t % cv.OH;
    const int n = t / cv.OH;
    const int ih0 = oh * cv.sh - cv.pt, iw0 = ow * cv.sw - cv.pl;
    origin[i] = (((long long)n * cv.H + ih0) * cv.W + iw0) * cv.Ci;
    origin_b[i] = 2u * ((unsigned)(int)origin[i] + (unsigned)scol);
    unsigned ok = 0, bit = 1u;
    for (int fy = 0; fy < cv.fh; ++fy)
      for (int fx = 0; fx < cv.fw; ++fx, bit <<= 1) {
        const int ih = ih0 + fy, iw = iw0 + fx;
        ok |= (ih >= 0 && ih < cv.H && iw >= 0 && iw < cv.W) ? bit : 0u;
      }
    tap_ok[i] = ok;
  }
  // this thread's k position in the slice being fetched: tap (kh, kw) and channel c (LEAN: the slice's first k,
  // uniform)
  int tap = LEAN ? 0 : scol / cv.Ci, c = LEAN ? 0 : scol % cv.Ci;
  int kh = tap / cv.fw, kw = tap % cv.fw;

  // B slots: k-rows 4 kq ... + 3 of the slice, columns n0 + 8 nb ... + 7 (threads with nb past the tile: none)
  const int kq = tid % 16, nb = tid / 16;
  const bool has_b = 8 * nb < kBN;
  const int bcol = n0 + 8 * nb < N ? n0 + 8 * nb : 0;  // past N: any valid column block (feeds no stored output)
  unsigned boff_b[kSlots];  // LEAN: byte offset of the slot at k0 = 0
#pragma unroll
  for (int j = 0; j < kSlots; ++j) boff_b[j] = 2u * ((unsigned)(4 * kq + j) * (unsigned)N + (unsigned)bcol);

  h8 ra[kSlotsA], rb[kSlots];
  unsigned a_ok = 0;  // bit i: A slot i of the fetched slice is inside the image and inside K
  const h8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
  auto load = [&](int k0) {
    if constexpr (LEAN) {
      const char* xb = reinterpret_cast<const char*>(cv.x);
      const unsigned tap_off_b = 2u * (unsigned)((kh * cv.W + kw) * cv.Ci + c);  // uniform
      a_ok = 0;
#pragma unroll
      for (int i = 0; i < kSlotsA; ++i) {
        const bool ok = ((tap_ok[i] >> tap) & 1u) != 0;
        const unsigned off = ok ? origin_b[i] + tap_off_b : 0u;  // inside the image: 0 <= offset < 2^32
        ra[i] = *reinterpret_cast<const h8*>(xb + off);
        a_ok |= ok ? 1u << i : 0u;
      }
      if (has_b) {
        const char* wb = reinterpret_cast<const char*>(w) + 2 * (size_t)k0 * (size_t)N;  // uniform
#pragma unroll
        for (int j = 0; j < kSlots; ++j) rb[j] = *reinterpret_cast<const h8*>(wb + boff_b[j]);
      }
      c += kBK;
      if (c >= cv.Ci) {
        c = 0;
        ++tap;
        if (++kw >= cv.fw) {
          kw = 0;
          ++kh;
        }
      }
      return;
    }
    const bool k_in = tap < cv.taps;  // k0 + scol < K
    const long long tap_off = ((long long)kh * cv.W + kw) * cv.Ci + c;
    a_ok = 0;
#pragma unroll
    for (int i = 0; i < kSlotsA; ++i) {
      const bool ok = k_in && ((tap_ok[i] >> tap) & 1u) != 0;
      const half_t* p = ok ? cv.x + (origin[i] + tap_off) : cv.x;  // unconditional load from a valid address
      ra[i] = *reinterpret_cast<const h8*>(p);
      a_ok |= ok ? 1u << i : 0u;
    }
    if (has_b) {
#pragma unroll
      for (int j = 0; j < kSlots; ++j) {
        const int k = k0 + 4 * kq + j;
        const half_t* p = w + (size_t)(k < K ? k : 0) * N + bcol;
        rb[j] = *reinterpret_cast<const h8*>(p);
        if (k >= K) rb[j] = zero8;
      }
    }
    // next slice: 64 channels further, carried into the tap index (Ci may be smaller than 64)
    c += kBK;
    for (int u = 0; u < wraps; ++u) {
      const bool carry = c >= cv.Ci;
      c -= carry ? cv.Ci : 0;
      tap += carry ? 1 : 0;
      kw += carry ? 1 : 0;
      const bool carry2 = kw >= cv.fw;
      kw -= carry2 ? cv.fw : 0;
      kh += carry2 ? 1 : 0;
    }
  };
  auto store = [&](int buf) {
    half_t* la = lds_a + buf * kTileA + srow * kLd + scol;
#pragma unroll
    for (int i = 0; i < kSlotsA; ++i)
      *reinterpret_cast<h8*>(la + 32 * i * kLd) = ((a_ok >> i) & 1u) ? ra[i] : zero8;
    if (has_b) {
      half_t* lb = lds_b + buf * kTileB + (8 * nb) * kLd + 4 * kq;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const h4 o = {rb[0][i], rb[1][i], rb[2][i], rb[3][i]};
        *reinterpret_cast<h4*>(lb + i * kLd) = o;
      }
    }
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

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
      // operands swapped (the filter's fragment first): a lane's registers then hold 4 consecutive output
      // columns of one row
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fb[s & 1][j], fa[s & 1][i], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) store(cur ^ 1);
    __syncthreads();
  }

  // acc[i][j][v] is the output at row m0 + wm0 + 32 i + li, column n0 + wn0 + 32 j + 8 (v / 4) + 4 hh + v % 4
  const ActClamp clamp = make_act(act);
  if (c_vec == 2) {
    // N % 8 == 0 and y 16-byte aligned: every wavefront converts its 32 TM x 32 TN block to binary16 in a private
    // LDS region (the slice buffers are free after the loop's last barrier), reads it back row-wise and
    // stores 16 bytes per lane, whole 128-byte lines per row
    constexpr int kWN = 32 * TN, kLs = kWN + 8;
    constexpr int kWM = 32 * TM;
    static_assert(4 * kWM * kLs <= 2 * (kTileA + kTileB), "staging fits in the slice buffers");
    half_t* stage = smem_h + wave * kWM * kLs;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int cl = 32 * j + 8 * g + 4 * hh;
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
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    constexpr int kLanesPerRow = kWN / 8, kRowsPerStep = 64 / kLanesPerRow;
    static_assert(kWM % kRowsPerStep == 0, "store steps cover the block");
    const int rr = lane / kLanesPerRow, cc = 8 * (lane % kLanesPerRow);
    const int col = n0 + wn0 + cc;
#pragma unroll
    for (int r0 = 0; r0 < kWM; r0 += kRowsPerStep) {
      const int row = m0 + wm0 + r0 + rr;
      const h8 v = *reinterpret_cast<const h8*>(stage + (r0 + rr) * kLs + cc);
      if (row < M && col < N) *reinterpret_cast<h8*>(y + (size_t)row * N + col) = v;
    }
    return;
  }
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int row = m0 + wm0 + 32 * i + li;
    if (row >= M) continue;
    half_t* yrow = y + (size_t)row * N;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int col = n0 + wn0 + 32 * j + 8 * g + 4 * hh;
        if (col >= N) continue;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (col + e >= N) continue;
          const float bv = bias != nullptr ? (float)bias[col + e] : 0.f;
          yrow[col + e] = (half_t)apply_act(acc[i][j][4 * g + e] + bv, clamp);
        }
      }
    }
  }
}

}  // namespace

bool conv2d_gemm_f16_supported(const void* x, const void* w, int ci, int fh, int fw, int co) {
  return ci % 8 == 0 && co % 8 == 0 && (long long)fh * fw <= 32 && reinterpret_cast<uintptr_t>(x) % 16 == 0 &&
         reinterpret_cast<uintptr_t>(w) % 16 == 0;
}

namespace {
template <int TM, int TN, bool LEAN>
int launch_tiles(const ConvGeomF16& cv, const half_t* w, const half_t* bias, half_t* y, long long m, int co, long long k,
                 int act, hipStream_t stream) {
  constexpr int kBM = 64 * TM, kBN = 64 * TN;
  constexpr size_t lds_bytes = 2 * (size_t)(kBM + kBN) * kLd * sizeof(half_t);
  const long long tiles_m = (m + kBM - 1) / kBM, tiles_n = (co + kBN - 1) / kBN;
  if (tiles_m * tiles_n > 0x7fffffffLL) return TFX_ERR_UNSUPPORTED;
  static std::atomic<uint64_t> lds_allowed{0};
  if (allow_dynamic_lds(reinterpret_cast<const void*>(conv_f16_gemm_kernel<TM, TN, LEAN>), lds_bytes, lds_allowed) != TFX_OK)
    return TFX_ERR_LAUNCH;
  const int wraps = (kBK + cv.Ci - 1) / cv.Ci;  // tap carries per 64-half step
  const int c_vec = reinterpret_cast<uintptr_t>(y) % 16 == 0 ? 2 : 0;
  const int total = (int)(tiles_m * tiles_n);
  hipLaunchKernelGGL((conv_f16_gemm_kernel<TM, TN, LEAN>), dim3((unsigned)total), dim3(kNT), lds_bytes, stream, cv, w, bias, y,
                     (int)m, co, (int)k, (int)tiles_n, total, wraps, act, c_vec);
  return check_launch();
}
}  // namespace

int launch_conv2d_gemm_f16(const uint16_t* x, const uint16_t* w, const uint16_t* bias, uint16_t* y, int n, int h, int wd,
                           int ci, int fh, int fw, int co, int oh, int ow, int sh, int sw, int pt, int pl, int act,
                           hipStream_t stream) {
  const long long m = (long long)n * oh * ow, k = (long long)fh * fw * ci;
  if (m > 0x7fffffffLL || k > 0x7fffffffLL) return TFX_ERR_UNSUPPORTED;
  const ConvGeomF16 cv{reinterpret_cast<const half_t*>(x), h, wd, ci, oh, ow, fh, fw, fh * fw, sh, sw, pt, pl};
  const half_t* wh = reinterpret_cast<const half_t*>(w);
  const half_t* bh = reinterpret_cast<const half_t*>(bias);
  half_t* yh = reinterpret_cast<half_t*>(y);
  // 64-column tiles when they cover the output channels with less padding than 128-column tiles.  64-row tiles
  // with those, and whenever 128-row tiles would leave CUs without a workgroup: more, smaller workgroups per CU
  // hide each other's memory latency (3x3, 56x56x64 -> 64 at batch 64: 70 -> 64 us; 28x28x256 -> 256 at batch 8:
  // 56 -> 47 us), at the price of less operand reuse (same layer at batch 64: 140 -> 205 us).
  const bool narrow = (co + 63) / 64 * 64 < (co + 127) / 128 * 128;
  const long long tiles128 = ((m + 127) / 128) * ((co + (narrow ? 63 : 127)) / (narrow ? 64 : 128));
  const bool low = narrow || tiles128 < 256;
  // scalar tap state and 32-bit offsets: 64-channel multiples, x and filter below 2^31 bytes
  const bool lean = ci % 64 == 0 && (long long)n * h * wd * ci < (1LL << 30) && k * co < (1LL << 30);
#define TFX_CONV16(TM, TN)                                                                   \
  (lean ? launch_tiles<TM, TN, true>(cv, wh, bh, yh, m, co, k, act, stream)                  \
        : launch_tiles<TM, TN, false>(cv, wh, bh, yh, m, co, k, act, stream))
  if (low) return narrow ? TFX_CONV16(1, 1) : TFX_CONV16(1, 2);
  return narrow ? TFX_CONV16(2, 1) : TFX_CONV16(2, 2);
#undef TFX_CONV16
}

}  // namespace tfx
