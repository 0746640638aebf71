// The small-map half of the batch-1 MobileNet v1 forward pass (Section 3.9, Table 1) as ONE kernel:
// the depthwise-separable blocks from the last 28 x 28 one (or the one after it) down to 7 x 7, the average pool, the fully
// connected layer and the softmax -- 20 dependent steps that, as 20 kernels of 3-6 us each, are
// bound by kernel boundaries and by each kernel's own start-up, not by their arithmetic.
//
// The kernel is persistent: 256 workgroups (one per CU) walk through the steps in order, and a step's
// work is cut into tasks that match the producers and consumers of the neighbouring steps:
//   depthwise task  = 16 consecutive output pixels x 32 channels (one output per thread),
//   pointwise task  = a 16-row x 16*TN-column tile of the pixel x channel GEMM, K split over the
//                     8 wavefronts, operands loaded straight into MFMA registers (the scheme of
//                     gemm_m16_direct_kernel), partial tiles added through LDS,
//   pool + fully connected task = 32 input channels x 128 classes, softmax = one task.
// There is no grid-wide barrier.  A task waits only for the tasks whose output it reads: every task
// has a flag word; the producer sets it after its stores have been acknowledged, the consumer polls the
// (at most a few dozen) flags it needs, one per lane.  Measured on the MI355X, a chain of such steps
// costs 1.6 us per step against 1.9 us for a kernel boundary in a graph and 2.5 us in a stream, and the
// per-kernel start-up (argument loads, address set-up, filter fetch) disappears: filters are fetched
// before the wait.
//
// Visibility between workgroups on different XCDs (each XCD has its own L2) without cache write-back /
// invalidate instructions: every activation that one task writes and another reads moves through
// device-coherent accesses (the sc1 cache policy of agent-scope atomics: stores write through to
// the memory side, loads do not hit a stale line), as do the flags.  A producer waits for its stores
// (vmcnt 0), the workgroup meets at a barrier, then one thread sets the flag; a consumer sees the flag,
// the workgroup meets at a barrier, then loads.  Filters and biases are read-only and use ordinary
// cached loads.  No location written inside the kernel is written twice (every step has its own
// output region), so a slow reader can never see a later value.
//
// Every wait is bounded: a poll loop gives up after kSpinLimit rounds (seconds), sets a failure word that makes
// every other wait give up too, and the softmax task then writes NaN to every output, so a workgroup that was
// never scheduled cannot hang the GPU and cannot yield plausible numbers.  The grid (256 workgroups, one per CU) is
// only launched where all of it is resident at once (chain_resident), and two such kernels never run side by side
// in one process: launch_chain orders them across streams (see there), because two half-resident grids would wait
// for workgroups that the other one keeps from being scheduled.
#include <cstdlib>
#include <mutex>

#include "tfx_internal.h"

namespace tfx {
namespace {

constexpr int kComputeThreads = 512;  // 8 wavefronts that compute
constexpr int kComputeWaves = kComputeThreads / 64;
constexpr int kChainThreads = kComputeThreads + 64;  // + one helper wavefront: polls flags, sets flags, warms L2
constexpr int kChainGrid = 256;
constexpr int kChainBlocks = 9;       // at most blocks 5 .. 13 of the network (0-based 4 .. 12)
constexpr int kFirstChainBlock = 4;   // a launch starts there or one block later (both read a 1/8-size map of 256 channels)
constexpr int kSpinLimit = 1 << 22;  // polls before a wait gives up (each poll is a memory round trip: seconds)
constexpr int kFcSliceChannels = 128;  // input channels of the fully connected layer per task (2 to 8 slices)
constexpr int kFcColBlock = 128;      // classes per fully connected task
constexpr int kFlagStride = 32;       // words between flags: one flag per 128-byte line.  Flags of neighbouring tasks
                                      // are set by different CUs at almost the same time; packed into one line their
                                      // write-throughs queue up behind each other (measured: 1.5 us until the last of
                                      // 16 is visible, against 0.6 us with a line each)
constexpr int kSc1 = 16;              // cache-policy operand of the buffer builtins: device-coherent access

typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

struct ChainBlock {
  const float *dw_w, *dw_b, *pw_w, *pw_b;
  int in_hw, out_hw, stride, pad;  // square maps; pad = zero rows / columns before the image
  int cin, cout;
  int tn;                          // 16-column blocks per pointwise tile
  int in_tn;                       // the same of the step that produced this block's input
  unsigned in_off, mid_off, out_off;  // float offsets in the chain workspace: input (0 for the first block, whose
                                   // input is a buffer of its own), depthwise output, pointwise output
  int flag_in, flag_mid, flag_out; // first flag of the tasks producing the input (-1: complete before launch),
                                   // the depthwise output, the pointwise output
};

struct ChainParams {
  ChainBlock blk[kChainBlocks];
  const float* in0;     // input of the first block (written by an earlier kernel)
  unsigned in0_bytes;
  float* act;           // chain workspace: every step's output
  unsigned act_bytes;
  int* flags;           // word 0: failure; task t's flag is word kFlagStride * t (t >= 1)
  const float *fc_w, *fc_b;
  unsigned partial_off; // float offset in act: [feat / 128][classes] partial logits
  float *probs, *logits;
  int classes, feat, last_hw;
  int flag_fc;          // first flag of the fully connected tasks
  int spin_limit;       // polls before a wait gives up
  int nblocks;          // blocks in blk[]
};

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, unsigned bytes) {
  // raw buffer (stride 0): an access at or past `bytes` returns 0 / is dropped by the hardware
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ float ld_f32(__amdgpu_buffer_rsrc_t r, unsigned byte_off) {
  return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, (int)byte_off, 0, kSc1));
}
__device__ __forceinline__ float4 ld_f32x4(__amdgpu_buffer_rsrc_t r, unsigned byte_off) {
  const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)byte_off, 0, kSc1);
  return make_float4(__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w));
}
__device__ __forceinline__ void st_f32(__amdgpu_buffer_rsrc_t r, unsigned byte_off, float v) {
  __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(v), r, (int)byte_off, 0, kSc1);
}
__device__ __forceinline__ void st_f32x2(__amdgpu_buffer_rsrc_t r, unsigned byte_off, float a, float b) {
  u32x2 v;
  v.x = __float_as_uint(a);
  v.y = __float_as_uint(b);
  __builtin_amdgcn_raw_buffer_store_b64(v, r, (int)byte_off, 0, kSc1);
}

__device__ __forceinline__ int flag_load(const int* f) {
  return __hip_atomic_load(f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void flag_store(int* f, int v) {
  __hip_atomic_store(f, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Wait until the producer tasks (rows r_lo..r_hi) x (columns c_lo..c_hi) of a step with `tiles_n` column tiles
// have set their flags.  Only the helper wavefront polls, one flag per lane: loads return in order within a
// wavefront, so a poll issued by a compute wavefront would wait behind that wavefront's filter loads.  Ends with a
// workgroup barrier.
__device__ __forceinline__ void wait_tiles(int* flags, int spin_limit, int first, int tiles_n, int r_lo, int r_hi,
                                           int c_lo, int c_hi) {
  if (threadIdx.x >= kComputeThreads) {
    const int nc = c_hi - c_lo + 1, n = (r_hi - r_lo + 1) * nc;
    for (int i = threadIdx.x - kComputeThreads; i < n; i += 64) {
      const int* f = flags + (size_t)(first + (r_lo + i / nc) * tiles_n + c_lo + i % nc) * kFlagStride;
      int spin = 0;
      while (flag_load(f) == 0) {
        if (++spin > spin_limit) {
          flag_store(flags, 1);
          break;
        }
        if ((spin & 255) == 0 && flag_load(flags) != 0) break;
        __builtin_amdgcn_s_sleep(1);
      }
    }
  }
  __syncthreads();
}

// After a task's stores: wait for their acknowledgement, meet, publish.
__device__ __forceinline__ void publish(int* flags, int index) {
  __builtin_amdgcn_s_waitcnt(0);  // vmcnt = expcnt = lgkmcnt = 0
  __syncthreads();
  if (threadIdx.x == kComputeThreads) flag_store(flags + (size_t)index * kFlagStride, 1);
}

// Tasks of a step with tiles_m x tiles_c tiles are dealt to workgroups so that a row tile's tasks fall on
// workgroups with the same id modulo 8, i.e. (workgroups are dealt to the 8 XCDs round robin) on one XCD -- or, with
// 1, 2 or 4 row tiles, on 8, 4 or 2 XCDs, so that no XCD stays idle: the exchange between a row tile's depthwise
// tasks and its pointwise tiles then stays inside an XCD's L2, which answers device-coherent accesses to lines it
// owns faster than the memory side does (measured: 1.3 against 1.8 us per dependent step).  Correctness does not
// depend on where workgroups run.  Workgroup w takes the virtual tasks vt = w, w + 256, ...; vt % 8 is the XCD.
struct TaskMap {
  int tiles_m, tiles_c, mode, f, count;
};
__device__ __forceinline__ TaskMap make_task_map(int tiles_m, int tiles_c) {
  TaskMap m;
  m.tiles_m = tiles_m;
  m.tiles_c = tiles_c;
  if (tiles_m >= 8) {
    m.mode = 0, m.f = 1, m.count = 8 * ((tiles_m + 7) / 8) * tiles_c;  // vt = r % 8 + 8 ((r / 8) tiles_c + c)
  } else if (tiles_m == 1 || tiles_m == 2 || tiles_m == 4) {
    m.mode = 1, m.f = 8 / tiles_m, m.count = 8 * ((tiles_c + m.f - 1) / m.f);  // XCD = r f + c % f, slot = c / f
  } else {
    m.mode = 2, m.f = 1, m.count = tiles_m * tiles_c;  // plain order
  }
  return m;
}
__device__ __forceinline__ bool task_of(const TaskMap& m, int vt, int* r, int* c) {
  if (m.mode == 0) {
    *r = vt % 8 + 8 * ((vt / 8) / m.tiles_c);
    *c = (vt / 8) % m.tiles_c;
  } else if (m.mode == 1) {
    *r = (vt % 8) / m.f;
    *c = (vt / 8) * m.f + (vt % 8) % m.f;
  } else {
    *r = vt / m.tiles_c;
    *c = vt % m.tiles_c;
  }
  return *r < m.tiles_m && *c < m.tiles_c;
}

// ---- depthwise 3x3 + bias + ReLU6: 16 output pixels x 32 channels, one output per compute thread ----
__device__ __forceinline__ void dw_task(const ChainParams& P, const ChainBlock& B, int r, int c,
                                        __amdgpu_buffer_rsrc_t in, __amdgpu_buffer_rsrc_t act) {
  const int tiles_c = B.cin / 32;
  const int m_out = B.out_hw * B.out_hw;
  const int t = threadIdx.x, px = (t / 32) % 16, ch = 32 * c + t % 32;
  const bool compute = t < kComputeThreads;
  // filter taps and bias first: they do not depend on anybody
  float w[9];
#pragma unroll
  for (int k = 0; k < 9; ++k) w[k] = compute ? B.dw_w[k * B.cin + ch] : 0.f;
  const float bias = compute ? B.dw_b[ch] : 0.f;

  if (B.flag_in >= 0) {
    // input rows under the 16 output pixels, as whole rows of the input map -> producer row tiles of 16 pixels
    const int p_lo = 16 * r, p_hi = min(16 * r + 15, m_out - 1);
    const int iy_lo = max((p_lo / B.out_hw) * B.stride - B.pad, 0);
    const int iy_hi = min((p_hi / B.out_hw) * B.stride - B.pad + 2, B.in_hw - 1);
    const int w16 = 16 * B.in_tn;  // channels per producer tile
    wait_tiles(P.flags, P.spin_limit, B.flag_in, B.cin / w16, iy_lo * B.in_hw / 16, (iy_hi * B.in_hw + B.in_hw - 1) / 16,
               32 * c / w16, (32 * c + 31) / w16);
  }
  if (compute) {
    const int p = 16 * r + px;
    const bool live = p < m_out;
    const int oy = p / B.out_hw, ox = p % B.out_hw;
    const int iy0 = oy * B.stride - B.pad, ix0 = ox * B.stride - B.pad;
    float v[9];
    bool ok[9];
#pragma unroll
    for (int kh = 0; kh < 3; ++kh)
#pragma unroll
      for (int kw = 0; kw < 3; ++kw) {
        const int iy = iy0 + kh, ix = ix0 + kw;
        ok[kh * 3 + kw] = live && iy >= 0 && iy < B.in_hw && ix >= 0 && ix < B.in_hw;
        // a tap outside the image reads past the end of the buffer: the hardware returns 0, no branch
        const unsigned off =
            ok[kh * 3 + kw] ? (B.in_off + (unsigned)((iy * B.in_hw + ix) * B.cin + ch)) * 4u : 0x80000000u;
        v[kh * 3 + kw] = ld_f32(in, off);
      }
    float acc = bias;
#pragma unroll
    for (int k = 0; k < 9; ++k) acc = ok[k] ? fmaf(v[k], w[k], acc) : acc;
    ActClamp clamp;
    clamp.on = true;
    clamp.hi = 6.0f;
    if (live) st_f32(act, (B.mid_off + (unsigned)(p * B.cin + ch)) * 4u, apply_act(acc, clamp));
  }
  publish(P.flags, B.flag_mid + r * tiles_c + c);
}

// ---- pointwise 1x1 + bias + ReLU6: 16 x (16 TN) tile, K = WAVES x CHUNK split over the first WAVES compute
// wavefronts (all 8 where K is a multiple of 128; 4 for the K = 64 and K = 192 of the narrower networks) ----
template <int CHUNK, int TN, int WAVES>
__device__ __forceinline__ void pw_task(const ChainParams& P, const ChainBlock& B, int tile_m, int tile_n,
                                        __amdgpu_buffer_rsrc_t act, float* red) {
  constexpr int G = CHUNK / 16;
  const int K = B.cin, N = B.cout, M = B.out_hw * B.out_hw;
  const int tiles_n = N / (16 * TN);
  const int tid = threadIdx.x, wk = (tid / 64) % kComputeWaves, lane = tid % 64, li = lane % 16, q = lane / 16;
  const bool compute = tid < 64 * WAVES;
  const int m0 = 16 * tile_m, n0 = 16 * TN * tile_n;

  // filter columns and bias before the wait (ordinary cached loads)
  const float* bp = B.pw_w + (size_t)(wk * CHUNK + 4 * q) * N + n0 + TN * li;
  float b[G][4][TN];
  if (compute) {
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const float* p = bp + (size_t)(16 * g + s) * N;
        if constexpr (TN == 2) {
          const float2 t2 = *reinterpret_cast<const float2*>(p);
          b[g][s][0] = t2.x;
          b[g][s][1] = t2.y;
        } else {
          b[g][s][0] = *p;
        }
      }
  }
  // epilogue thread e < 256 owns register v = e / 64 of lane l = e % 64: row 4 (l / 16) + v, columns TN (l % 16) ...
  const int ev = tid / 64, el = tid % 64;
  const int erow = m0 + 4 * (el / 16) + ev, ecol = n0 + TN * (el % 16);
  float ebias[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) ebias[j] = tid < 256 ? B.pw_b[ecol + j] : 0.f;

  // the depthwise tasks of this row tile, all channel groups
  wait_tiles(P.flags, P.spin_limit, B.flag_mid, K / 32, tile_m, tile_m, 0, K / 32 - 1);

  if (compute) {
    const int arow = min(m0 + li, M - 1);  // rows past M repeat the last one (they feed outputs that are not stored)
    const unsigned a_off = (B.mid_off + (unsigned)(arow * K + wk * CHUNK + 4 * q)) * 4u;
    float4 a[G];
#pragma unroll
    for (int g = 0; g < G; ++g) a[g] = ld_f32x4(act, a_off + 64u * g);

    floatx4 acc[2][TN];
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[c][j][v] = 0.f;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float av[4] = {a[g].x, a[g].y, a[g].z, a[g].w};
#pragma unroll
      for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[s & 1][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[s], b[g][s][j], acc[s & 1][j], 0, 0, 0);
    }
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) red[((wk * TN + j) * 4 + v) * 64 + lane] = acc[0][j][v] + acc[1][j][v];
  }
  __syncthreads();
  if (tid < 256 && erow < M) {
    ActClamp clamp;
    clamp.on = true;
    clamp.hi = 6.0f;
    float o[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      float sum = ebias[j];
#pragma unroll
      for (int w = 0; w < WAVES; ++w) sum += red[((w * TN + j) * 4 + ev) * 64 + el];
      o[j] = apply_act(sum, clamp);
    }
    const unsigned off = (B.out_off + (unsigned)(erow * N + ecol)) * 4u;
    if constexpr (TN == 2) st_f32x2(act, off, o[0], o[1]);
    else st_f32(act, off, o[0]);
  }
  publish(P.flags, B.flag_out + tile_m * tiles_n + tile_n);  // its barrier also protects `red` from the next task's writes
}

__device__ __forceinline__ float block_sum_or_max(float v, bool is_max, float* scratch) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const float o = __shfl_xor(v, off, 64);
    v = is_max ? fmaxf(v, o) : v + o;
  }
  __syncthreads();
  if (threadIdx.x % 64 == 0) scratch[threadIdx.x / 64] = v;
  __syncthreads();
  float r = scratch[0];
#pragma unroll
  for (int i = 1; i < kComputeWaves; ++i) r = is_max ? fmaxf(r, scratch[i]) : r + scratch[i];
  return r;
}

// The pointwise task for a layer of K input channels: the K split, and 32-column tiles only below K = 1024.
template <int K>
__device__ __forceinline__ void pw_task_for(const ChainParams& P, const ChainBlock& B, int r, int c,
                                            __amdgpu_buffer_rsrc_t act, float* red) {
  constexpr int WAVES = K % 128 == 0 ? 8 : 4, CHUNK = K / WAVES;
  static_assert(CHUNK % 16 == 0 && CHUNK <= 128, "a wavefront takes whole groups of 16 values of K");
  if constexpr (K < 1024) {
    if (B.tn == 2) return pw_task<CHUNK, 2, WAVES>(P, B, r, c, act, red);
  }
  pw_task<CHUNK, 1, WAVES>(P, B, r, c, act, red);
}

// Q = width multiplier in quarters: the chained blocks have 64 Q, 128 Q and 256 Q input channels, the fully
// connected layer 256 Q = 2 Q slices of 128.
template <int Q>
__global__ __launch_bounds__(kChainThreads) void mobilenet_chain_kernel(const ChainParams P) {
  constexpr int kSlices = 2 * Q;
  __shared__ float red[kComputeWaves * 2 * 4 * 64];  // 16 KB: split-K partial tiles; reused by the tail
  const int wg = blockIdx.x, tid = threadIdx.x;
  const bool compute = tid < kComputeThreads;
  {
    // The block descriptors are read at every block change, on the critical path, and the first touch of a line of
    // the kernel argument segment misses the scalar cache: touch every line now.
    typedef __attribute__((address_space(4))) const int* KernargInts;
    KernargInts karg = (KernargInts)__builtin_amdgcn_kernarg_segment_ptr();
    int warm = 0;
#pragma unroll
    for (int i = 0; i < (int)sizeof(ChainParams) / 4; i += 16) warm += karg[i];
    asm volatile("" ::"s"(warm));
  }
  const __amdgpu_buffer_rsrc_t in0 = make_rsrc(P.in0, P.in0_bytes);
  const __amdgpu_buffer_rsrc_t act = make_rsrc(P.act, P.act_bytes);

  // this workgroup's slice of the fully connected weights (128 input channels x 128 classes, 32 values per
  // compute thread), fetched now: nothing in the kernel depends on it for the next 50 us
  const int fc_tasks_c = (P.classes + kFcColBlock - 1) / kFcColBlock;
  const int fc_tasks = kSlices * fc_tasks_c;
  constexpr int kper = 128;  // input channels per task, 8 per thread
  float4 fw[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) fw[i] = make_float4(0.f, 0.f, 0.f, 0.f);
  const bool fvec = P.classes % 4 == 0;
  auto load_fc = [&](int task, float4 (&dst)[8]) {
    const int ks = task / fc_tasks_c, cb = task % fc_tasks_c;
    const int col = kFcColBlock * cb + 4 * (tid % 32), k0 = kper * ks + 8 * ((tid / 32) % 16);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float* p = P.fc_w + (size_t)(k0 + i) * P.classes + col;
      if (fvec && col + 3 < P.classes) {
        dst[i] = *reinterpret_cast<const float4*>(p);
      } else {
        dst[i].x = col < P.classes ? p[0] : 0.f;
        dst[i].y = col + 1 < P.classes ? p[1] : 0.f;
        dst[i].z = col + 2 < P.classes ? p[2] : 0.f;
        dst[i].w = col + 3 < P.classes ? p[3] : 0.f;
      }
    }
  };
  if (wg < fc_tasks && compute) load_fc(wg, fw);
  for (int bi = 0; bi < P.nblocks; ++bi) {
    const ChainBlock& B = P.blk[bi];
    const int tiles_m = (B.out_hw * B.out_hw + 15) / 16;
    const TaskMap dw_map = make_task_map(tiles_m, B.cin / 32), pw_map = make_task_map(tiles_m, B.cout / (16 * B.tn));
    for (int vt = wg; vt < dw_map.count; vt += kChainGrid) {
      int r, c;
      if (task_of(dw_map, vt, &r, &c)) dw_task(P, B, r, c, bi == 0 ? in0 : act, act);
    }
    for (int vt = wg; vt < pw_map.count; vt += kChainGrid) {
      int r, c;
      if (!task_of(pw_map, vt, &r, &c)) continue;
      if (B.cin == 64 * Q) pw_task_for<64 * Q>(P, B, r, c, act, red);
      else if (B.cin == 128 * Q) pw_task_for<128 * Q>(P, B, r, c, act, red);
      else pw_task_for<256 * Q>(P, B, r, c, act, red);
    }
  }

  // ---- average pool + fully connected: task (ks, cb) = 128 input channels x 128 classes ----
  const ChainBlock& L = P.blk[P.nblocks - 1];
  const int hw2 = P.last_hw * P.last_hw;
  for (int task = wg; task < fc_tasks; task += kChainGrid) {
    const int ks = task / fc_tasks_c, cb = task % fc_tasks_c;
    if (task != wg && compute) load_fc(task, fw);
    // the last pointwise layer's tiles holding channels kper ks .. kper ks + kper - 1, every pixel row tile
    const int w16 = 16 * L.tn;
    wait_tiles(P.flags, P.spin_limit, L.flag_out, L.cout / w16, 0, (hw2 + 15) / 16 - 1, kper * ks / w16,
               (kper * ks + kper - 1) / w16);
    float* pooled = red;             // [128]
    float* psum = red + 128;         // [4][128]
    float* fsum = red + 128 + 512;   // [16][128]
    if (compute) {
      // thread (pixel group pg of 4, channel chn of 128) sums pixels pg, pg + 4, ... (at most 64 pixels)
      const int chn = tid % 128, pg = tid / 128;
      float x[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int p = pg + 4 * i;
        x[i] = ld_f32(act, p < hw2 ? (L.out_off + (unsigned)(p * P.feat + kper * ks + chn)) * 4u : 0x80000000u);
      }
      float s = 0.f;
#pragma unroll
      for (int i = 0; i < 16; ++i) s += x[i];
      psum[pg * 128 + chn] = s;
    }
    __syncthreads();
    if (tid < 128) pooled[tid] = (psum[tid] + psum[128 + tid] + psum[256 + tid] + psum[384 + tid]) / (float)hw2;
    __syncthreads();
    if (compute) {
      const int kq = tid / 32, c4 = tid % 32;
      float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float pv = pooled[8 * kq + i];
        s.x = fmaf(pv, fw[i].x, s.x);
        s.y = fmaf(pv, fw[i].y, s.y);
        s.z = fmaf(pv, fw[i].z, s.z);
        s.w = fmaf(pv, fw[i].w, s.w);
      }
      *reinterpret_cast<float4*>(fsum + kq * 128 + 4 * c4) = s;
    }
    __syncthreads();
    if (tid < kFcColBlock) {
      float s = 0.f;
#pragma unroll
      for (int g = 0; g < 16; ++g) s += fsum[g * 128 + tid];
      const int col = kFcColBlock * cb + tid;
      if (col < P.classes) st_f32(act, (P.partial_off + (unsigned)(ks * P.classes + col)) * 4u, s);
    }
    publish(P.flags, P.flag_fc + task);
  }

  // ---- bias + softmax: one task, two classes per compute thread ----
  if (wg == 0) {
    wait_tiles(P.flags, P.spin_limit, P.flag_fc, fc_tasks_c, 0, kSlices - 1, 0, fc_tasks_c - 1);
    float l[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int j = tid + kComputeThreads * h;
      const bool in = compute && j < P.classes;
      float part[kSlices];
#pragma unroll
      for (int s = 0; s < kSlices; ++s)
        part[s] = ld_f32(act, in ? (P.partial_off + (unsigned)(s * P.classes + j)) * 4u : 0x80000000u);
      float v = in ? P.fc_b[j] : 0.f;
#pragma unroll
      for (int s = 0; s < kSlices; ++s) v += part[s];
      l[h] = in ? v : -INFINITY;
    }
    const bool failed = flag_load(P.flags) != 0;
    const float mx = block_sum_or_max(fmaxf(l[0], l[1]), true, red);
    float e[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) e[h] = (compute && tid + kComputeThreads * h < P.classes) ? __expf(l[h] - mx) : 0.f;
    const float sum = block_sum_or_max(e[0] + e[1], false, red + 16);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int j = tid + kComputeThreads * h;
      if (compute && j < P.classes) {
        const float nan = __uint_as_float(0x7fc00000u);
        if (P.logits) P.logits[j] = failed ? nan : l[h];
        P.probs[j] = failed ? nan : e[h] / sum;
      }
    }
  }
}

struct ChainPlanHost {
  int flags;            // number of flag words
  size_t act_floats;    // chain workspace in floats
};

}  // namespace

bool chain_supported(int image_size, int width_quarters, int classes, long long batch) {
  // the 1/8-size map of 64 q channels is what the first chained block reads; channel counts 64 q / 128 q / 256 q
  return batch == 1 && width_quarters >= 1 && width_quarters <= 4 && image_size >= 32 && image_size <= 256 &&
         classes >= 1 && classes <= 1024;
}

namespace {
typedef void (*ChainKernel)(const ChainParams);
ChainKernel chain_kernel(int width_quarters) {
  switch (width_quarters) {
    case 1: return mobilenet_chain_kernel<1>;
    case 2: return mobilenet_chain_kernel<2>;
    case 3: return mobilenet_chain_kernel<3>;
    default: return mobilenet_chain_kernel<4>;
  }
}
}  // namespace

// Whether 256 workgroups of the chain kernel are resident at once on the current device (looked up once per device).
bool chain_resident(int width_quarters) {
  static std::atomic<int> states[4][64];  // 0 unknown, 1 yes, 2 no
  int dev = 0;
  if (width_quarters < 1 || width_quarters > 4 || hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return false;
  std::atomic<int>* const state = states[width_quarters - 1];
  const int s = state[dev].load(std::memory_order_acquire);
  if (s) return s == 1;
  int cus = 0, per_cu = 0;
  bool ok = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess &&
            hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, chain_kernel(width_quarters), kChainThreads, 0) == hipSuccess;
  ok = ok && (long long)cus * per_cu >= kChainGrid;
  state[dev].store(ok ? 1 : 2, std::memory_order_release);
  return ok;
}

namespace {
constexpr int kNetChannels[13] = {64, 128, 128, 256, 256, 512, 512, 512, 512, 512, 512, 1024, 1024};
constexpr int kNetStrides[13] = {1, 2, 1, 2, 1, 2, 1, 1, 1, 1, 1, 2, 1};

// Sizes of the chained part for an input map of in_hw x in_hw x 64 q (the output of block 4) at width q / 4.
ChainPlanHost chain_layout(int in_hw, int classes, int q, ChainParams* P, int first = kFirstChainBlock) {
  ChainPlanHost h{};
  int flags = 1;  // [0] = failure word
  size_t off = 0;
  const int nblocks = 13 - first;
  int hw = in_hw, cin = kNetChannels[first - 1] * q / 4, prev_flags = -1, prev_tn = 2;
  size_t prev_out = 0;
  for (int bi = 0; bi < nblocks; ++bi) {
    const int net = first + bi, s = kNetStrides[net], cout = kNetChannels[net] * q / 4;
    const int out_hw = (hw + s - 1) / s;
    const int need = (out_hw - 1) * s + 3 - hw;
    const int pad = need > 0 ? need / 2 : 0;
    const int m = out_hw * out_hw, tiles_m = (m + 15) / 16;
    // 16-column tiles when 32-column ones would leave CUs idle (always for K = 1024: 32 values of K per lane)
    const int tn = (tiles_m * (cout / 32) >= 160 && cin < 1024) ? 2 : 1;
    if (P) {
      ChainBlock& B = P->blk[bi];
      B.in_hw = hw, B.out_hw = out_hw, B.stride = s, B.pad = pad, B.cin = cin, B.cout = cout, B.tn = tn, B.in_tn = prev_tn;
      B.flag_in = prev_flags;
      B.flag_mid = flags;
      B.flag_out = flags + tiles_m * (cin / 32);
      B.in_off = (unsigned)prev_out;
      B.mid_off = (unsigned)off;
      B.out_off = (unsigned)(off + (size_t)m * cin);
    }
    prev_out = off + (size_t)m * cin;
    prev_flags = flags + tiles_m * (cin / 32);
    flags = prev_flags + tiles_m * (cout / (16 * tn));
    off += (size_t)m * cin + (size_t)m * cout;
    hw = out_hw, cin = cout, prev_tn = tn;
  }
  const int slices = cin / kFcSliceChannels;
  const int fc_tasks = slices * ((classes + kFcColBlock - 1) / kFcColBlock);
  if (P) {
    P->flag_fc = flags;
    P->partial_off = (unsigned)off;
    P->last_hw = hw;
    P->feat = cin;
    P->classes = classes;
    P->nblocks = nblocks;
  }
  flags += fc_tasks;
  off += (size_t)slices * classes;
  h.flags = flags;
  h.act_floats = off;
  return h;
}
}  // namespace

size_t chain_workspace_bytes(int image_size, int classes, int width_quarters) {
  const int half = (image_size + 1) / 2, quarter = (half + 1) / 2, eighth = (quarter + 1) / 2;
  const ChainPlanHost h = chain_layout(eighth, classes, width_quarters, nullptr);
  const size_t flag_bytes = (size_t)(h.flags + block_chain_flag_words(half, half)) * kFlagStride * sizeof(int);
  return flag_bytes + (h.act_floats * sizeof(float) + 255) / 256 * 256;
}

// The flags at the start of the chain workspace: `count` words, chain_flag_stride() words apart, that must be zero
// when the first kernel that uses them starts: the chain kernel's own (word 0 = failure word), then, from
// chain_head_flag_base() on, those of the launch that runs blocks 2 - 4 as stages (block.hip).
int chain_flag_words(int image_size, int classes, int width_quarters) {
  const int half = (image_size + 1) / 2, quarter = (half + 1) / 2, eighth = (quarter + 1) / 2;
  return chain_layout(eighth, classes, width_quarters, nullptr).flags + block_chain_flag_words(half, half);
}
int chain_head_flag_base(int image_size, int classes) {
  const int half = (image_size + 1) / 2, quarter = (half + 1) / 2, eighth = (quarter + 1) / 2;
  return chain_layout(eighth, classes, 4, nullptr).flags;
}
int chain_spin_limit() {
  // Test hook: TFX_CHAIN_SPIN_LIMIT=<n> makes every wait give up after n polls, which exercises the failure
  // path (all outputs NaN, the kernels still run to their end) without any workgroup actually missing.
  if (const char* e = getenv("TFX_CHAIN_SPIN_LIMIT")) {
    const long v = strtol(e, nullptr, 10);
    if (v >= 1 && v <= kSpinLimit) return (int)v;
  }
  return kSpinLimit;
}
int chain_flag_stride() { return kFlagStride; }

namespace {
// Chain kernels of one process are kept from overlapping on a device.  The last stream that launched one is
// remembered per device; a launch on another stream first records an event behind everything queued on that
// stream and makes the new stream wait for it.  Launches that stay on one stream (the usual case) pay nothing.
// A stream that is being captured into a graph is left alone (an event of another stream cannot be recorded into
// the capture): replays of such graphs on several streams at once are the caller's to order.
struct ChainOrder {
  std::mutex lock;
  hipStream_t last[64];
  hipEvent_t event[64];
  bool launched[64], have_event[64];
};
ChainOrder g_order;

void order_after_other_streams(int dev, hipStream_t stream) {
  hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(stream, &capturing) != hipSuccess || capturing != hipStreamCaptureStatusNone) {
    (void)hipGetLastError();
    return;
  }
  if (g_order.launched[dev] && g_order.last[dev] != stream) {
    if (!g_order.have_event[dev])
      g_order.have_event[dev] = hipEventCreateWithFlags(&g_order.event[dev], hipEventDisableTiming) == hipSuccess;
    // a stream that has been destroyed since is refused by the runtime: nothing of it can still be running
    if (g_order.have_event[dev] && hipEventRecord(g_order.event[dev], g_order.last[dev]) == hipSuccess)
      (void)hipStreamWaitEvent(stream, g_order.event[dev], 0);
    (void)hipGetLastError();
  }
  g_order.last[dev] = stream;
  g_order.launched[dev] = true;
}
}  // namespace

// Runs fn(arg) -- which enqueues a kernel whose workgroups wait for each other -- once `stream` has been ordered behind
// the last such kernel of any other stream.
int launch_ordered(hipStream_t stream, int (*fn)(void*), void* arg) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return TFX_ERR_LAUNCH;
  std::lock_guard<std::mutex> guard(g_order.lock);
  order_after_other_streams(dev, stream);
  return fn(arg);
}

int launch_chain(const float* in0, int in_hw, const tfx_mobilenet_v1_weights* w, void* chain_ws, int head_flags,
                 float* probs, float* logits, int classes, int width_quarters, hipStream_t stream, int (*before)(void*),
                 void* before_arg, int first_block) {
  if (first_block != kFirstChainBlock && first_block != kFirstChainBlock + 1) return TFX_ERR_ARG;
  if (width_quarters < 1 || width_quarters > 4) return TFX_ERR_ARG;
  ChainParams P{};
  // the workspace is laid out for the longer chain; a launch that starts one block later uses a part of it
  const ChainPlanHost h = chain_layout(in_hw, classes, width_quarters, nullptr);
  const ChainPlanHost used = chain_layout(in_hw, classes, width_quarters, &P, first_block);
  if (used.flags > h.flags || used.act_floats > h.act_floats) return TFX_ERR_LAUNCH;
  for (int bi = 0; bi < P.nblocks; ++bi) {
    const int net = first_block + bi;
    P.blk[bi].dw_w = w->dw_w[net];
    P.blk[bi].dw_b = w->dw_b[net];
    P.blk[bi].pw_w = w->pw_w[net];
    P.blk[bi].pw_b = w->pw_b[net];
  }
  const size_t flag_bytes = (size_t)(h.flags + head_flags) * kFlagStride * sizeof(int);
  P.in0 = in0;
  P.in0_bytes = (unsigned)((size_t)in_hw * in_hw * (kNetChannels[first_block - 1] * width_quarters / 4) * sizeof(float));
  P.flags = static_cast<int*>(chain_ws);
  P.act = reinterpret_cast<float*>(static_cast<char*>(chain_ws) + flag_bytes);
  P.act_bytes = (unsigned)(h.act_floats * sizeof(float));
  P.fc_w = w->fc_w;
  P.fc_b = w->fc_b;
  P.probs = probs;
  P.logits = logits;
  P.spin_limit = chain_spin_limit();
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return TFX_ERR_LAUNCH;
  std::lock_guard<std::mutex> guard(g_order.lock);
  order_after_other_streams(dev, stream);
  // a launch of waiting workgroups that belongs in front of this one (blocks 2 - 4 as stages, block.hip) is enqueued
  // under the same lock, so that the pair is ordered against other streams' pairs as one
  if (before != nullptr) {
    const int rc = before(before_arg);
    if (rc != TFX_OK) return rc;
  }
  hipLaunchKernelGGL(chain_kernel(width_quarters), dim3(kChainGrid), dim3(kChainThreads), 0, stream, P);
  return check_launch();
}

}  // namespace tfx
