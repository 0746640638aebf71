// Element-wise addition for gfx950, C = A + B with one output value per thread-slot
// (the example program of Section 4.1, Fig. 3), in fp32 and in 16-bit float storage
// (the second precision of Section 4.1).  Pure streaming: three HBM streams, no reuse.
#include "tfx_internal.h"

namespace tfx {
namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));

constexpr int kThreads = 256;
constexpr int kVecPerThread = 4;  // 16-byte vectors per thread, all loads issued before the first add

// V: 16-byte vector type, E: element type.  Full workgroups use unconditional vector accesses;
// c may alias a or b (every slot is read before it is written, by the same thread).
// the elements past the last full workgroup (and everything, when a pointer is not 16-byte
// aligned) go through the scalar loop of the trailing workgroup(s).
template <typename V, typename E>
__global__ __launch_bounds__(kThreads) void add_kernel(const E* a, const E* b, E* c, long long n, long long full_blocks) {
  constexpr int kPerVec = sizeof(V) / sizeof(E);
  constexpr long long kPerBlock = (long long)kThreads * kVecPerThread * kPerVec;
  const long long blk = blockIdx.x;
  if (blk < full_blocks) {
    const long long base = blk * (kThreads * kVecPerThread) + threadIdx.x;
    const V* av = reinterpret_cast<const V*>(a);
    const V* bv = reinterpret_cast<const V*>(b);
    V* cv = reinterpret_cast<V*>(c);
    V x[kVecPerThread], y[kVecPerThread];
#pragma unroll
    for (int i = 0; i < kVecPerThread; ++i) x[i] = av[base + i * kThreads];
#pragma unroll
    for (int i = 0; i < kVecPerThread; ++i) y[i] = bv[base + i * kThreads];
#pragma unroll
    for (int i = 0; i < kVecPerThread; ++i) cv[base + i * kThreads] = x[i] + y[i];
    return;
  }
  const long long start = full_blocks * kPerBlock + (blk - full_blocks) * kPerBlock;
  const long long stop = start + kPerBlock < n ? start + kPerBlock : n;
  for (long long i = start + threadIdx.x; i < stop; i += kThreads) c[i] = a[i] + b[i];
}

template <typename V, typename E>
int launch_add_t(const E* a, const E* b, E* c, long long n, hipStream_t stream) {
  if (n == 0) return TFX_OK;
  constexpr long long kPerBlock = (long long)kThreads * kVecPerThread * (sizeof(V) / sizeof(E));
  const bool aligned = ((reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b) | reinterpret_cast<uintptr_t>(c)) & 15) == 0;
  const long long full = aligned ? n / kPerBlock : 0;
  const long long blocks = full + (n - full * kPerBlock + kPerBlock - 1) / kPerBlock;
  if (blocks > 0x7fffffffLL) return TFX_ERR_UNSUPPORTED;
  hipLaunchKernelGGL((add_kernel<V, E>), dim3((unsigned)blocks), dim3(kThreads), 0, stream, a, b, c, n, full);
  return check_launch();
}

}  // namespace

int launch_add_f32(const float* a, const float* b, float* c, long long n, hipStream_t stream) {
  return launch_add_t<v4f, float>(a, b, c, n, stream);
}

int launch_add_f16(const uint16_t* a, const uint16_t* b, uint16_t* c, long long n, hipStream_t stream) {
  return launch_add_t<v8h, _Float16>(reinterpret_cast<const _Float16*>(a), reinterpret_cast<const _Float16*>(b),
                                     reinterpret_cast<_Float16*>(c), n, stream);
}

}  // namespace tfx
