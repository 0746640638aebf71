// MobileNet v1 tail for gfx950: global average pool, fully connected layer, softmax
// (the last three steps of the network timed in Section 3.9, Table 1).
// All three are bound by memory latency and traffic (the 4 MB fully connected weight matrix
// dominates), so the pool is fused into the fully connected kernel, that kernel is split over
// K across many workgroups with all of a thread's loads in flight at once, and the partial
// sums are combined by the softmax kernel.
#include "tfx_internal.h"

namespace tfx {
namespace {

constexpr int kFcSlices = 32;   // K-slices of the fully connected layer
constexpr int kFcKMax = 32;     // K elements per slice (so K <= 1024)
constexpr int kFcBatchMax = 4;  // images handled per weight read

// partial[slice][n][j] = sum_{k in slice} mean_p(a[n,p,k]) * w[k,j].
// grid = (column blocks, slices, image groups); a is the last feature map [n, hw, k].
__global__ __launch_bounds__(256) void pool_fc_partial_kernel(const float* __restrict__ a, const float* __restrict__ w,
                                                              float* __restrict__ partial, int n, int hw, int k,
                                                              int classes, int kslice) {
  const int j = blockIdx.x * 256 + threadIdx.x;
  const int slice = blockIdx.y;
  const int n0 = blockIdx.z * kFcBatchMax;
  const int nb = min(kFcBatchMax, n - n0);
  const int k0 = slice * kslice;
  const int kn = min(kslice, k - k0);
  __shared__ float ps[kFcBatchMax][kFcKMax];

  // this thread's weight column slice first, so the loads overlap the pooling below
  float wv[kFcKMax];
#pragma unroll
  for (int kk = 0; kk < kFcKMax; ++kk) wv[kk] = (kk < kn && j < classes) ? w[(size_t)(k0 + kk) * classes + j] : 0.f;

  // global average pool of this K-slice: thread t sums pixels t/32, t/32 + 8, ... of channel t % 32.
  // The loads are unconditional from clamped addresses so that all of them are in flight at once.
  {
    constexpr int kPixPerLane = 8;  // hw <= 64
    const int kk = threadIdx.x % kFcKMax, p0 = threadIdx.x / kFcKMax;  // 8 pixel lanes
    __shared__ float red[kFcBatchMax][8][kFcKMax];
    const int kc = kk < kn ? kk : 0;
#pragma unroll
    for (int b = 0; b < kFcBatchMax; ++b) {
      const int bc = b < nb ? b : 0;
      const float* ap = a + ((size_t)(n0 + bc) * hw) * k + k0 + kc;
      float v[kPixPerLane];
#pragma unroll
      for (int q = 0; q < kPixPerLane; ++q) {
        const int p = p0 + 8 * q;
        v[q] = ap[(size_t)(p < hw ? p : hw - 1) * k];
      }
      float acc = 0.f;
#pragma unroll
      for (int q = 0; q < kPixPerLane; ++q) acc += (p0 + 8 * q < hw) ? v[q] : 0.f;
      red[b][p0][kk] = (b < nb && kk < kn) ? acc : 0.f;
    }
    __syncthreads();
    if (threadIdx.x < kFcBatchMax * kFcKMax) {
      const int b = threadIdx.x / kFcKMax, c = threadIdx.x % kFcKMax;
      float s = 0.f;
#pragma unroll
      for (int q = 0; q < 8; ++q) s += red[b][q][c];
      ps[b][c] = s / (float)hw;
    }
    __syncthreads();
  }
  if (j >= classes) return;
  float acc[kFcBatchMax];
#pragma unroll
  for (int b = 0; b < kFcBatchMax; ++b) acc[b] = 0.f;
#pragma unroll
  for (int kk = 0; kk < kFcKMax; ++kk) {
#pragma unroll
    for (int b = 0; b < kFcBatchMax; ++b) acc[b] = fmaf(ps[b][kk], wv[kk], acc[b]);
  }
  for (int b = 0; b < nb; ++b) partial[((size_t)slice * n + n0 + b) * classes + j] = acc[b];
}

__device__ __forceinline__ float block_reduce(float v, bool is_max, float* scratch) {
  // wave reduction by shuffles, then across the workgroup's waves through LDS
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const float o = __shfl_xor(v, off, 64);
    v = is_max ? fmaxf(v, o) : v + o;
  }
  const int wave = threadIdx.x / 64;
  __syncthreads();
  if (threadIdx.x % 64 == 0) scratch[wave] = v;
  __syncthreads();
  float r = scratch[0];
  for (int i = 1; i < (int)blockDim.x / 64; ++i) r = is_max ? fmaxf(r, scratch[i]) : r + scratch[i];
  return r;
}

// One workgroup per image, one thread per class (all of a thread's 32 partial sums in flight at once):
// logits = bias + sum of the K-slice partials, then probs = exp(l - max l) / sum exp(l - max l).
constexpr int kSoftmaxThreads = 1024;  // classes <= 1024
__global__ __launch_bounds__(kSoftmaxThreads) void softmax_kernel(const float* __restrict__ partial,
                                                                  const float* __restrict__ bias,
                                                                  float* __restrict__ logits, float* __restrict__ probs,
                                                                  int n, int classes) {
  __shared__ float scratch[kSoftmaxThreads / 64];
  const int img = blockIdx.x;
  const int j = threadIdx.x;
  float l = -INFINITY;
  if (j < classes) {
    float part[kFcSlices];
#pragma unroll
    for (int s = 0; s < kFcSlices; ++s) part[s] = partial[((size_t)s * n + img) * classes + j];
    float v = bias ? bias[j] : 0.f;
#pragma unroll
    for (int s = 0; s < kFcSlices; ++s) v += part[s];
    if (logits) logits[(size_t)img * classes + j] = v;
    l = v;
  }
  const float mx = block_reduce(l, true, scratch);
  const float e = j < classes ? __expf(l - mx) : 0.f;
  const float sum = block_reduce(e, false, scratch);
  if (j < classes) probs[(size_t)img * classes + j] = e / sum;
}

}  // namespace

size_t fc_partial_floats(int n, int k, int classes) {
  (void)k;
  return (size_t)kFcSlices * n * classes;
}

int launch_pool_fc_softmax(const float* a, const float* w, const float* bias, float* partial, float* logits,
                           float* probs, int n, int hw, int k, int classes, hipStream_t stream) {
  if (classes > kSoftmaxThreads) return TFX_ERR_UNSUPPORTED;
  const int kslice = (k + kFcSlices - 1) / kFcSlices;
  if (kslice > kFcKMax || hw > 64) return TFX_ERR_UNSUPPORTED;
  dim3 grid((classes + 255) / 256, kFcSlices, (n + kFcBatchMax - 1) / kFcBatchMax);
  hipLaunchKernelGGL(pool_fc_partial_kernel, grid, dim3(256), 0, stream, a, w, partial, n, hw, k, classes, kslice);
  int rc = check_launch();
  if (rc) return rc;
  hipLaunchKernelGGL(softmax_kernel, dim3(n), dim3(kSoftmaxThreads), 0, stream, (const float*)partial, bias, logits, probs, n,
                     classes);
  return check_launch();
}

}  // namespace tfx
