// MobileNet v1 tail for gfx950: global average pool, fully connected layer, softmax
// (the last three steps of the network timed in Section 3.9, Table 1).
// All three are bound by memory traffic (the 4 MB fully connected weight matrix dominates),
// so the fully connected layer is split over K across many workgroups and the partial
// sums are combined by the softmax kernel.
#include "tfx_internal.h"

namespace tfx {
namespace {

constexpr int kFcSlices = 32;   // K-slices of the fully connected layer
constexpr int kFcBatchMax = 8;  // images handled per weight read in the split-K kernel

// p[n,c] = (1/hw) * sum_i a[n,i,c]; one thread per (n,c), coalesced over c.
__global__ __launch_bounds__(256) void global_avg_pool_kernel(const float* __restrict__ a, float* __restrict__ p, int hw,
                                                              int c, int total) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const int n = idx / c, ch = idx % c;
  const float* ap = a + (size_t)n * hw * c + ch;
  float acc = 0.f;
  for (int i = 0; i < hw; ++i) acc += ap[(size_t)i * c];
  p[idx] = acc / (float)hw;
}

// partial[slice][n][j] = sum_{k in slice} pooled[n,k] * w[k,j].  grid = (column blocks, slices, image groups).
__global__ __launch_bounds__(256) void fc_partial_kernel(const float* __restrict__ pooled, const float* __restrict__ w,
                                                         float* __restrict__ partial, int n, int k, int classes,
                                                         int kslice) {
  const int j = blockIdx.x * 256 + threadIdx.x;
  const int slice = blockIdx.y;
  const int n0 = blockIdx.z * kFcBatchMax;
  const int nb = min(kFcBatchMax, n - n0);
  const int k0 = slice * kslice, k1 = min(k0 + kslice, k);
  __shared__ float ps[kFcBatchMax][64];
  // stage this slice of the pooled vectors (kslice <= 64)
  for (int i = threadIdx.x; i < kFcBatchMax * 64; i += 256) {
    const int b = i / 64, kk = i % 64;
    ps[b][kk] = (b < nb && k0 + kk < k1) ? pooled[(size_t)(n0 + b) * k + k0 + kk] : 0.f;
  }
  __syncthreads();
  if (j >= classes) return;
  float acc[kFcBatchMax];
#pragma unroll
  for (int b = 0; b < kFcBatchMax; ++b) acc[b] = 0.f;
  for (int kk = k0; kk < k1; ++kk) {
    const float wv = w[(size_t)kk * classes + j];
#pragma unroll
    for (int b = 0; b < kFcBatchMax; ++b) acc[b] = fmaf(ps[b][kk - k0], wv, acc[b]);
  }
  for (int b = 0; b < nb; ++b) partial[((size_t)slice * n + n0 + b) * classes + j] = acc[b];
}

__device__ __forceinline__ float block_reduce(float v, bool is_max, float* scratch) {
  // wave reduction by shuffles, then across the 4 waves through LDS
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
  for (int i = 1; i < 4; ++i) r = is_max ? fmaxf(r, scratch[i]) : r + scratch[i];
  return r;
}

// One workgroup per image: logits = bias + sum of partials (or the given logits), then
// probs = exp(l - max l) / sum exp(l - max l).
constexpr int kMaxPerThread = 8;  // classes <= 256 * 8
__global__ __launch_bounds__(256) void softmax_kernel(const float* __restrict__ partial, int slices,
                                                      const float* __restrict__ bias, float* __restrict__ logits,
                                                      float* __restrict__ probs, int n, int classes) {
  __shared__ float scratch[4];
  const int img = blockIdx.x;
  float l[kMaxPerThread];
  float mx = -INFINITY;
#pragma unroll
  for (int i = 0; i < kMaxPerThread; ++i) {
    const int j = threadIdx.x + 256 * i;
    l[i] = -INFINITY;
    if (j < classes) {
      float v;
      if (partial) {
        v = bias ? bias[j] : 0.f;
        for (int s = 0; s < slices; ++s) v += partial[((size_t)s * n + img) * classes + j];
        if (logits) logits[(size_t)img * classes + j] = v;
      } else {
        v = logits[(size_t)img * classes + j];
      }
      l[i] = v;
      mx = fmaxf(mx, v);
    }
  }
  mx = block_reduce(mx, true, scratch);
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < kMaxPerThread; ++i) {
    const int j = threadIdx.x + 256 * i;
    if (j < classes) {
      l[i] = __expf(l[i] - mx);
      sum += l[i];
    }
  }
  sum = block_reduce(sum, false, scratch);
  const float inv = 1.0f / sum;
#pragma unroll
  for (int i = 0; i < kMaxPerThread; ++i) {
    const int j = threadIdx.x + 256 * i;
    if (j < classes) probs[(size_t)img * classes + j] = l[i] * inv;
  }
}

}  // namespace

int launch_global_avg_pool(const float* a, float* p, int n, int hw, int c, hipStream_t stream) {
  const long long total = (long long)n * c;
  if (total > 0x7fffffffLL) return TFX_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(global_avg_pool_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, a, p, hw, c,
                     (int)total);
  return check_launch();
}

size_t fc_partial_floats(int n, int k, int classes) {
  (void)k;
  return (size_t)kFcSlices * n * classes;
}

int launch_fc_softmax(const float* pooled, const float* w, const float* bias, float* partial, float* logits,
                      float* probs, int n, int k, int classes, hipStream_t stream) {
  if (classes > 256 * kMaxPerThread) return TFX_ERR_UNSUPPORTED;
  const int kslice = (k + kFcSlices - 1) / kFcSlices;
  if (kslice > 64) return TFX_ERR_UNSUPPORTED;
  dim3 grid((classes + 255) / 256, kFcSlices, (n + kFcBatchMax - 1) / kFcBatchMax);
  hipLaunchKernelGGL(fc_partial_kernel, grid, dim3(256), 0, stream, pooled, w, partial, n, k, classes, kslice);
  int rc = check_launch();
  if (rc) return rc;
  hipLaunchKernelGGL(softmax_kernel, dim3(n), dim3(256), 0, stream, (const float*)partial, kFcSlices, bias, logits,
                     probs, n, classes);
  return check_launch();
}

}  // namespace tfx
