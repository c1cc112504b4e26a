// Sparsity and variance of the attention for Dynamic Pivot Layer Detection (paper Eq. 5-6), from the
// per-head in-degree vectors D_h (what structkv_score_layer_groups returns when every query head is its own
// group).  Reading of the paper's free row index: a head's attention is pooled over the window rows,
// a_h[j] = D_h[j] / w, a probability vector over the keys.
//   variance_h = (1/n) sum_j (a_h[j] - 1/n)^2          (the mean of a probability vector is 1/n)
//   sparsity_h = sum of a_h over the k keys selected by structkv_select_topk
// A head's keys are cut into up to kPivotMaxSlices slices, one workgroup each; all sums follow a fixed order,
// so results are bit-reproducible.
#include "common.h"

namespace skv {
namespace {

// sum over the workgroup in a fixed order (256 threads); result valid in thread 0
__device__ inline float block_sum(float v, float* sh /*[256]*/) {
  sh[threadIdx.x] = v;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if ((int)threadIdx.x < off) sh[threadIdx.x] += sh[threadIdx.x + off];
    __syncthreads();
  }
  return sh[0];
}

// grid (H, P): workgroup (h, p) takes the p-th slice of head h's keys and of its selected indices and writes
// two partial sums; heads [H][n], idx [H][k] (head-local key indices), part [H][P][2]
__global__ __launch_bounds__(256) void pivot_head_kernel(const float* __restrict__ heads, int64_t n,
                                                         const int32_t* __restrict__ idx, int64_t k, float inv_w,
                                                         float* __restrict__ part) {
  __shared__ float sh[256];
  const int h = blockIdx.x, p = blockIdx.y, P = gridDim.y;
  const float* d = heads + (int64_t)h * n;
  const float mean = 1.0f / (float)n;
  const int64_t per = (n + P - 1) / P, lo = (int64_t)p * per, hi = lo + per < n ? lo + per : n;
  float v = 0.f;
  for (int64_t j = lo + threadIdx.x; j < hi; j += 256) {
    const float a = d[j] * inv_w - mean;
    v = fmaf(a, a, v);
  }
  const float vs = block_sum(v, sh);
  __syncthreads();
  const int64_t kper = (k + P - 1) / P, klo = (int64_t)p * kper, khi = klo + kper < k ? klo + kper : k;
  float r = 0.f;
  const int32_t* ix = idx + (int64_t)h * k;
  for (int64_t i = klo + threadIdx.x; i < khi; i += 256) {
    int64_t j = ix[i];
    if (j < 0 || j >= n) j = 0;
    r += d[j];
  }
  const float rs = block_sum(r, sh);
  if (threadIdx.x == 0) {
    part[((int64_t)h * P + p) * 2 + 0] = vs;
    part[((int64_t)h * P + p) * 2 + 1] = rs;
  }
}

// per head: the partial sums in slice order; then the means over the heads, in head order (valid == 0: zeros)
__global__ __launch_bounds__(256) void pivot_finish_kernel(const float* __restrict__ part, int H, int P, int64_t n,
                                                           float inv_w, int valid, float* __restrict__ sparsity,
                                                           float* __restrict__ variance) {
  __shared__ float sv[256], sr[256];
  float rt = 0.f, vt = 0.f;
  if (valid) {
    for (int h0 = 0; h0 < H; h0 += 256) {   // heads in rounds of 256, each round summed in head order
      const int h = h0 + (int)threadIdx.x;
      float vs = 0.f, rs = 0.f;
      if (h < H)
        for (int p = 0; p < P; ++p) { vs += part[((int64_t)h * P + p) * 2]; rs += part[((int64_t)h * P + p) * 2 + 1]; }
      sv[threadIdx.x] = vs / (float)n;
      sr[threadIdx.x] = rs * inv_w;
      __syncthreads();
      if (threadIdx.x == 0)
        for (int i = 0; i < 256 && h0 + i < H; ++i) { vt += sv[i]; rt += sr[i]; }
      __syncthreads();
    }
  }
  if (threadIdx.x == 0) {
    *sparsity = rt / (float)H;
    *variance = vt / (float)H;
  }
}

__global__ void zero_floats_kernel(float* __restrict__ p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0.f;
}

}  // namespace

hipError_t launch_zero_floats(float* p, int n, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(zero_floats_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, n);
  return hipGetLastError();
}

int pivot_slices(int64_t n) {
  const int64_t p = (n + 8191) / 8192;
  return (int)(p < 1 ? 1 : (p > kPivotMaxSlices ? kPivotMaxSlices : p));
}

hipError_t launch_pivot_heads(const float* heads, int H, int64_t n, const int32_t* idx, int64_t k, float inv_w,
                              float* part, hipStream_t st) {
  if (H == 0 || n == 0) return hipSuccess;
  hipLaunchKernelGGL(pivot_head_kernel, dim3((unsigned)H, (unsigned)pivot_slices(n)), dim3(256), 0, st, heads, n,
                     idx, k, inv_w, part);
  return hipGetLastError();
}

hipError_t launch_pivot_finish(const float* part, int H, int64_t n, float inv_w, int valid, float* sparsity,
                               float* variance, hipStream_t st) {
  hipLaunchKernelGGL(pivot_finish_kernel, dim3(1), dim3(256), 0, st, part, H, pivot_slices(n), n, inv_w, valid,
                     sparsity, variance);
  return hipGetLastError();
}

}  // namespace skv
