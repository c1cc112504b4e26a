// Sparsity and variance of the attention for Dynamic Pivot Layer Detection (paper Eq. 5-6), from the
// per-head in-degree vectors D_h (what structkv_score_layer_groups returns when every query head is its own
// group).  Reading of the paper's free row index: a head's attention is pooled over the window rows,
// a_h[j] = D_h[j] / w, a probability vector over the keys.
//   variance_h = (1/n) sum_j (a_h[j] - 1/n)^2          (the mean of a probability vector is 1/n)
//   sparsity_h = sum of a_h over the k keys selected by structkv_select_topk
// Fixed reduction trees: results are bit-reproducible.
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

// one workgroup per head: heads [H][n], idx [H][k] (head-local key indices), out_rho / out_var [H]
__global__ __launch_bounds__(256) void pivot_head_kernel(const float* __restrict__ heads, int64_t n,
                                                         const int32_t* __restrict__ idx, int64_t k, float inv_w,
                                                         float* __restrict__ out_rho, float* __restrict__ out_var) {
  __shared__ float sh[256];
  const int h = blockIdx.x;
  const float* d = heads + (int64_t)h * n;
  const float mean = 1.0f / (float)n;
  float v = 0.f;
  for (int64_t j = threadIdx.x; j < n; j += 256) {
    const float a = d[j] * inv_w - mean;
    v = fmaf(a, a, v);
  }
  const float vs = block_sum(v, sh);
  __syncthreads();
  float r = 0.f;
  const int32_t* ix = idx + (int64_t)h * k;
  for (int64_t i = threadIdx.x; i < k; i += 256) {
    int64_t j = ix[i];
    if (j < 0 || j >= n) j = 0;
    r += d[j];
  }
  const float rs = block_sum(r, sh);
  if (threadIdx.x == 0) {
    out_var[h] = vs / (float)n;
    out_rho[h] = rs * inv_w;
  }
}

// means over the heads, in head order (n == 0: zeros)
__global__ void pivot_finish_kernel(const float* __restrict__ rho_h, const float* __restrict__ var_h, int H, int valid,
                                    float* __restrict__ sparsity, float* __restrict__ variance) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  float r = 0.f, v = 0.f;
  if (valid)
    for (int h = 0; h < H; ++h) { r += rho_h[h]; v += var_h[h]; }
  *sparsity = r / (float)H;
  *variance = v / (float)H;
}

}  // namespace

hipError_t launch_pivot_heads(const float* heads, int H, int64_t n, const int32_t* idx, int64_t k, float inv_w,
                              float* rho_h, float* var_h, hipStream_t st) {
  if (H == 0 || n == 0) return hipSuccess;
  hipLaunchKernelGGL(pivot_head_kernel, dim3((unsigned)H), dim3(256), 0, st, heads, n, idx, k, inv_w, rho_h, var_h);
  return hipGetLastError();
}

hipError_t launch_pivot_finish(const float* rho_h, const float* var_h, int H, int valid, float* sparsity,
                               float* variance, hipStream_t st) {
  hipLaunchKernelGGL(pivot_finish_kernel, dim3(1), dim3(64), 0, st, rho_h, var_h, H, valid, sparsity, variance);
  return hipGetLastError();
}

}  // namespace skv
