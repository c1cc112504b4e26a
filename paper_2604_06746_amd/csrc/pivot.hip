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

// First pass over the per-head in-degrees that a scoring call leaves in its column-sum planes (pass 2 with one
// plane per query head): the first radix digit of their selection and the variance partials.
//   hist[h][digit of heads[h][j]] += 1;   part[h P + p] = sum over the workgroup's keys of (heads/w - 1/n)^2
// grid (P, H): workgroup (p, h) takes keys [p*kPlaneShare, ...) of head h.
constexpr int kPlaneShare = 2048;

__global__ __launch_bounds__(256) void pivot_planes_kernel(const float* __restrict__ heads, int64_t n, float inv_w,
                                                           uint32_t* __restrict__ hist, float* __restrict__ part) {
  short_kernel_priority();
  __shared__ uint32_t h0[kTopkBins];
  __shared__ float sh[256];
  const int p = blockIdx.x, h = blockIdx.y, P = gridDim.x;
  const float* d = heads + (int64_t)h * n;
  const int64_t lo = (int64_t)p * kPlaneShare;
  float x[kPlaneShare / 256];
#pragma unroll
  for (int i = 0; i < kPlaneShare / 256; ++i) {   // loads first, the histogram's clearing under them
    const int64_t j = lo + threadIdx.x + i * 256;
    x[i] = j < n ? d[j] : 0.f;
  }
  for (int i = threadIdx.x; i < kTopkBins; i += 256) h0[i] = 0u;
  __syncthreads();
  const float mean = 1.0f / (float)n;
  float v = 0.f;
#pragma unroll
  for (int i = 0; i < kPlaneShare / 256; ++i) {
    if (lo + threadIdx.x + i * 256 < n) {
      atomicAdd(&h0[score_key(x[i]) >> 21], 1u);
      const float a = x[i] * inv_w - mean;
      v = fmaf(a, a, v);
    }
  }
  const float vs = block_sum(v, sh);   // its barriers also complete the LDS histogram
  uint32_t* gh = hist + (size_t)h * 3 * kTopkBins;
  for (int i = threadIdx.x; i < kTopkBins; i += 256)
    if (h0[i]) atomicAdd(&gh[i], h0[i]);
  if (threadIdx.x == 0) part[(int64_t)h * P + p] = vs;
}

// the means from the partials of the planes path: variance partials var_part [H][Pv] (pivot_planes_kernel),
// mass partials mass_part [H][Pm][2] (second of each pair; topk_mass_kernel) and, per head, tail[2h] selected keys
// that tie with the k-th largest, of value tail[2h+1].  Eight lanes share a head: each adds every eighth
// partial, then a fixed shuffle tree; the heads are added in order by one thread.
__global__ __launch_bounds__(256) void pivot_finish_planes_kernel(const float* __restrict__ var_part, int Pv,
                                                                  const float* __restrict__ mass_part, int Pm,
                                                                  const float* __restrict__ tail, int H, int64_t n,
                                                                  float inv_w, float* __restrict__ sparsity,
                                                                  float* __restrict__ variance) {
  __shared__ float sv[32], sr[32];
  float rt = 0.f, vt = 0.f;
  const int sub = threadIdx.x & 7;
  for (int h0 = 0; h0 < H; h0 += 32) {   // heads in rounds of 32
    const int h = h0 + (int)(threadIdx.x >> 3);
    float vs = 0.f, rs = 0.f;
    if (h < H) {
      for (int p = sub; p < Pv; p += 8) vs += var_part[(int64_t)h * Pv + p];
      for (int p = sub; p < Pm; p += 8) rs += mass_part[((int64_t)h * Pm + p) * 2 + 1];
    }
    vs += __shfl_xor(vs, 1); vs += __shfl_xor(vs, 2); vs += __shfl_xor(vs, 4);
    rs += __shfl_xor(rs, 1); rs += __shfl_xor(rs, 2); rs += __shfl_xor(rs, 4);
    if (sub == 0) {
      if (h < H) rs = fmaf(tail[2 * h], tail[2 * h + 1], rs);
      sv[threadIdx.x >> 3] = vs / (float)n;
      sr[threadIdx.x >> 3] = rs * inv_w;
    }
    __syncthreads();
    if (threadIdx.x == 0)
      for (int i = 0; i < 32 && h0 + i < H; ++i) { vt += sv[i]; rt += sr[i]; }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    *sparsity = rt / (float)H;
    *variance = vt / (float)H;
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

int pivot_plane_shares(int64_t n) { return (int)((n + kPlaneShare - 1) / kPlaneShare); }

hipError_t launch_pivot_planes(const float* heads, int H, int64_t n, float inv_w, uint32_t* hist, float* part,
                               hipStream_t st) {
  if (H == 0 || n == 0) return hipSuccess;
  hipLaunchKernelGGL(pivot_planes_kernel, dim3((unsigned)pivot_plane_shares(n), (unsigned)H), dim3(256), 0, st, heads,
                     n, inv_w, hist, part);
  return hipGetLastError();
}

hipError_t launch_pivot_finish_planes(const float* var_part, int Pv, const float* mass_part, int Pm, const float* tail,
                                      int H, int64_t n, float inv_w, float* sparsity, float* variance, hipStream_t st) {
  hipLaunchKernelGGL(pivot_finish_planes_kernel, dim3(1), dim3(256), 0, st, var_part, Pv, mass_part, Pm, tail, H, n,
                     inv_w, sparsity, variance);
  return hipGetLastError();
}

}  // namespace skv
