// SIMT scoring kernels: fp32 inputs (the exact-arithmetic path) and any shape the MFMA kernels
// do not cover.  Same two-pass scheme and the same partial-result layout as the MFMA path:
//   pass 1: per (row, key-chunk) running (M, Z, E) in the log2 domain        (paper Eq. 1, Eq. 4)
//   pass 2: p = 2^(x - lse2), column sums over a row-chunk's rows            (paper Eq. 2)
// A workgroup = 16 query rows x 16 key lanes; K tiles and the 16 query rows live in LDS as fp32.
#include "common.h"
#include <hip/hip_bf16.h>

namespace skv {
namespace {

constexpr int kRows = 16;     // rows per workgroup (RPC of the SIMT plan)
constexpr int kLanes = 16;    // key lanes per row
constexpr float kNegBig = -1.0e30f;

__device__ inline float ld_elem(const float* p, int64_t i) { return p[i]; }
__device__ inline float ld_elem(const __hip_bfloat16* p, int64_t i) {
  return __uint_as_float(((uint32_t)reinterpret_cast<const uint16_t*>(p)[i]) << 16);
}

template <typename T>
__global__ __launch_bounds__(256) void score_simt_kernel(
    const T* __restrict__ q, const T* __restrict__ k, int64_t ksh, int64_t kst, int kshare, SeqTable seq,
    int Hq, int G, int d, int w, int causal, float c2, int R, int RC, int KC, int TKS,
    int64_t n_chunks, float* __restrict__ stats, const float* __restrict__ lse2,
    float* __restrict__ colsum, int64_t total, float* __restrict__ probs, int pass) {
  extern __shared__ float smem[];
  const int pitch = d + 1;
  float* qs = smem;                       // [16][d]
  float* ks = qs + kRows * d;             // [TKS][d+1]
  float* cs = ks + TKS * pitch;           // [16][TKS]

  const int GRC = G * RC;
  const int grc = blockIdx.x % GRC;
  const int64_t chunk = blockIdx.x / GRC;
  const int g = grc / RC, rc = grc % RC;
  int b = 0;
  while (b + 1 < seq.batch && chunk >= seq.chunk_start[b + 1]) ++b;
  const int64_t tok0 = seq.cu[b];
  const int64_t n = seq.cu[b + 1] - tok0;
  const int64_t key0 = (chunk - seq.chunk_start[b]) * (int64_t)KC;
  const int64_t key_end = min(n, key0 + KC);

  const int tid = threadIdx.x;
  const int r = tid / kLanes, kl = tid % kLanes;
  const int row = rc * kRows + r;                 // row inside the KV group: (h_local * w + i)
  const bool row_ok = row < R;
  const int64_t n_vis = !row_ok ? 0 : (causal ? (n - w + (row % w) + 1) : n);

  // the 16 query rows of this workgroup -> LDS (fp32)
  const T* qg = q + ((int64_t)b * Hq * w + (int64_t)g * R) * d;
  for (int e = tid; e < kRows * d; e += 256) {
    const int rr = e / d, c = e % d;
    const int grow = rc * kRows + rr;
    qs[e] = grow < R ? ld_elem(qg, (int64_t)grow * d + c) : 0.f;
  }

  float M = kNegBig, Z = 0.f, E = 0.f;
  float nl = 0.f;
  if (pass == 2) nl = row_ok ? -lse2[(int64_t)b * G * R + (int64_t)g * R + row] : 0.f;
  const T* kg = k + (int64_t)(g / kshare) * ksh + tok0 * kst;   // kshare consecutive groups read one K head

  for (int64_t t0 = key0; t0 < key_end; t0 += TKS) {
    __syncthreads();
    for (int e = tid; e < TKS * d; e += 256) {
      const int jj = e / d, c = e % d;
      const int64_t j = min(t0 + jj, n - 1);
      ks[jj * pitch + c] = ld_elem(kg, j * kst + c);
    }
    __syncthreads();
    for (int jj = kl; jj < TKS; jj += kLanes) {
      const int64_t j = t0 + jj;
      float acc = 0.f;
      const float* qr = qs + r * d;
      const float* kr = ks + jj * pitch;
      for (int c = 0; c < d; ++c) acc = fmaf(qr[c], kr[c], acc);
      const float x = acc * c2;
      const bool vis = j < key_end && j < n_vis;
      if (pass == 1) {
        if (vis) {
          const float Mn = fmaxf(M, x);
          const float dl = M - Mn;
          const float f = __builtin_amdgcn_exp2f(dl);
          const float t = x - Mn;
          const float p = __builtin_amdgcn_exp2f(t);
          E = (E + dl * Z) * f + p * t;
          Z = Z * f + p;
          M = Mn;
        }
      } else {
        const float p = vis ? __builtin_amdgcn_exp2f(x + nl) : 0.f;
        cs[r * TKS + jj] = p;
        if (probs != nullptr && row_ok && j < key_end)
          probs[((int64_t)g * R + row) * n + j] = p;
      }
    }
    if (pass == 2) {
      __syncthreads();
      if (tid < TKS && t0 + tid < key_end) {
        float s = 0.f;
        for (int rr = 0; rr < kRows; ++rr) s += cs[rr * TKS + tid];
        colsum[(int64_t)grc * total + tok0 + t0 + tid] = s;
      }
    }
  }

  if (pass == 1) {
    // fixed-shape tree over the 16 key lanes of a row (lanes of one wave)
    for (int off = 1; off < kLanes; off <<= 1) {
      const float M2 = __shfl_xor(M, off), Z2 = __shfl_xor(Z, off), E2 = __shfl_xor(E, off);
      merge_stats(M, Z, E, M2, Z2, E2);
    }
    if (kl == 0) {
      float* sp = stats + (((int64_t)grc * n_chunks + chunk) * 3) * kRows;
      sp[0 * kRows + r] = M;
      sp[1 * kRows + r] = Z;
      sp[2 * kRows + r] = E;
    }
  }
}

}  // namespace

hipError_t launch_score_simt(const structkv_shape& s, const ScorePlan& p, const SeqTable& seq,
                             const void* q, const void* k, int64_t ksh, int64_t kst, float c2,
                             float* stats, const float* lse2, float* colsum, int64_t total,
                             float* probs, int pass, hipStream_t st) {
  if (p.grid_chunks == 0) return hipSuccess;
  const int d = s.head_dim;
  const int TKS = d <= 128 ? 64 : 16;
  const size_t smem = sizeof(float) * ((size_t)kRows * d + (size_t)TKS * (d + 1) + (size_t)kRows * TKS);
  const int64_t grid = (int64_t)s.n_kv_heads * p.RC * p.grid_chunks;
  dim3 g((unsigned)grid), blk(256);
  if (s.dtype == STRUCTKV_DTYPE_F32) {
    hipLaunchKernelGGL(score_simt_kernel<float>, g, blk, smem, st, (const float*)q, (const float*)k, ksh,
                       kst, p.kshare, seq, s.n_q_heads, s.n_kv_heads, d, s.window, s.causal, c2, p.R, p.RC, p.KC,
                       TKS, p.n_chunks, stats, lse2, colsum, total, probs, pass);
  } else {
    hipLaunchKernelGGL(score_simt_kernel<__hip_bfloat16>, g, blk, smem, st, (const __hip_bfloat16*)q,
                       (const __hip_bfloat16*)k, ksh, kst, p.kshare, seq, s.n_q_heads, s.n_kv_heads, d, s.window,
                       s.causal, c2, p.R, p.RC, p.KC, TKS, p.n_chunks, stats, lse2, colsum, total, probs,
                       pass);
  }
  return hipGetLastError();
}

}  // namespace skv
