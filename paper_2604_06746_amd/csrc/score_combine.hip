// Small kernels around the two scoring passes:
//   combine : merge the per-key-chunk softmax statistics of every query row into
//             lse2 = M + log2 Z (what pass 2 normalises with) and the row entropies of Eq. 4.
//   reduce  : D_j = sum over KV heads / row-chunks of the pass-2 column sums (Eq. 2 without 1/w),
//             plus the means over window rows and heads that finish Eq. 4; optionally also the
//             centrality update below on the value it has just formed.
//   accumulate : C <- lambda C + inv_w D   (Alg. 1 line 6 / Eq. 3).
//   group sums : the same column sums per KV head only (Eq. 2's inner sum over h in H_g), on request.
#include "common.h"

namespace skv {
namespace {

constexpr float kLn2 = 0.6931471805599453f;

// one workgroup of 1024 threads per (sequence b, KV head g, block of 32 query rows): thread = (row,
// slot); the 32 slots of a row split its partial statistics (consecutive threads read consecutive rows,
// the contiguous direction of the partials), then merge in a fixed order: lane pairs, then waves
constexpr int kCombRows = 32, kCombSlots = 32;

__global__ __launch_bounds__(kCombRows* kCombSlots) void score_combine_kernel(
    SeqTable seq, int G, int R, int RPC, int RC, int WK, int64_t n_chunks, int row_blocks,
    const float* __restrict__ stats, float* __restrict__ lse2, float* __restrict__ row_ent,
    uint32_t* __restrict__ zero_ptr, int64_t zero_words) {
  short_kernel_priority();
  __shared__ float sM[kCombSlots / 2][kCombRows], sZ[kCombSlots / 2][kCombRows], sE[kCombSlots / 2][kCombRows];
  // fused layer step: clear the digit histograms of the selection that follows the scoring
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < zero_words; i += (int64_t)gridDim.x * blockDim.x)
    zero_ptr[i] = 0u;
  const int rblk = blockIdx.x % row_blocks;
  const int bg = blockIdx.x / row_blocks;
  const int b = bg / G, g = bg % G;
  const int rl = threadIdx.x & (kCombRows - 1);
  const int slot = threadIdx.x / kCombRows;
  const int row = rblk * kCombRows + rl;
  const int64_t c0 = seq.chunk_start[b], c1 = seq.chunk_start[b + 1];
  const int rowc = min(row, R - 1);
  const int rc = rowc / RPC, rr = rowc % RPC;
  const int grc = g * RC + rc;
  float M = -1.0e30f, Z = 0.f, E = 0.f;
  const int64_t np = (c1 - c0) * WK;
  const float* base = stats + (((int64_t)grc * n_chunks + c0) * WK * 3) * RPC + rr;
  int64_t p = slot;
  for (; p + 3 * kCombSlots < np; p += 4 * kCombSlots) {   // four partials in flight
    float m[4], z[4], e[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const float* sp = base + (p + u * kCombSlots) * 3 * RPC;
      m[u] = sp[0]; z[u] = sp[RPC]; e[u] = sp[2 * RPC];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) merge_stats(M, Z, E, m[u], z[u], e[u]);
  }
  for (; p < np; p += kCombSlots) {
    const float* sp = base + p * 3 * RPC;
    merge_stats(M, Z, E, sp[0], sp[RPC], sp[2 * RPC]);
  }
  {  // the two slots of a wave
    const float M2 = __shfl_xor(M, 32), Z2 = __shfl_xor(Z, 32), E2 = __shfl_xor(E, 32);
    merge_stats(M, Z, E, M2, Z2, E2);
  }
  const int wv = threadIdx.x >> 6;
  if ((threadIdx.x & 63) < kCombRows) { sM[wv][rl] = M; sZ[wv][rl] = Z; sE[wv][rl] = E; }
  __syncthreads();
  if (threadIdx.x < kCombRows && row < R) {
    for (int k = 1; k < kCombSlots / 2; ++k) merge_stats(M, Z, E, sM[k][rl], sZ[k][rl], sE[k][rl]);
    float ent = 0.f, l2 = 0.f;
    if (c1 > c0) {
      const float lz = __log2f(Z);
      l2 = M + lz;
      ent = kLn2 * (lz - E / Z);   // -sum a ln a  with a = 2^(x-M)/Z
    }
    const int64_t o = (int64_t)b * G * R + (int64_t)g * R + row;
    lse2[o] = l2;
    row_ent[o] = ent;
  }
}

// grid covers the tokens, V floats per thread (V = 4 for long inputs, else 1 so that enough workgroups
// exist to use every CU); planes are added in ascending order, eight loads in flight.
// Workgroups b < B also finish Eq. 4 for sequence b.  With `cen` != NULL the kernel also applies
// C <- lambda C + inv_w D with the arithmetic of accumulate_kernel (one fma on the rounded product).
// FUSED (a fused layer step, Eq. 13 follows Eq. 2 directly): the kernel also starts the selection on the
// scores it has just formed -- the histogram of their first radix digit (what topk_hist0_kernel builds
// from memory) and the kept window's indices.
template <int V, bool FUSED>
__global__ __launch_bounds__(256) void score_reduce_kernel(
    const float* __restrict__ colsum, int GRC, int64_t total, float* __restrict__ indeg,
    const float* __restrict__ row_ent, float* __restrict__ ent_head, float* __restrict__ entropy, int B,
    int Hq, int w, float* __restrict__ cen, float lambda, float inv_w, SeqTable seq, SelectFusion fs) {
  short_kernel_priority();
  __shared__ float hsum[256];
  __shared__ uint32_t h0[FUSED ? kTopkBins : 1];
  const int64_t i0 = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * V;
  int b_wg = 0;   // FUSED: the sequence of the workgroup's first token; its digits are counted in LDS
  if constexpr (FUSED) {
    for (int i = threadIdx.x; i < kTopkBins; i += 256) h0[i] = 0u;
    const int64_t first = min((int64_t)blockIdx.x * blockDim.x * V, total > 0 ? total - 1 : 0);
    while (b_wg + 1 < B && first >= seq.cu[b_wg + 1]) ++b_wg;
    __syncthreads();
  }
  if (i0 < total) {   // V == 4 only when total % 4 == 0
    float a[V], c[V];
#pragma unroll
    for (int j = 0; j < V; ++j) a[j] = 0.f;
    if (cen) {
      if constexpr (V == 4) {
        const float4 t = *reinterpret_cast<const float4*>(cen + i0);
        c[0] = t.x; c[1] = t.y; c[2] = t.z; c[3] = t.w;
      } else {
        c[0] = cen[i0];
      }
    }
    const float* cp = colsum + i0;
    int p = 0;
    for (; p + 8 <= GRC; p += 8) {
      float v[8][V];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if constexpr (V == 4) {
          const float4 t = *reinterpret_cast<const float4*>(cp + (int64_t)(p + u) * total);
          v[u][0] = t.x; v[u][1] = t.y; v[u][2] = t.z; v[u][3] = t.w;
        } else {
          v[u][0] = cp[(int64_t)(p + u) * total];
        }
      }
#pragma unroll
      for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int j = 0; j < V; ++j) a[j] += v[u][j];
    }
    for (; p < GRC; ++p)
#pragma unroll
      for (int j = 0; j < V; ++j) a[j] += cp[(int64_t)p * total + j];
    if constexpr (V == 4) *reinterpret_cast<float4*>(indeg + i0) = make_float4(a[0], a[1], a[2], a[3]);
    else indeg[i0] = a[0];
    if (cen) {
#pragma unroll
      for (int j = 0; j < V; ++j) c[j] = fmaf(lambda, c[j], inv_w * a[j]);
      if constexpr (V == 4) *reinterpret_cast<float4*>(cen + i0) = make_float4(c[0], c[1], c[2], c[3]);
      else cen[i0] = c[0];
    }
    if constexpr (FUSED) {
      int b = b_wg;
#pragma unroll
      for (int j = 0; j < V; ++j) {
        const int64_t i = i0 + j;
        while (b + 1 < B && i >= seq.cu[b + 1]) ++b;
        // only the prefix [0, n_b - keep_tail) of a sequence with a budget is searched
        if (seq.k[b] > 0 && i - seq.cu[b] < seq.cu[b + 1] - seq.cu[b] - fs.keep_tail) {
          const uint32_t digit = score_key(a[j]) >> 21;
          if (b == b_wg) atomicAdd(&h0[digit], 1u);
          else atomicAdd(&fs.hist[(size_t)b * 3 * kTopkBins + digit], 1u);
        }
      }
    }
  }
  if constexpr (FUSED) {
    __syncthreads();
    uint32_t* gh = fs.hist + (size_t)b_wg * 3 * kTopkBins;
    for (int i = threadIdx.x; i < kTopkBins; i += 256)
      if (h0[i]) atomicAdd(&gh[i], h0[i]);
    // the kept window: indices n_b - keep_tail .. n_b - 1 behind the k_b selected ones
    const int64_t gtid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x, gsz = (int64_t)gridDim.x * blockDim.x;
    const int64_t tail = fs.keep_tail;
    for (int64_t u = gtid; u < (int64_t)B * tail; u += gsz) {
      const int b = (int)(u / tail);
      const int64_t i = u - (int64_t)b * tail;
      fs.idx_out[seq.out_off[b] + seq.k[b] + i] = (int32_t)(seq.cu[b + 1] - seq.cu[b] - tail + i);
    }
  }
  for (int b = blockIdx.x; b < B; b += gridDim.x) {   // uniform per workgroup
    // eight lanes share a head: each sums every eighth window row, then a fixed shuffle tree
    float part = 0.f;
    for (int h0i = 0; h0i < Hq; h0i += 32) {
      const int h = h0i + (threadIdx.x >> 3);
      float s = 0.f;
      if (h < Hq) {
        const float* re = row_ent + ((int64_t)b * Hq + h) * w;
        for (int i = threadIdx.x & 7; i < w; i += 8) s += re[i];
      }
      s += __shfl_xor(s, 1);
      s += __shfl_xor(s, 2);
      s += __shfl_xor(s, 4);
      if (h < Hq && (threadIdx.x & 7) == 0) {
        s /= (float)w;
        ent_head[(int64_t)b * Hq + h] = s;
        part += s;
      }
    }
    hsum[threadIdx.x] = part;
    __syncthreads();
    if (threadIdx.x == 0) {
      float s = 0.f;
      for (int t = 0; t < 256; t += 8) s += hsum[t];
      entropy[b] = s / (float)Hq;
    }
    __syncthreads();
  }
}

// per-KV-head in-degree: the column-sum planes of head g added up in plane order
__global__ __launch_bounds__(256) void group_sums_kernel(const float* __restrict__ colsum, int CP, int64_t total,
                                                         float* __restrict__ groups) {
  short_kernel_priority();
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int g = blockIdx.y;
  if (i >= total) return;
  float a = 0.f;
  for (int c = 0; c < CP; ++c) a += colsum[((int64_t)g * CP + c) * total + i];
  groups[(int64_t)g * total + i] = a;
}

__global__ __launch_bounds__(256) void accumulate_kernel(float* __restrict__ c, const float* __restrict__ d,
                                                         int64_t n, float lambda, float inv_w, int vec) {
  short_kernel_priority();
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (vec) {
    const int64_t i4 = i * 4;
    if (i4 + 3 < n) {
      float4 cv = *reinterpret_cast<float4*>(c + i4);
      const float4 dv = *reinterpret_cast<const float4*>(d + i4);
      cv.x = fmaf(lambda, cv.x, inv_w * dv.x);
      cv.y = fmaf(lambda, cv.y, inv_w * dv.y);
      cv.z = fmaf(lambda, cv.z, inv_w * dv.z);
      cv.w = fmaf(lambda, cv.w, inv_w * dv.w);
      *reinterpret_cast<float4*>(c + i4) = cv;
    } else {
      for (int64_t j = i4; j < n; ++j) c[j] = fmaf(lambda, c[j], inv_w * d[j]);
    }
  } else if (i < n) {
    c[i] = fmaf(lambda, c[i], inv_w * d[i]);
  }
}

}  // namespace

hipError_t launch_score_combine(const structkv_shape& s, const ScorePlan& p, const SeqTable& seq,
                                const float* stats, float* lse2, float* row_ent, uint32_t* zero_ptr,
                                int64_t zero_words, hipStream_t st) {
  const int row_blocks = (int)ceil_div(p.R, kCombRows);
  const int64_t blocks = (int64_t)seq.batch * s.n_kv_heads * row_blocks;
  if (blocks == 0) return hipSuccess;
  hipLaunchKernelGGL(score_combine_kernel, dim3((unsigned)blocks), dim3(kCombRows * kCombSlots), 0, st, seq, s.n_kv_heads, p.R,
                     p.RPC, p.RC, p.WK, p.n_chunks, row_blocks, stats, lse2, row_ent, zero_ptr, zero_words);
  return hipGetLastError();
}

hipError_t launch_score_reduce(const structkv_shape& s, const ScorePlan& p, const SeqTable& seq,
                               const float* colsum, int64_t total, float* indeg, const float* row_ent,
                               float* ent_head, float* entropy, float* centrality, float lambda, float inv_w,
                               const SelectFusion* fuse, hipStream_t st) {
  const bool vec = (total % 4 == 0) && (((uintptr_t)indeg | (uintptr_t)colsum | (uintptr_t)centrality) & 15) == 0 &&
                   total >= (int64_t)4 * 256 * 1024;
  int64_t blocks = ceil_div(ceil_div(total, vec ? 4 : 1), 256);
  if (blocks == 0) blocks = 1;
  const bool fused = fuse != nullptr && fuse->hist != nullptr;
  const SelectFusion fs = fused ? *fuse : SelectFusion{};
#define SKV_REDUCE(V, F)                                                                                       \
  hipLaunchKernelGGL((score_reduce_kernel<V, F>), dim3((unsigned)blocks), dim3(256), 0, st, colsum,            \
                     s.n_kv_heads * p.CP, total, indeg, row_ent, ent_head, entropy, seq.batch, s.n_q_heads,    \
                     s.window, centrality, lambda, inv_w, seq, fs)
  if (vec) { if (fused) SKV_REDUCE(4, true); else SKV_REDUCE(4, false); }
  else     { if (fused) SKV_REDUCE(1, true); else SKV_REDUCE(1, false); }
#undef SKV_REDUCE
  return hipGetLastError();
}

hipError_t launch_group_sums(const structkv_shape& s, const ScorePlan& p, const float* colsum, int64_t total,
                             float* groups, hipStream_t st) {
  if (total == 0) return hipSuccess;
  hipLaunchKernelGGL(group_sums_kernel, dim3((unsigned)ceil_div(total, 256), (unsigned)s.n_kv_heads), dim3(256), 0,
                     st, colsum, p.CP, total, groups);
  return hipGetLastError();
}

hipError_t launch_accumulate(float* c, const float* d, int64_t n, float lambda, float inv_w, hipStream_t st) {
  if (n == 0) return hipSuccess;
  // four floats per thread only when that still leaves enough workgroups to use every CU
  const int vec = (((uintptr_t)c | (uintptr_t)d) & 15) == 0 && n >= (int64_t)4 * 256 * 1024;
  const int64_t work = vec ? ceil_div(n, 4) : n;
  hipLaunchKernelGGL(accumulate_kernel, dim3((unsigned)ceil_div(work, 256)), dim3(256), 0, st, c, d, n,
                     lambda, inv_w, vec);
  return hipGetLastError();
}

}  // namespace skv
