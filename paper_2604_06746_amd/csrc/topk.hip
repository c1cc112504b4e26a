// Exact, deterministic top-k selection (paper Eq. 10 / Eq. 13): radix select on order-preserving
// 32-bit keys (three digit passes 11/11/10 bits from the top), then an index-ordered compaction.
//   init    : zero histograms / tickets, set the per-sequence search state, write the kept window
//   hist<P> : per-sequence digit histogram of the still-matching candidates; the last workgroup to
//             finish (atomic ticket, no spinning) scans the bins from the top and narrows the search
//   count   : per-workgroup counts of keys above / equal to the threshold key
//   write   : each workgroup sums the counts before it and writes its selected indices in order
// Ties at the threshold go to the lowest indices; output is ascending; no floating-point atomics.
#include "common.h"

namespace skv {
namespace {

#ifndef SKV_TOPK_CHUNK
#define SKV_TOPK_CHUNK 4096
#endif
constexpr int kChunk = SKV_TOPK_CHUNK;   // scores per workgroup
constexpr int kThreads = 256;
constexpr int kPer = kChunk / kThreads;
constexpr int kBins = 2048;

struct TopkWs {
  uint32_t* hist;     // [3][B][kBins]
  uint32_t* ticket;   // [3][B]
  uint32_t* prefix;   // [B] key bits fixed so far
  uint32_t* krem;     // [B] how many still to take among the matching candidates
  uint32_t* blkcnt;   // [total_blocks][2] (above, equal)
};

__device__ inline uint32_t score_key(float f) {
  uint32_t u = __float_as_uint(f);
  if (u == 0x80000000u) u = 0u;                         // -0.0 orders as +0.0
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);    // larger float <=> larger key
}

template <int P> struct Digit;
template <> struct Digit<0> { static constexpr int shift = 21, bits = 11; };
template <> struct Digit<1> { static constexpr int shift = 10, bits = 11; };
template <> struct Digit<2> { static constexpr int shift = 0, bits = 10; };

__global__ __launch_bounds__(kThreads) void topk_init_kernel(SeqTable seq, int keep_tail, TopkWs ws,
                                                             int32_t* __restrict__ idx_out) {
  const int b = blockIdx.y;
  const int B = seq.batch;
  const int tid = blockIdx.x * kThreads + threadIdx.x;
  const int stride = gridDim.x * kThreads;
  for (int p = 0; p < 3; ++p)
    for (int i = tid; i < kBins; i += stride) ws.hist[((size_t)p * B + b) * kBins + i] = 0u;
  const int64_t n = seq.cu[b + 1] - seq.cu[b];
  const int64_t m = n - keep_tail;
  if (tid == 0) {
    for (int p = 0; p < 3; ++p) ws.ticket[p * B + b] = 0u;
    ws.prefix[b] = 0u;
    ws.krem[b] = (uint32_t)seq.k[b];
  }
  for (int i = tid; i < keep_tail; i += stride)
    idx_out[seq.out_off[b] + seq.k[b] + i] = (int32_t)(m + i);
}

// exclusive scan of one value per thread over the workgroup (256 threads), result in *excl, total returned
__device__ inline uint32_t block_excl_scan(uint32_t v, uint32_t* sh /*[256]*/, uint32_t* excl) {
  const int t = threadIdx.x;
  sh[t] = v;
  __syncthreads();
  for (int off = 1; off < kThreads; off <<= 1) {
    const uint32_t add = t >= off ? sh[t - off] : 0u;
    __syncthreads();
    sh[t] += add;
    __syncthreads();
  }
  *excl = sh[t] - v;
  const uint32_t total = sh[kThreads - 1];
  __syncthreads();
  return total;
}

template <int P>
__global__ __launch_bounds__(kThreads) void topk_hist_kernel(const float* __restrict__ scores, SeqTable seq,
                                                             int keep_tail, TopkWs ws) {
  constexpr int shift = Digit<P>::shift, bits = Digit<P>::bits, nb = 1 << bits;
  __shared__ uint32_t h[kBins];
  __shared__ uint32_t scan[kThreads];
  __shared__ uint32_t is_last;
  const int b = blockIdx.y;
  const int nblk = seq.chunk_start[b + 1] - seq.chunk_start[b];
  if ((int)blockIdx.x >= nblk) return;
  const int B = seq.batch;
  const int64_t m = seq.cu[b + 1] - seq.cu[b] - keep_tail;
  const float* sc = scores + seq.cu[b];
  const int t = threadIdx.x;
  for (int i = t; i < nb; i += kThreads) h[i] = 0u;
  __syncthreads();
  const uint32_t prefix = P == 0 ? 0u : ws.prefix[b];
  const int64_t base = (int64_t)blockIdx.x * kChunk;
#pragma unroll
  for (int e = 0; e < kPer; ++e) {
    const int64_t j = base + e * kThreads + t;
    if (j < m) {
      const uint32_t key = score_key(sc[j]);
      const bool match = P == 0 ? true : ((key >> (shift + bits)) == prefix);
      if (match) atomicAdd(&h[(key >> shift) & (nb - 1)], 1u);
    }
  }
  __syncthreads();
  uint32_t* gh = ws.hist + ((size_t)P * B + b) * kBins;
  for (int i = t; i < nb; i += kThreads)
    if (h[i]) atomicAdd(&gh[i], h[i]);
  __threadfence();
  __syncthreads();
  if (t == 0) is_last = (atomicAdd(&ws.ticket[P * B + b], 1u) == (uint32_t)(nblk - 1)) ? 1u : 0u;
  __syncthreads();
  if (!is_last) return;
  __threadfence();
  // last workgroup of this sequence: walk the bins from the top until krem candidates are covered
  const uint32_t krem = ws.krem[b];
  constexpr int per = nb / kThreads;
  uint32_t mine[per];
  uint32_t sum = 0;
#pragma unroll
  for (int i = 0; i < per; ++i) {
    mine[i] = __hip_atomic_load(&gh[nb - 1 - (t * per + i)], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    sum += mine[i];
  }
  uint32_t excl;
  block_excl_scan(sum, scan, &excl);
  if (excl < krem && excl + sum >= krem) {
    uint32_t run = excl;
#pragma unroll
    for (int i = 0; i < per; ++i) {
      if (run < krem && run + mine[i] >= krem) {
        const uint32_t bin = (uint32_t)(nb - 1 - (t * per + i));
        ws.prefix[b] = (prefix << bits) | bin;
        ws.krem[b] = krem - run;
      }
      run += mine[i];
    }
  }
}

__global__ __launch_bounds__(kThreads) void topk_count_kernel(const float* __restrict__ scores, SeqTable seq,
                                                              int keep_tail, TopkWs ws) {
  __shared__ uint32_t cnt[2];
  const int b = blockIdx.y;
  const int nblk = seq.chunk_start[b + 1] - seq.chunk_start[b];
  if ((int)blockIdx.x >= nblk) return;
  const int64_t m = seq.cu[b + 1] - seq.cu[b] - keep_tail;
  const float* sc = scores + seq.cu[b];
  const int t = threadIdx.x;
  if (t < 2) cnt[t] = 0u;
  __syncthreads();
  const uint32_t T = ws.prefix[b];
  const int64_t base = (int64_t)blockIdx.x * kChunk;
  uint32_t gt = 0, eq = 0;
#pragma unroll
  for (int e = 0; e < kPer; ++e) {
    const int64_t j = base + e * kThreads + t;
    if (j < m) {
      const uint32_t key = score_key(sc[j]);
      gt += key > T;
      eq += key == T;
    }
  }
  if (gt) atomicAdd(&cnt[0], gt);
  if (eq) atomicAdd(&cnt[1], eq);
  __syncthreads();
  if (t < 2) ws.blkcnt[((size_t)seq.chunk_start[b] + blockIdx.x) * 2 + t] = cnt[t];
}

__global__ __launch_bounds__(kThreads) void topk_write_kernel(const float* __restrict__ scores, SeqTable seq,
                                                              int keep_tail, TopkWs ws,
                                                              int32_t* __restrict__ idx_out) {
  __shared__ uint32_t keys[kChunk];
  __shared__ uint32_t scan[kThreads];
  __shared__ uint32_t pre[2];
  const int b = blockIdx.y;
  const int nblk = seq.chunk_start[b + 1] - seq.chunk_start[b];
  if ((int)blockIdx.x >= nblk) return;
  const int64_t m = seq.cu[b + 1] - seq.cu[b] - keep_tail;
  const float* sc = scores + seq.cu[b];
  const int t = threadIdx.x;
  const uint32_t T = ws.prefix[b];
  const uint32_t need = ws.krem[b];            // equal-to-threshold keys to take (lowest indices)
  const int64_t base = (int64_t)blockIdx.x * kChunk;
  if (t < 2) pre[t] = 0u;
#pragma unroll
  for (int e = 0; e < kPer; ++e) {
    const int64_t j = base + e * kThreads + t;
    keys[e * kThreads + t] = j < m ? score_key(sc[j]) : 0u;
  }
  __syncthreads();
  // counts of all earlier workgroups of this sequence
  uint32_t g0 = 0, e0 = 0;
  const uint32_t* bc = ws.blkcnt + (size_t)seq.chunk_start[b] * 2;
  for (int i = t; i < (int)blockIdx.x; i += kThreads) { g0 += bc[2 * i]; e0 += bc[2 * i + 1]; }
  if (g0) atomicAdd(&pre[0], g0);
  if (e0) atomicAdd(&pre[1], e0);
  // this thread's 16 consecutive scores
  uint32_t gt = 0, eq = 0;
#pragma unroll
  for (int e = 0; e < kPer; ++e) {
    const int64_t j = base + t * kPer + e;
    const uint32_t key = keys[t * kPer + e];
    if (j < m) { gt += key > T; eq += key == T; }
  }
  uint32_t gt_before, eq_before;
  block_excl_scan(gt, scan, &gt_before);
  block_excl_scan(eq, scan, &eq_before);
  gt_before += pre[0];
  eq_before += pre[1];
  int32_t* out = idx_out + seq.out_off[b];
#pragma unroll
  for (int e = 0; e < kPer; ++e) {
    const int64_t j = base + t * kPer + e;
    if (j >= m) break;
    const uint32_t key = keys[t * kPer + e];
    if (key > T) {
      out[gt_before + min(eq_before, need)] = (int32_t)j;
      ++gt_before;
    } else if (key == T) {
      if (eq_before < need) out[gt_before + eq_before] = (int32_t)j;
      ++eq_before;
    }
  }
}

TopkWs carve(void* ws, int B, int64_t total_blocks) {
  TopkWs w;
  uint8_t* p = (uint8_t*)ws;
  w.hist = (uint32_t*)p;   p += align_up(sizeof(uint32_t) * 3 * (size_t)B * kBins, 256);
  w.ticket = (uint32_t*)p; p += align_up(sizeof(uint32_t) * 3 * (size_t)B, 256);
  w.prefix = (uint32_t*)p; p += align_up(sizeof(uint32_t) * (size_t)B, 256);
  w.krem = (uint32_t*)p;   p += align_up(sizeof(uint32_t) * (size_t)B, 256);
  w.blkcnt = (uint32_t*)p;
  (void)total_blocks;
  return w;
}

}  // namespace

size_t topk_workspace_bytes(int batch, int64_t total_tokens) {
  const size_t B = (size_t)(batch > 0 ? batch : 1);
  const size_t blocks = (size_t)(total_tokens / kChunk) + B;
  return align_up(sizeof(uint32_t) * 3 * B * kBins, 256) + align_up(sizeof(uint32_t) * 3 * B, 256) +
         2 * align_up(sizeof(uint32_t) * B, 256) + align_up(sizeof(uint32_t) * 2 * blocks, 256);
}

// seq.chunk_start must hold the cumulative workgroup counts (kChunk scores each, sequences with
// k_b == 0 get none); seq.out_off the output offsets.
hipError_t launch_topk(const float* scores, const SeqTable& seq_in, int keep_tail, int32_t* idx_out,
                       void* wsp, hipStream_t st) {
  SeqTable seq = seq_in;
  const int B = seq.batch;
  if (B == 0) return hipSuccess;
  int max_blk = 0;
  seq.chunk_start[0] = 0;
  for (int b = 0; b < B; ++b) {
    const int64_t m = seq.cu[b + 1] - seq.cu[b] - keep_tail;
    const int nblk = seq.k[b] > 0 ? (int)ceil_div(m, kChunk) : 0;
    seq.chunk_start[b + 1] = seq.chunk_start[b] + nblk;
    if (nblk > max_blk) max_blk = nblk;
  }
  TopkWs ws = carve(wsp, B, seq.chunk_start[B]);
  hipLaunchKernelGGL(topk_init_kernel, dim3(2, B), dim3(kThreads), 0, st, seq, keep_tail, ws, idx_out);
  if (max_blk > 0) {
    dim3 grid(max_blk, B), blk(kThreads);
    hipLaunchKernelGGL(topk_hist_kernel<0>, grid, blk, 0, st, scores, seq, keep_tail, ws);
    hipLaunchKernelGGL(topk_hist_kernel<1>, grid, blk, 0, st, scores, seq, keep_tail, ws);
    hipLaunchKernelGGL(topk_hist_kernel<2>, grid, blk, 0, st, scores, seq, keep_tail, ws);
    hipLaunchKernelGGL(topk_count_kernel, grid, blk, 0, st, scores, seq, keep_tail, ws);
    hipLaunchKernelGGL(topk_write_kernel, grid, blk, 0, st, scores, seq, keep_tail, ws, idx_out);
  }
  return hipGetLastError();
}

}  // namespace skv
