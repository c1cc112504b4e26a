// Exact, deterministic top-k selection (paper Eq. 10 / Eq. 13): radix select on order-preserving
// 32-bit keys (three digit passes, 11/11/10 bits from the top), then an index-ordered compaction.
//
// Two launches per call.  `topk_init_kernel` zeroes the histograms and barrier words and writes the
// kept window.  `topk_select_kernel` is one resident grid (at most 1024 workgroups in all, so every
// workgroup is on the chip at once) in which the workgroups of a sequence move through five phases
// separated by a counter barrier in global memory:
//   digit histogram (LDS, merged with integer atomics)  x3, each followed by every workgroup scanning the
//   2048 bins from the top to narrow the search;  per-workgroup counts of keys above / equal to the
//   threshold key;  ordered write (each workgroup adds the counts of the workgroups before it).
// Ties at the threshold go to the lowest indices; output is ascending; no floating-point atomics.
// The barrier wait is bounded: a workgroup that waits too long gives up, raises an error word in the
// workspace and still runs to the end, so the kernel always terminates.
#include "common.h"

namespace skv {
namespace {

constexpr int kThreads = 256;
constexpr int kBins = 2048;
constexpr int kMaxBlocksPerSeq = 128;
constexpr int kMaxBlocksTotal = 1024;
constexpr int kTargetPerBlock = 2048;        // scores per workgroup when the sequence is short enough
constexpr uint32_t kSpinLimit = 1u << 22;    // barrier polls (about a microsecond each) before a workgroup gives up

struct TopkWs {
  uint32_t* hist;     // [B][3][kBins]
  uint32_t* bar;      // [B][4]: arrivals, error flag, unused, unused
  uint32_t* blkcnt;   // [total_blocks][2] (above, equal)
};

__device__ inline uint32_t score_key(float f) {
  uint32_t u = __float_as_uint(f);
  if (u == 0x80000000u) u = 0u;                         // -0.0 orders as +0.0
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);    // larger float <=> larger key
}

__device__ inline uint32_t ld_agent(const uint32_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__global__ __launch_bounds__(kThreads) void topk_init_kernel(SeqTable seq, int keep_tail, TopkWs ws,
                                                             int32_t* __restrict__ idx_out) {
  const int b = blockIdx.y;
  const int tid = blockIdx.x * kThreads + threadIdx.x;
  const int stride = gridDim.x * kThreads;
  for (int i = tid; i < 3 * kBins; i += stride) ws.hist[(size_t)b * 3 * kBins + i] = 0u;
  if (tid < 4) ws.bar[b * 4 + tid] = 0u;
  const int64_t m = seq.cu[b + 1] - seq.cu[b] - keep_tail;
  for (int i = tid; i < keep_tail; i += stride)
    idx_out[seq.out_off[b] + seq.k[b] + i] = (int32_t)(m + i);
}

// exclusive scan of one value per thread over the workgroup (256 threads = 4 waves); returns the total.
// Shuffle scan inside each wave, then the four wave totals through LDS.
__device__ inline uint32_t block_excl_scan(uint32_t v, uint32_t* sh /*[>=4]*/, uint32_t* excl) {
  const int t = threadIdx.x, lane = t & 63, wv = t >> 6;
  uint32_t x = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t y = __shfl_up(x, off);
    if (lane >= off) x += y;
  }
  if (lane == 63) sh[wv] = x;
  __syncthreads();
  const uint32_t w0 = sh[0], w1 = sh[1], w2 = sh[2], w3 = sh[3];
  const uint32_t base = wv == 0 ? 0u : (wv == 1 ? w0 : (wv == 2 ? w0 + w1 : w0 + w1 + w2));
  *excl = base + x - v;
  __syncthreads();
  return w0 + w1 + w2 + w3;
}

// All workgroups of a sequence meet here; `phase` counts from 1.  Arrivals only ever grow during a call,
// so phase p is complete when the counter reaches p * nblk.
__device__ inline void seq_barrier(uint32_t* bar, uint32_t nblk, uint32_t phase) {
  __syncthreads();
  if (threadIdx.x == 0) {
    __threadfence();
    atomicAdd(&bar[0], 1u);
    const uint32_t target = phase * nblk;
    uint32_t spins = 0;
    while (ld_agent(&bar[0]) < target) {
      if (++spins > kSpinLimit) { atomicExch(&bar[1], 1u); break; }   // give up rather than hang
    }
    __threadfence();
  }
  __syncthreads();
}

// Scan `nb` bins of a merged histogram from the top until `krem` candidates are covered.
// Returns the bin (all threads), and how many candidates lie above it.
__device__ inline void select_bin(const uint32_t* gh, int nb, uint32_t krem, uint32_t* scan, uint32_t* res,
                                  uint32_t* bin_out, uint32_t* above_out) {
  const int t = threadIdx.x;
  const int per = nb / kThreads;   // 8 or 4
  uint32_t mine[8];
  uint32_t sum = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    mine[i] = i < per ? ld_agent(&gh[nb - 1 - (t * per + i)]) : 0u;
    sum += mine[i];
  }
  uint32_t excl;
  block_excl_scan(sum, scan, &excl);
  if (excl < krem && excl + sum >= krem) {
    uint32_t run = excl;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (i < per && run < krem && run + mine[i] >= krem) {
        res[0] = (uint32_t)(nb - 1 - (t * per + i));
        res[1] = run;
      }
      run += mine[i];
    }
  }
  __syncthreads();
  *bin_out = res[0];
  *above_out = res[1];
  __syncthreads();
}

__global__ __launch_bounds__(kThreads) void topk_select_kernel(const float* __restrict__ scores, SeqTable seq,
                                                               int keep_tail, TopkWs ws,
                                                               int32_t* __restrict__ idx_out) {
  __shared__ uint32_t h[kBins];
  __shared__ uint32_t scan[kThreads];
  __shared__ uint32_t res[2];
  __shared__ uint32_t cnt[2];
  int b = 0;
  while (b + 1 < seq.batch && (int)blockIdx.x >= seq.chunk_start[b + 1]) ++b;
  const uint32_t nblk = (uint32_t)(seq.chunk_start[b + 1] - seq.chunk_start[b]);
  const uint32_t blk = blockIdx.x - (uint32_t)seq.chunk_start[b];
  const int64_t m = seq.cu[b + 1] - seq.cu[b] - keep_tail;
  const float* sc = scores + seq.cu[b];
  uint32_t* bar = ws.bar + b * 4;
  uint32_t* gh = ws.hist + (size_t)b * 3 * kBins;
  const int t = threadIdx.x;
  // this workgroup's contiguous share of the sequence
  const int64_t per = (m + nblk - 1) / nblk;
  const int64_t lo = min(m, (int64_t)blk * per), hi = min(m, lo + per);

  uint32_t prefix = 0, krem = (uint32_t)seq.k[b];
  // ---- three digit passes ----
  for (int pass = 0; pass < 3; ++pass) {
    const int shift = pass == 0 ? 21 : (pass == 1 ? 10 : 0);
    const int bits = pass == 2 ? 10 : 11;
    const int nb = 1 << bits;
    for (int i = t; i < nb; i += kThreads) h[i] = 0u;
    __syncthreads();
    for (int64_t j = lo + t; j < hi; j += kThreads) {
      const uint32_t key = score_key(sc[j]);
      const bool match = pass == 0 ? true : ((key >> (shift + bits)) == prefix);
      if (match) atomicAdd(&h[(key >> shift) & (nb - 1)], 1u);
    }
    __syncthreads();
    for (int i = t; i < nb; i += kThreads)
      if (h[i]) atomicAdd(&gh[pass * kBins + i], h[i]);
    seq_barrier(bar, nblk, (uint32_t)pass + 1);
    uint32_t bin, above;
    select_bin(gh + pass * kBins, nb, krem, scan, res, &bin, &above);
    prefix = (prefix << bits) | bin;
    krem -= above;
  }
  const uint32_t T = prefix;      // the k-th largest key
  const uint32_t need = krem;     // how many keys equal to T are taken (lowest indices first)

  // ---- counts of this workgroup's share; thread t owns a contiguous slice of it ----
  const int64_t sub = (hi - lo + kThreads - 1) / kThreads;
  const int64_t tlo = min(hi, lo + t * sub), thi = min(hi, tlo + sub);
  uint32_t gt = 0, eq = 0;
  for (int64_t j = tlo; j < thi; ++j) {
    const uint32_t key = score_key(sc[j]);
    gt += key > T;
    eq += key == T;
  }
  uint32_t gt_before, eq_before;
  const uint32_t gt_blk = block_excl_scan(gt, scan, &gt_before);
  const uint32_t eq_blk = block_excl_scan(eq, scan, &eq_before);
  uint32_t* bc = ws.blkcnt + (size_t)seq.chunk_start[b] * 2;
  if (t == 0) {
    __hip_atomic_store(&bc[2 * blk], gt_blk, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(&bc[2 * blk + 1], eq_blk, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    cnt[0] = 0u; cnt[1] = 0u;
  }
  seq_barrier(bar, nblk, 4u);

  // ---- ordered write: counts of the workgroups before this one, then of the threads before this one ----
  uint32_t g0 = 0, e0 = 0;
  for (uint32_t i = t; i < blk; i += kThreads) { g0 += ld_agent(&bc[2 * i]); e0 += ld_agent(&bc[2 * i + 1]); }
  if (g0) atomicAdd(&cnt[0], g0);
  if (e0) atomicAdd(&cnt[1], e0);
  __syncthreads();
  gt_before += cnt[0];
  eq_before += cnt[1];
  int32_t* out = idx_out + seq.out_off[b];
  for (int64_t j = tlo; j < thi; ++j) {
    const uint32_t key = score_key(sc[j]);
    if (key > T) {
      out[gt_before + min(eq_before, need)] = (int32_t)j;
      ++gt_before;
    } else if (key == T) {
      if (eq_before < need) out[gt_before + eq_before] = (int32_t)j;
      ++eq_before;
    }
  }
}

TopkWs carve(void* ws, int B) {
  TopkWs w;
  uint8_t* p = (uint8_t*)ws;
  w.hist = (uint32_t*)p;   p += align_up(sizeof(uint32_t) * 3 * (size_t)B * kBins, 256);
  w.bar = (uint32_t*)p;    p += align_up(sizeof(uint32_t) * 4 * (size_t)B, 256);
  w.blkcnt = (uint32_t*)p;
  return w;
}

}  // namespace

size_t topk_workspace_bytes(int batch, int64_t total_tokens) {
  (void)total_tokens;
  const size_t B = (size_t)(batch > 0 ? batch : 1);
  return align_up(sizeof(uint32_t) * 3 * B * kBins, 256) + align_up(sizeof(uint32_t) * 4 * B, 256) +
         align_up(sizeof(uint32_t) * 2 * (size_t)kMaxBlocksTotal, 256);
}

// seq.out_off must hold the output offsets, seq.k the budgets.
hipError_t launch_topk(const float* scores, const SeqTable& seq_in, int keep_tail, int32_t* idx_out,
                       void* wsp, hipStream_t st) {
  SeqTable seq = seq_in;
  const int B = seq.batch;
  if (B == 0) return hipSuccess;
  // workgroups per sequence: about kTargetPerBlock scores each, at most kMaxBlocksPerSeq, and few enough
  // in all that the whole grid is resident at once (the phases meet at a barrier)
  const int cap = kMaxBlocksTotal / B < kMaxBlocksPerSeq ? kMaxBlocksTotal / B : kMaxBlocksPerSeq;
  seq.chunk_start[0] = 0;
  for (int b = 0; b < B; ++b) {
    const int64_t m = seq.cu[b + 1] - seq.cu[b] - keep_tail;
    int64_t nblk = seq.k[b] > 0 ? ceil_div(m, kTargetPerBlock) : 0;
    if (nblk > cap) nblk = cap;
    seq.chunk_start[b + 1] = seq.chunk_start[b] + (int)nblk;
  }
  TopkWs ws = carve(wsp, B);
  hipLaunchKernelGGL(topk_init_kernel, dim3(4, B), dim3(kThreads), 0, st, seq, keep_tail, ws, idx_out);
  if (seq.chunk_start[B] > 0)
    hipLaunchKernelGGL(topk_select_kernel, dim3(seq.chunk_start[B]), dim3(kThreads), 0, st, scores, seq,
                       keep_tail, ws, idx_out);
  return hipGetLastError();
}

}  // namespace skv
