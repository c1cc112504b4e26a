// Exact, deterministic top-k selection (paper Eq. 10 / Eq. 13): radix select on order-preserving
// 32-bit keys (three digit passes, 11/11/10 bits from the top), then an index-ordered compaction.
//
// Five short launches per call; the stream order between them is the only synchronisation (no
// workgroup ever waits for another one, so there is no residency requirement and nothing can hang):
//   init   : zero the three digit histograms, write the kept window
//   hist0  : histogram of the top 11 key bits (LDS, merged into global memory with integer atomics)
//   hist1  : every workgroup scans histogram 0 from the top to find the digit of the k-th key, then
//            histograms the next 11 bits of the keys that carry that digit
//   hist2  : same for digit 1; then one sweep that counts the keys above the 22-bit prefix and
//            histograms the last 10 bits of the keys equal to it.  Each workgroup also publishes the
//            suffix sums of its own last-digit histogram, so that once the last digit T is known
//            anyone can read "keys of workgroup w above T" and "equal to T" with two loads
//   write  : find the last digit, add up the counts of the workgroups before this one, and write the
//            selected indices in ascending order.
// Ties at the threshold go to the lowest indices; no floating-point atomics anywhere.
#include "common.h"

#include <mutex>

namespace skv {
namespace {

// Scratch of structkv_select_topk_static, the entry point for callers that cannot allocate: the histograms,
// search state and per-workgroup suffix sums that structkv_select_topk takes from the caller's workspace live
// here instead.  Every GPU the library runs on holds its own copy until the process ends.  In host code the
// array's name is only a handle for hipGetSymbolAddress; kernels get the address that call returns.
constexpr size_t kStaticScratchBytes = (size_t)4 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kThreads = 256;
constexpr int kBins = kTopkBins;          // digits 0 and 1: 11 bits
constexpr int kLowBins = 1024;            // digit 2: 10 bits
constexpr int kTargetPerBlock = 2048;     // most scores a workgroup holds in registers (eight per thread)
constexpr int kSmallTarget = 1024;        // share of a workgroup when the whole call is short: more, lighter
constexpr int64_t kSmallTotal = 262144;   // workgroups shorten each kernel's serial part
constexpr int kMaxBlocksPerSeq = 1024;    // beyond that a workgroup's share grows instead

// the calling workgroup's sequence and its contiguous share [lo, hi) of the prefix that is searched
struct Share {
  int b;
  uint32_t nblk, blk, first;   // workgroups of the sequence, rank of this one, global id of rank 0
  int64_t lo, hi;
  const float* sc;
};

__device__ inline Share my_share(const float* scores, const SeqTable& seq, int keep_tail) {
  Share s;
  int b = 0;
  while (b + 1 < seq.batch && (int)blockIdx.x >= seq.chunk_start[b + 1]) ++b;
  s.b = b;
  s.first = (uint32_t)seq.chunk_start[b];
  s.nblk = (uint32_t)(seq.chunk_start[b + 1] - seq.chunk_start[b]);
  s.blk = blockIdx.x - s.first;
  const int64_t m = seq.cu[b + 1] - seq.cu[b] - keep_tail;
  const int64_t per = (m + s.nblk - 1) / s.nblk;
  s.lo = min(m, (int64_t)s.blk * per);
  s.hi = min(m, s.lo + per);
  s.sc = scores + seq.cu[b];
  return s;
}

__global__ __launch_bounds__(kThreads) void topk_init_kernel(SeqTable seq, int keep_tail, TopkWs ws,
                                                             int32_t* __restrict__ idx_out) {
  short_kernel_priority();
  const int b = blockIdx.y;
  const int tid = blockIdx.x * kThreads + threadIdx.x;
  const int stride = gridDim.x * kThreads;
  for (int i = tid; i < 3 * kBins; i += stride) ws.hist[(size_t)b * 3 * kBins + i] = 0u;
  const int64_t m = seq.cu[b + 1] - seq.cu[b] - keep_tail;
  for (int i = tid; i < keep_tail; i += stride)
    idx_out[seq.out_off[b] + seq.k[b] + i] = (int32_t)(m + i);
}

// exclusive scan of one value per thread over the workgroup (THREADS / 64 waves); returns the total.
// Shuffle scan inside each wave, then the wave totals through LDS.
template <int THREADS = kThreads>
__device__ inline uint32_t block_excl_scan(uint32_t v, uint32_t* sh /*[>= THREADS / 64]*/, uint32_t* excl) {
  constexpr int NWV = THREADS / 64;
  const int t = threadIdx.x, lane = t & 63, wv = t >> 6;
  uint32_t x = v;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t y = __shfl_up(x, off);
    if (lane >= off) x += y;
  }
  if (lane == 63) sh[wv] = x;
  __syncthreads();
  uint32_t base = 0u, total = 0u;
#pragma unroll
  for (int i = 0; i < NWV; ++i) {
    const uint32_t wsum = sh[i];
    if (i < wv) base += wsum;
    total += wsum;
  }
  *excl = base + x - v;
  __syncthreads();
  return total;
}

// Scan `nb` bins of a merged histogram from the top until `krem` keys are covered.
// Returns the bin (all threads), and how many keys lie above it.
template <int THREADS = kThreads>
__device__ inline void select_bin(const uint32_t* __restrict__ gh, int nb, uint32_t krem, uint32_t* scan /*[>= THREADS / 64]*/,
                                  uint32_t* res, uint32_t* bin_out, uint32_t* above_out) {
  const int t = threadIdx.x;
  const int per = nb / THREADS;   // 8 or 4 with 256 threads, 2 or 1 with 1024
  uint32_t mine[8];
  uint32_t sum = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    mine[i] = i < per ? gh[nb - 1 - (t * per + i)] : 0u;
    sum += mine[i];
  }
  if (t == 0) { res[0] = 0u; res[1] = 0u; }
  uint32_t excl;
  block_excl_scan<THREADS>(sum, scan, &excl);
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

// add a workgroup's LDS histogram into the merged one
__device__ inline void merge_hist(const uint32_t* h, int nb, uint32_t* __restrict__ gh) {
  for (int i = threadIdx.x; i < nb; i += kThreads)
    if (h[i]) atomicAdd(&gh[i], h[i]);
}

// A workgroup's share normally fits eight scores per thread; those are loaded into registers before the
// histogram scan so that the two latencies overlap.  Longer shares (capped workgroup count) loop instead.
constexpr int kPerThread = kTargetPerBlock / kThreads;

// thread t takes scores lo + t, lo + t + 256, ...
__device__ inline bool preload_strided(const Share& s, float (&v)[kPerThread]) {
  const bool fast = s.hi - s.lo <= kTargetPerBlock;
  if (fast) {
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
      const int64_t j = s.lo + threadIdx.x + i * kThreads;
      v[i] = j < s.hi ? s.sc[j] : 0.f;
    }
  }
  return fast;
}

template <class F>
__device__ inline void for_each_strided(const Share& s, const float (&v)[kPerThread], bool fast, F f) {
  if (fast) {
#pragma unroll
    for (int i = 0; i < kPerThread; ++i)
      if (s.lo + threadIdx.x + i * kThreads < s.hi) f(score_key(v[i]));
  } else {
    for (int64_t j = s.lo + threadIdx.x; j < s.hi; j += kThreads) f(score_key(s.sc[j]));
  }
}

__global__ __launch_bounds__(kThreads) void topk_hist0_kernel(const float* __restrict__ scores, SeqTable seq,
                                                              int keep_tail, TopkWs ws) {
  short_kernel_priority();
  __shared__ uint32_t h[kBins];
  const Share s = my_share(scores, seq, keep_tail);
  const int t = threadIdx.x;
  float v[kPerThread];
  const bool fast = preload_strided(s, v);
  for (int i = t; i < kBins; i += kThreads) h[i] = 0u;
  __syncthreads();
  for_each_strided(s, v, fast, [&](uint32_t key) { atomicAdd(&h[key >> 21], 1u); });
  __syncthreads();
  merge_hist(h, kBins, ws.hist + (size_t)s.b * 3 * kBins);
}

__global__ __launch_bounds__(kThreads) void topk_hist1_kernel(const float* __restrict__ scores, SeqTable seq,
                                                              int keep_tail, TopkWs ws) {
  short_kernel_priority();
  __shared__ uint32_t h[kBins];
  __shared__ uint32_t scan[4];
  __shared__ uint32_t res[2];
  const Share s = my_share(scores, seq, keep_tail);
  const int t = threadIdx.x;
  uint32_t* gh = ws.hist + (size_t)s.b * 3 * kBins;
  float v[kPerThread];
  const bool fast = preload_strided(s, v);
  for (int i = t; i < kBins; i += kThreads) h[i] = 0u;
  uint32_t bin0, above0;
  select_bin(gh, kBins, (uint32_t)seq.k[s.b], scan, res, &bin0, &above0);   // its barriers cover h[] = 0
  if (s.blk == 0 && t == 0) {
    ws.state[s.b * 4 + 0] = bin0;
    ws.state[s.b * 4 + 1] = (uint32_t)seq.k[s.b] - above0;
  }
  for_each_strided(s, v, fast, [&](uint32_t key) {
    if ((key >> 21) == bin0) atomicAdd(&h[(key >> 10) & (kBins - 1)], 1u);
  });
  __syncthreads();
  merge_hist(h, kBins, gh + kBins);
}

__global__ __launch_bounds__(kThreads) void topk_hist2_kernel(const float* __restrict__ scores, SeqTable seq,
                                                              int keep_tail, TopkWs ws) {
  short_kernel_priority();
  __shared__ uint32_t h[kLowBins];
  __shared__ uint32_t scan[4];
  __shared__ uint32_t res[2];
  __shared__ uint32_t above_cnt;
  const Share s = my_share(scores, seq, keep_tail);
  const int t = threadIdx.x;
  uint32_t* gh = ws.hist + (size_t)s.b * 3 * kBins;
  float v[kPerThread];
  const bool fast = preload_strided(s, v);
  for (int i = t; i < kLowBins; i += kThreads) h[i] = 0u;
  if (t == 0) above_cnt = 0u;
  const uint32_t bin0 = ws.state[s.b * 4 + 0], krem0 = ws.state[s.b * 4 + 1];
  uint32_t bin1, above1;
  select_bin(gh + kBins, kBins, krem0, scan, res, &bin1, &above1);   // its barriers cover h[], above_cnt = 0
  const uint32_t prefix = (bin0 << 11) | bin1;     // the top 22 bits of the k-th largest key
  if (s.blk == 0 && t == 0) {
    ws.state[s.b * 4 + 2] = prefix;
    ws.state[s.b * 4 + 3] = krem0 - above1;
  }
  uint32_t above = 0;
  for_each_strided(s, v, fast, [&](uint32_t key) {
    const uint32_t hi = key >> 10;
    above += hi > prefix;
    if (hi == prefix) atomicAdd(&h[key & (kLowBins - 1)], 1u);
  });
  if (above) atomicAdd(&above_cnt, above);
  __syncthreads();
  merge_hist(h, kLowBins, gh + 2 * kBins);
  // suffix sums of h: thread t owns the four bins 1023-4t .. 1020-4t (descending), scanned from the top
  uint32_t own[4];
  uint32_t sum = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) { own[i] = h[kLowBins - 1 - (4 * t + i)]; sum += own[i]; }
  uint32_t run;
  const uint32_t ncand = block_excl_scan(sum, scan, &run);
  if (ncand) {
    uint32_t* suf = ws.suf + (size_t)blockIdx.x * kLowBins;
#pragma unroll
    for (int i = 0; i < 4; ++i) { run += own[i]; suf[kLowBins - 1 - (4 * t + i)] = run; }
  }
  if (t == 0) {
    ws.meta[2 * (size_t)blockIdx.x] = above_cnt;
    ws.meta[2 * (size_t)blockIdx.x + 1] = ncand;
  }
}

__global__ __launch_bounds__(kThreads) void topk_write_kernel(const float* __restrict__ scores, SeqTable seq,
                                                              int keep_tail, TopkWs ws,
                                                              int32_t* __restrict__ idx_out) {
  short_kernel_priority();
  __shared__ uint32_t scan[4];
  __shared__ uint32_t res[2];
  __shared__ uint32_t cnt[2];
  const Share s = my_share(scores, seq, keep_tail);
  const int t = threadIdx.x;
  const uint32_t* gh = ws.hist + (size_t)s.b * 3 * kBins;
  if (t == 0) { cnt[0] = 0u; cnt[1] = 0u; }
  // this workgroup's share; thread t owns a contiguous slice of it (loaded before the histogram scan)
  const int64_t sub = (s.hi - s.lo + kThreads - 1) / kThreads;
  const int64_t tlo = min(s.hi, s.lo + t * sub), thi = min(s.hi, tlo + sub);
  const bool fast = sub <= kPerThread;
  float v[kPerThread];
  if (fast) {
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) v[i] = tlo + i < thi ? s.sc[tlo + i] : 0.f;
  }
  // counts of the first workgroup this thread will add up, also requested before the scan
  const bool has0 = (uint32_t)t < s.blk;
  const uint2 m0 = has0 ? *reinterpret_cast<const uint2*>(ws.meta + 2 * ((size_t)s.first + t)) : make_uint2(0u, 0u);
  const uint32_t prefix = ws.state[s.b * 4 + 2], krem1 = ws.state[s.b * 4 + 3];
  uint32_t t10, above2;
  select_bin(gh + 2 * kBins, kLowBins, krem1, scan, res, &t10, &above2);   // its barriers cover cnt[] = 0
  const uint32_t T = (prefix << 10) | t10;   // the k-th largest key
  const uint32_t need = krem1 - above2;      // how many keys equal to T are taken (lowest indices first)

  // selected keys in the workgroups before this one
  uint32_t g0 = 0, e0 = 0;
  auto add_block = [&](size_t w, uint32_t above, uint32_t ncand) {
    g0 += above;
    if (ncand) {
      const uint32_t* suf = ws.suf + w * kLowBins;
      const uint32_t ge = suf[t10];
      const uint32_t gt = t10 + 1 < (uint32_t)kLowBins ? suf[t10 + 1] : 0u;
      g0 += gt;
      e0 += ge - gt;
    }
  };
  if (has0) add_block((size_t)s.first + t, m0.x, m0.y);
  for (uint32_t i = t + kThreads; i < s.blk; i += kThreads) {
    const size_t w = (size_t)s.first + i;
    add_block(w, ws.meta[2 * w], ws.meta[2 * w + 1]);
  }
  if (g0) atomicAdd(&cnt[0], g0);
  if (e0) atomicAdd(&cnt[1], e0);

  uint32_t gt = 0, eq = 0;
  if (fast) {
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
      const uint32_t key = score_key(v[i]);
      gt += tlo + i < thi && key > T;
      eq += tlo + i < thi && key == T;
    }
  } else {
    for (int64_t j = tlo; j < thi; ++j) {
      const uint32_t key = score_key(s.sc[j]);
      gt += key > T;
      eq += key == T;
    }
  }
  uint32_t gt_before, eq_before;
  block_excl_scan(gt, scan, &gt_before);
  block_excl_scan(eq, scan, &eq_before);   // the barriers inside also order the cnt[] atomics above
  gt_before += cnt[0];
  eq_before += cnt[1];
  int32_t* out = idx_out + seq.out_off[s.b];
  auto place = [&](uint32_t key, int64_t j) {
    if (key > T) {
      out[gt_before + min(eq_before, need)] = (int32_t)j;
      ++gt_before;
    } else if (key == T) {
      if (eq_before < need) out[gt_before + eq_before] = (int32_t)j;
      ++eq_before;
    }
  };
  if (fast) {
#pragma unroll
    for (int i = 0; i < kPerThread; ++i)
      if (tlo + i < thi) place(score_key(v[i]), tlo + i);
  } else {
    for (int64_t j = tlo; j < thi; ++j) place(score_key(s.sc[j]), j);
  }
}

// Sum of the k largest scores of each of H equally long rows instead of their indices (the top-k mass of the pivot
// detector's sparsity, Eq. 5), after the first digit's histogram of every row has been built by whoever formed the
// rows.  Two kernels:
//   compact : every workgroup finds the first digit t0 of the k-th largest key from the row's histogram, adds up
//             its scores ABOVE that digit (a partial sum per workgroup, fixed order) and appends its scores WITH that
//             digit -- the candidates -- to the row's candidate list (one integer atomic per workgroup reserves the
//             place; the order of the list differs from run to run, and nothing below depends on it);
//   select  : one workgroup of 1024 threads per row takes the candidates (the first 32768 in registers), finds the two remaining
//             digits with histograms in LDS, and adds the candidates above the k-th key T as integers (they share
//             their exponent: exact, whatever the order), `need` copies of T's own value for the ties, and the
//             partial sums.
// Scores must be non-negative (in-degrees), rows at most 2^24 long.
__device__ inline float key_score(uint32_t key) {
  return __uint_as_float((key & 0x80000000u) ? (key & 0x7FFFFFFFu) : ~key);
}

constexpr int kSelThreads = 1024;             // the select kernel: sixteen waves per row
constexpr int kCandPerThread = 32;            // candidates one of its threads keeps in registers (32768 in all)

__global__ __launch_bounds__(kThreads) void mass_compact_kernel(const float* __restrict__ rows, int64_t n, uint32_t kk,
                                                                TopkWs ws, float* __restrict__ cand,
                                                                float* __restrict__ part_above) {
  short_kernel_priority();
  __shared__ uint32_t scan[4];
  __shared__ uint32_t res[2];
  __shared__ float red[kThreads];
  __shared__ float stage[kTargetPerBlock];
  __shared__ uint32_t cnt, gbase;
  const int p = blockIdx.x, h = blockIdx.y, P = gridDim.x, t = threadIdx.x, lane = t & 63;
  const float* d = rows + (int64_t)h * n;
  const int64_t lo = (int64_t)p * kTargetPerBlock;
  float x[kPerThread];
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) {   // loads first, the histogram scan under them
    const int64_t j = lo + t + i * kThreads;
    x[i] = j < n ? d[j] : 0.f;
  }
  if (t == 0) cnt = 0u;
  uint32_t* gh = ws.hist + (size_t)h * 3 * kBins;
  uint32_t t0, above0;
  select_bin(gh, kBins, kk, scan, res, &t0, &above0);   // its barriers cover cnt = 0
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) {
    const bool in = lo + t + i * kThreads < n;
    const uint32_t dg = score_key(x[i]) >> 21;
    if (in && dg > t0) sum += x[i];
    const bool c = in && dg == t0;
    const unsigned long long m = __ballot(c);
    if (m) {   // one LDS atomic per wave and step reserves the wave's places
      const int first = __ffsll((long long)m) - 1;
      uint32_t base = 0u;
      if (lane == first) base = atomicAdd(&cnt, (uint32_t)__popcll(m));
      base = __shfl(base, first);
      if (c) stage[base + (uint32_t)__popcll(m & ((1ull << lane) - 1ull))] = x[i];
    }
  }
  red[t] = sum;
  __syncthreads();
  for (int off = kThreads / 2; off > 0; off >>= 1) {
    if (t < off) red[t] += red[t + off];
    __syncthreads();
  }
  if (t == 0) {
    part_above[(int64_t)h * P + p] = red[0];
    gbase = cnt ? atomicAdd(&gh[kBins], cnt) : 0u;   // the row's candidate counter: first word of the (unused, zeroed) digit-1 histogram
    if (p == 0) {
      ws.state[h * 4 + 0] = t0;
      ws.state[h * 4 + 1] = kk - above0;
    }
  }
  __syncthreads();
  float* out = cand + (int64_t)h * n + gbase;
  for (uint32_t i = t; i < cnt; i += kThreads) out[i] = stage[i];
}

__global__ __launch_bounds__(kSelThreads) void mass_select_kernel(const float* __restrict__ cand, int64_t n, TopkWs ws,
                                                                  const float* __restrict__ part_above, int P,
                                                                  float* __restrict__ mass, float* __restrict__ tail) {
  short_kernel_priority();
  constexpr int NT = kSelThreads;
  __shared__ uint32_t hh[kBins];
  __shared__ uint32_t scan[NT / 64];
  __shared__ uint32_t res[2];
  __shared__ unsigned long long red64[NT];
  __shared__ float redf[NT];
  const int h = blockIdx.x, t = threadIdx.x;
  const uint32_t* gh = ws.hist + (size_t)h * 3 * kBins;
  const uint32_t t0 = ws.state[h * 4 + 0], krem0 = ws.state[h * 4 + 1];
  const uint32_t c0 = gh[kBins];   // candidates = keys whose first digit is t0
  const float* c = cand + (int64_t)h * n;
  float v[kCandPerThread];
#pragma unroll
  for (int r = 0; r < kCandPerThread; ++r) {
    const uint32_t i = (uint32_t)(r * NT + t);
    v[r] = i < c0 ? c[i] : 0.f;
  }
  auto each = [&](auto f) {
#pragma unroll
    for (int r = 0; r < kCandPerThread; ++r)
      if ((uint32_t)(r * NT + t) < c0) f(score_key(v[r]));
    for (uint32_t i = (uint32_t)(kCandPerThread * NT + t); i < c0; i += NT) f(score_key(c[i]));
  };
  for (int i = t; i < kBins; i += NT) hh[i] = 0u;
  __syncthreads();
  each([&](uint32_t key) { atomicAdd(&hh[(key >> 10) & (kBins - 1)], 1u); });
  __syncthreads();
  uint32_t t1, above1;
  select_bin<NT>(hh, kBins, krem0, scan, res, &t1, &above1);
  const uint32_t krem1 = krem0 - above1;
  for (int i = t; i < kLowBins; i += NT) hh[i] = 0u;
  __syncthreads();
  each([&](uint32_t key) {
    if (((key >> 10) & (kBins - 1)) == t1) atomicAdd(&hh[key & (kLowBins - 1)], 1u);
  });
  __syncthreads();
  uint32_t t2, above2;
  select_bin<NT>(hh, kLowBins, krem1, scan, res, &t2, &above2);
  const uint32_t T = (t0 << 21) | (t1 << 10) | t2;
  // every candidate carries the first digit t0 -- sign, exponent and two mantissa bits -- so the candidates share
  // one exponent and their 24-bit significands add up exactly as integers, in any order
  unsigned long long acc = 0ull;
  const uint32_t expo = (t0 >> 2) & 0xFFu;            // biased exponent (scores are non-negative)
  const uint32_t hidden = expo ? 0x00800000u : 0u;    // (subnormals have no hidden one)
  each([&](uint32_t key) {
    if (key > T) acc += (unsigned long long)((key & 0x007FFFFFu) | hidden);
  });
  red64[t] = acc;
  float pa = 0.f;
  for (int p = t; p < P; p += NT) pa += part_above[(int64_t)h * P + p];
  redf[t] = pa;
  __syncthreads();
  for (int off = NT / 2; off > 0; off >>= 1) {
    if (t < off) { red64[t] += red64[t + off]; redf[t] += redf[t + off]; }
    __syncthreads();
  }
  if (t == 0) {
    const double m = ldexp((double)red64[0], (int)(expo ? expo : 1u) - 150) + (double)(krem1 - above2) * (double)key_score(T) +
                     (double)redf[0];
    mass[2 * h + 1] = (float)m;
    tail[2 * h] = 0.f;
    tail[2 * h + 1] = 0.f;
  }
}

// upper bound of the workgroups one call launches
inline int share_target(int64_t total_tokens) {
  return total_tokens <= kSmallTotal ? kSmallTarget : kTargetPerBlock;
}

size_t max_blocks(int batch, int64_t total_tokens) {
  const size_t B = (size_t)(batch > 0 ? batch : 1);
  // monotone in total_tokens, so a workspace sized for a long call also serves every shorter one
  const int64_t small = total_tokens < kSmallTotal ? total_tokens : kSmallTotal;
  const int64_t by_small = small / kSmallTarget, by_large = total_tokens / kTargetPerBlock;
  size_t nb = (size_t)(by_small > by_large ? by_small : by_large) + B;
  if (nb > B * kMaxBlocksPerSeq) nb = B * kMaxBlocksPerSeq;
  return nb;
}

}  // namespace

size_t topk_workspace_bytes(int batch, int64_t total_tokens) {
  const size_t B = (size_t)(batch > 0 ? batch : 1);
  const size_t nb = max_blocks(batch, total_tokens);
  return align_up(sizeof(uint32_t) * 3 * B * kBins, 256) + align_up(sizeof(uint32_t) * 4 * B, 256) +
         align_up(sizeof(uint32_t) * kLowBins * nb, 256) + align_up(sizeof(uint32_t) * 2 * nb, 256);
}

// Device address and size of the static scratch on the CURRENT device (looked up once per device).
hipError_t topk_static_scratch(void** ptr, size_t* bytes) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* dev_ptr[kMaxDevices] = {};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (dev_ptr[dev] == nullptr) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (p == nullptr || ((uintptr_t)p & 255)) return hipErrorInvalidSymbol;
    dev_ptr[dev] = p;
  }
  *ptr = dev_ptr[dev];
  *bytes = kStaticScratchBytes;
  return hipSuccess;
}

// workgroups per sequence (about `target` scores each, at most kMaxBlocksPerSeq; none where nothing is
// selected) and the workspace carve
void topk_plan(const SeqTable& seq_in, int keep_tail, void* wsp, SeqTable* plan, TopkWs* ws, unsigned* blocks) {
  *plan = seq_in;
  const int B = plan->batch;
  const int target = share_target(plan->cu[B]);
  plan->chunk_start[0] = 0;
  for (int b = 0; b < B; ++b) {
    const int64_t m = plan->cu[b + 1] - plan->cu[b] - keep_tail;
    int64_t nblk = plan->k[b] > 0 ? ceil_div(m, target) : 0;
    if (nblk > kMaxBlocksPerSeq) nblk = kMaxBlocksPerSeq;
    plan->chunk_start[b + 1] = plan->chunk_start[b] + (int)nblk;
  }
  *blocks = (unsigned)plan->chunk_start[B];
  const size_t nb = max_blocks(B, plan->cu[B]);   // blocks <= nb: sum of ceil(m_b / target) <= total / target + B
  const size_t Bz = (size_t)(B > 0 ? B : 1);
  uint8_t* p = (uint8_t*)wsp;
  ws->hist = (uint32_t*)p;    p += align_up(sizeof(uint32_t) * 3 * Bz * kBins, 256);
  ws->state = (uint32_t*)p;   p += align_up(sizeof(uint32_t) * 4 * Bz, 256);
  ws->suf = (uint32_t*)p;     p += align_up(sizeof(uint32_t) * kLowBins * nb, 256);
  ws->meta = (uint32_t*)p;
}

hipError_t launch_topk_rest(const float* scores, const SeqTable& plan, int keep_tail, const TopkWs& ws,
                            unsigned blocks, int32_t* idx_out, hipStream_t st) {
  if (blocks == 0) return hipSuccess;
  hipLaunchKernelGGL(topk_hist1_kernel, dim3(blocks), dim3(kThreads), 0, st, scores, plan, keep_tail, ws);
  hipLaunchKernelGGL(topk_hist2_kernel, dim3(blocks), dim3(kThreads), 0, st, scores, plan, keep_tail, ws);
  hipLaunchKernelGGL(topk_write_kernel, dim3(blocks), dim3(kThreads), 0, st, scores, plan, keep_tail, ws, idx_out);
  return hipGetLastError();
}

// The sum of the kk largest scores of each of H rows of n scores (see mass_compact_kernel).  ws.hist[h][0][.] must
// hold the histogram of the rows' first digits and ws.hist[h][1][0] must be zero; cand: H x n floats of scratch;
// part_above: H x ceil(n / 2048) floats; the sums land in mass[2h + 1], and tail[2h], tail[2h + 1] are cleared.
hipError_t launch_topk_mass(const float* rows, int H, int64_t n, uint32_t kk, const TopkWs& ws, float* cand,
                            float* part_above, float* mass, float* tail, hipStream_t st) {
  if (H == 0 || n == 0) return hipSuccess;
  const unsigned P = (unsigned)((n + kTargetPerBlock - 1) / kTargetPerBlock);
  hipLaunchKernelGGL(mass_compact_kernel, dim3(P, (unsigned)H), dim3(kThreads), 0, st, rows, n, kk, ws, cand, part_above);
  hipLaunchKernelGGL(mass_select_kernel, dim3((unsigned)H), dim3(kSelThreads), 0, st, cand, n, ws, part_above, (int)P, mass,
                     tail);
  return hipGetLastError();
}

// seq.out_off must hold the output offsets, seq.k the budgets.
hipError_t launch_topk(const float* scores, const SeqTable& seq_in, int keep_tail, int32_t* idx_out,
                       void* wsp, hipStream_t st) {
  if (seq_in.batch == 0) return hipSuccess;
  SeqTable seq;
  TopkWs ws;
  unsigned blocks = 0;
  topk_plan(seq_in, keep_tail, wsp, &seq, &ws, &blocks);
  hipLaunchKernelGGL(topk_init_kernel, dim3(4, seq.batch), dim3(kThreads), 0, st, seq, keep_tail, ws, idx_out);
  if (blocks > 0)
    hipLaunchKernelGGL(topk_hist0_kernel, dim3(blocks), dim3(kThreads), 0, st, scores, seq, keep_tail, ws);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_topk_rest(scores, seq, keep_tail, ws, blocks, idx_out, st);
}

}  // namespace skv
