// Two small steps next to the selection:
//   block scores : S_block_k = sum of the centralities of the tokens of cache block k (paper Sec. 4.1,
//                  implementation details: block-level aggregation for paged caches)
//   positions    : P' = P[I_struct] (paper Eq. 11-12), the position ids that go with the hidden states
//                  kept at the structural indices (the hidden rows themselves go through the row gather).
#include "common.h"

namespace skv {
namespace {

// one thread per cache block, left-to-right fp32 sum (deterministic); seq.out_off holds the block offsets
__global__ __launch_bounds__(256) void block_scores_kernel(const float* __restrict__ scores, SeqTable seq,
                                                           int block, float* __restrict__ out) {
  const int64_t gb = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (gb >= seq.out_off[seq.batch]) return;
  int b = 0;
  for (int bb = 1; bb < seq.batch; ++bb) b += gb >= seq.out_off[bb];
  const int64_t n = seq.cu[b + 1] - seq.cu[b];
  const int64_t lo = (gb - seq.out_off[b]) * block;
  const int64_t hi = min(n, lo + block);
  const float* sc = scores + seq.cu[b];
  float s = 0.f;
  for (int64_t t = lo; t < hi; ++t) s += sc[t];
  out[gb] = s;
}

// pos_dst[row] = pos_src ? pos_src[cu[b] + idx[row]] : idx[row]; out-of-range indices read position 0
__global__ __launch_bounds__(256) void positions_kernel(const int64_t* __restrict__ pos_src, SeqTable seq,
                                                        const int32_t* __restrict__ idx,
                                                        int64_t* __restrict__ pos_dst) {
  const int64_t row = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (row >= seq.out_off[seq.batch]) return;
  int b = 0;
  for (int bb = 1; bb < seq.batch; ++bb) b += row >= seq.out_off[bb];
  const int64_t n = seq.cu[b + 1] - seq.cu[b];
  int64_t j = idx[row];
  if (j < 0 || j >= n) j = 0;
  pos_dst[row] = pos_src ? pos_src[seq.cu[b] + j] : j;
}

}  // namespace

hipError_t launch_block_scores(const float* scores, const SeqTable& seq, int block, float* out, hipStream_t st) {
  const int64_t nb = seq.out_off[seq.batch];
  if (nb == 0) return hipSuccess;
  hipLaunchKernelGGL(block_scores_kernel, dim3((unsigned)ceil_div(nb, 256)), dim3(256), 0, st, scores, seq, block,
                     out);
  return hipGetLastError();
}

hipError_t launch_positions(const int64_t* pos_src, const SeqTable& seq, const int32_t* idx, int64_t* pos_dst,
                            hipStream_t st) {
  const int64_t rows = seq.out_off[seq.batch];
  if (rows == 0) return hipSuccess;
  hipLaunchKernelGGL(positions_kernel, dim3((unsigned)ceil_div(rows, 256)), dim3(256), 0, st, pos_src, seq, idx,
                     pos_dst);
  return hipGetLastError();
}

}  // namespace skv
