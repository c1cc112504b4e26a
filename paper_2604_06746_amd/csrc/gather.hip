// Index-driven K/V row gather (paper Alg. 1 line 17: the decoupled cache store).
// One thread moves one vector unit (16, 4 or 2 bytes) of one row; consecutive threads cover a row,
// then the next row, so reads are 256-byte row bursts and writes are fully contiguous.  One unit per
// thread measured fastest on MI355X (about half the time of 2-8 units per thread): the copy is a
// single wave of requests, and more, lighter waves issue it sooner than fewer waves with deeper queues.
#include "common.h"

namespace skv {
namespace {

constexpr int kThreads = 256;
constexpr int kUnroll = 1;   // units per thread

// Every row is read once and written once and neither is touched again by this kernel: the 16-byte units move with
// the non-temporal policy, which keeps them from displacing what the next layer's scoring will read (measured on
// back-to-back launches: 16.0 -> 14.2 us at 34 MB, 52.6 -> 47.2 us at 221 MB; non-temporal stores alone were slower
// at 34 MB).  The builtins take clang's own vector types, not HIP's structs.
typedef unsigned __attribute__((ext_vector_type(4))) u32x4;
template <typename V> __device__ inline V load_once(const uint8_t* p) {
  if constexpr (sizeof(V) == 16) {
    const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    V r; r.x = t[0]; r.y = t[1]; r.z = t[2]; r.w = t[3];
    return r;
  } else {
    return *reinterpret_cast<const V*>(p);
  }
}
template <typename V> __device__ inline void store_once(uint8_t* p, V v) {
  if constexpr (sizeof(V) == 16) {
    const u32x4 t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, reinterpret_cast<u32x4*>(p));
  } else {
    *reinterpret_cast<V*>(p) = v;
  }
}

template <typename V, bool POW2>
__global__ __launch_bounds__(kThreads) void gather_rows_kernel(
    const uint8_t* __restrict__ src0, const uint8_t* __restrict__ src1, uint8_t* __restrict__ dst0,
    uint8_t* __restrict__ dst1, int64_t ssh, int64_t sst, int64_t dsh, int64_t dst_tok, uint32_t units_per_row,
    uint32_t upr_shift, uint32_t total_units, SeqTable seq, const int32_t* __restrict__ idx) {
  short_kernel_priority();
  const int g = blockIdx.y;
  const uint8_t* src = (blockIdx.z == 0 ? src0 : src1) + (int64_t)g * ssh;
  uint8_t* dst = (blockIdx.z == 0 ? dst0 : dst1) + (int64_t)g * dsh;
  const uint32_t base = blockIdx.x * (uint32_t)(kThreads * kUnroll) + threadIdx.x;
  V val[kUnroll];
  int64_t doff[kUnroll];
#pragma unroll
  for (int i = 0; i < kUnroll; ++i) {
    const uint32_t lin = base + (uint32_t)i * kThreads;
    doff[i] = -1;
    if (lin < total_units) {
      const uint32_t row = POW2 ? lin >> upr_shift : lin / units_per_row;
      const uint32_t u = lin - row * units_per_row;
      int b = 0;
      for (int bb = 1; bb < seq.batch; ++bb) b += (int64_t)row >= seq.out_off[bb];
      const int64_t n = seq.cu[b + 1] - seq.cu[b];
      int64_t j = idx[row];
      if (j < 0 || j >= n) j = 0;
      val[i] = load_once<V>(src + (seq.cu[b] + j) * sst + (int64_t)u * sizeof(V));
      doff[i] = (int64_t)row * dst_tok + (int64_t)u * sizeof(V);
    }
  }
#pragma unroll
  for (int i = 0; i < kUnroll; ++i)
    if (doff[i] >= 0) store_once<V>(dst + doff[i], val[i]);
}

}  // namespace

// strides in BYTES here
hipError_t launch_gather(const void* k_src, const void* v_src, int64_t ssh, int64_t sst, void* k_dst,
                         void* v_dst, int64_t dsh, int64_t dst_tok, int G, int row_bytes,
                         const SeqTable& seq, const int32_t* idx, hipStream_t st) {
  const int64_t rows = seq.out_off[seq.batch];
  if (rows == 0 || G == 0) return hipSuccess;
  const uint8_t* s0 = (const uint8_t*)k_src;
  const uint8_t* s1 = (const uint8_t*)v_src;
  uint8_t* d0 = (uint8_t*)k_dst;
  uint8_t* d1 = (uint8_t*)v_dst;
  int nz = 2;
  if (s0 == nullptr) { s0 = s1; d0 = d1; nz = 1; }
  else if (s1 == nullptr) { nz = 1; }
  if (s0 == nullptr) return hipSuccess;
  uintptr_t bits = (uintptr_t)s0 | (uintptr_t)d0 | (uintptr_t)ssh | (uintptr_t)sst | (uintptr_t)dsh |
                   (uintptr_t)dst_tok | (uintptr_t)row_bytes;
  if (nz == 2) bits |= (uintptr_t)s1 | (uintptr_t)d1;
  const int vec = (bits & 15) == 0 ? 16 : ((bits & 3) == 0 ? 4 : 2);
  const int upr = row_bytes / vec;
  const int64_t total_units = rows * upr;
  if (total_units >= ((int64_t)1 << 31) - kThreads * kUnroll) return hipErrorInvalidValue;  // host checks this first
  const bool pow2 = (upr & (upr - 1)) == 0;
  uint32_t sh = 0;
  while ((1 << sh) < upr) ++sh;
  dim3 grid((unsigned)ceil_div(total_units, kThreads * kUnroll), (unsigned)G, (unsigned)nz), blk(kThreads);
#define SKV_GATHER(V, P)                                                                              \
  hipLaunchKernelGGL((gather_rows_kernel<V, P>), grid, blk, 0, st, s0, s1, d0, d1, ssh, sst, dsh, dst_tok, \
                     (uint32_t)upr, sh, (uint32_t)total_units, seq, idx)
  if (vec == 16) { if (pow2) SKV_GATHER(uint4, true); else SKV_GATHER(uint4, false); }
  else if (vec == 4) { if (pow2) SKV_GATHER(uint32_t, true); else SKV_GATHER(uint32_t, false); }
  else { if (pow2) SKV_GATHER(uint16_t, true); else SKV_GATHER(uint16_t, false); }
#undef SKV_GATHER
  return hipGetLastError();
}

}  // namespace skv
