// Internal declarations shared by the libstructkv translation units (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/structkv.h"

namespace skv {

// Record a thread-local error message and return the status.
structkv_status fail(structkv_status st, const char* fmt, ...);
void clear_error();

#define SKV_HIP_CHECK(expr)                                                              \
  do {                                                                                   \
    hipError_t _e = (expr);                                                              \
    if (_e != hipSuccess)                                                                \
      return skv::fail(STRUCTKV_ERR_HIP, "%s: %s", #expr, hipGetErrorString(_e));        \
  } while (0)

constexpr int kMaxBatch = STRUCTKV_MAX_BATCH;

// Per-sequence table passed by value in kernel arguments (host arrays never touch the device heap).
struct SeqTable {
  int64_t cu[kMaxBatch + 1];        // token offsets
  int64_t out_off[kMaxBatch + 1];   // output-row offsets (top-k / gather)
  int32_t k[kMaxBatch];             // top-k budget
  int32_t chunk_start[kMaxBatch + 1]; // cumulative key-chunk counts (scoring) / block counts (top-k)
  int32_t batch;
};

// The short, latency-bound kernels of a layer (combine, reduce, accumulate, top-k, gather) call this first.  When
// layers run as chains on several streams such a kernel shares a SIMD with waves of another layer's scoring
// kernel, which run at priority 1 while they have MFMAs to issue: at the default priority the short kernel would
// queue behind them, and it is the short kernels that sit on a chain's critical path.
#ifdef __HIPCC__
__device__ __forceinline__ void short_kernel_priority() { __builtin_amdgcn_s_setprio(2); }

// merge partial softmax statistics (M, Z, E) of two disjoint key sets, log2 domain:
//   Z = sum 2^(x-M),  E = sum 2^(x-M) (x-M)
__device__ inline void merge_stats(float& M, float& Z, float& E, float M2, float Z2, float E2) {
  const float Mn = fmaxf(M, M2);
  const float d1 = M - Mn, d2 = M2 - Mn;
  const float f1 = __builtin_amdgcn_exp2f(d1), f2 = __builtin_amdgcn_exp2f(d2);
  E = (E + d1 * Z) * f1 + (E2 + d2 * Z2) * f2;
  Z = Z * f1 + Z2 * f2;
  M = Mn;
}
#endif

// ---- selection (radix select on order-preserving keys) ---------------------------------------
constexpr int kTopkBins = 2048;      // digits 0 and 1: 11 bits each; digit 2: the last 10 bits

#ifdef __HIPCC__
// order-preserving 32-bit key of a score: larger float <=> larger key; -0.0 orders as +0.0
__device__ inline uint32_t score_key(float f) {
  uint32_t u = __float_as_uint(f);
  if (u == 0x80000000u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
#endif

struct TopkWs {
  uint32_t* hist;    // [B][3][kTopkBins]
  uint32_t* state;   // [B][4]: digit 0, k left after it, 22-bit prefix, k left after it
  uint32_t* suf;     // [blocks][1024]: suffix sums of the workgroup's last-digit histogram
  uint32_t* meta;    // [blocks][2]: keys above the 22-bit prefix, keys equal to it
};

// What the scoring call's small kernels do for the selection that follows it in a fused layer step: the
// combine kernel zeroes the digit histograms, the reduce kernel histograms the first digit of the scores
// it has just formed and writes the kept window's indices.
struct SelectFusion {
  uint32_t* hist;        // [B][3][kTopkBins]; NULL = no fusion
  int32_t* idx_out;
  int keep_tail;
};

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---- scoring plan: how one structkv_score_layer call is cut into workgroups ----------------
struct ScorePlan {
  int path;          // 0 = bf16 MFMA kernels, 1 = SIMT kernels
  int R;             // query rows per KV head: (H_q/G) * w
  int RPC;           // rows per row-chunk (a workgroup's share of R)
  int RC;            // row-chunks per KV head
  int KC;            // keys per key-chunk (one workgroup)
  int WK;            // partial statistics written per (row-chunk, key-chunk)
  int RB;            // MFMA path: 32-row blocks per wave (1, 2 or 4)
  int NW;            // MFMA path: waves (row-chunks) per workgroup sharing the key tiles (1, 2 or 4)
  int CP;            // pass-2 column-sum planes per KV head (the waves of a workgroup add theirs up first)
  int planes;        // MFMA path, pass 2: 0, or column-sum planes per WAVE (1: a wave's rows are one query head's
                     // window; 2: each of its two 32-row blocks is) instead of one per workgroup: CP = RC * planes =
                     // query heads per KV head, and the planes are the per-head in-degrees
  int kshare;        // consecutive groups that read the same K head (1 in ordinary scoring; the per-head
                     // scoring of the pivot metrics runs every query head as its own group: H_q/G)
  int64_t n_chunks;  // sum over sequences of ceil(n_b / KC): the stride of the per-chunk statistics
  int64_t grid_chunks;  // key chunks covered by ONE launch (= n_chunks unless the batch is scored in groups)
  int stream_k;      // MFMA path: 1 = fetch K with the non-temporal policy (K is larger than the memory-side cache)
  // workspace carve (byte offsets)
  size_t off_stats, off_lse, off_rowent, off_colsum, off_enthead, total_bytes;
};

// Launchers (each enqueues on `stream`, returns hipGetLastError()).
hipError_t launch_score_mfma_ring(const structkv_shape& s, const ScorePlan& p, const SeqTable& seq,
                                  const void* q, const void* k, int64_t ksh, int64_t kst, float c2,
                                  float* stats, const float* lse2, float* colsum, int64_t total,
                                  float* probs, int pass, hipStream_t st);
hipError_t launch_score_simt(const structkv_shape& s, const ScorePlan& p, const SeqTable& seq,
                             const void* q, const void* k, int64_t ksh, int64_t kst, float c2,
                             float* stats, const float* lse2, float* colsum, int64_t total,
                             float* probs, int pass, hipStream_t st);
// zero_words > 0: the kernel also clears that many 32-bit words at zero_ptr (the selection's histograms)
hipError_t launch_score_combine(const structkv_shape& s, const ScorePlan& p, const SeqTable& seq,
                                const float* stats, float* lse2, float* row_ent, uint32_t* zero_ptr,
                                int64_t zero_words, hipStream_t st);
// fuse != NULL: seq.k / seq.out_off must hold the selection's budgets and output offsets
hipError_t launch_score_reduce(const structkv_shape& s, const ScorePlan& p, const SeqTable& seq,
                               const float* colsum, int64_t total, float* indeg, const float* row_ent,
                               float* ent_head, float* entropy, float* centrality, float lambda, float inv_w,
                               const SelectFusion* fuse, hipStream_t st);
hipError_t launch_group_sums(const structkv_shape& s, const ScorePlan& p, const float* colsum, int64_t total,
                             float* groups, hipStream_t st);
hipError_t launch_accumulate(float* c, const float* d, int64_t n, float lambda, float inv_w, hipStream_t st);
hipError_t launch_topk(const float* scores, const SeqTable& seq, int keep_tail, int32_t* idx_out,
                       void* ws, hipStream_t st);
// The same selection split for a fused layer step.  topk_plan: workgroups per sequence (into plan->chunk_start)
// and the workspace carve.  launch_topk_rest: digits 1 and 2 and the ordered write, for a call whose histograms
// were zeroed, whose first digit was histogrammed and whose window indices were written by the scoring kernels
// (SelectFusion).
void topk_plan(const SeqTable& seq_in, int keep_tail, void* wsp, SeqTable* plan, TopkWs* ws, unsigned* blocks);
hipError_t launch_topk_rest(const float* scores, const SeqTable& plan, int keep_tail, const TopkWs& ws,
                            unsigned blocks, int32_t* idx_out, hipStream_t st);
size_t topk_workspace_bytes(int batch, int64_t total_tokens);
// the library's own top-k scratch on the current device (structkv_select_topk_static); no allocation
hipError_t topk_static_scratch(void** ptr, size_t* bytes);
// pivot metrics: partial sums part [H][kPivotMaxSlices][2] of every head, then the means over the heads
constexpr int kPivotMaxSlices = 64;
hipError_t launch_pivot_heads(const float* heads, int H, int64_t n, const int32_t* idx, int64_t k, float inv_w,
                              float* part, hipStream_t st);
hipError_t launch_zero_floats(float* p, int n, hipStream_t st);   // a fill kernel (safe inside a captured graph)
hipError_t launch_pivot_finish(const float* part, int H, int64_t n, float inv_w, int valid, float* sparsity,
                               float* variance, hipStream_t st);
// pivot metrics from the hot path's own scoring, whose pass 2 leaves the per-head in-degrees [H][n] in its
// column-sum planes: first radix digit + variance partials, the top-k mass by radix select, the means over the heads
int pivot_plane_shares(int64_t n);
hipError_t launch_pivot_planes(const float* heads, int H, int64_t n, float inv_w, uint32_t* hist, float* part,
                               hipStream_t st);
hipError_t launch_topk_mass(const float* rows, int H, int64_t n, uint32_t kk, const TopkWs& ws, float* cand,
                            float* part_above, float* mass, float* tail, hipStream_t st);
hipError_t launch_pivot_finish_planes(const float* var_part, int Pv, const float* mass_part, int Pm, const float* tail,
                                      int H, int64_t n, float inv_w, float* sparsity, float* variance, hipStream_t st);
hipError_t launch_block_scores(const float* scores, const SeqTable& seq, int block, float* out, hipStream_t st);
hipError_t launch_positions(const int64_t* pos_src, const SeqTable& seq, const int32_t* idx, int64_t* pos_dst,
                            hipStream_t st);
hipError_t launch_gather(const void* k_src, const void* v_src, int64_t ssh, int64_t sst, void* k_dst,
                         void* v_dst, int64_t dsh, int64_t dst_, int G, int row_bytes,
                         const SeqTable& seq, const int32_t* idx, hipStream_t st);

}  // namespace skv
