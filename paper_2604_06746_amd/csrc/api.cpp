// C-ABI entry points of libstructkv: argument validation, work planning, workspace carving and
// kernel launches.  No device memory is allocated here; nothing synchronises the device.
#include "common.h"
#include "../../include/structkv_debug.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>

namespace skv {

static thread_local char g_err[512] = "";

structkv_status fail(structkv_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return st;
}
void clear_error() { g_err[0] = 0; }

namespace {

structkv_status check_shape(const structkv_shape* s) {
  if (!s) return fail(STRUCTKV_ERR_INVALID_ARG, "shape is NULL");
  if (s->n_q_heads < 1 || s->n_kv_heads < 1 || s->n_q_heads % s->n_kv_heads)
    return fail(STRUCTKV_ERR_INVALID_ARG, "n_kv_heads (%d) must be >= 1 and divide n_q_heads (%d)",
                s->n_kv_heads, s->n_q_heads);
  if (s->window < 1) return fail(STRUCTKV_ERR_INVALID_ARG, "window must be >= 1, got %d", s->window);
  if (s->head_dim < 1) return fail(STRUCTKV_ERR_INVALID_ARG, "head_dim must be >= 1, got %d", s->head_dim);
  if (s->head_dim > 256) return fail(STRUCTKV_ERR_UNSUPPORTED, "head_dim %d > 256", s->head_dim);
  if (s->dtype != STRUCTKV_DTYPE_F32 && s->dtype != STRUCTKV_DTYPE_BF16)
    return fail(STRUCTKV_ERR_UNSUPPORTED, "dtype %d is neither f32 (0) nor bf16 (1)", s->dtype);
  if (s->causal != 0 && s->causal != 1) return fail(STRUCTKV_ERR_INVALID_ARG, "causal must be 0 or 1");
  if (!(s->scale >= 0.f) || !std::isfinite(s->scale))
    return fail(STRUCTKV_ERR_INVALID_ARG, "scale must be finite and >= 0 (0 = 1/sqrt(head_dim))");
  if ((int64_t)(s->n_q_heads / s->n_kv_heads) * s->window > 65536)
    return fail(STRUCTKV_ERR_UNSUPPORTED, "more than 65536 query rows per KV head");
  return STRUCTKV_OK;
}

structkv_status check_cu(int32_t batch, const int64_t* cu, SeqTable* seq) {
  if (batch < 0) return fail(STRUCTKV_ERR_INVALID_ARG, "batch must be >= 0, got %d", batch);
  if (batch > kMaxBatch)
    return fail(STRUCTKV_ERR_UNSUPPORTED, "batch %d exceeds STRUCTKV_MAX_BATCH (%d)", batch, kMaxBatch);
  if (!cu) return fail(STRUCTKV_ERR_INVALID_ARG, "cu_seqlens is NULL");
  if (cu[0] != 0) return fail(STRUCTKV_ERR_INVALID_ARG, "cu_seqlens[0] must be 0");
  memset(seq, 0, sizeof(*seq));
  seq->batch = batch;
  for (int b = 0; b < batch; ++b) {
    if (cu[b + 1] < cu[b]) return fail(STRUCTKV_ERR_INVALID_ARG, "cu_seqlens decreases at %d", b);
    if (cu[b + 1] - cu[b] >= ((int64_t)1 << 31))
      return fail(STRUCTKV_ERR_UNSUPPORTED, "sequence %d has 2^31 or more tokens", b);
  }
  for (int b = 0; b <= batch; ++b) seq->cu[b] = cu[b];
  return STRUCTKV_OK;
}

// Decide path, tiling and workspace layout.  `n_chunk_bound` < 0: exact from seq; otherwise an upper bound.
void make_plan(const structkv_shape& s, const SeqTable* seq, int batch, int64_t total, bool mfma_ok,
               ScorePlan* p, bool planes = false) {
  const int gs = s.n_q_heads / s.n_kv_heads;
  p->R = gs * s.window;
  p->kshare = 1;
  p->path = mfma_ok ? 0 : 1;
  p->planes = 0;
  // a K of at least the memory-side cache's 256 MiB streams through the caches (see the kernel's NT parameter)
  p->stream_k = p->path == 0 && total * s.n_kv_heads * s.head_dim * 2 >= ((int64_t)256 << 20);
  if (p->path == 0) {
    // MFMA kernels: one wave owns RPC = 32*RB <= 64 rows and a chunk of KC keys.  A KV group with more rows is
    // cut into row-chunks whose waves form one four-wave workgroup and share the key tiles.  More than 128 rows
    // (GQA 4 x w 64 = 256): row-chunks of 64 rows; at 168 registers three such waves fit a SIMD, and waves of 64
    // rows beat waves of 128 rows (256 registers, two per SIMD) by 6 %: more waves hide more of the MFMA -> softmax
    // latency.  65..128 rows (GQA 4 x w 32): row-chunks of 32 rows, again four waves -- against two waves of 64
    // rows twice as many waves for the same keys per workgroup (a 32K-token layer then puts two waves on every
    // SIMD instead of one: both passes -20 %) and a workgroup may take 2048 keys instead of 1024, so that sizes
    // between whole rounds of resident workgroups quantise better (48K..512K tokens: -2 % .. -10 %, except
    // exactly 128K, one full round either way: +2 %).  With 256 rows, 32-row waves LOSE 10-20 % (each wave reads
    // the whole key tile from LDS for half the rows).
    p->RB = (p->R > 32 && p->R <= 64) || p->R > 128 ? 2 : 1;
    p->RPC = 32 * p->RB; p->WK = 1;
    p->RC = (int)ceil_div(p->R, p->RPC);
    p->NW = p->RC > 1 ? 4 : 1;
    // keys per workgroup: whole rounds of resident workgroups over the chip (256 CUs x 3 four-wave or 8 one-wave
    // workgroups), at most kMaxKC keys each, and at least 256 so that loading the query operands
    // (RPC*d*2 bytes per wave) stays small against the K stream
    // per-head planes: a wave's RPC rows must be one head's window (w = RPC) or two (w = 32, RPC = 64)
    if (planes && (s.window == p->RPC || (s.window == 32 && p->RPC == 64 && gs % 2 == 0)))
      p->planes = p->RPC / s.window;
    // the kernels' LDS column-sum capacity
    const int64_t kMaxKC = p->planes ? (p->NW == 4 ? (p->planes == 1 ? 1376 : 736) : 1024 / p->planes)
                                     : (p->NW == 4 ? 2048 : 896);
    const int64_t slots = 256 * (p->NW == 4 ? 3 : 8);
    const int64_t wg_per_chunk = s.n_kv_heads * ceil_div(p->RC, p->NW);
    const int64_t chunks_per_round = slots / wg_per_chunk > 0 ? slots / wg_per_chunk : 1;
    const int64_t rounds = ceil_div(total > 0 ? total : 1, chunks_per_round * kMaxKC);
    int64_t kc = ceil_div(ceil_div(total, chunks_per_round * rounds), 32) * 32;
    // Short inputs: at least 512 keys per workgroup while that still fills half of the resident slots (a
    // workgroup's fixed costs -- query operands, the first tiles' latency, the partial results -- weigh as much
    // as 6-8 tiles; with layers running as chains the other half of the chip is another layer's), else 256.
    const int64_t kc_min = ceil_div(total, 512) * wg_per_chunk * 2 >= slots ? 512 : 256;
    if (kc < kc_min) kc = kc_min;
    if (kc > kMaxKC) kc = kMaxKC;
    p->KC = (int)kc;
    p->CP = p->planes ? p->RC * p->planes : (int)ceil_div(p->RC, p->NW);
  } else {
    p->RPC = 16; p->RB = 0; p->NW = 0; p->WK = 1;
    p->RC = (int)ceil_div(p->R, p->RPC);
    p->KC = 256;
    p->CP = p->RC;
  }
  if (seq) {
    p->n_chunks = 0;
    for (int b = 0; b < batch; ++b) p->n_chunks += ceil_div(seq->cu[b + 1] - seq->cu[b], p->KC);
  } else {
    p->n_chunks = total / 256 + batch;   // KC is at least 256 on either path
  }
  p->grid_chunks = p->n_chunks;
  const size_t GRC = (size_t)s.n_kv_heads * p->RC;
  size_t off = 0;
  p->off_stats = off;   off += align_up(sizeof(float) * GRC * (size_t)p->n_chunks * p->WK * 3 * p->RPC, 256);
  p->off_lse = off;     off += align_up(sizeof(float) * (size_t)batch * s.n_q_heads * s.window, 256);
  p->off_rowent = off;  off += align_up(sizeof(float) * (size_t)batch * s.n_q_heads * s.window, 256);
  p->off_colsum = off;  off += align_up(sizeof(float) * (size_t)s.n_kv_heads * p->CP * (size_t)total, 256);
  p->off_enthead = off; off += align_up(sizeof(float) * (size_t)batch * s.n_q_heads, 256);
  p->total_bytes = off;
}

bool mfma_eligible(const structkv_shape& s, const void* q, const void* k, int64_t ksh, int64_t kst) {
  if (s.dtype != STRUCTKV_DTYPE_BF16) return false;
  if (s.head_dim != 64 && s.head_dim != 128) return false;
  if (s.causal && (s.window % 32) != 0) return false;   // the MFMA kernels' causal masks assume whole 32-row blocks per head
  if ((((uintptr_t)q | (uintptr_t)k) & 15) != 0) return false;
  if ((ksh % 8) != 0 || (kst % 8) != 0) return false;
  return true;
}

// Keys (bytes of one layer's K) that a group of sequences may hold when a batch is scored group by group so that
// the second pass over a group's keys is served by the 256 MB memory-side cache.
constexpr int64_t kCacheGroupBytes = (int64_t)192 << 20;

// What a scoring call does beyond structkv_score_layer itself.
struct ScoreOpts {
  int step_mask = 15;          // which of the four kernels are enqueued (profiling hook)
  float* centrality = nullptr; // the reduce kernel also applies C <- lambda C + inv_w D
  float lambda = 0.f, inv_w = 0.f;
  float* groups = nullptr;     // per-KV-head in-degree [G][total]
  int kshare = 1;              // consecutive groups that read one K head (per-head scoring)
  bool force_simt = false;     // test hook: SIMT kernels even where the MFMA kernels apply
  bool cache_groups = false;   // measurement hook: score a batch in cache-sized groups of sequences
  bool flip_stream_k = false;  // test hook: the other cache policy for the K tiles than the size rule picks
  float* probs = nullptr;      // test hook: the attention rows themselves
  const SelectFusion* fuse = nullptr;   // fused layer step: the small kernels also start the selection
  bool planes = false;         // pass 2 keeps one column-sum plane per query head (the pivot metrics' input)
  uint32_t* zero_ptr = nullptr;   // words the combine kernel clears on the way (someone's histograms)
  int64_t zero_words = 0;
};

structkv_status run_score(const structkv_shape* shape, const void* q_win, const void* k, int64_t ksh,
                          int64_t kst, const SeqTable& seq_in, float* indeg, float* entropy,
                          float* ent_head_out, void* ws, size_t ws_bytes, hipStream_t st, const ScoreOpts& o) {
  const structkv_shape& s = *shape;
  SeqTable seq = seq_in;
  const int B = seq.batch;
  const int64_t total = seq.cu[B];
  ScorePlan p;
  make_plan(s, &seq, B, total, !o.force_simt && mfma_eligible(s, q_win, k, ksh, kst), &p, o.planes);
  if (o.planes && !p.planes) return fail(STRUCTKV_ERR_UNSUPPORTED, "per-head planes need the MFMA kernels and a window of 32 or 64");
  p.kshare = o.kshare;   // s.n_kv_heads % kshare == 0 (the caller's business)
  if (o.flip_stream_k && p.path == 0) p.stream_k = !p.stream_k;
  if (p.total_bytes > ws_bytes)
    return fail(STRUCTKV_ERR_WORKSPACE, "workspace has %zu bytes, this call needs %zu", ws_bytes, p.total_bytes);
  if ((int64_t)s.n_kv_heads * p.RC * p.n_chunks >= ((int64_t)1 << 31))
    return fail(STRUCTKV_ERR_UNSUPPORTED, "too many workgroups for one launch");
  seq.chunk_start[0] = 0;
  for (int b = 0; b < B; ++b) {
    const int64_t c = seq.chunk_start[b] + ceil_div(seq.cu[b + 1] - seq.cu[b], p.KC);
    if (c >= ((int64_t)1 << 31)) return fail(STRUCTKV_ERR_UNSUPPORTED, "too many key chunks");
    seq.chunk_start[b + 1] = (int32_t)c;
  }
  uint8_t* w8 = (uint8_t*)ws;
  float* stats = (float*)(w8 + p.off_stats);
  float* lse2 = (float*)(w8 + p.off_lse);
  float* colsum = (float*)(w8 + p.off_colsum);
  float* row_ent = (float*)(w8 + p.off_rowent);
  float* ent_head = ent_head_out ? ent_head_out : (float*)(w8 + p.off_enthead);
  const float scale = s.scale > 0.f ? s.scale : 1.0f / std::sqrt((float)s.head_dim);
  const float c2 = (float)((double)scale * 1.4426950408889634);
  auto pass = p.path == 0 ? launch_score_mfma_ring : launch_score_simt;

  // Cache-resident second pass (a measurement hook, not the default).  A batch whose keys exceed the 256 MB
  // memory-side cache can be scored in groups of consecutive sequences whose keys fit it: pass 1, combine and
  // pass 2 of a group back to back, so that pass 2 finds in the cache what pass 1 has just streamed.  The plan
  // (keys per workgroup, summation order) stays the whole batch's, so every output is bit-identical to the
  // ungrouped call.  Measured on the ragged batch of 8 (1.1 GB of keys per layer, window 32, where HBM binds): a
  // pass 2 that follows its pass 1 directly is 13-15 % shorter for a lone sequence, but six groups cost 15 more
  // launches per layer, each with its own ramp and
  // tail on a chip that one launch over the whole batch keeps full: 20.6 ms per sweep against 16.9 ms on one
  // stream (18.6 ms with every group planned as a batch of its own), no gain with layers on several streams,
  // whose K streams share the cache anyway.  So structkv_score_layer scores a batch with one launch per kernel.
  int group_end[kMaxBatch + 1];
  int n_groups = 0;
  {
    const int64_t bytes_per_token = (int64_t)s.n_kv_heads * s.head_dim * (s.dtype == STRUCTKV_DTYPE_BF16 ? 2 : 4);
    const bool grouped = o.cache_groups && p.path == 0 && B > 1 && o.probs == nullptr &&
                         total * bytes_per_token > kCacheGroupBytes;
    if (!grouped) {
      group_end[n_groups++] = B;
    } else {
      int64_t in_group = 0;
      for (int b = 0; b < B; ++b) {
        const int64_t nb = (seq.cu[b + 1] - seq.cu[b]) * bytes_per_token;
        if (b > 0 && in_group > 0 && in_group + nb > kCacheGroupBytes) { group_end[n_groups++] = b; in_group = 0; }
        in_group += nb;
      }
      group_end[n_groups++] = B;
    }
  }
  const size_t esz = s.dtype == STRUCTKV_DTYPE_BF16 ? 2 : 4;
  // the launches of group gi for the steps in `mask` (1: pass 1, 2: combine, 4: pass 2)
  auto run_group = [&](int gi, int mask) -> structkv_status {
    const int b0 = gi == 0 ? 0 : group_end[gi - 1], b1 = group_end[gi];
    SeqTable sub = seq;
    ScorePlan gp = p;
    const uint8_t* q_g = (const uint8_t*)q_win;
    float *stats_g = stats, *lse2_g = lse2, *row_ent_g = row_ent;
    if (n_groups > 1) {
      const int32_t c0 = seq.chunk_start[b0];
      sub.batch = b1 - b0;
      for (int i = 0; i <= b1 - b0; ++i) {
        sub.cu[i] = seq.cu[b0 + i];                           // absolute token offsets: K and the column sums are not shifted
        sub.chunk_start[i] = seq.chunk_start[b0 + i] - c0;    // launch-local key chunks
      }
      gp.grid_chunks = seq.chunk_start[b1] - c0;
      gp.stream_k = 0;                                        // a group's keys are meant to stay in the cache
      q_g += (size_t)b0 * s.n_q_heads * s.window * s.head_dim * esz;
      stats_g += (size_t)c0 * p.WK * 3 * p.RPC;               // chunk c of row-chunk r sits at (r * n_chunks + c) * WK * 3 * RPC
      lse2_g += (size_t)b0 * s.n_q_heads * s.window;
      row_ent_g += (size_t)b0 * s.n_q_heads * s.window;
    }
    if (mask & 1)
      SKV_HIP_CHECK(pass(s, gp, sub, q_g, k, ksh, kst, c2, stats_g, lse2_g, colsum, total, nullptr, 1, st));
    if (mask & 2)
      SKV_HIP_CHECK(launch_score_combine(s, gp, sub, stats_g, lse2_g, row_ent_g,
                                         gi != 0 ? nullptr : (o.fuse ? o.fuse->hist : o.zero_ptr),
                                         gi != 0 ? 0 : (o.fuse ? (int64_t)3 * kTopkBins * B : o.zero_words), st));
    if (mask & 4)
      SKV_HIP_CHECK(pass(s, gp, sub, q_g, k, ksh, kst, c2, stats_g, lse2_g, colsum, total, o.probs, 2, st));
    return STRUCTKV_OK;
  };
  if ((o.step_mask & 7) == 7) {
    for (int gi = 0; gi < n_groups; ++gi) {
      const structkv_status gs = run_group(gi, 7);
      if (gs != STRUCTKV_OK) return gs;
    }
  } else {   // profiling hook: one kind of kernel at a time, over all groups
    for (int bit = 1; bit <= 4; bit <<= 1)
      if (o.step_mask & bit)
        for (int gi = 0; gi < n_groups; ++gi) {
          const structkv_status gs = run_group(gi, bit);
          if (gs != STRUCTKV_OK) return gs;
        }
  }
  if (o.step_mask & 8)
    SKV_HIP_CHECK(launch_score_reduce(s, p, seq, colsum, total, indeg, row_ent, ent_head, entropy, o.centrality,
                                      o.lambda, o.inv_w, o.fuse, st));
  if (o.groups) SKV_HIP_CHECK(launch_group_sums(s, p, colsum, total, o.groups, st));
  return STRUCTKV_OK;
}

}  // namespace
}  // namespace skv

using namespace skv;

extern "C" {

const char* structkv_last_error(void) { return g_err; }

int32_t structkv_version(void) { return 204; }

size_t structkv_workspace_bytes(const structkv_shape* shape, int32_t batch, int64_t total_tokens) {
  if (batch < 0 || batch > kMaxBatch || total_tokens < 0) return 0;
  size_t need = topk_workspace_bytes(batch, total_tokens);
  if (shape) {
    if (check_shape(shape) != STRUCTKV_OK) return 0;
    for (int mfma = 0; mfma < 2; ++mfma) {
      ScorePlan p;
      make_plan(*shape, nullptr, batch, total_tokens, mfma == 1, &p);
      if (p.total_bytes > need) need = p.total_bytes;
    }
  }
  return align_up(need, 256);
}

static structkv_status score_layer_impl(const structkv_shape* shape, const void* q_win, const void* k,
                                        int64_t k_stride_head, int64_t k_stride_tok, int32_t batch,
                                        const int64_t* cu_seqlens, float* indeg_out, float* entropy_out,
                                        float* entropy_per_head_out, void* workspace, size_t workspace_bytes,
                                        void* stream, const ScoreOpts& opts = ScoreOpts(),
                                        const SeqTable* selection = nullptr) {
  clear_error();
  structkv_status st = check_shape(shape);
  if (st != STRUCTKV_OK) return st;
  SeqTable seq;
  st = check_cu(batch, cu_seqlens, &seq);
  if (st != STRUCTKV_OK) return st;
  if (batch == 0) return STRUCTKV_OK;
  if (selection) {   // a fused layer step: budgets and output offsets of the selection travel with the table
    for (int b = 0; b < batch; ++b) { seq.k[b] = selection->k[b]; seq.out_off[b] = selection->out_off[b]; }
    seq.out_off[batch] = selection->out_off[batch];
  }
  const int64_t total = seq.cu[batch];
  if (!q_win || !entropy_out) return fail(STRUCTKV_ERR_INVALID_ARG, "q_win or entropy_out is NULL");
  if (total > 0 && (!k || !indeg_out)) return fail(STRUCTKV_ERR_INVALID_ARG, "k or indeg_out is NULL");
  if (k_stride_tok < shape->head_dim)
    return fail(STRUCTKV_ERR_INVALID_ARG, "k_stride_tok (%lld) < head_dim", (long long)k_stride_tok);
  if (shape->n_kv_heads > 1 && k_stride_head < 0) return fail(STRUCTKV_ERR_INVALID_ARG, "k_stride_head < 0");
  for (int b = 0; b < batch; ++b) {
    const int64_t n = seq.cu[b + 1] - seq.cu[b];
    if (shape->causal && n != 0 && n < shape->window)
      return fail(STRUCTKV_ERR_INVALID_ARG, "sequence %d: causal scoring needs n (%lld) >= window (%d)", b,
                  (long long)n, shape->window);
  }
  if (!workspace || ((uintptr_t)workspace & 255))
    return fail(STRUCTKV_ERR_WORKSPACE, "workspace is NULL or not 256-byte aligned");
  return run_score(shape, q_win, k, k_stride_head, k_stride_tok, seq, indeg_out, entropy_out,
                   entropy_per_head_out, workspace, workspace_bytes, (hipStream_t)stream, opts);
}

structkv_status structkv_score_layer(const structkv_shape* shape, const void* q_win, const void* k,
                                     int64_t k_stride_head, int64_t k_stride_tok, int32_t batch,
                                     const int64_t* cu_seqlens, float* indeg_out, float* entropy_out,
                                     float* entropy_per_head_out, void* workspace, size_t workspace_bytes,
                                     void* stream) {
  return score_layer_impl(shape, q_win, k, k_stride_head, k_stride_tok, batch, cu_seqlens, indeg_out,
                          entropy_out, entropy_per_head_out, workspace, workspace_bytes, stream);
}

structkv_status structkv_score_layer_accumulate(const structkv_shape* shape, const void* q_win, const void* k,
                                                int64_t k_stride_head, int64_t k_stride_tok, int32_t batch,
                                                const int64_t* cu_seqlens, float* indeg_out, float* centrality,
                                                float lambda, float inv_w, float* entropy_out,
                                                float* entropy_per_head_out, void* workspace,
                                                size_t workspace_bytes, void* stream) {
  clear_error();
  if (!(lambda > 0.f && lambda <= 1.f)) return fail(STRUCTKV_ERR_INVALID_ARG, "lambda must be in (0,1]");
  if (!(inv_w > 0.f) || !std::isfinite(inv_w)) return fail(STRUCTKV_ERR_INVALID_ARG, "inv_w must be > 0");
  if (batch != 0 && (!centrality || ((uintptr_t)centrality & 3)))
    return fail(STRUCTKV_ERR_INVALID_ARG, "centrality is NULL or not 4-byte aligned");
  if (centrality && centrality == indeg_out)
    return fail(STRUCTKV_ERR_INVALID_ARG, "centrality must not alias indeg_out");
  ScoreOpts o;
  o.centrality = centrality; o.lambda = lambda; o.inv_w = inv_w;
  return score_layer_impl(shape, q_win, k, k_stride_head, k_stride_tok, batch, cu_seqlens, indeg_out,
                          entropy_out, entropy_per_head_out, workspace, workspace_bytes, stream, o);
}

structkv_status structkv_score_layer_groups(const structkv_shape* shape, const void* q_win, const void* k,
                                            int64_t k_stride_head, int64_t k_stride_tok, int32_t batch,
                                            const int64_t* cu_seqlens, float* indeg_out, float* indeg_groups_out,
                                            float* entropy_out, float* entropy_per_head_out, void* workspace,
                                            size_t workspace_bytes, void* stream) {
  clear_error();
  if (batch != 0 && (!indeg_groups_out || ((uintptr_t)indeg_groups_out & 3)))
    return fail(STRUCTKV_ERR_INVALID_ARG, "indeg_groups_out is NULL or not 4-byte aligned");
  ScoreOpts o;
  o.groups = indeg_groups_out;
  return score_layer_impl(shape, q_win, k, k_stride_head, k_stride_tok, batch, cu_seqlens, indeg_out,
                          entropy_out, entropy_per_head_out, workspace, workspace_bytes, stream, o);
}

structkv_status structkv_debug_score_steps(const structkv_shape* shape, const void* q_win, const void* k,
                                           int64_t k_stride_head, int64_t k_stride_tok, int32_t batch,
                                           const int64_t* cu_seqlens, float* indeg_out, float* entropy_out,
                                           float* entropy_per_head_out, void* workspace,
                                           size_t workspace_bytes, void* stream, int32_t step_mask,
                                           int32_t force_simt) {
  ScoreOpts o;
  o.step_mask = step_mask & 15;
  o.cache_groups = (step_mask & 16) != 0;
  o.flip_stream_k = (step_mask & 32) != 0;
  o.force_simt = force_simt != 0;
  return score_layer_impl(shape, q_win, k, k_stride_head, k_stride_tok, batch, cu_seqlens, indeg_out,
                          entropy_out, entropy_per_head_out, workspace, workspace_bytes, stream, o);
}

structkv_status structkv_debug_probs(const structkv_shape* shape, const void* q_win, const void* k,
                                     int64_t k_stride_head, int64_t k_stride_tok, int64_t n,
                                     float* probs_out, void* workspace, size_t workspace_bytes,
                                     void* stream, int32_t force_simt) {
  clear_error();
  structkv_status st = check_shape(shape);
  if (st != STRUCTKV_OK) return st;
  if (n < 1 || (shape->causal && n < shape->window)) return fail(STRUCTKV_ERR_INVALID_ARG, "bad n");
  if ((int64_t)shape->n_q_heads * shape->window * n > ((int64_t)1 << 26))
    return fail(STRUCTKV_ERR_UNSUPPORTED, "H_q*w*n exceeds 2^26");
  if (!q_win || !k || !probs_out) return fail(STRUCTKV_ERR_INVALID_ARG, "NULL pointer");
  if (!workspace || ((uintptr_t)workspace & 255))
    return fail(STRUCTKV_ERR_WORKSPACE, "workspace is NULL or not 256-byte aligned");
  // indeg / entropy land in scratch behind the scoring workspace
  const size_t base = structkv_workspace_bytes(shape, 1, n);
  const size_t extra = align_up(sizeof(float) * (size_t)n, 256) + 256;
  if (workspace_bytes < base + extra)
    return fail(STRUCTKV_ERR_WORKSPACE, "workspace has %zu bytes, debug_probs needs %zu", workspace_bytes,
                base + extra);
  const int64_t cu[2] = {0, n};
  SeqTable seq;
  st = check_cu(1, cu, &seq);
  if (st != STRUCTKV_OK) return st;
  float* indeg = (float*)((uint8_t*)workspace + base);
  float* ent = (float*)((uint8_t*)workspace + base + align_up(sizeof(float) * (size_t)n, 256));
  ScoreOpts o;
  o.probs = probs_out;
  o.force_simt = force_simt != 0;
  return run_score(shape, q_win, k, k_stride_head, k_stride_tok, seq, indeg, ent, nullptr, workspace, base,
                   (hipStream_t)stream, o);
}

structkv_status structkv_accumulate_centrality(float* centrality, const float* indeg, int64_t total_tokens,
                                               float lambda, float inv_w, void* stream) {
  clear_error();
  if (total_tokens < 0) return fail(STRUCTKV_ERR_INVALID_ARG, "total_tokens < 0");
  if (!(lambda > 0.f && lambda <= 1.f)) return fail(STRUCTKV_ERR_INVALID_ARG, "lambda must be in (0,1]");
  if (!(inv_w > 0.f) || !std::isfinite(inv_w)) return fail(STRUCTKV_ERR_INVALID_ARG, "inv_w must be > 0");
  if (total_tokens == 0) return STRUCTKV_OK;
  if (!centrality || !indeg) return fail(STRUCTKV_ERR_INVALID_ARG, "NULL pointer");
  if ((((uintptr_t)centrality | (uintptr_t)indeg) & 3) != 0)
    return fail(STRUCTKV_ERR_INVALID_ARG, "pointers must be 4-byte aligned");
  if (ceil_div(total_tokens, 256) >= ((int64_t)1 << 31))
    return fail(STRUCTKV_ERR_UNSUPPORTED, "total_tokens too large for one launch");
  SKV_HIP_CHECK(launch_accumulate(centrality, indeg, total_tokens, lambda, inv_w, (hipStream_t)stream));
  return STRUCTKV_OK;
}

// shared by the two selection entry points: validates, fills seq.k / seq.out_off; *rows_out = output entries
static structkv_status check_topk_args(const float* scores, int32_t batch, const int64_t* cu_seqlens,
                                       const int64_t* k_per_seq, int32_t keep_tail, int32_t* idx_out, SeqTable* seq,
                                       int64_t* rows_out) {
  *rows_out = 0;
  structkv_status st = check_cu(batch, cu_seqlens, seq);
  if (st != STRUCTKV_OK) return st;
  if (batch == 0) return STRUCTKV_OK;
  if (!k_per_seq) return fail(STRUCTKV_ERR_INVALID_ARG, "k_per_seq is NULL");
  if (keep_tail < 0) return fail(STRUCTKV_ERR_INVALID_ARG, "keep_tail < 0");
  int64_t out = 0;
  for (int b = 0; b < batch; ++b) {
    const int64_t n = seq->cu[b + 1] - seq->cu[b];
    if (keep_tail > n)
      return fail(STRUCTKV_ERR_INVALID_ARG, "sequence %d: keep_tail (%d) > n (%lld)", b, keep_tail, (long long)n);
    if (k_per_seq[b] < 0 || k_per_seq[b] > n - keep_tail)
      return fail(STRUCTKV_ERR_INVALID_ARG, "sequence %d: k (%lld) outside [0, n - keep_tail = %lld]", b,
                  (long long)k_per_seq[b], (long long)(n - keep_tail));
    seq->k[b] = (int32_t)k_per_seq[b];
    seq->out_off[b] = out;
    out += k_per_seq[b] + keep_tail;
  }
  seq->out_off[batch] = out;
  if (out == 0) return STRUCTKV_OK;
  if (!scores || !idx_out) return fail(STRUCTKV_ERR_INVALID_ARG, "scores or idx_out is NULL");
  *rows_out = out;
  return STRUCTKV_OK;
}

structkv_status structkv_select_topk(const float* scores, int32_t batch, const int64_t* cu_seqlens,
                                     const int64_t* k_per_seq, int32_t keep_tail, int32_t* idx_out,
                                     void* workspace, size_t workspace_bytes, void* stream) {
  clear_error();
  SeqTable seq;
  int64_t rows = 0;
  structkv_status st = check_topk_args(scores, batch, cu_seqlens, k_per_seq, keep_tail, idx_out, &seq, &rows);
  if (st != STRUCTKV_OK || rows == 0) return st;
  if (!workspace || ((uintptr_t)workspace & 255))
    return fail(STRUCTKV_ERR_WORKSPACE, "workspace is NULL or not 256-byte aligned");
  const size_t need = topk_workspace_bytes(batch, seq.cu[batch]);
  if (workspace_bytes < need)
    return fail(STRUCTKV_ERR_WORKSPACE, "workspace has %zu bytes, top-k needs %zu", workspace_bytes, need);
  SKV_HIP_CHECK(launch_topk(scores, seq, keep_tail, idx_out, workspace, (hipStream_t)stream));
  return STRUCTKV_OK;
}

structkv_status structkv_select_topk_static(const float* scores, int32_t batch, const int64_t* cu_seqlens,
                                            const int64_t* k_per_seq, int32_t keep_tail, int32_t* idx_out,
                                            void* stream) {
  clear_error();
  SeqTable seq;
  int64_t rows = 0;
  structkv_status st = check_topk_args(scores, batch, cu_seqlens, k_per_seq, keep_tail, idx_out, &seq, &rows);
  if (st != STRUCTKV_OK || rows == 0) return st;
  void* scratch_ptr = nullptr;
  size_t scratch_bytes = 0;
  SKV_HIP_CHECK(topk_static_scratch(&scratch_ptr, &scratch_bytes));
  const size_t need = topk_workspace_bytes(batch, seq.cu[batch]);
  if (need > scratch_bytes)
    return fail(STRUCTKV_ERR_UNSUPPORTED,
                "this selection needs %zu bytes of scratch, the library's static scratch holds %zu "
                "(enough for %d sequences with %d tokens in all); use structkv_select_topk with a workspace",
                need, scratch_bytes, kMaxBatch, STRUCTKV_STATIC_TOPK_MAX_TOKENS);
  SKV_HIP_CHECK(launch_topk(scores, seq, keep_tail, idx_out, scratch_ptr, (hipStream_t)stream));
  return STRUCTKV_OK;
}

// shared by structkv_gather_kv and structkv_layer_step: validates, fills seq->out_off from rows_per_seq
static structkv_status check_gather_args(const void* k_src, const void* v_src, int64_t src_stride_head,
                                         int64_t src_stride_tok, void* k_dst, void* v_dst, int64_t dst_stride_head,
                                         int64_t dst_stride_tok, int32_t n_kv_heads, int32_t head_dim,
                                         int32_t elem_bytes, int32_t batch, const int64_t* cu_seqlens,
                                         const int64_t* rows_per_seq, const int32_t* idx, bool idx_needed,
                                         SeqTable* seq, bool* nothing_to_do) {
  *nothing_to_do = true;
  structkv_status st = check_cu(batch, cu_seqlens, seq);
  if (st != STRUCTKV_OK) return st;
  if (n_kv_heads < 1 || head_dim < 1) return fail(STRUCTKV_ERR_INVALID_ARG, "n_kv_heads and head_dim must be >= 1");
  if (n_kv_heads > 65535) return fail(STRUCTKV_ERR_UNSUPPORTED, "n_kv_heads > 65535");
  if (elem_bytes != 2 && elem_bytes != 4) return fail(STRUCTKV_ERR_UNSUPPORTED, "elem_bytes must be 2 or 4");
  if (batch == 0) return STRUCTKV_OK;
  if (!rows_per_seq) return fail(STRUCTKV_ERR_INVALID_ARG, "rows_per_seq is NULL");
  if (src_stride_tok < head_dim || dst_stride_tok < head_dim)
    return fail(STRUCTKV_ERR_INVALID_ARG, "token strides must be >= head_dim");
  if (src_stride_head < 0 || dst_stride_head < 0) return fail(STRUCTKV_ERR_INVALID_ARG, "negative head stride");
  int64_t out = 0;
  for (int b = 0; b < batch; ++b) {
    const int64_t n = seq->cu[b + 1] - seq->cu[b];
    if (rows_per_seq[b] < 0) return fail(STRUCTKV_ERR_INVALID_ARG, "rows_per_seq[%d] < 0", b);
    if (rows_per_seq[b] > 0 && n == 0)
      return fail(STRUCTKV_ERR_INVALID_ARG, "sequence %d is empty but rows_per_seq is %lld", b,
                  (long long)rows_per_seq[b]);
    seq->out_off[b] = out;
    out += rows_per_seq[b];
  }
  seq->out_off[batch] = out;
  if (out == 0) return STRUCTKV_OK;
  if (idx_needed && !idx) return fail(STRUCTKV_ERR_INVALID_ARG, "idx is NULL");
  if ((k_src == nullptr) != (k_dst == nullptr) || (v_src == nullptr) != (v_dst == nullptr))
    return fail(STRUCTKV_ERR_INVALID_ARG, "src/dst of a pair must both be given or both be NULL");
  if (!k_src && !v_src) return STRUCTKV_OK;
  const uintptr_t ptrs = (uintptr_t)k_src | (uintptr_t)v_src | (uintptr_t)k_dst | (uintptr_t)v_dst;
  if (ptrs & (uintptr_t)(elem_bytes - 1)) return fail(STRUCTKV_ERR_INVALID_ARG, "pointers not aligned to the element size");
  if (out * head_dim * (int64_t)elem_bytes / 2 >= ((int64_t)1 << 31) - 4096)
    return fail(STRUCTKV_ERR_UNSUPPORTED, "too many rows for one launch (rows*head_dim*elem_bytes/2 must stay below 2^31)");
  *nothing_to_do = false;
  return STRUCTKV_OK;
}

structkv_status structkv_gather_kv(const void* k_src, const void* v_src, int64_t src_stride_head,
                                   int64_t src_stride_tok, void* k_dst, void* v_dst, int64_t dst_stride_head,
                                   int64_t dst_stride_tok, int32_t n_kv_heads, int32_t head_dim,
                                   int32_t elem_bytes, int32_t batch, const int64_t* cu_seqlens,
                                   const int64_t* rows_per_seq, const int32_t* idx, void* stream) {
  clear_error();
  SeqTable seq;
  bool nothing = true;
  structkv_status st = check_gather_args(k_src, v_src, src_stride_head, src_stride_tok, k_dst, v_dst, dst_stride_head,
                                         dst_stride_tok, n_kv_heads, head_dim, elem_bytes, batch, cu_seqlens,
                                         rows_per_seq, idx, true, &seq, &nothing);
  if (st != STRUCTKV_OK || nothing) return st;
  const int64_t e = elem_bytes;
  SKV_HIP_CHECK(launch_gather(k_src, v_src, src_stride_head * e, src_stride_tok * e, k_dst, v_dst,
                              dst_stride_head * e, dst_stride_tok * e, n_kv_heads, head_dim * elem_bytes, seq,
                              idx, (hipStream_t)stream));
  return STRUCTKV_OK;
}

size_t structkv_layer_step_workspace_bytes(const structkv_shape* shape, int32_t batch, int64_t total_tokens) {
  const size_t a = structkv_workspace_bytes(shape, batch, total_tokens);
  const size_t b = structkv_workspace_bytes(nullptr, batch, total_tokens);
  if (!shape || a == 0 || b == 0) return 0;
  return a + b;   // scoring scratch and selection scratch are live at the same time
}

namespace {
// Everything a fused layer step derives from its arguments: validated once, used by both halves.
struct LayerStepPlan {
  SeqTable sel;          // cu, budgets, output offsets
  SeqTable blocks;       // the selection's workgroups per sequence
  SeqTable gseq;         // the row gather's table (fallback path)
  TopkWs tws;
  unsigned n_blocks = 0;
  int64_t rows = 0;      // output entries in all
  bool no_rows = true;
  SelectFusion fuse{};
  size_t score_bytes = 0;
  int elem_bytes = 2;
};

// *done = true: nothing to enqueue (empty batch)
structkv_status plan_layer_step(const structkv_shape* shape, const void* k, const void* v, int64_t kv_stride_head,
                                int64_t kv_stride_tok, int32_t batch, const int64_t* cu_seqlens,
                                const int64_t* k_per_seq, int32_t keep_tail, const float* indeg, int32_t* idx_out,
                                void* k_dst, void* v_dst, int64_t dst_stride_head, int64_t dst_stride_tok,
                                void* workspace, size_t workspace_bytes, LayerStepPlan* p, bool* done) {
  *done = false;
  structkv_status st = check_shape(shape);
  if (st != STRUCTKV_OK) return st;
  // the selection's arguments (budgets, window, output offsets) ...
  st = check_topk_args(indeg, batch, cu_seqlens, k_per_seq, keep_tail, idx_out, &p->sel, &p->rows);
  if (st != STRUCTKV_OK) return st;
  if (batch == 0) { *done = true; return STRUCTKV_OK; }
  // ... and the cache store's: rows_b = k_b + keep_tail
  int64_t rows_per_seq[kMaxBatch];
  for (int b = 0; b < batch; ++b) rows_per_seq[b] = k_per_seq[b] + keep_tail;
  p->elem_bytes = shape->dtype == STRUCTKV_DTYPE_BF16 ? 2 : 4;
  st = check_gather_args(k_dst ? k : nullptr, v_dst ? v : nullptr, kv_stride_head, kv_stride_tok, k_dst, v_dst,
                         dst_stride_head, dst_stride_tok, shape->n_kv_heads, shape->head_dim, p->elem_bytes, batch,
                         cu_seqlens, rows_per_seq, idx_out, false, &p->gseq, &p->no_rows);
  if (st != STRUCTKV_OK) return st;
  if (v_dst && !v) return fail(STRUCTKV_ERR_INVALID_ARG, "v_dst given without v");
  if (k_dst && !k) return fail(STRUCTKV_ERR_INVALID_ARG, "k_dst given without k");
  if (!workspace || ((uintptr_t)workspace & 255))
    return fail(STRUCTKV_ERR_WORKSPACE, "workspace is NULL or not 256-byte aligned");
  const int64_t total = p->sel.cu[batch];
  p->score_bytes = structkv_workspace_bytes(shape, batch, total);
  const size_t topk_bytes = topk_workspace_bytes(batch, total);
  if (workspace_bytes < p->score_bytes + topk_bytes)
    return fail(STRUCTKV_ERR_WORKSPACE, "workspace has %zu bytes, a layer step needs %zu", workspace_bytes,
                p->score_bytes + topk_bytes);
  topk_plan(p->sel, keep_tail, (uint8_t*)workspace + p->score_bytes, &p->blocks, &p->tws, &p->n_blocks);
  p->fuse.hist = p->tws.hist;
  p->fuse.idx_out = idx_out;
  p->fuse.keep_tail = keep_tail;
  return STRUCTKV_OK;
}

structkv_status layer_finish_impl(const structkv_shape* shape, const LayerStepPlan& p, const void* k, const void* v,
                                  int64_t kv_stride_head, int64_t kv_stride_tok, int32_t keep_tail, const float* indeg,
                                  int32_t* idx_out, void* k_dst, void* v_dst, int64_t dst_stride_head,
                                  int64_t dst_stride_tok, hipStream_t hs) {
  if (p.rows == 0) return STRUCTKV_OK;
  SKV_HIP_CHECK(launch_topk_rest(indeg, p.blocks, keep_tail, p.tws, p.n_blocks, idx_out, hs));
  const int64_t e = p.elem_bytes;
  if (!p.no_rows)
    SKV_HIP_CHECK(launch_gather(k_dst ? k : nullptr, v_dst ? v : nullptr, kv_stride_head * e, kv_stride_tok * e, k_dst,
                                v_dst, dst_stride_head * e, dst_stride_tok * e, shape->n_kv_heads,
                                shape->head_dim * p.elem_bytes, p.gseq, idx_out, hs));
  return STRUCTKV_OK;
}
}  // namespace

structkv_status structkv_layer_begin(const structkv_shape* shape, const void* q_win, const void* k, const void* v,
                                     int64_t kv_stride_head, int64_t kv_stride_tok, int32_t batch,
                                     const int64_t* cu_seqlens, const int64_t* k_per_seq, int32_t keep_tail,
                                     float* indeg_out, float* centrality, float lambda, float inv_w,
                                     float* entropy_out, float* entropy_per_head_out, int32_t* idx_out, void* k_dst,
                                     void* v_dst, int64_t dst_stride_head, int64_t dst_stride_tok, void* workspace,
                                     size_t workspace_bytes, void* stream) {
  clear_error();
  if (centrality) {
    if (!(lambda > 0.f && lambda <= 1.f)) return fail(STRUCTKV_ERR_INVALID_ARG, "lambda must be in (0,1]");
    if (!(inv_w > 0.f) || !std::isfinite(inv_w)) return fail(STRUCTKV_ERR_INVALID_ARG, "inv_w must be > 0");
    if ((uintptr_t)centrality & 3) return fail(STRUCTKV_ERR_INVALID_ARG, "centrality is not 4-byte aligned");
    if (centrality == indeg_out) return fail(STRUCTKV_ERR_INVALID_ARG, "centrality must not alias indeg_out");
  }
  LayerStepPlan p;
  bool done = false;
  structkv_status st = plan_layer_step(shape, k, v, kv_stride_head, kv_stride_tok, batch, cu_seqlens, k_per_seq,
                                       keep_tail, indeg_out, idx_out, k_dst, v_dst, dst_stride_head, dst_stride_tok,
                                       workspace, workspace_bytes, &p, &done);
  if (st != STRUCTKV_OK || done) return st;
  ScoreOpts o;
  o.centrality = centrality; o.lambda = lambda; o.inv_w = inv_w;
  o.fuse = p.rows > 0 ? &p.fuse : nullptr;
  return score_layer_impl(shape, q_win, k, kv_stride_head, kv_stride_tok, batch, cu_seqlens, indeg_out, entropy_out,
                          entropy_per_head_out, workspace, p.score_bytes, stream, o, &p.sel);
}

structkv_status structkv_layer_finish(const structkv_shape* shape, const void* k, const void* v,
                                      int64_t kv_stride_head, int64_t kv_stride_tok, int32_t batch,
                                      const int64_t* cu_seqlens, const int64_t* k_per_seq, int32_t keep_tail,
                                      const float* indeg, int32_t* idx_out, void* k_dst, void* v_dst,
                                      int64_t dst_stride_head, int64_t dst_stride_tok, void* workspace,
                                      size_t workspace_bytes, void* stream) {
  clear_error();
  LayerStepPlan p;
  bool done = false;
  structkv_status st = plan_layer_step(shape, k, v, kv_stride_head, kv_stride_tok, batch, cu_seqlens, k_per_seq,
                                       keep_tail, indeg, idx_out, k_dst, v_dst, dst_stride_head, dst_stride_tok,
                                       workspace, workspace_bytes, &p, &done);
  if (st != STRUCTKV_OK || done) return st;
  return layer_finish_impl(shape, p, k, v, kv_stride_head, kv_stride_tok, keep_tail, indeg, idx_out, k_dst, v_dst,
                           dst_stride_head, dst_stride_tok, (hipStream_t)stream);
}

structkv_status structkv_layer_step(const structkv_shape* shape, const void* q_win, const void* k, const void* v,
                                    int64_t kv_stride_head, int64_t kv_stride_tok, int32_t batch,
                                    const int64_t* cu_seqlens, const int64_t* k_per_seq, int32_t keep_tail,
                                    float* indeg_out, float* centrality, float lambda, float inv_w,
                                    float* entropy_out, float* entropy_per_head_out, int32_t* idx_out, void* k_dst,
                                    void* v_dst, int64_t dst_stride_head, int64_t dst_stride_tok, void* workspace,
                                    size_t workspace_bytes, void* stream) {
  structkv_status st = structkv_layer_begin(shape, q_win, k, v, kv_stride_head, kv_stride_tok, batch, cu_seqlens,
                                            k_per_seq, keep_tail, indeg_out, centrality, lambda, inv_w, entropy_out,
                                            entropy_per_head_out, idx_out, k_dst, v_dst, dst_stride_head,
                                            dst_stride_tok, workspace, workspace_bytes, stream);
  if (st != STRUCTKV_OK) return st;
  return structkv_layer_finish(shape, k, v, kv_stride_head, kv_stride_tok, batch, cu_seqlens, k_per_seq, keep_tail,
                               indeg_out, idx_out, k_dst, v_dst, dst_stride_head, dst_stride_tok, workspace,
                               workspace_bytes, stream);
}

structkv_status structkv_truncate_hidden(const void* h_src, int64_t src_stride_tok, void* h_dst,
                                         int64_t dst_stride_tok, int32_t hidden_dim, int32_t elem_bytes,
                                         const int64_t* pos_src, int64_t* pos_dst, int32_t batch,
                                         const int64_t* cu_seqlens, const int64_t* rows_per_seq,
                                         const int32_t* idx, void* stream) {
  // the hidden rows are one "head" of row gather; argument checks are shared with structkv_gather_kv
  if (h_src || h_dst) {
    structkv_status st = structkv_gather_kv(h_src, nullptr, 0, src_stride_tok, h_dst, nullptr, 0, dst_stride_tok, 1,
                                            hidden_dim, elem_bytes, batch, cu_seqlens, rows_per_seq, idx, stream);
    if (st != STRUCTKV_OK) return st;
  } else {
    clear_error();
  }
  if (!pos_dst) {
    if (pos_src) return fail(STRUCTKV_ERR_INVALID_ARG, "pos_src given without pos_dst");
    return STRUCTKV_OK;
  }
  SeqTable seq;
  structkv_status st = check_cu(batch, cu_seqlens, &seq);
  if (st != STRUCTKV_OK) return st;
  if (batch == 0) return STRUCTKV_OK;
  if (!rows_per_seq) return fail(STRUCTKV_ERR_INVALID_ARG, "rows_per_seq is NULL");
  int64_t out = 0;
  for (int b = 0; b < batch; ++b) {
    if (rows_per_seq[b] < 0) return fail(STRUCTKV_ERR_INVALID_ARG, "rows_per_seq[%d] < 0", b);
    if (rows_per_seq[b] > 0 && seq.cu[b + 1] == seq.cu[b])
      return fail(STRUCTKV_ERR_INVALID_ARG, "sequence %d is empty but rows_per_seq is %lld", b,
                  (long long)rows_per_seq[b]);
    seq.out_off[b] = out;
    out += rows_per_seq[b];
  }
  seq.out_off[batch] = out;
  if (out == 0) return STRUCTKV_OK;
  if (!idx) return fail(STRUCTKV_ERR_INVALID_ARG, "idx is NULL");
  if (((uintptr_t)pos_src | (uintptr_t)pos_dst) & 7) return fail(STRUCTKV_ERR_INVALID_ARG, "positions not 8-byte aligned");
  if (ceil_div(out, 256) >= ((int64_t)1 << 31)) return fail(STRUCTKV_ERR_UNSUPPORTED, "too many rows for one launch");
  SKV_HIP_CHECK(launch_positions(pos_src, seq, idx, pos_dst, (hipStream_t)stream));
  return STRUCTKV_OK;
}

structkv_status structkv_block_scores(const float* scores, int32_t batch, const int64_t* cu_seqlens,
                                      int32_t block_size, float* block_scores_out, void* stream) {
  clear_error();
  SeqTable seq;
  structkv_status st = check_cu(batch, cu_seqlens, &seq);
  if (st != STRUCTKV_OK) return st;
  if (block_size < 1) return fail(STRUCTKV_ERR_INVALID_ARG, "block_size must be >= 1");
  if (batch == 0) return STRUCTKV_OK;
  int64_t nb = 0;
  for (int b = 0; b < batch; ++b) {
    seq.out_off[b] = nb;
    nb += ceil_div(seq.cu[b + 1] - seq.cu[b], block_size);
  }
  seq.out_off[batch] = nb;
  if (nb == 0) return STRUCTKV_OK;
  if (!scores || !block_scores_out) return fail(STRUCTKV_ERR_INVALID_ARG, "scores or block_scores_out is NULL");
  if (((uintptr_t)scores | (uintptr_t)block_scores_out) & 3) return fail(STRUCTKV_ERR_INVALID_ARG, "pointers must be 4-byte aligned");
  if (ceil_div(nb, 256) >= ((int64_t)1 << 31)) return fail(STRUCTKV_ERR_UNSUPPORTED, "too many blocks for one launch");
  SKV_HIP_CHECK(launch_block_scores(scores, seq, block_size, block_scores_out, (hipStream_t)stream));
  return STRUCTKV_OK;
}

// ---- Dynamic Pivot Layer Detection: metrics (Eq. 5-6) and transition score (Eq. 7-9) --------------------------

namespace {
struct PivotCarve {
  size_t off_heads, off_indeg, off_idx, off_small, off_score_ws, off_topk_ws, total;
  size_t score_ws_bytes, topk_ws_bytes;
};
// scratch for ONE sequence of at most n_max tokens at a time (sequences are processed one after the other)
bool pivot_carve(const structkv_shape& s, int64_t n_max, structkv_shape* sub, PivotCarve* c) {
  *sub = s;
  sub->n_kv_heads = s.n_q_heads;   // every query head as a group of its own; gs consecutive ones share a K head
  const int hb = s.n_q_heads < kMaxBatch ? s.n_q_heads : kMaxBatch;   // heads per top-k call
  const size_t N = (size_t)(n_max > 0 ? n_max : 1);
  c->score_ws_bytes = structkv_workspace_bytes(sub, 1, n_max);
  c->topk_ws_bytes = structkv_workspace_bytes(nullptr, hb, (int64_t)hb * n_max);
  if (c->score_ws_bytes == 0 || c->topk_ws_bytes == 0) return false;
  {  // the scoring call with one column-sum plane per 32-row block (the path that needs no per-head re-scoring)
    ScorePlan pp;
    make_plan(s, nullptr, 1, n_max, true, &pp, true);
    if (pp.total_bytes > c->score_ws_bytes) c->score_ws_bytes = align_up(pp.total_bytes, 256);
  }
  size_t off = 0;
  c->off_heads = off;     off += align_up(sizeof(float) * (size_t)s.n_q_heads * N, 256);
  c->off_indeg = off;     off += align_up(sizeof(float) * N, 256);
  c->off_idx = off;       off += align_up(sizeof(int32_t) * (size_t)s.n_q_heads * N, 256);
  c->off_small = off;     off += align_up(sizeof(float) * (size_t)((2 * kPivotMaxSlices + 1) * s.n_q_heads + 8), 256);
  c->off_score_ws = off;  off += align_up(c->score_ws_bytes, 256);
  c->off_topk_ws = off;   off += align_up(c->topk_ws_bytes, 256);
  c->total = off;
  return true;
}
}  // namespace

size_t structkv_pivot_workspace_bytes(const structkv_shape* shape, int64_t max_seq_len) {
  if (!shape || check_shape(shape) != STRUCTKV_OK || max_seq_len < 0) return 0;
  structkv_shape sub;
  PivotCarve c;
  if (!pivot_carve(*shape, max_seq_len, &sub, &c)) return 0;
  return c.total;
}

// indeg_out / entropy_out / entropy_head_out: optional, the per-head scoring call's own totals
static structkv_status pivot_impl(const structkv_shape* shape, const void* q_win, const void* k,
                                  int64_t k_stride_head, int64_t k_stride_tok, int32_t batch,
                                  const int64_t* cu_seqlens, double top_frac, float* indeg_out, float* entropy_out,
                                  float* entropy_head_out, float* sparsity_out, float* variance_out,
                                  void* workspace, size_t workspace_bytes, void* stream) {
  clear_error();
  structkv_status st = check_shape(shape);
  if (st != STRUCTKV_OK) return st;
  SeqTable seq;
  st = check_cu(batch, cu_seqlens, &seq);
  if (st != STRUCTKV_OK) return st;
  if (!(top_frac > 0.0 && top_frac <= 1.0)) return fail(STRUCTKV_ERR_INVALID_ARG, "top_frac must be in (0,1]");
  if (batch == 0) return STRUCTKV_OK;
  if (!q_win || !sparsity_out || !variance_out) return fail(STRUCTKV_ERR_INVALID_ARG, "NULL pointer");
  const int64_t total = seq.cu[batch];
  if (total > 0 && !k) return fail(STRUCTKV_ERR_INVALID_ARG, "k is NULL");
  if (k_stride_tok < shape->head_dim) return fail(STRUCTKV_ERR_INVALID_ARG, "k_stride_tok < head_dim");
  if (shape->n_kv_heads > 1 && k_stride_head < 0) return fail(STRUCTKV_ERR_INVALID_ARG, "k_stride_head < 0");
  int64_t n_max = 0;
  for (int b = 0; b < batch; ++b) {
    const int64_t n = seq.cu[b + 1] - seq.cu[b];
    if (n > n_max) n_max = n;
    if (n >= ((int64_t)1 << 31)) return fail(STRUCTKV_ERR_UNSUPPORTED, "sequence %d is too long", b);
    if (shape->causal && n != 0 && n < shape->window)
      return fail(STRUCTKV_ERR_INVALID_ARG, "sequence %d: causal scoring needs n >= window", b);
  }
  if (!workspace || ((uintptr_t)workspace & 255))
    return fail(STRUCTKV_ERR_WORKSPACE, "workspace is NULL or not 256-byte aligned");
  structkv_shape sub;
  PivotCarve c;
  if (!pivot_carve(*shape, n_max, &sub, &c)) return fail(STRUCTKV_ERR_UNSUPPORTED, "cannot size the scratch");
  if (workspace_bytes < c.total)
    return fail(STRUCTKV_ERR_WORKSPACE, "workspace has %zu bytes, pivot metrics need %zu", workspace_bytes, c.total);

  uint8_t* w8 = (uint8_t*)workspace;
  float* heads = (float*)(w8 + c.off_heads);
  float* indeg = (float*)(w8 + c.off_indeg);
  int32_t* idx = (int32_t*)(w8 + c.off_idx);
  float* part = (float*)(w8 + c.off_small);        // [Hq][slices][2] partial sums
  float* ent = part + (size_t)2 * kPivotMaxSlices * shape->n_q_heads;   // entropy outputs of the scoring call: not used
  float* ent_h = ent + 4;
  const int Hq = shape->n_q_heads, gs = Hq / shape->n_kv_heads, w = shape->window, d = shape->head_dim;
  const size_t e = shape->dtype == STRUCTKV_DTYPE_BF16 ? 2 : 4;
  hipStream_t hs = (hipStream_t)stream;
  // Where the bf16 MFMA kernels apply and a wave's rows are one head's window (or two), the metrics come out of the
  // hot path's own scoring: pass 2 keeps one column-sum plane per query head -- the per-head in-degrees -- and
  // nothing is scored twice.  Otherwise the layer is re-scored with every head as its own group.
  bool from_planes = false;
  if (mfma_eligible(*shape, q_win, k, k_stride_head, k_stride_tok) && Hq <= kMaxBatch) {
    ScorePlan probe;
    make_plan(*shape, nullptr, 1, n_max, true, &probe, true);
    from_planes = probe.planes != 0 && probe.CP == gs;
  }
  for (int b = 0; b < batch; ++b) {
    const int64_t n = seq.cu[b + 1] - seq.cu[b];
    const int64_t cu1[2] = {0, n};
    const uint8_t* qs = (const uint8_t*)q_win + (size_t)b * Hq * w * d * e;
    const uint8_t* ks = (const uint8_t*)k + (size_t)seq.cu[b] * k_stride_tok * e;
    int64_t kk = (int64_t)std::ceil(top_frac * (double)n);   // the ceil(top_frac n) largest keys of every head
    if (kk < 1) kk = 1;
    if (kk > n) kk = n;
    // (the planes path keeps its partial sums where the other path keeps indices: Hq x n words)
    if (n > 0 && from_planes && 2 * ceil_div(n, 2048) + 4 <= n && n <= ((int64_t)1 << 24)) {
      // selection scratch for the Hq heads as "sequences" of one call; its histograms are cleared by the
      // scoring call's combine kernel and their first digit is filled by the kernel that forms the variance
      SeqTable hseq;
      memset(&hseq, 0, sizeof(hseq));
      hseq.batch = Hq;
      for (int i = 0; i <= Hq; ++i) hseq.cu[i] = (int64_t)i * n;
      for (int i = 0; i < Hq; ++i) hseq.k[i] = (int32_t)kk;
      SeqTable hplan;
      TopkWs tws;
      unsigned blocks = 0;
      topk_plan(hseq, 0, w8 + c.off_topk_ws, &hplan, &tws, &blocks);
      const int Pv = pivot_plane_shares(n);
      float* var_part = (float*)idx;                       // the index scratch of the other path is free here
      float* part_above = var_part + (size_t)Hq * Pv;      // ... Hq x n words of it: 2 Pv + 4 per head are used
      float* mass_part = part_above + (size_t)Hq * Pv;
      float* tail = mass_part + (size_t)Hq * 2;
      ScoreOpts o;
      o.planes = true;
      o.zero_ptr = tws.hist;
      o.zero_words = (int64_t)3 * kTopkBins * Hq;
      st = score_layer_impl(shape, qs, ks, k_stride_head, k_stride_tok, 1, cu1,
                            indeg_out ? indeg_out + seq.cu[b] : indeg, entropy_out ? entropy_out + b : ent,
                            entropy_head_out ? entropy_head_out + (size_t)b * Hq : ent_h, w8 + c.off_score_ws,
                            c.score_ws_bytes, stream, o);
      if (st != STRUCTKV_OK) return st;
      // where that call left its planes: the same plan, made again
      ScorePlan pp;
      SeqTable one;
      memset(&one, 0, sizeof(one));
      one.batch = 1; one.cu[1] = n;
      make_plan(*shape, &one, 1, n, true, &pp, true);
      const float* planes = (const float*)(w8 + c.off_score_ws + pp.off_colsum);   // [Hq][n]: plane g*gs + hl is head h
      SKV_HIP_CHECK(launch_pivot_planes(planes, Hq, n, 1.0f / (float)w, tws.hist, var_part, hs));
      // (the per-head in-degrees of the other path's scratch hold the candidate lists here)
      SKV_HIP_CHECK(launch_topk_mass(planes, Hq, n, (uint32_t)kk, tws, heads, part_above, mass_part, tail, hs));
      SKV_HIP_CHECK(launch_pivot_finish_planes(var_part, Pv, mass_part, 1, tail, Hq, n, 1.0f / (float)w, sparsity_out + b,
                                               variance_out + b, hs));
      continue;
    }
    if (n > 0) {
      // per-head in-degree D_h [Hq][n]: one scoring call in which every query head is a group of its own
      // and the gs heads of a KV head read the same K head
      ScoreOpts o;
      o.groups = heads; o.kshare = gs;
      st = score_layer_impl(&sub, qs, ks, k_stride_head, k_stride_tok, 1, cu1,
                            indeg_out ? indeg_out + seq.cu[b] : indeg, entropy_out ? entropy_out + b : ent,
                            entropy_head_out ? entropy_head_out + (size_t)b * Hq : ent_h, w8 + c.off_score_ws,
                            c.score_ws_bytes, stream, o);
      if (st != STRUCTKV_OK) return st;
      for (int h0 = 0; h0 < Hq; h0 += kMaxBatch) {
        const int hb = Hq - h0 < kMaxBatch ? Hq - h0 : kMaxBatch;
        int64_t cuh[kMaxBatch + 1], kh[kMaxBatch];
        for (int i = 0; i <= hb; ++i) cuh[i] = (int64_t)i * n;
        for (int i = 0; i < hb; ++i) kh[i] = kk;
        st = structkv_select_topk(heads + (size_t)h0 * n, hb, cuh, kh, 0, idx + (size_t)h0 * kk,
                                  w8 + c.off_topk_ws, c.topk_ws_bytes, stream);
        if (st != STRUCTKV_OK) return st;
      }
      SKV_HIP_CHECK(launch_pivot_heads(heads, Hq, n, idx, kk, 1.0f / (float)w, part, hs));
    }
    SKV_HIP_CHECK(launch_pivot_finish(part, Hq, n, 1.0f / (float)w, n > 0 ? 1 : 0, sparsity_out + b,
                                      variance_out + b, hs));
    if (n == 0) {   // an empty sequence scores nothing: its entropies are zero, as in structkv_score_layer
      if (entropy_out) SKV_HIP_CHECK(launch_zero_floats(entropy_out + b, 1, hs));
      if (entropy_head_out) SKV_HIP_CHECK(launch_zero_floats(entropy_head_out + (size_t)b * Hq, Hq, hs));
    }
  }
  return STRUCTKV_OK;
}

structkv_status structkv_pivot_metrics(const structkv_shape* shape, const void* q_win, const void* k,
                                       int64_t k_stride_head, int64_t k_stride_tok, int32_t batch,
                                       const int64_t* cu_seqlens, double top_frac, float* sparsity_out,
                                       float* variance_out, void* workspace, size_t workspace_bytes, void* stream) {
  return pivot_impl(shape, q_win, k, k_stride_head, k_stride_tok, batch, cu_seqlens, top_frac, nullptr, nullptr,
                    nullptr, sparsity_out, variance_out, workspace, workspace_bytes, stream);
}

structkv_status structkv_score_layer_pivot(const structkv_shape* shape, const void* q_win, const void* k,
                                           int64_t k_stride_head, int64_t k_stride_tok, int32_t batch,
                                           const int64_t* cu_seqlens, double top_frac, float* indeg_out,
                                           float* entropy_out, float* entropy_per_head_out, float* sparsity_out,
                                           float* variance_out, void* workspace, size_t workspace_bytes,
                                           void* stream) {
  if (batch > 0 && !entropy_out) { clear_error(); return fail(STRUCTKV_ERR_INVALID_ARG, "entropy_out is NULL"); }
  if (batch > 0 && cu_seqlens && cu_seqlens[batch] > 0 && !indeg_out) {
    clear_error();
    return fail(STRUCTKV_ERR_INVALID_ARG, "indeg_out is NULL");
  }
  return pivot_impl(shape, q_win, k, k_stride_head, k_stride_tok, batch, cu_seqlens, top_frac, indeg_out,
                    entropy_out, entropy_per_head_out, sparsity_out, variance_out, workspace, workspace_bytes,
                    stream);
}

// Eq. 7: t[l] += weight * (g_l - min g) / (max g - min g) for l >= 1, with g_l = direction * (m[l] - m[l-1]);
// a metric whose steps are all equal has no transition to point at and adds nothing.
static void add_normalised_gradient(const double* m, int n_layers, double direction, double weight, double* t) {
  double g_min = 0.0, g_max = 0.0;
  for (int l = 1; l < n_layers; ++l) {
    const double g = direction * (m[l] - m[l - 1]);
    if (l == 1 || g < g_min) g_min = g;
    if (l == 1 || g > g_max) g_max = g;
  }
  const double span = g_max - g_min;
  if (!(span > 0.0)) return;
  for (int l = 1; l < n_layers; ++l) t[l] += weight * ((direction * (m[l] - m[l - 1]) - g_min) / span);
}

structkv_status structkv_transition_scores(const double* entropy, const double* sparsity, const double* variance,
                                           int32_t n_layers, double w1, double w2, double w3, double* t_out,
                                           int32_t* pivot_layer_out) {
  clear_error();
  if (n_layers < 0) return fail(STRUCTKV_ERR_INVALID_ARG, "n_layers < 0");
  if (n_layers > 0 && (!entropy || !sparsity || !variance || !t_out))
    return fail(STRUCTKV_ERR_INVALID_ARG, "NULL pointer");
  if (!pivot_layer_out) return fail(STRUCTKV_ERR_INVALID_ARG, "pivot_layer_out is NULL");
  for (int l = 0; l < n_layers; ++l) t_out[l] = 0.0;
  if (n_layers < 2) { *pivot_layer_out = n_layers; return STRUCTKV_OK; }
  // Eq. 8: the detector looks for a DROP in entropy together with a RISE in sparsity and in variance
  add_normalised_gradient(entropy, n_layers, -1.0, w1, t_out);
  add_normalised_gradient(sparsity, n_layers, +1.0, w2, t_out);
  add_normalised_gradient(variance, n_layers, +1.0, w3, t_out);
  // Eq. 9: the first layer after the strongest transition (the lowest such layer on ties)
  int32_t at = 1;
  for (int32_t l = 2; l < n_layers; ++l)
    if (t_out[l] > t_out[at]) at = l;
  *pivot_layer_out = at + 1;
  return STRUCTKV_OK;
}

}  // extern "C"
