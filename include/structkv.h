/*
 * libstructkv -- StructKV prefill scoring / selection / gather path for AMD MI355X (gfx950).
 *
 * C ABI.  Every tensor pointer is a DEVICE pointer unless marked "host".  The
 * library owns no memory, reads no environment variable and keeps no state
 * between calls: the caller owns all buffers, including the scratch
 * `workspace` (size it with structkv_workspace_bytes); the one exception is
 * structkv_select_topk_static, whose scratch is an array inside the library.  All work is enqueued
 * on `stream` (a hipStream_t passed as void*; NULL = the default stream); no
 * call synchronises the device.  Every entry point returns a structkv_status; on failure nothing has
 * been enqueued unless the status is STRUCTKV_ERR_HIP, and
 * structkv_last_error() holds a thread-local message.  Inputs are assumed
 * finite (NaN/Inf behaviour is undefined).  Strides count ELEMENTS and are
 * 64-bit.  Outputs are overwritten in full except `centrality` (in/out).
 *
 * Notation (StructKV paper, Sec. 3.2): H_q query heads, G KV heads (GQA group
 * size H_q/G), d head dim, n cached tokens of a sequence, w observation
 * window (the last w positions n-w .. n-1), k selection budget, lambda decay.
 * A call handles a ragged batch of B sequences packed along the token axis:
 * sequence b owns tokens cu_seqlens[b] .. cu_seqlens[b+1]-1.
 */
#ifndef STRUCTKV_H
#define STRUCTKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  STRUCTKV_OK = 0,
  STRUCTKV_ERR_INVALID_ARG = 1, /* NULL pointer, bad size, inconsistent cu_seqlens, k out of range */
  STRUCTKV_ERR_UNSUPPORTED = 2, /* dtype / head_dim / batch beyond what the kernels implement */
  STRUCTKV_ERR_WORKSPACE = 3,   /* workspace NULL, misaligned or smaller than required */
  STRUCTKV_ERR_HIP = 4          /* a HIP runtime call failed (message has hipGetErrorString) */
} structkv_status;

enum { STRUCTKV_DTYPE_F32 = 0, STRUCTKV_DTYPE_BF16 = 1 };

/* Largest batch one call accepts. */
#define STRUCTKV_MAX_BATCH 64

typedef struct {
  int32_t n_q_heads;  /* H_q >= 1 */
  int32_t n_kv_heads; /* G >= 1, divides H_q */
  int32_t head_dim;   /* d: 1..256; the bf16 MFMA path needs d in {64,128}, other shapes take a SIMT path */
  int32_t window;     /* w >= 1 */
  int32_t dtype;      /* STRUCTKV_DTYPE_F32 or STRUCTKV_DTYPE_BF16: element type of q_win and k */
  int32_t causal;     /* 0 (Eq. 1 as written): each window query sees all n keys;
                         1: window row i (position n-w+i) sees keys j <= n-w+i only (needs n >= w) */
  float scale;        /* logit scale, >= 0; 0 selects 1/sqrt(head_dim) (Eq. 1) */
} structkv_shape;

/* Thread-local message of the last failing call on this thread ("" if none). */
const char* structkv_last_error(void);

/* Library version, major*10000 + minor*100 + patch. */
int32_t structkv_version(void);

/*
 * Bytes of scratch that structkv_score_layer (shape != NULL) and structkv_select_topk need
 * for a batch of `batch` sequences holding `total_tokens` tokens in all.  With shape == NULL
 * only the top-k requirement is returned.  Returns 0 on invalid arguments.  The workspace must
 * be 256-byte aligned; its contents need not be preserved between calls and need no initialisation.
 */
size_t structkv_workspace_bytes(const structkv_shape* shape, int32_t batch, int64_t total_tokens);

/*
 * Per-layer scoring pass (paper Eq. 1, Eq. 2 without its 1/w, Eq. 4).
 * For every sequence b, every query head h (KV head g = h / (H_q/G)) and every window row i:
 *   a_{h,i,j} = softmax_j( scale * q_win[b][h][i] . k[g][cu[b]+j] ),  j in [0, n_b)
 *   indeg_out[cu[b]+j]  = sum_{h,i} a_{h,i,j}            (raw in-degree D_j; sums to w*H_q per sequence)
 *   entropy_out[b]      = -(1/(H_q w)) sum_{h,i,j} a ln a (natural log, 0 ln 0 = 0)
 *   entropy_per_head_out[b][h] = -(1/w) sum_{i,j} a ln a  (optional, may be NULL)
 * q_win : [B][H_q][w][d] contiguous, dtype per shape.
 * k     : element (g, token t, c) at k[g*k_stride_head + t*k_stride_tok + c], c contiguous, t packed over the batch.
 * cu_seqlens : HOST pointer, [B+1], cu[0]=0, non-decreasing, cu[B] = total tokens; n_b = 0 is allowed
 *              (no output, entropy 0), otherwise n_b >= 1 (and n_b >= w if causal).
 * indeg_out [total], entropy_out [B], entropy_per_head_out [B][H_q]: fp32.
 * Deterministic: the same inputs give bit-identical outputs (no floating-point atomics).
 */
structkv_status structkv_score_layer(const structkv_shape* shape, const void* q_win, const void* k,
                                     int64_t k_stride_head, int64_t k_stride_tok, int32_t batch,
                                     const int64_t* cu_seqlens, float* indeg_out, float* entropy_out,
                                     float* entropy_per_head_out, void* workspace,
                                     size_t workspace_bytes, void* stream);

/*
 * Global in-degree centrality update (paper Eq. 3 as the recurrence of Alg. 1 line 6, with
 * Eq. 2's 1/w applied here):  centrality[t] = lambda*centrality[t] + inv_w*indeg[t], t < total_tokens.
 * lambda in (0,1]; inv_w > 0 (normally 1/w).  centrality is in/out, fp32; start it at zero.
 */
structkv_status structkv_accumulate_centrality(float* centrality, const float* indeg,
                                               int64_t total_tokens, float lambda, float inv_w,
                                               void* stream);

/*
 * structkv_score_layer followed by structkv_accumulate_centrality in one call (paper Eq. 1-4 and the
 * recurrence of Alg. 1 line 6): the kernel that forms indeg_out also updates
 *   centrality[t] = lambda*centrality[t] + inv_w*indeg_out[t]
 * with the same arithmetic, so every output is bit-identical to the two separate calls; it saves one
 * launch and one read of indeg per layer.  Arguments as for those two entry points; centrality
 * [total] fp32 in/out, non-NULL whenever batch > 0, must not alias indeg_out.
 */
structkv_status structkv_score_layer_accumulate(const structkv_shape* shape, const void* q_win, const void* k,
                                                int64_t k_stride_head, int64_t k_stride_tok, int32_t batch,
                                                const int64_t* cu_seqlens, float* indeg_out, float* centrality,
                                                float lambda, float inv_w, float* entropy_out,
                                                float* entropy_per_head_out, void* workspace,
                                                size_t workspace_bytes, void* stream);

/*
 * structkv_score_layer that also returns the in-degree per KV head (paper Eq. 2 before its outer sum
 * over the KV groups):  indeg_groups_out[g][cu[b]+j] = sum_{h in H_g} sum_i a_{h,i,j},  [G][total] fp32,
 * so that sum_g indeg_groups_out[g][t] = indeg_out[t] up to fp32 rounding.  For callers that keep one index
 * set per KV head.  indeg_groups_out must be given whenever batch > 0.  Other arguments and outputs as
 * structkv_score_layer.
 */
structkv_status structkv_score_layer_groups(const structkv_shape* shape, const void* q_win, const void* k,
                                            int64_t k_stride_head, int64_t k_stride_tok, int32_t batch,
                                            const int64_t* cu_seqlens, float* indeg_out, float* indeg_groups_out,
                                            float* entropy_out, float* entropy_per_head_out, void* workspace,
                                            size_t workspace_bytes, void* stream);

/*
 * Token selection (paper Eq. 10 on the centrality, Eq. 13 on a layer's scores): per sequence b the
 * k_b largest of scores[cu[b] .. cu[b+1]-keep_tail) -- ties go to the lower index -- united with the
 * last keep_tail positions (the observation window I_win).  Written in ascending order as
 * sequence-local int32 indices at idx_out + sum_{b'<b}(k_b' + keep_tail);  k_b + keep_tail entries.
 * scores : [total] fp32.  cu_seqlens, k_per_seq : HOST pointers ([B+1], [B]).
 * Requires 0 <= keep_tail <= n_b and 0 <= k_b <= n_b - keep_tail for every b; n_b < 2^31.
 * Deterministic and exact: the result is the unique set defined above for the given fp32 scores
 * (-0.0 and +0.0 compare equal).
 */
structkv_status structkv_select_topk(const float* scores, int32_t batch, const int64_t* cu_seqlens,
                                     const int64_t* k_per_seq, int32_t keep_tail, int32_t* idx_out,
                                     void* workspace, size_t workspace_bytes, void* stream);

/*
 * structkv_select_topk for callers that cannot allocate or hold a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): same arguments without the workspace, same result
 * bit for bit.  Its scratch (digit histograms, search state, per-workgroup suffix sums) is a fixed 4 MiB
 * array inside the library, one copy per GPU, held until the process ends; the call allocates nothing.
 * Limit: the scratch covers any batch of up to STRUCTKV_MAX_BATCH sequences with at most
 * STRUCTKV_STATIC_TOPK_MAX_TOKENS tokens in all (a single sequence may be about twice that long); a larger
 * call returns STRUCTKV_ERR_UNSUPPORTED with nothing enqueued.  All calls on one GPU share the array: calls
 * that overlap in time on the same GPU (different streams, different threads) race; serialise them, or use
 * structkv_select_topk with separate workspaces.  Nothing needs clearing between calls (every call starts
 * by zeroing the histograms it uses, on the stream).
 */
#define STRUCTKV_STATIC_TOPK_MAX_TOKENS 1048576
structkv_status structkv_select_topk_static(const float* scores, int32_t batch, const int64_t* cu_seqlens,
                                            const int64_t* k_per_seq, int32_t keep_tail, int32_t* idx_out,
                                            void* stream);

/*
 * Decoupled cache store (paper Alg. 1 line 17): compact the selected K and V rows.
 *   dst[g][o_b + i][:] = src[g][cu[b] + idx[o_b + i]][:],  o_b = sum_{b'<b} rows_b',  i < rows_b
 * for K and V (either pair may be NULL to skip it), bit-exact copy of head_dim*elem_bytes bytes per row.
 * idx : DEVICE pointer, sequence-local int32 indices laid out as structkv_select_topk writes them;
 *       every index must lie in [0, n_b) (checked on the device: an out-of-range index copies row 0
 *       of the sequence instead of faulting).
 * rows_per_seq : HOST pointer [B] (k_b + keep_tail).  elem_bytes in {2,4}.
 */
structkv_status structkv_gather_kv(const void* k_src, const void* v_src, int64_t src_stride_head,
                                   int64_t src_stride_tok, void* k_dst, void* v_dst,
                                   int64_t dst_stride_head, int64_t dst_stride_tok, int32_t n_kv_heads,
                                   int32_t head_dim, int32_t elem_bytes, int32_t batch,
                                   const int64_t* cu_seqlens, const int64_t* rows_per_seq,
                                   const int32_t* idx, void* stream);

/*
 * One layer of the hot path in one call (paper Alg. 1 lines 4, 6, 16, 17; Eq. 1-4, Eq. 13):
 *   structkv_score_layer            -> indeg_out, entropy_out, entropy_per_head_out
 *   structkv_accumulate_centrality  -> centrality (skipped when centrality == NULL: a caller that runs layers
 *                                      on several streams applies the recurrence itself, in layer order)
 *   structkv_select_topk(indeg_out, k_per_seq, keep_tail) -> idx_out
 *   structkv_gather_kv(k, v, idx_out) -> k_dst, v_dst   (rows_b = k_b + keep_tail; either dst may be NULL)
 * with the results of those four calls bit for bit, in eight kernel launches instead of eleven: the kernel
 * that forms the in-degree also applies the recurrence, histograms the first radix digit of the selection and
 * writes the kept window's indices (the scoring kernel before it has cleared the histograms).
 * v shares k's strides (kv_stride_head, kv_stride_tok) and element type; k_dst / v_dst share
 * dst_stride_head / dst_stride_tok.  Other arguments as in the four calls.
 * workspace: structkv_layer_step_workspace_bytes(shape, batch, total_tokens) bytes (scoring and selection
 * scratch are live together), 256-byte aligned, no initialisation needed.
 */
size_t structkv_layer_step_workspace_bytes(const structkv_shape* shape, int32_t batch, int64_t total_tokens);
structkv_status structkv_layer_step(const structkv_shape* shape, const void* q_win, const void* k, const void* v,
                                    int64_t kv_stride_head, int64_t kv_stride_tok, int32_t batch,
                                    const int64_t* cu_seqlens, const int64_t* k_per_seq, int32_t keep_tail,
                                    float* indeg_out, float* centrality, float lambda, float inv_w,
                                    float* entropy_out, float* entropy_per_head_out, int32_t* idx_out,
                                    void* k_dst, void* v_dst, int64_t dst_stride_head, int64_t dst_stride_tok,
                                    void* workspace, size_t workspace_bytes, void* stream);

/*
 * structkv_layer_step in two halves, for callers that run the layers of a prefill on several streams and must
 * apply the centrality recurrence (paper Eq. 3 / Alg. 1 line 6) in layer order BETWEEN the halves:
 *   structkv_layer_begin  : the scoring (Eq. 1, 2, 4) -> indeg_out, entropies; the first radix digit of the
 *                           selection and the kept window's indices; with centrality != NULL also the
 *                           recurrence (then this is the first four kernels of structkv_layer_step)
 *   (the caller: wait for the previous layer's update, structkv_accumulate_centrality, signal)
 *   structkv_layer_finish : the rest of the selection (Eq. 13) -> idx_out, and the selected rows -> k_dst, v_dst
 * Both take the same arguments as structkv_layer_step (finish only those it uses), on the same stream, with the
 * same workspace, whose contents must survive from begin to finish; indeg must not change in between.
 */
structkv_status structkv_layer_begin(const structkv_shape* shape, const void* q_win, const void* k, const void* v,
                                     int64_t kv_stride_head, int64_t kv_stride_tok, int32_t batch,
                                     const int64_t* cu_seqlens, const int64_t* k_per_seq, int32_t keep_tail,
                                     float* indeg_out, float* centrality, float lambda, float inv_w,
                                     float* entropy_out, float* entropy_per_head_out, int32_t* idx_out,
                                     void* k_dst, void* v_dst, int64_t dst_stride_head, int64_t dst_stride_tok,
                                     void* workspace, size_t workspace_bytes, void* stream);
structkv_status structkv_layer_finish(const structkv_shape* shape, const void* k, const void* v,
                                      int64_t kv_stride_head, int64_t kv_stride_tok, int32_t batch,
                                      const int64_t* cu_seqlens, const int64_t* k_per_seq, int32_t keep_tail,
                                      const float* indeg, int32_t* idx_out, void* k_dst, void* v_dst,
                                      int64_t dst_stride_head, int64_t dst_stride_tok, void* workspace,
                                      size_t workspace_bytes, void* stream);

/*
 * Structural truncation (paper Eq. 11-12): keep the hidden states and the position ids of the
 * structural indices, in index order.
 *   h_dst[o_b + i][:]  = h_src[cu[b] + idx[o_b + i]][:]          (hidden_dim*elem_bytes bytes, bit-exact)
 *   pos_dst[o_b + i]   = pos_src ? pos_src[cu[b] + idx[o_b + i]] : idx[o_b + i]
 * h_src : [total][hidden] rows, src_stride_tok elements apart; h_dst likewise with dst_stride_tok.
 *         Both NULL skips the hidden states.
 * pos_src : DEVICE int64 [total] position ids (for RoPE re-alignment), or NULL for the identity
 *           0..n_b-1 of every sequence; pos_dst : DEVICE int64 [rows] or NULL to skip positions.
 * idx, rows_per_seq, cu_seqlens, elem_bytes and the out-of-range rule: as for structkv_gather_kv.
 */
structkv_status structkv_truncate_hidden(const void* h_src, int64_t src_stride_tok, void* h_dst,
                                         int64_t dst_stride_tok, int32_t hidden_dim, int32_t elem_bytes,
                                         const int64_t* pos_src, int64_t* pos_dst, int32_t batch,
                                         const int64_t* cu_seqlens, const int64_t* rows_per_seq,
                                         const int32_t* idx, void* stream);

/*
 * Block-level aggregation for paged caches (paper Sec. 4.1, implementation details): the score of
 * cache block k of sequence b is the sum of the scores (normally the centrality) of its tokens,
 *   out[B_b + k] = sum_{t = k*block_size}^{min(n_b, (k+1)*block_size) - 1} scores[cu[b] + t],
 *   k < ceil(n_b / block_size),  B_b = sum_{b' < b} ceil(n_b' / block_size),
 * added left to right in fp32 (deterministic).  scores, block_scores_out : DEVICE fp32.
 * Lowest-score blocks are then found with structkv_select_topk on block_scores_out (cu = the B_b),
 * and kept blocks are moved with structkv_gather_kv on K/V viewed as [G][n/block_size][block_size*d].
 */
structkv_status structkv_block_scores(const float* scores, int32_t batch, const int64_t* cu_seqlens,
                                      int32_t block_size, float* block_scores_out, void* stream);

/*
 * Dynamic Pivot Layer Detection, the two metrics the scoring pass does not already produce (paper Eq. 5-6;
 * the entropy of Eq. 4 comes from structkv_score_layer).  The paper leaves the row index of a^(l,h) free;
 * here a head's attention is pooled over the window rows, a_h[j] = (1/w) sum_i a_{h,i,j}, a probability
 * vector over the n_b keys of sequence b.  Per sequence:
 *   sparsity_out[b] = (1/H_q) sum_h ( sum of the k largest a_h[j] ),   k = ceil(top_frac * n_b) in double arithmetic (paper: 0.1)
 *   variance_out[b] = (1/H_q) sum_h (1/n_b) sum_j (a_h[j] - 1/n_b)^2
 * (0 for an empty sequence).  With bf16 inputs, head_dim 64 or 128 and a window of 32 or 64 the per-head in-degrees
 * come out of the scoring pass itself (its second pass keeps one column-sum plane per query head) and the call
 * costs one scoring of the layer plus four short kernels over those planes (a radix select for the top-k mass);
 * other shapes are re-scored head by head, which costs about as much as scoring the layer twice.
 * q_win, k, strides, cu_seqlens, shape: as structkv_score_layer.  sparsity_out, variance_out: DEVICE fp32 [B].
 * workspace: structkv_pivot_workspace_bytes(shape, longest sequence) bytes, 256-byte aligned.
 */
size_t structkv_pivot_workspace_bytes(const structkv_shape* shape, int64_t max_seq_len);
structkv_status structkv_pivot_metrics(const structkv_shape* shape, const void* q_win, const void* k,
                                       int64_t k_stride_head, int64_t k_stride_tok, int32_t batch,
                                       const int64_t* cu_seqlens, double top_frac, float* sparsity_out,
                                       float* variance_out, void* workspace, size_t workspace_bytes,
                                       void* stream);

/*
 * structkv_score_layer and structkv_pivot_metrics from ONE scoring of the layer, for the layers on which the
 * pivot detector is still running (paper Eq. 2, 4, 5, 6): the scoring that the metrics need also yields
 * the in-degree and the entropies.  Outputs as in structkv_score_layer (indeg_out DEVICE fp32 [total],
 * entropy_out DEVICE fp32 [B], entropy_per_head_out DEVICE fp32 [B][H_q] or NULL) and structkv_pivot_metrics.
 * indeg_out sums the heads in another order than structkv_score_layer does: equal to it within fp32 rounding, not
 * bit for bit.  Workspace and errors as structkv_pivot_metrics.
 */
structkv_status structkv_score_layer_pivot(const structkv_shape* shape, const void* q_win, const void* k,
                                           int64_t k_stride_head, int64_t k_stride_tok, int32_t batch,
                                           const int64_t* cu_seqlens, double top_frac, float* indeg_out,
                                           float* entropy_out, float* entropy_per_head_out, float* sparsity_out,
                                           float* variance_out, void* workspace, size_t workspace_bytes,
                                           void* stream);

/*
 * Transition score and pivot layer (paper Eq. 7-9), HOST arithmetic on HOST arrays of per-layer metrics
 * (layers 0 .. n_layers-1 of the un-pruned prefix):  dM_l = M_l - M_{l-1} for l >= 1; each metric's differences
 * are min-max scaled to [0,1] over l = 1 .. n_layers-1 (a metric whose differences are all equal contributes 0);
 *   t_out[l] = w1 * grad(-entropy)_l + w2 * grad(sparsity)_l + w3 * grad(variance)_l,   t_out[0] = 0;
 *   *pivot_layer_out = argmax_{l >= 1} t_out[l] + 1   (lowest l on ties; n_layers < 2: n_layers).
 * The paper's weights are (0.2, 0.3, 0.5).
 */
structkv_status structkv_transition_scores(const double* entropy, const double* sparsity, const double* variance,
                                           int32_t n_layers, double w1, double w2, double w3, double* t_out,
                                           int32_t* pivot_layer_out);

#ifdef __cplusplus
}
#endif
#endif /* STRUCTKV_H */
