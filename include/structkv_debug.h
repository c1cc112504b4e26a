/*
 * libstructkv -- test and profiling hooks.  Not part of the product interface: nothing on the hot path
 * calls these; tests use them to look inside the scoring pass (the attention rows of paper Eq. 1) and
 * bench.py to time its four kernels one at a time.  Conventions as in structkv.h.
 */
#ifndef STRUCTKV_DEBUG_H
#define STRUCTKV_DEBUG_H

#include "structkv.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * The attention rows themselves (paper Eq. 1) for ONE sequence of n tokens, probs_out [H_q][w][n] fp32,
 * computed by the same kernels as structkv_score_layer.  H_q*w*n must not exceed 2^26.
 * workspace: structkv_workspace_bytes(shape, 1, n) + 4 n + 512 bytes.
 * force_simt != 0 takes the SIMT kernels even where the bf16 MFMA kernels apply.
 */
structkv_status structkv_debug_probs(const structkv_shape* shape, const void* q_win, const void* k,
                                     int64_t k_stride_head, int64_t k_stride_tok, int64_t n,
                                     float* probs_out, void* workspace, size_t workspace_bytes,
                                     void* stream, int32_t force_simt);

/*
 * structkv_score_layer with only some of its four kernels enqueued, so a caller can bracket each with
 * events.  step_mask bits: 1 = pass 1 (row statistics, Eq. 4), 2 = combine (lse, entropy per row),
 * 4 = pass 2 (column sums, Eq. 2), 8 = reduce (in-degree, entropy).  Steps read what earlier steps left
 * in the workspace; mask 15 is structkv_score_layer itself.  Bit 16: go through a batch whose keys exceed 192 MB
 * in groups of consecutive sequences that fit the memory-side cache -- pass 1, combine, pass 2 of a group back
 * to back -- instead of one launch per kernel over the whole batch (same results, bit for bit; kept for
 * measuring the two schedules: the grouped one fetches less from HBM in pass 2 and is slower).  Bit 32: fetch
 * the K tiles with the other cache policy than the library's size rule picks (non-temporal below 256 MiB of K per
 * layer, cached from there on); a cache policy changes no result.
 * force_simt as above.
 */
structkv_status structkv_debug_score_steps(const structkv_shape* shape, const void* q_win, const void* k,
                                           int64_t k_stride_head, int64_t k_stride_tok, int32_t batch,
                                           const int64_t* cu_seqlens, float* indeg_out, float* entropy_out,
                                           float* entropy_per_head_out, void* workspace,
                                           size_t workspace_bytes, void* stream, int32_t step_mask,
                                           int32_t force_simt);

#ifdef __cplusplus
}
#endif
#endif /* STRUCTKV_DEBUG_H */
