// Stand-ins for the kernel launchers of libstructkv, for the host-only sanitizer build of its C ABI:
// api.cpp is compiled with -fsanitize=address,undefined and linked against these instead of the HIP
// kernels, so that argument validation, work planning and workspace carving run under the sanitizers
// on a machine without a GPU.  The stubs launch nothing and count the calls; the one that stands in for the MFMA
// scoring kernels also checks the plan it is handed against what those kernels assume about it (tilings that are
// instantiated, key chunks within the LDS capacity, chunk bookkeeping) and keeps it for the tests to look at.
#include "../../paper_2604_06746_amd/csrc/common.h"

namespace skv {

static int g_launches = 0;
static int32_t g_last_plan[8];
extern "C" int structkv_stub_launch_count(void) { return g_launches; }
// RB, NW, KC, planes, stream_k, RC, grid_chunks, path of the latest MFMA scoring launch
extern "C" void structkv_stub_last_plan(int32_t* out) { for (int i = 0; i < 8; ++i) out[i] = g_last_plan[i]; }

hipError_t launch_score_mfma_ring(const structkv_shape& s, const ScorePlan& p, const SeqTable& seq, const void*,
                                  const void*, int64_t, int64_t, float, float*, const float*, float*, int64_t total,
                                  float* probs, int pass, hipStream_t) {
  ++g_launches;
  const int32_t plan[8] = {p.RB, p.NW, p.KC, p.planes, p.stream_k, p.RC, (int32_t)p.grid_chunks, p.path};
  for (int i = 0; i < 8; ++i) g_last_plan[i] = plan[i];
  if (p.grid_chunks == 0) return hipSuccess;
  bool ok = p.path == 0 && (s.head_dim == 64 || s.head_dim == 128) && (pass == 1 || pass == 2);
  ok = ok && ((p.RB == 2 && p.NW == 4) || (p.RB == 1 && p.NW == 4) || (p.RB == 2 && p.NW == 1) || (p.RB == 1 && p.NW == 1));
  ok = ok && p.RPC == 32 * p.RB && p.R == (s.n_q_heads / s.n_kv_heads) * s.window && p.RC == (p.R + p.RPC - 1) / p.RPC;
  ok = ok && (p.NW == 4 || p.RC == 1);                          // one-wave workgroups hold a KV group's only row-chunk
  const int planes = pass == 2 && probs == nullptr ? p.planes : 0;
  ok = ok && (planes == 0 || planes == 1 || (planes == 2 && p.RB == 2));
  const int cap = planes ? (p.NW == 4 ? (planes == 1 ? 1376 : 736) : 1024 / planes) : (p.NW == 4 ? 2048 : 896);   // keys whose sums fit the LDS
  ok = ok && p.KC >= 32 && p.KC % 32 == 0 && (pass == 1 || p.KC <= cap);
  ok = ok && (int64_t)s.n_kv_heads * ((p.RC + p.NW - 1) / p.NW) * p.grid_chunks < ((int64_t)1 << 31);
  ok = ok && seq.batch >= 1 && seq.batch <= kMaxBatch && seq.chunk_start[0] == 0 && seq.chunk_start[seq.batch] == p.grid_chunks;
  for (int b = 0; ok && b < seq.batch; ++b) {
    const int64_t n = seq.cu[b + 1] - seq.cu[b];
    ok = n >= 0 && seq.chunk_start[b + 1] - seq.chunk_start[b] == (n + p.KC - 1) / p.KC && seq.cu[b + 1] <= total;
  }
  return ok ? hipSuccess : hipErrorInvalidValue;
}
hipError_t launch_score_simt(const structkv_shape&, const ScorePlan&, const SeqTable&, const void*, const void*,
                             int64_t, int64_t, float, float*, const float*, float*, int64_t, float*, int,
                             hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_score_combine(const structkv_shape&, const ScorePlan&, const SeqTable&, const float*, float*,
                                float*, uint32_t*, int64_t, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_score_reduce(const structkv_shape&, const ScorePlan&, const SeqTable&, const float*, int64_t,
                               float*, const float*, float*, float*, float*, float, float, const SelectFusion*,
                               hipStream_t) {
  ++g_launches; return hipSuccess;
}
void topk_plan(const SeqTable& seq_in, int, void* wsp, SeqTable* plan, TopkWs* ws, unsigned* blocks) {
  *plan = seq_in;
  *blocks = 1;
  ws->hist = ws->state = ws->suf = ws->meta = (uint32_t*)wsp;
}
hipError_t launch_topk_rest(const float*, const SeqTable&, int, const TopkWs&, unsigned, int32_t*, hipStream_t) {
  ++g_launches; return hipSuccess;
}
hipError_t launch_group_sums(const structkv_shape&, const ScorePlan&, const float*, int64_t, float*, hipStream_t) {
  ++g_launches; return hipSuccess;
}
hipError_t launch_accumulate(float*, const float*, int64_t, float, float, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_topk(const float*, const SeqTable&, int, int32_t*, void*, hipStream_t) { ++g_launches; return hipSuccess; }
size_t topk_workspace_bytes(int batch, int64_t total_tokens) {
  return 256 * (size_t)(batch > 0 ? batch : 1) + 4 * (size_t)(total_tokens > 0 ? total_tokens : 0) + 256;
}
hipError_t topk_static_scratch(void** ptr, size_t* bytes) {
  alignas(256) static unsigned char host_stand_in[(size_t)4 << 20];   // never touched: the launchers are stubs
  *ptr = host_stand_in;
  *bytes = sizeof(host_stand_in);
  return hipSuccess;
}
int pivot_plane_shares(int64_t n) { return (int)((n + 2047) / 2048); }
hipError_t launch_pivot_planes(const float*, int, int64_t, float, uint32_t*, float*, hipStream_t) {
  ++g_launches; return hipSuccess;
}
hipError_t launch_topk_mass(const float*, int, int64_t, uint32_t, const TopkWs&, float*, float*, float*, float*, hipStream_t) {
  ++g_launches; return hipSuccess;
}
hipError_t launch_pivot_finish_planes(const float*, int, const float*, int, const float*, int, int64_t, float, float*,
                                      float*, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_pivot_heads(const float*, int, int64_t, const int32_t*, int64_t, float, float*, hipStream_t) {
  ++g_launches; return hipSuccess;
}
hipError_t launch_zero_floats(float*, int, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_pivot_finish(const float*, int, int64_t, float, int, float*, float*, hipStream_t) {
  ++g_launches; return hipSuccess;
}
hipError_t launch_block_scores(const float*, const SeqTable&, int, float*, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_positions(const int64_t*, const SeqTable&, const int32_t*, int64_t*, hipStream_t) {
  ++g_launches; return hipSuccess;
}
hipError_t launch_gather(const void*, const void*, int64_t, int64_t, void*, void*, int64_t, int64_t, int, int,
                         const SeqTable&, const int32_t*, hipStream_t) { ++g_launches; return hipSuccess; }

}  // namespace skv
