// Stand-ins for the kernel launchers of libstructkv, for the host-only sanitizer build of its C ABI:
// api.cpp is compiled with -fsanitize=address,undefined and linked against these instead of the HIP
// kernels, so that argument validation, work planning and workspace carving run under the sanitizers
// on a machine without a GPU.  Each stub checks nothing and launches nothing; it only counts the call.
#include "../../paper_2604_06746_amd/csrc/common.h"

namespace skv {

static int g_launches = 0;
extern "C" int structkv_stub_launch_count(void) { return g_launches; }

hipError_t launch_score_mfma_ring(const structkv_shape&, const ScorePlan&, const SeqTable&, const void*, const void*,
                                  int64_t, int64_t, float, float*, const float*, float*, int64_t, float*, int,
                                  hipStream_t) { ++g_launches; return hipSuccess; }
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
hipError_t launch_topk_mass(const float*, const SeqTable&, const TopkWs&, unsigned, int, float*, float*, hipStream_t) {
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
