// The whole decode step of one layer in one call: insertion of the new token,
// criticality estimate, Top-K selection and sparse attention (Algorithm 1 and
// Figure 5 of arXiv 2406.10774), as two launches:
//   1. quest_append_estimate (quest_estimate without a new token): the metadata stream;
//   2. quest_select_decode: the attention kernel with the selection inside
//      (quest_decode.hip): every work-group selects the pages of its head itself from
//      the scores, keeps the list in LDS and attends over its slice; one of them writes
//      the list out.
// Same arithmetic as the separate calls (shared device cores): metadata, scores
// and the page list are bit-equal to theirs.  When a row of scores or the list is
// too long for that, the selection runs as its own launch (three launches).
//
// A single launch for the whole step (teams of work-groups per head that wait for
// each other through L2) was built and measured twice: 24.2 us against 23.5 us for
// these two launches at 32 heads / 32k context in its first form, 28.5 us against
// 21.6 us in its second (the estimate's pages spread over the attention launch's 256
// work-groups).  The metadata scan wants tens of thousands of waves, the attention
// part 256 work-groups of 8; one grid cannot be both, and the wait needs the whole grid
// resident at once.  It is not part of the library.
#include "quest_common.h"

namespace quest {

size_t step_workspace_bytes(const quest_cache& c, int k_pages) {
  return decode_workspace_bytes(c, k_pages) + topk_scratch_bytes(c, k_pages);
}

int launch_decode_step(const quest_cache& c, const void* k_new, const void* v_new, int k_pool_write,
                       const void* q, int k_pages, float sm_scale, float* scores, int32_t* topk_idx,
                       int32_t* k_eff, void* out, int out_is_fp16, float* lse, void* workspace,
                       size_t workspace_bytes, hipStream_t s) {
  (void)workspace_bytes;  // checked by the caller
  int r = k_new ? launch_append_estimate(c, k_new, v_new, k_pool_write, q, scores, s)
                : launch_estimate(c, q, scores, s);
  if (r != QUEST_OK) return r;
  return launch_select_decode(c, q, scores, k_pages, sm_scale, topk_idx, k_eff, out, out_is_fp16, lse,
                              workspace, s);
}

}  // namespace quest
