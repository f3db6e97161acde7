// C ABI of the Quest decode hot path: argument validation and dispatch to the
// kernel launchers.  Nothing here allocates, frees or synchronises.
#include "quest_common.h"

#include <cstdarg>
#include <cstdio>

namespace quest {

namespace {
thread_local char g_error[512] = "";
}

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_error, sizeof(g_error), fmt, ap);
  va_end(ap);
}

int check_launch(const char* who) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    set_error("%s: launch failed: %s", who, hipGetErrorString(e));
    return QUEST_ERR_HIP;
  }
  return QUEST_OK;
}

int check_cache(const quest_cache* c, const char* who) {
  if (c == nullptr) {
    set_error("%s: cache is NULL", who);
    return QUEST_ERR_NULL;
  }
  if (c->head_dim != kHeadDim || page_shift_of(c->page_size) < 0) {
    set_error("%s: only head_dim == 128 and page_size 8, 16, 32 or 64 are supported (got %d, %d)",
              who, c->head_dim, c->page_size);
    return QUEST_ERR_UNSUPPORTED;
  }
  if (c->batch < 1 || c->num_heads < 1 || c->max_pages_per_seq < 1 || c->num_phys_pages < 1) {
    set_error("%s: batch, num_heads, max_pages_per_seq and num_phys_pages must be >= 1", who);
    return QUEST_ERR_SHAPE;
  }
  if (c->batch > 65535 || c->num_heads > 65535) {
    set_error("%s: batch and num_heads are limited to 65535 (grid dimensions)", who);
    return QUEST_ERR_SHAPE;
  }
  if ((int64_t)c->max_pages_per_seq * c->page_size > INT32_MAX) {
    set_error("%s: max_pages_per_seq * page_size exceeds the int32 range of seq_lens", who);
    return QUEST_ERR_SHAPE;
  }
  if (c->num_kv_heads < 0 || (c->num_kv_heads > 0 && c->num_heads % c->num_kv_heads != 0)) {
    set_error("%s: num_kv_heads must be 0 or a divisor of num_heads (got %d, %d)", who,
              c->num_kv_heads, c->num_heads);
    return QUEST_ERR_SHAPE;
  }
  if (c->page_table == nullptr || c->seq_lens == nullptr) {
    set_error("%s: page_table and seq_lens must not be NULL", who);
    return QUEST_ERR_NULL;
  }
  return QUEST_OK;
}

}  // namespace quest

using namespace quest;

extern "C" {

const char* quest_last_error(void) { return g_error; }

int quest_workspace_bytes(const quest_cache* cache, int32_t k_pages, size_t* out_bytes) {
  int r = check_cache(cache, "quest_workspace_bytes");
  if (r != QUEST_OK) return r;
  if (out_bytes == nullptr) {
    set_error("quest_workspace_bytes: out_bytes is NULL");
    return QUEST_ERR_NULL;
  }
  // with a page list: enough for quest_select_decode and quest_decode_step as well
  *out_bytes = k_pages > 0 ? step_workspace_bytes(*cache, k_pages) : decode_workspace_bytes(*cache, 0);
  return QUEST_OK;
}

int quest_build_meta(const quest_cache* cache, void* stream) {
  int r = check_cache(cache, "quest_build_meta");
  if (r != QUEST_OK) return r;
  if (cache->k_pool == nullptr || cache->meta == nullptr) {
    set_error("quest_build_meta: k_pool and meta must not be NULL");
    return QUEST_ERR_NULL;
  }
  return launch_build_meta(*cache, (hipStream_t)stream);
}

int quest_append_meta(const quest_cache* cache, const void* k_new, const void* v_new,
                      int32_t k_pool_write, void* stream) {
  int r = check_cache(cache, "quest_append_meta");
  if (r != QUEST_OK) return r;
  if (cache->meta == nullptr || k_new == nullptr) {
    set_error("quest_append_meta: meta and k_new must not be NULL");
    return QUEST_ERR_NULL;
  }
  if (k_pool_write &&
      (v_new == nullptr || cache->k_pool == nullptr || cache->v_pool == nullptr)) {
    set_error("quest_append_meta: k_pool_write needs v_new, k_pool and v_pool");
    return QUEST_ERR_NULL;
  }
  return launch_append_meta(*cache, k_new, v_new, k_pool_write != 0, (hipStream_t)stream);
}

int quest_estimate(const quest_cache* cache, const void* q, float* scores, void* stream) {
  int r = check_cache(cache, "quest_estimate");
  if (r != QUEST_OK) return r;
  if (cache->meta == nullptr || q == nullptr || scores == nullptr) {
    set_error("quest_estimate: meta, q and scores must not be NULL");
    return QUEST_ERR_NULL;
  }
  return launch_estimate(*cache, q, scores, (hipStream_t)stream);
}

int quest_append_estimate(const quest_cache* cache, const void* k_new, const void* v_new,
                          int32_t k_pool_write, const void* q, float* scores, void* stream) {
  int r = check_cache(cache, "quest_append_estimate");
  if (r != QUEST_OK) return r;
  if (cache->meta == nullptr || k_new == nullptr || q == nullptr || scores == nullptr) {
    set_error("quest_append_estimate: meta, k_new, q and scores must not be NULL");
    return QUEST_ERR_NULL;
  }
  if (k_pool_write &&
      (v_new == nullptr || cache->k_pool == nullptr || cache->v_pool == nullptr)) {
    set_error("quest_append_estimate: k_pool_write needs v_new, k_pool and v_pool");
    return QUEST_ERR_NULL;
  }
  return launch_append_estimate(*cache, k_new, v_new, k_pool_write != 0, q, scores,
                                (hipStream_t)stream);
}

int quest_topk_workspace_bytes(const quest_cache* cache, int32_t k_pages, size_t* out_bytes) {
  int r = check_cache(cache, "quest_topk_workspace_bytes");
  if (r != QUEST_OK) return r;
  if (out_bytes == nullptr) {
    set_error("quest_topk_workspace_bytes: out_bytes is NULL");
    return QUEST_ERR_NULL;
  }
  *out_bytes = k_pages >= 1 ? topk_scratch_bytes(*cache, k_pages) : 0;
  return QUEST_OK;
}

int quest_topk(const quest_cache* cache, const float* scores, int32_t k_pages, int32_t* topk_idx,
               int32_t* k_eff, void* workspace, size_t workspace_bytes, void* stream) {
  int r = check_cache(cache, "quest_topk");
  if (r != QUEST_OK) return r;
  if (scores == nullptr || topk_idx == nullptr) {
    set_error("quest_topk: scores and topk_idx must not be NULL");
    return QUEST_ERR_NULL;
  }
  if (k_pages < 1) {
    set_error("quest_topk: k_pages must be >= 1 (got %d)", k_pages);
    return QUEST_ERR_SHAPE;
  }
  const size_t need = topk_scratch_bytes(*cache, k_pages);
  if (workspace == nullptr || need == 0)  // one work-group per row
    return launch_topk(*cache, scores, k_pages, topk_idx, k_eff, (hipStream_t)stream);
  if (workspace_bytes < need) {
    set_error("quest_topk: workspace of %zu bytes needed for the two-stage selection, %zu given "
              "(pass NULL for the single-stage selection)", need, workspace_bytes);
    return QUEST_ERR_WORKSPACE;
  }
  return launch_topk_chunked(*cache, scores, k_pages, topk_idx, k_eff, workspace,
                             (hipStream_t)stream);
}

int quest_sparse_decode(const quest_cache* cache, const void* q, const int32_t* topk_idx,
                        int32_t k_pages, float sm_scale, void* out, int32_t out_is_fp16, float* lse,
                        void* workspace, size_t workspace_bytes, void* stream) {
  int r = check_cache(cache, "quest_sparse_decode");
  if (r != QUEST_OK) return r;
  if (cache->k_pool == nullptr || cache->v_pool == nullptr || q == nullptr || out == nullptr) {
    set_error("quest_sparse_decode: k_pool, v_pool, q and out must not be NULL");
    return QUEST_ERR_NULL;
  }
  if (topk_idx != nullptr && k_pages < 1) {
    set_error("quest_sparse_decode: k_pages must be >= 1 with a page list (got %d)", k_pages);
    return QUEST_ERR_SHAPE;
  }
  const size_t need = decode_workspace_bytes(*cache, topk_idx ? k_pages : 0);
  if (need > 0 && (workspace == nullptr || workspace_bytes < need)) {
    set_error("quest_sparse_decode: workspace of %zu bytes needed, %zu given", need,
              workspace ? workspace_bytes : (size_t)0);
    return QUEST_ERR_WORKSPACE;
  }
  return launch_sparse_decode(*cache, q, topk_idx, k_pages, sm_scale, out, out_is_fp16 != 0, lse,
                              workspace, (hipStream_t)stream);
}

int quest_select_decode(const quest_cache* cache, const void* q, const float* scores,
                        int32_t k_pages, float sm_scale, int32_t* topk_idx, int32_t* k_eff,
                        void* out, int32_t out_is_fp16, float* lse, void* workspace,
                        size_t workspace_bytes, void* stream) {
  int r = check_cache(cache, "quest_select_decode");
  if (r != QUEST_OK) return r;
  if (cache->k_pool == nullptr || cache->v_pool == nullptr || q == nullptr || scores == nullptr ||
      topk_idx == nullptr || out == nullptr) {
    set_error("quest_select_decode: k_pool, v_pool, q, scores, topk_idx and out must not be NULL");
    return QUEST_ERR_NULL;
  }
  if (k_pages < 1) {
    set_error("quest_select_decode: k_pages must be >= 1 (got %d)", k_pages);
    return QUEST_ERR_SHAPE;
  }
  const size_t need = step_workspace_bytes(*cache, k_pages);
  if (need > 0 && (workspace == nullptr || workspace_bytes < need)) {
    set_error("quest_select_decode: workspace of %zu bytes needed, %zu given", need,
              workspace ? workspace_bytes : (size_t)0);
    return QUEST_ERR_WORKSPACE;
  }
  return launch_select_decode(*cache, q, scores, k_pages, sm_scale, topk_idx, k_eff, out,
                              out_is_fp16 != 0, lse, workspace, (hipStream_t)stream);
}

int quest_step_workspace_bytes(const quest_cache* cache, int32_t k_pages, size_t* out_bytes) {
  int r = check_cache(cache, "quest_step_workspace_bytes");
  if (r != QUEST_OK) return r;
  if (out_bytes == nullptr) {
    set_error("quest_step_workspace_bytes: out_bytes is NULL");
    return QUEST_ERR_NULL;
  }
  if (k_pages < 1) {
    set_error("quest_step_workspace_bytes: k_pages must be >= 1 (got %d)", k_pages);
    return QUEST_ERR_SHAPE;
  }
  *out_bytes = step_workspace_bytes(*cache, k_pages);
  return QUEST_OK;
}

int quest_decode_step(const quest_cache* cache, const void* k_new, const void* v_new,
                      int32_t k_pool_write, const void* q, int32_t k_pages, float sm_scale,
                      float* scores, int32_t* topk_idx, int32_t* k_eff, void* out,
                      int32_t out_is_fp16, float* lse, void* workspace, size_t workspace_bytes,
                      void* stream) {
  int r = check_cache(cache, "quest_decode_step");
  if (r != QUEST_OK) return r;
  if (cache->k_pool == nullptr || cache->v_pool == nullptr || cache->meta == nullptr ||
      q == nullptr || scores == nullptr || topk_idx == nullptr || out == nullptr) {
    set_error("quest_decode_step: k_pool, v_pool, meta, q, scores, topk_idx and out must not be NULL");
    return QUEST_ERR_NULL;
  }
  if (k_new != nullptr && k_pool_write && v_new == nullptr) {
    set_error("quest_decode_step: k_pool_write needs v_new");
    return QUEST_ERR_NULL;
  }
  if (k_pages < 1) {
    set_error("quest_decode_step: k_pages must be >= 1 (got %d)", k_pages);
    return QUEST_ERR_SHAPE;
  }
  const size_t need = step_workspace_bytes(*cache, k_pages);
  if (need > 0 && (workspace == nullptr || workspace_bytes < need)) {
    set_error("quest_decode_step: workspace of %zu bytes needed, %zu given", need,
              workspace ? workspace_bytes : (size_t)0);
    return QUEST_ERR_WORKSPACE;
  }
  return launch_decode_step(*cache, k_new, v_new, k_pool_write != 0, q, k_pages, sm_scale, scores,
                            topk_idx, k_eff, out, out_is_fp16 != 0, lse, workspace, workspace_bytes,
                            (hipStream_t)stream);
}

int quest_decode_step_static(const quest_cache* cache, const void* k_new, const void* v_new,
                             int32_t k_pool_write, const void* q, int32_t k_pages, float sm_scale,
                             float* scores, int32_t* topk_idx, int32_t* k_eff, void* out,
                             int32_t out_is_fp16, float* lse, void* stream) {
  int r = check_cache(cache, "quest_decode_step_static");
  if (r != QUEST_OK) return r;
  if (cache->k_pool == nullptr || cache->v_pool == nullptr || cache->meta == nullptr ||
      q == nullptr || scores == nullptr || topk_idx == nullptr || out == nullptr) {
    set_error("quest_decode_step_static: k_pool, v_pool, meta, q, scores, topk_idx and out must not be NULL");
    return QUEST_ERR_NULL;
  }
  if (k_new != nullptr && k_pool_write && v_new == nullptr) {
    set_error("quest_decode_step_static: k_pool_write needs v_new");
    return QUEST_ERR_NULL;
  }
  if (k_pages < 1) {
    set_error("quest_decode_step_static: k_pages must be >= 1 (got %d)", k_pages);
    return QUEST_ERR_SHAPE;
  }
  return launch_decode_step_static(*cache, k_new, v_new, k_pool_write != 0, q, k_pages, sm_scale,
                                   scores, topk_idx, k_eff, out, out_is_fp16 != 0, lse,
                                   (hipStream_t)stream);
}

}  // extern "C"
