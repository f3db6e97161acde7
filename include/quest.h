/*
 * quest.h -- C ABI of the Quest decode hot path for AMD MI355X (gfx950).
 *
 * Quest (arXiv 2406.10774) keeps the whole KV cache, organised in pages, and
 * at every decode step (i) scores each page with an upper bound of the
 * attention logit any of its tokens can reach, computed from the channel-wise
 * min and max of the page's keys, (ii) keeps the K best pages and (iii) runs
 * ordinary decode attention over those pages only (Section 3.4, Algorithm 1
 * and Figure 5 of the paper).  This library is that path, one call per step:
 *
 *     after prefill :  quest_build_meta
 *     every token   :  quest_append_meta -> quest_estimate -> quest_topk
 *                      -> quest_sparse_decode
 *                      (quest_append_estimate fuses the first two launches,
 *                       quest_select_decode the last two; quest_decode_step
 *                       is the whole step in one call)
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller.  The library
 *     never allocates or frees device memory and keeps no state between calls
 *     (quest_decode_step_static alone works in a static device array of the
 *     library instead of a caller's workspace: see there).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work on that stream; they never synchronise.
 *   - The return value is a quest_status; 0 means "enqueued".  Only facts the
 *     host can see are validated (null pointers, unsupported head_dim /
 *     page_size, k_pages < 1, workspace too small, a failed launch).  What
 *     lives in device memory (seq_lens, page_table, topk_idx) is trusted:
 *     1 <= seq_lens[b] <= max_pages_per_seq * page_size, and every logical
 *     page that holds a token maps to a physical page < num_phys_pages.
 *   - fp16 means IEEE binary16.  Keys, values and queries must be finite
 *     (NaN/Inf in a *valid* slot is undefined behaviour; stale slots beyond
 *     seq_lens are never used, whatever they contain).
 *   - Supported shapes: head_dim == 128; page_size 8, 16, 32 or 64 tokens (the
 *     paper's default is 16; Figure 8 sweeps the page size); multi-head
 *     attention (one KV head per query head) or grouped-query attention (below).
 *
 * Layouts (row-major, innermost last)
 *   k_pool, v_pool : fp16  [num_phys_pages][num_heads][page_size][head_dim]
 *   meta           : fp16  [num_heads][num_phys_pages][2][head_dim]  (head-major:
 *                          the estimate scans all pages of a head)
 *                          [..][0][:] = channel-wise min, [..][1][:] = max
 *   page_table     : int32 [batch][max_pages_per_seq]; logical page p of
 *                          sequence b (tokens [p*S, p*S+S)) -> physical page
 *   seq_lens       : int32 [batch], tokens currently valid
 *   q, k_new, v_new: fp16  [batch][num_heads][head_dim]
 *   scores         : fp32  [batch][num_heads][max_pages_per_seq]
 *   topk_idx       : int32 [batch][num_heads][k_pages]
 *   out            : fp32 or fp16 [batch][num_heads][head_dim]
 *   lse            : fp32  [batch][num_heads]
 *
 * Grouped-query attention (num_kv_heads = Hkv < num_heads = H, G = H / Hkv; the
 * paper's models have G == 1 and it gives no rule for groups, this is the
 * library's reading): query heads [g G, (g + 1) G) share KV head g.  k_pool,
 * v_pool, meta, k_new, v_new, scores and topk_idx then have Hkv where the
 * layouts above say num_heads; q, out and lse keep H.  A page's score for a KV
 * head is the largest of the scores of the group's query heads (each computed
 * as in quest_estimate against that KV head's metadata): still an upper bound
 * of every attention logit any head of the group can reach in the page.  One
 * page list per KV head; every query head of the group attends over it.
 */
#ifndef QUEST_H_
#define QUEST_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum quest_status {
  QUEST_OK = 0,
  QUEST_ERR_NULL = -1,        /* a required pointer is NULL                  */
  QUEST_ERR_SHAPE = -2,       /* a size is < 1 or exceeds a launch limit     */
  QUEST_ERR_UNSUPPORTED = -3, /* head_dim != 128, page_size not 8/16/32/64    */
  QUEST_ERR_WORKSPACE = -4,   /* workspace NULL or smaller than required     */
  QUEST_ERR_HIP = -5          /* the HIP runtime refused the launch          */
} quest_status;

/* quest_cache.flags.
 *  QUEST_FLAG_SEPARATE_LAUNCHES: quest_decode_step always enqueues the three
 *    separate launches (estimate, Top-K, attention) instead of letting the
 *    attention launch select its pages (see there; changes no result except
 *    the rounding of out / lse).
 *  QUEST_FLAG_DEVICE_FENCES: work-groups that exchange partial results inside a
 *    launch put device-scope release/acquire fences around their arrival
 *    counter (the textbook form of the hand-over; by default the results
 *    travel through device-scope stores and loads and need no fence).  For
 *    testing that path: slower, changes no result.
 *  QUEST_FLAG_KEEP_FIRST_PAGE, QUEST_FLAG_KEEP_NEWEST_PAGE: selection policy of
 *    quest_topk and quest_decode_step.  The paper selects purely by score
 *    (Section 3.4) and that is the default; with these flags logical page 0
 *    (the first tokens of the sequence) and / or the page that holds the newest
 *    token are in the list whatever their score: they rank above every score
 *    and among themselves by page index, so they take the first places of the K
 *    and the remaining places are filled by score. */
enum {
  QUEST_FLAG_SEPARATE_LAUNCHES = 1,
  QUEST_FLAG_DEVICE_FENCES = 2,
  QUEST_FLAG_KEEP_FIRST_PAGE = 4,
  QUEST_FLAG_KEEP_NEWEST_PAGE = 8
};

/* Description of one layer's paged KV cache.  Host struct, passed by pointer;
 * the library reads it during the call only. */
typedef struct quest_cache {
  int32_t batch;              /* B >= 1                                      */
  int32_t num_heads;          /* H >= 1                                      */
  int32_t head_dim;           /* D, must be 128                              */
  int32_t page_size;          /* S: 8, 16, 32 or 64                          */
  int32_t max_pages_per_seq;  /* row stride of page_table and of scores      */
  int32_t flags;              /* QUEST_FLAG_* bits, normally 0               */
  int64_t num_phys_pages;     /* capacity of the pools, in pages             */
  void* k_pool;               /* device, fp16                                */
  void* v_pool;               /* device, fp16                                */
  void* meta;                 /* device, fp16                                */
  const int32_t* page_table;  /* device                                      */
  const int32_t* seq_lens;    /* device                                      */
  int32_t num_kv_heads;       /* 0 or num_heads: one KV head per query head;
                                 else a divisor of num_heads (see below)     */
} quest_cache;

/* Bytes of device workspace quest_sparse_decode, quest_select_decode and
 * quest_decode_step need for this cache and k_pages (k_pages <= 0: the dense
 * path of quest_sparse_decode over all pages).  Pure host function.
 * The workspace holds one arrival counter per (sequence, head) and the split-K
 * partial results (running max, denominator and un-normalised accumulator of
 * each split); for rows of 16384 pages or more also the candidates of the
 * two-stage selection that quest_select_decode and quest_decode_step then use
 * (the best k_pages of every 4096-page chunk of a row, when there are at most
 * 8192 of them per row).  *out_bytes may be 0.
 * A workspace must be zero-filled once, after it is allocated and before its
 * first use (e.g. hipMemset); every call leaves the counters at zero again, so
 * the same workspace serves later calls, sparse or dense, on the same cache
 * shape.  Calls that share a workspace must not overlap in time. */
int quest_workspace_bytes(const quest_cache* cache, int32_t k_pages, size_t* out_bytes);

/* Metadata of every page that holds at least one token (Section 3.4): per
 * head and channel, the smallest and the largest key value among the page's
 * tokens:
 *   meta[h][phys][0][i] = min_j k[j][i],  meta[h][phys][1][i] = max_j k[j][i]
 * over the valid tokens j of the page (a partial last page: its first
 * seq_len - p*S slots).  Comparison is by value with -0 ordered below +0, so
 * the result is independent of reduction order and bit-exact.  Entries of
 * pages without tokens are not written.  To be called once after prefill;
 * also the recovery path (metadata is a pure function of the keys). */
int quest_build_meta(const quest_cache* cache, void* stream);

/* Insertion half of Algorithm 1.  seq_lens[b] already counts the new token,
 * which sits at position L-1: slot (L-1) % S of logical page (L-1) / S.
 * If k_pool_write != 0 the token's key and value (v_new must then be
 * non-NULL) are first stored into that slot of k_pool / v_pool.  Then the key
 * is folded into the page's entry: slot 0 opens the page (min = max = k),
 * otherwise max = max(max, k), min = min(min, k) per channel, same ordering
 * as quest_build_meta.  v_new may be NULL when k_pool_write == 0. */
int quest_append_meta(const quest_cache* cache, const void* k_new, const void* v_new,
                      int32_t k_pool_write, void* stream);

/* Attention half of Algorithm 1: for every sequence b, head h and logical
 * page p < ceil(seq_lens[b] / S),
 *   scores[b][h][p] = sum_i max(q[i] * min[p][i], q[i] * max[p][i]),
 * unscaled; fp16 products are exact in fp32, accumulation is fp32.  Entries
 * p >= ceil(seq_lens[b]/S) of a row are not written. */
int quest_estimate(const quest_cache* cache, const void* q, float* scores, void* stream);

/* quest_append_meta followed by quest_estimate in one launch (both halves of
 * Algorithm 1 for the step's new token and new query): same arguments, same
 * results in k_pool / v_pool / meta / scores, bit for bit.  The wave that scores
 * the newest token's page performs the insertion on the metadata it holds in
 * registers. */
int quest_append_estimate(const quest_cache* cache, const void* k_new, const void* v_new,
                          int32_t k_pool_write, const void* q, float* scores, void* stream);

/* Top-K filtering (Section 3.4): for every (b, h) the K_b = min(k_pages, P_b)
 * pages with the largest score among the P_b = ceil(seq_lens[b]/S) valid ones.
 * Scores compare by value (-0 == +0); of equal scores the lower page index is
 * kept.  QUEST_FLAG_KEEP_* in cache->flags force pages into the list (see
 * there).  topk_idx[b][h][0..K_b) receives the chosen logical page ids in
 * ascending order, the rest of the row is set to -1.  k_eff (nullable, int32
 * [batch], device) receives K_b.  Deterministic.
 * workspace (nullable): one work-group per row needs none, and that is what runs
 * with workspace == NULL at any row length.  Rows of 16384 pages or more are
 * selected faster in two stages (a work-group per 4096-page chunk keeps the
 * chunk's best k_pages, a second launch selects among those candidates; same
 * result bit for bit, ties and forced pages included) when a workspace of at
 * least quest_topk_workspace_bytes(cache, k_pages) bytes is given; for shapes
 * where that size is 0 the workspace is ignored. */
int quest_topk(const quest_cache* cache, const float* scores, int32_t k_pages,
               int32_t* topk_idx, int32_t* k_eff, void* workspace, size_t workspace_bytes,
               void* stream);

/* Bytes of device workspace with which quest_topk selects in two stages (0: this
 * shape is always selected by one work-group per row and needs none).  Pure host
 * function.  The workspace holds the candidates of the first stage (score and page
 * of the best k_pages of every 4096-page chunk of a row); it need not be
 * initialised and keeps nothing between calls. */
int quest_topk_workspace_bytes(const quest_cache* cache, int32_t k_pages, size_t* out_bytes);

/* Approximate attention (Figure 5, stage 2): ordinary softmax attention of q
 * over the valid tokens of the listed pages only,
 *   out[b][h][:] = sum_j softmax_j(sm_scale * q.k_j) * v_j,
 *   lse[b][h]    = log sum_j exp(sm_scale * q.k_j)            (nullable).
 * The first min(k_pages, max_pages_per_seq) entries of a topk_idx row are
 * read; an entry that is negative, or the id of a page without
 * tokens (>= P_b), is skipped wherever it stands, so lists padded with -1 as
 * quest_topk writes them need no length.  A page listed twice is attended
 * twice.  topk_idx == NULL selects every page: the dense baseline (k_pages is
 * then ignored).  fp16 inputs, fp32 dot products, fp32 online
 * softmax over splits of the page list; the split that finishes last merges
 * them.  out is fp32
 * if out_is_fp16 == 0, else fp16 (rounded once, from the fp32 result).
 * workspace: at least quest_workspace_bytes(cache, topk_idx ? k_pages : 0). */
int quest_sparse_decode(const quest_cache* cache, const void* q, const int32_t* topk_idx,
                        int32_t k_pages, float sm_scale, void* out, int32_t out_is_fp16,
                        float* lse, void* workspace, size_t workspace_bytes, void* stream);

/* quest_topk followed by quest_sparse_decode with the list just selected
 * (Section 3.4 and Figure 5, stage 2), for scores that already exist.  topk_idx
 * / k_eff receive exactly what quest_topk would write, bit for bit; out and lse
 * are the attention result of quest_sparse_decode over that list (equal within
 * fp32 rounding: the list is split differently).  One launch, in which every
 * work-group first selects the pages of its (sequence, KV head) from the scores
 * and keeps the list in on-chip memory, when k_pages <= 2048 and
 * max_pages_per_seq <= 4096 and QUEST_FLAG_SEPARATE_LAUNCHES is not set; else
 * the selection and the attention as launches of their own (the selection in
 * two stages for very long rows, see quest_workspace_bytes).
 * workspace: at least quest_workspace_bytes(cache, k_pages). */
int quest_select_decode(const quest_cache* cache, const void* q, const float* scores,
                        int32_t k_pages, float sm_scale, int32_t* topk_idx, int32_t* k_eff,
                        void* out, int32_t out_is_fp16, float* lse, void* workspace,
                        size_t workspace_bytes, void* stream);

/* The whole decode step of one layer in one call (Algorithm 1 and
 * Figure 5): quest_append_estimate (quest_estimate if k_new == NULL), then
 * quest_topk, then quest_sparse_decode with the list just selected.  k_pool /
 * v_pool / meta / scores / topk_idx / k_eff receive exactly what those calls
 * would write, bit for bit; out and lse are the same attention result,
 * accumulated over a different split of the page list (so equal within fp32
 * rounding, not bit for bit).  scores and topk_idx are outputs and also the
 * buffers the phases hand to each other, so they must be provided.
 * workspace: at least quest_step_workspace_bytes(cache, k_pages) bytes (the
 * same size as quest_workspace_bytes gives for k_pages), zero-filled once after
 * allocation (same rule as for quest_sparse_decode; one buffer may serve both
 * calls); calls sharing a workspace must not overlap in time.
 * The call enqueues the estimate, then what quest_select_decode enqueues: two
 * launches in all when k_pages <= 2048 and max_pages_per_seq <= 4096 and
 * QUEST_FLAG_SEPARATE_LAUNCHES is not set, else three (four with the two-stage
 * selection of very long rows). */
int quest_step_workspace_bytes(const quest_cache* cache, int32_t k_pages, size_t* out_bytes);
int quest_decode_step(const quest_cache* cache, const void* k_new, const void* v_new,
                      int32_t k_pool_write, const void* q, int32_t k_pages, float sm_scale,
                      float* scores, int32_t* topk_idx, int32_t* k_eff, void* out,
                      int32_t out_is_fp16, float* lse, void* workspace, size_t workspace_bytes,
                      void* stream);

/* quest_decode_step for callers that cannot allocate or carry a workspace: code
 * that runs under HIP graph capture in a harness that forbids hipMalloc, tight
 * serving loops, test harnesses.  Same arguments, launches and results as
 * quest_decode_step, but the decode workspace lives in a static device array of
 * the library (4 MiB per GPU, held until the process ends) instead of caller
 * memory.  The call allocates and frees nothing.  Shapes whose workspace
 * (quest_step_workspace_bytes) exceeds 4 MiB are refused with
 * QUEST_ERR_WORKSPACE.  The call first enqueues a small kernel that zeroes the
 * arrival counters it is going to use (the array keeps the previous call's
 * contents).  All calls on one GPU share the one array: calls that overlap in
 * time on the same GPU (different streams, or graphs replayed concurrently) race;
 * serialise them, or use quest_decode_step with a workspace per stream.  The
 * first call on a device looks the array's address up (no stream work); make
 * that first call outside stream capture. */
int quest_decode_step_static(const quest_cache* cache, const void* k_new, const void* v_new,
                             int32_t k_pool_write, const void* q, int32_t k_pages,
                             float sm_scale, float* scores, int32_t* topk_idx, int32_t* k_eff,
                             void* out, int32_t out_is_fp16, float* lse, void* stream);

/* Human-readable description of the last error on the calling thread.  Host
 * string owned by the library, valid until the thread's next failing call. */
const char* quest_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* QUEST_H_ */
