// Top-K page selection (Section 3.4 of arXiv 2406.10774: the K pages with the
// largest criticality score are the ones attended).  One work-group per
// (sequence, head).
//
// Scores are mapped to unsigned 32-bit keys whose integer order equals the
// order of the float values (-0 folded onto +0), taken relative to the row's
// smallest key and shifted left so that the leading bit of the row's range is
// bit 31.  An MSB-first radix select (8-bit digits, LDS histogram per digit)
// narrows down the key of the K-th largest score; it stops as soon as every key
// left in the threshold bin belongs to the selection, or the range's bits are
// used up.  A final pass in page order emits every page above
// the threshold bin plus the first `need` pages inside it, each at the position
// given by a block-wide prefix count, so the output is ascending and the lowest
// page index wins among equal scores.
//
// The kernel is latency-bound (a few thousand keys per head), so the work is
// organised to shorten the dependent chain: keys live in registers (thread t
// owns pages [t*ITEMS, (t+1)*ITEMS)), the score loads are issued before
// seq_lens is known, the range normalisation makes the first digit spread the
// row over the whole histogram (scores of one head share sign and most of the
// exponent: on raw keys the first one or two digits would decide nothing, and
// their LDS atomics would all hit the same few bins), every wave searches the
// histogram for the threshold bin itself so a pass needs a single barrier, and
// lanes that carry the first lane's digit share one LDS atomic in the first
// pass (a row with outliers still puts most keys into one bin there).
#include "quest_common.h"
#include "quest_topk_core.h"

namespace quest {

namespace {

template <int kThreads, int kItems>
__global__ __launch_bounds__(kThreads) void topk_kernel(
    const float* __restrict__ scores, const int32_t* __restrict__ seq_lens,
    int32_t* __restrict__ topk_idx, int32_t* __restrict__ k_eff, int num_heads, int max_pages,
    int k_pages, int page_shift, int policy) {
  __shared__ TopkShared<kThreads> sm;
  const int h = blockIdx.x;
  const int b = blockIdx.y;
  const size_t bh = (size_t)b * num_heads + h;
  topk_block<kThreads, kItems>(sm, scores + bh * max_pages, seq_lens + b, max_pages, k_pages,
                                      topk_idx + bh * k_pages,
                                      (h == 0 && k_eff != nullptr) ? k_eff + b : nullptr, page_shift,
                                      policy);
}

// Fallback for rows too long for register-resident keys: keys are re-read from
// global memory (L2) in every pass; same algorithm without the shortcuts.
constexpr int kBigThreads = 1024;
__global__ __launch_bounds__(kBigThreads) void topk_big_kernel(
    const float* __restrict__ scores, const int32_t* __restrict__ seq_lens,
    int32_t* __restrict__ topk_idx, int32_t* __restrict__ k_eff, int num_heads, int max_pages,
    int k_pages, int page_shift, int policy) {
  constexpr int kWaves = kBigThreads / kWave;
  __shared__ uint32_t hist[256];
  __shared__ int wave_gt[kWaves], wave_eq[kWaves];
  const int h = blockIdx.x;
  const int b = blockIdx.y;
  const int tid = threadIdx.x;
  const int lane = lane_id();
  const int wave = tid >> 6;
  const int num_pages = (seq_lens[b] + (1 << page_shift) - 1) >> page_shift;
  const int K = min(k_pages, num_pages);
  const float* row = scores + ((size_t)b * num_heads + h) * max_pages;
  int32_t* out = topk_idx + ((size_t)b * num_heads + h) * k_pages;
  if (h == 0 && tid == 0 && k_eff != nullptr) k_eff[b] = K;
  if (K == num_pages) {
    for (int i = tid; i < k_pages; i += kBigThreads) out[i] = i < K ? i : -1;
    return;
  }
  const ForcedPages forced = forced_pages(policy, num_pages);
  if (forced.count >= K) {
    if (tid == 0) {
      out[0] = forced.first ? 0 : num_pages - 1;
      if (K == 2) out[1] = num_pages - 1;
    }
    return;
  }
  auto key_of = [&](int i) { return forced.is(i) ? 0xffffffffu : score_key(row[i]); };
  uint32_t prefix = 0;
  int need = K;
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    const uint32_t high_mask = pass == 0 ? 0u : (0xffffffffu << (shift + 8));
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    for (int i = tid; i < num_pages; i += kBigThreads) {
      const uint32_t key = key_of(i);
      if ((key & high_mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
    }
    __syncthreads();
    const BinHit hit = find_bin(hist, need, lane);
    prefix |= (uint32_t)hit.bin << shift;
    need -= hit.above;
    __syncthreads();
  }
  const uint32_t T = prefix;
  const int items = (num_pages + kBigThreads - 1) / kBigThreads;
  const int begin = min(tid * items, num_pages);
  const int end = min(begin + items, num_pages);
  int n_gt = 0, n_eq = 0;
  for (int i = begin; i < end; ++i) {
    const uint32_t key = key_of(i);
    n_gt += key > T;
    n_eq += key == T;
  }
  const int gt_incl = wave_incl_scan(n_gt, lane);
  const int eq_incl = wave_incl_scan(n_eq, lane);
  if (lane == kWave - 1) {
    wave_gt[wave] = gt_incl;
    wave_eq[wave] = eq_incl;
  }
  __syncthreads();
  int gt_before = gt_incl - n_gt, eq_before = eq_incl - n_eq;
  for (int w = 0; w < kWaves; ++w) {
    if (w < wave) {
      gt_before += wave_gt[w];
      eq_before += wave_eq[w];
    }
  }
  for (int i = begin; i < end; ++i) {
    const uint32_t key = key_of(i);
    if (key > T) {
      out[gt_before + min(eq_before, need)] = i;
      ++gt_before;
    } else if (key == T) {
      if (eq_before < need) out[gt_before + eq_before] = i;
      ++eq_before;
    }
  }
}

// ---- Selection in two stages for very long rows.  One work-group per row is bound by
// what one compute unit can issue (about 0.75 us per key and thread at 1024 threads);
// here the row is cut into chunks of kChunkPages pages, a work-group per chunk selects
// the chunk's own best K pages (the K best of the row are among them, ties included:
// fewer than K pages of the chunk rank above any of them), and a second launch selects
// among the candidates.  Candidates are stored densely in page order (every chunk
// before the last non-empty one is full and yields exactly k_pages of them), so
// positions in the candidate row order like pages do: equal scores still go to the
// lower page, page 0 is candidate 0 and the newest page is the last candidate whenever
// the policy flags keep them in their chunks.
constexpr int kChunkThreads = 1024;  // 16 waves x 4 keys: 0.3 us faster than 8 waves x 8 keys
constexpr int kChunkItems = 4;
constexpr int kChunkPages = kChunkThreads * kChunkItems;

struct ChunkOfRow {
  int page_shift, policy, chunk;
  __device__ __forceinline__ RowShape operator()(int seq_len) const {
    const int pages = (seq_len + (1 << page_shift) - 1) >> page_shift;
    const int local = min(max(pages - chunk * kChunkPages, 0), kChunkPages);
    int pol = 0;
    if (chunk == 0) pol |= policy & QUEST_FLAG_KEEP_FIRST_PAGE;
    if (local > 0 && (chunk + 1) * kChunkPages >= pages) pol |= policy & QUEST_FLAG_KEEP_NEWEST_PAGE;
    return {local, pol};
  }
};

__global__ __launch_bounds__(kChunkThreads) void topk_chunk_kernel(
    const float* __restrict__ scores, const int32_t* __restrict__ seq_lens,
    float* __restrict__ cand_score, int32_t* __restrict__ cand_page, int num_heads, int max_pages,
    int k_pages, int num_chunks, int page_shift, int policy) {
  __shared__ TopkShared<kChunkThreads> sm;
  // chunk-major launch order: the last chunk of a row, often a short one, must not take
  // the place of a full one on a compute unit that is still free
  const int h = blockIdx.x;
  const int chunk = blockIdx.y;
  const int b = blockIdx.z;
  const size_t bh = (size_t)b * num_heads + h;
  const float* row = scores + bh * max_pages + (size_t)chunk * kChunkPages;
  const size_t at = (bh * num_chunks + chunk) * k_pages;
  float* out_score = cand_score + at;
  int32_t* out_page = cand_page + at;
  topk_block_put<kChunkThreads, kChunkItems>(
      sm, row, seq_lens + b, min(kChunkPages, max_pages - chunk * kChunkPages), k_pages,
      [=](int pos, int page, int j, float score) {
        if (page >= 0) {
          out_page[pos] = page + chunk * kChunkPages;
          out_score[pos] = j >= 0 ? score : row[page];
        }
      },
      nullptr, ChunkOfRow{page_shift, policy, chunk}, [] {});
}

struct CandidateRow {
  int page_shift, policy, k_pages;
  __device__ __forceinline__ RowShape operator()(int seq_len) const {
    const int pages = (seq_len + (1 << page_shift) - 1) >> page_shift;
    const int full = pages / kChunkPages;
    return {full * k_pages + min(k_pages, pages - full * kChunkPages), policy};
  }
};

template <int kThreads, int kItems>
__global__ __launch_bounds__(kThreads) void topk_candidates_kernel(
    const float* __restrict__ cand_score, const int32_t* __restrict__ cand_page,
    const int32_t* __restrict__ seq_lens, int32_t* __restrict__ topk_idx,
    int32_t* __restrict__ k_eff, int num_heads, int row_len, int k_pages, int page_shift,
    int policy) {
  __shared__ TopkShared<kThreads> sm;
  const int h = blockIdx.x;
  const int b = blockIdx.y;
  const size_t bh = (size_t)b * num_heads + h;
  const int32_t* pages = cand_page + bh * row_len;
  int32_t* out = topk_idx + bh * k_pages;
  // the pages of this thread's candidates travel behind their scores (entries past the
  // stored candidates are inside the row: never selected, safe to read)
  int32_t my_page[kItems];
  topk_block_put<kThreads, kItems>(
      sm, cand_score + bh * row_len, seq_lens + b, row_len, k_pages,
      [&](int pos, int cand, int j, float) {
        int32_t page = -1;
        if (j >= 0) {
#pragma unroll
          for (int jj = 0; jj < kItems; ++jj)
            if (jj == j) page = my_page[jj];
        } else if (cand >= 0) {
          page = pages[cand];
        }
        out[pos] = page;
      },
      (h == 0 && k_eff != nullptr) ? k_eff + b : nullptr, CandidateRow{page_shift, policy, k_pages},
      [&] {
#pragma unroll
        for (int jj = 0; jj < kItems; ++jj)
          my_page[jj] = pages[min((int)threadIdx.x * kItems + jj, row_len - 1)];
      });
}

template <int kThreads, int kItems>
int launch_one(const quest_cache& c, const float* scores, int k_pages, int32_t* topk_idx,
               int32_t* k_eff, hipStream_t s) {
  hipLaunchKernelGGL((topk_kernel<kThreads, kItems>), dim3(kv_heads(c), c.batch), dim3(kThreads), 0,
                     s, scores, c.seq_lens, topk_idx, k_eff, kv_heads(c), c.max_pages_per_seq,
                     k_pages, page_shift_of(c.page_size), c.flags);
  return check_launch("quest_topk");
}

}  // namespace

int launch_topk(const quest_cache& c, const float* scores, int k_pages, int32_t* topk_idx,
                int32_t* k_eff, hipStream_t s) {
  const int mp = c.max_pages_per_seq;
#define QUEST_TOPK_CASE(T, I) \
  if (mp <= (T) * (I)) return launch_one<T, I>(c, scores, k_pages, topk_idx, k_eff, s)
  // up to 8192 pages: 512 threads, smallest ITEMS that covers the row
  QUEST_TOPK_CASE(512, 1);
  QUEST_TOPK_CASE(512, 2);
  QUEST_TOPK_CASE(512, 3);
  QUEST_TOPK_CASE(512, 4);
  QUEST_TOPK_CASE(512, 5);
  QUEST_TOPK_CASE(512, 6);
  QUEST_TOPK_CASE(512, 8);
  QUEST_TOPK_CASE(512, 10);
  QUEST_TOPK_CASE(512, 12);
  QUEST_TOPK_CASE(512, 16);
  QUEST_TOPK_CASE(512, 20);
  // up to 65536 pages (the packed prefix counts hold 16 bits each)
  QUEST_TOPK_CASE(1024, 12);
  QUEST_TOPK_CASE(1024, 17);
  QUEST_TOPK_CASE(1024, 24);
  QUEST_TOPK_CASE(1024, 33);
  QUEST_TOPK_CASE(1024, 48);
  if (mp < 65536) return launch_one<1024, 64>(c, scores, k_pages, topk_idx, k_eff, s);
#undef QUEST_TOPK_CASE
  hipLaunchKernelGGL(topk_big_kernel, dim3(kv_heads(c), c.batch), dim3(kBigThreads), 0, s, scores,
                     c.seq_lens, topk_idx, k_eff, kv_heads(c), c.max_pages_per_seq, k_pages,
                     page_shift_of(c.page_size), c.flags);
  return check_launch("quest_topk");
}

// Rows from kChunkedFromPages pages on are selected in two stages when the caller
// brings scratch memory for the candidates (quest_select_decode, quest_decode_step).
constexpr int kChunkedFromPages = 16384;
constexpr int kMaxCandidates = 512 * 16;

static int num_chunks(const quest_cache& c) {
  return (c.max_pages_per_seq + kChunkPages - 1) / kChunkPages;
}

size_t topk_scratch_bytes(const quest_cache& c, int k_pages) {
  const long cand = (long)num_chunks(c) * k_pages;
  if (c.max_pages_per_seq < kChunkedFromPages || k_pages < 1 || k_pages > kChunkPages ||
      cand > kMaxCandidates || 2 * cand > c.max_pages_per_seq)
    return 0;
  return (size_t)c.batch * kv_heads(c) * cand * (sizeof(float) + sizeof(int32_t));
}

int launch_topk_chunked(const quest_cache& c, const float* scores, int k_pages, int32_t* topk_idx,
                        int32_t* k_eff, void* scratch, hipStream_t s) {
  const int chunks = num_chunks(c);
  const int row_len = chunks * k_pages;
  float* cand_score = (float*)scratch;
  int32_t* cand_page = (int32_t*)(cand_score + (size_t)c.batch * kv_heads(c) * row_len);
  hipLaunchKernelGGL(topk_chunk_kernel, dim3(kv_heads(c), chunks, c.batch), dim3(kChunkThreads), 0, s,
                     scores, c.seq_lens, cand_score, cand_page, kv_heads(c), c.max_pages_per_seq,
                     k_pages, chunks, page_shift_of(c.page_size), c.flags);
  int r = check_launch("quest_select_decode");
  if (r != QUEST_OK) return r;
#define QUEST_CAND_CASE(I)                                                                       \
  if (row_len <= 512 * (I)) {                                                                    \
    hipLaunchKernelGGL((topk_candidates_kernel<512, I>), dim3(kv_heads(c), c.batch), dim3(512), 0, \
                       s, cand_score, cand_page, c.seq_lens, topk_idx, k_eff, kv_heads(c), row_len, \
                       k_pages, page_shift_of(c.page_size), c.flags);                            \
    return check_launch("quest_select_decode");                                                  \
  }
  QUEST_CAND_CASE(2)
  QUEST_CAND_CASE(5)
  QUEST_CAND_CASE(8)
  QUEST_CAND_CASE(16)
#undef QUEST_CAND_CASE
  set_error("quest_select_decode: internal: %d candidates per row", row_len);
  return QUEST_ERR_SHAPE;
}

}  // namespace quest
