// Top-K page selection (Section 3.4 of arXiv 2406.10774: "choose the top K
// pages as critical").  One work-group per (sequence, head).
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
#ifdef QUEST_STEP_TRACE
  if (threadIdx.x == 0) sm.trace = nullptr;
#endif
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

}  // namespace quest
