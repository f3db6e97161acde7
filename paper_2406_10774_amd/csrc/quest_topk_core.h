// Device-side core of the Top-K page selection (Section 3.4 of arXiv
// 2406.10774), shared by the stand-alone kernel and the attention launch that
// selects its pages itself.  See quest_topk.hip for the algorithm.
#pragma once

#include "quest_common.h"

namespace quest {

#if defined(__HIPCC__)

__device__ __forceinline__ uint32_t score_key(float s) {
  uint32_t u = __builtin_bit_cast(uint32_t, s);
  if (u == 0x80000000u) u = 0;  // -0 ranks equal to +0
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Inclusive prefix sum over the 64 lanes: DPP row shifts inside each 16-lane
// row, then the totals of the preceding rows.
__device__ __forceinline__ int wave_incl_scan(int v, int lane) {
  v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);  // row_shr:1
  v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);  // row_shr:2
  v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);  // row_shr:4
  v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);  // row_shr:8
  const int r0 = __builtin_amdgcn_readlane(v, 15);
  const int r1 = __builtin_amdgcn_readlane(v, 31);
  const int r2 = __builtin_amdgcn_readlane(v, 47);
  const int row = lane >> 4;
  return v + (row >= 1 ? r0 : 0) + (row >= 2 ? r1 : 0) + (row >= 3 ? r2 : 0);
}

// Minimum / maximum over the 64 lanes, returned in every lane (wave-uniform): DPP
// row shifts gather each 16-lane row's result in its last lane (a lane without a
// source keeps its own value), the four rows are combined on the scalar side.
__device__ __forceinline__ uint32_t wave_min(uint32_t v) {
  v = min(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x111, 0xf, 0xf, false));
  v = min(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x112, 0xf, 0xf, false));
  v = min(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x114, 0xf, 0xf, false));
  v = min(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x118, 0xf, 0xf, false));
  return min(min((uint32_t)__builtin_amdgcn_readlane((int)v, 15), (uint32_t)__builtin_amdgcn_readlane((int)v, 31)),
             min((uint32_t)__builtin_amdgcn_readlane((int)v, 47), (uint32_t)__builtin_amdgcn_readlane((int)v, 63)));
}
__device__ __forceinline__ uint32_t wave_max(uint32_t v) { return ~wave_min(~v); }

// Scan the 256-bin histogram from the top bin down for the bin that holds the
// need-th largest key.  Lane l owns bins 255-4l .. 252-4l.  Every lane returns
// the same (bin, keys above the bin, keys in the bin).
struct BinHit {
  int bin, above, count;
};
template <int kCopies = 1>  // the histogram is the sum of kCopies arrays of 256 bins
__device__ __forceinline__ BinHit find_bin(const uint32_t* hist, int need, int lane) {
  const int top = 255 - 4 * lane;
  int c0 = hist[top], c1 = hist[top - 1], c2 = hist[top - 2], c3 = hist[top - 3];
#pragma unroll
  for (int r = 1; r < kCopies; ++r) {
    c0 += hist[r * 256 + top], c1 += hist[r * 256 + top - 1];
    c2 += hist[r * 256 + top - 2], c3 += hist[r * 256 + top - 3];
  }
  const int tot = c0 + c1 + c2 + c3;
  const int incl = wave_incl_scan(tot, lane);
  int above = incl - tot;
  const bool mine = above < need && need <= incl;
  int bin = top, count = c0;
  if (need > above + c0) {
    above += c0, bin = top - 1, count = c1;
    if (need > above + c1) {
      above += c1, bin = top - 2, count = c2;
      if (need > above + c2) above += c2, bin = top - 3, count = c3;
    }
  }
  const int src = __ffsll((long long)__ballot(mine)) - 1;  // exactly one lane
  BinHit r;
  r.bin = __builtin_amdgcn_readlane(bin, src);
  r.above = __builtin_amdgcn_readlane(above, src);
  r.count = __builtin_amdgcn_readlane(count, src);
  return r;
}

// Pages kept whatever their score (quest.h: QUEST_FLAG_KEEP_FIRST_PAGE,
// QUEST_FLAG_KEEP_NEWEST_PAGE); the page of the newest token is the last valid one.
struct ForcedPages {
  bool first, newest;
  int newest_page, count;
  __device__ __forceinline__ bool is(int page) const {
    return (first && page == 0) || (newest && page == newest_page);
  }
};
__device__ __forceinline__ ForcedPages forced_pages(int policy, int num_pages) {
  ForcedPages f;
  f.newest_page = num_pages - 1;
  f.first = (policy & QUEST_FLAG_KEEP_FIRST_PAGE) != 0;
  f.newest = (policy & QUEST_FLAG_KEEP_NEWEST_PAGE) != 0 && !(f.first && f.newest_page == 0);
  f.count = (int)f.first + (int)f.newest;
  return f;
}

// The first digit is counted for every key of the row, and lanes with the same digit
// serialise on one LDS address: with many keys per thread it gets several copies of its
// histogram, chosen by lane (with few keys the extra clearing and summing cost more than
// the conflicts: 23.0 us vs 22.7 us per step at 2049 pages, 25 us vs 30 us at 32769).
constexpr int kMaxHistCopies0 = 4;
constexpr int hist_copies0(int items) { return items >= 10 ? kMaxHistCopies0 : 1; }

template <int kThreads>
struct TopkShared {
  uint32_t hist[kMaxHistCopies0 + 3][256];  // copies for the first digit, then one per later digit
  int wave_tot[kThreads / kWave];
  uint32_t range[kThreads / kWave][2];  // smallest and largest key seen by each wave
};

// What a row of scores is, given the sequence length: its number of valid entries and
// which of them are kept whatever their score (QUEST_FLAG_KEEP_* bits).
struct RowShape {
  int num_pages, policy;
};
// The row holds the scores of all pages of the sequence.
struct WholeRow {
  int page_shift, policy;
  __device__ __forceinline__ RowShape operator()(int seq_len) const {
    return {(seq_len + (1 << page_shift) - 1) >> page_shift, policy};
  }
};

// Selection for one row of scores by one work-group of kThreads threads (all of
// them must call).  shape(seq_len) describes the row (it has room for max_pages
// entries); put(position, page, j, score) receives the list: positions 0 .. k_pages-1,
// pages ascending, -1 past the K_b selected ones; j >= 0 says that the page is the calling
// thread's j-th one (page == threadIdx.x * kItems + j) and `score` its score as loaded,
// j < 0 that it is not (then `score` carries nothing).  A put that needs per-page data
// takes it from what the thread already holds whenever j >= 0: a load issued from inside
// put is waited for before the next page's put starts.
// after_loads() is called once, right after the loads of the scores have been issued:
// the place for loads the caller wants in flight behind them.
template <int kThreads, int kItems, class Put, class Shape, class AfterLoads>
__device__ __forceinline__ void topk_block_put(TopkShared<kThreads>& sm,
                                               const float* __restrict__ row,
                                               const int32_t* __restrict__ seq_len_ptr,
                                               int max_pages, int k_pages, Put put,
                                               int32_t* __restrict__ k_eff_slot, Shape shape,
                                               AfterLoads after_loads) {
  constexpr int kWaves = kThreads / kWave;
  constexpr int kCopies0 = hist_copies0(kItems);
  uint32_t(&hist)[kMaxHistCopies0 + 3][256] = sm.hist;
  int(&wave_tot)[kWaves] = sm.wave_tot;
  uint32_t(&range)[kWaves][2] = sm.range;
  const int tid = threadIdx.x;
  const int lane = lane_id();
  const int wave = tid >> 6;

  // issue every load first: this thread's scores (entries past the valid pages
  // are inside the row, so reading them is safe; they are masked below) and the
  // sequence length
  const int base = tid * kItems;
  float raw[kItems];
#pragma unroll
  for (int j = 0; j < kItems; ++j) {
    // clamped, not predicated: the loads stay independent and all in flight at once
    const int i = min(base + j, max_pages - 1);
    raw[j] = row[i];
  }
  const int seq_len = *seq_len_ptr;
  after_loads();

  for (int i = tid; i < (kCopies0 + 3) * 256; i += kThreads) (&hist[0][0])[i] = 0;

  const RowShape row_shape = shape(seq_len);
  const int num_pages = row_shape.num_pages;
  const int K = min(k_pages, num_pages);
  if (tid == 0 && k_eff_slot != nullptr) *k_eff_slot = K;
  if (K == num_pages) {  // everything is selected: identity list, padded with -1
    for (int i = tid; i < k_pages; i += kThreads) put(i, i < K ? i : -1, -1, 0.f);
    return;
  }

  // Pages that are kept whatever their score rank above every score and, like
  // equal scores, by page index: they stay out of the histograms, take their
  // places off the count, and are emitted with the keys above the threshold.
  const ForcedPages forced = forced_pages(row_shape.policy, num_pages);
  if (forced.count >= K) {  // K is 1 or 2 here: the list is the forced pages, lowest first
    if (tid == 0) {
      put(0, forced.first ? 0 : num_pages - 1, -1, 0.f);
      if (K == 2) put(1, num_pages - 1, -1, 0.f);
    }
    return;
  }

  // Keys of the valid, not forced pages; their range over the row.
  uint32_t key[kItems];
  bool valid[kItems], kept[kItems];
  uint32_t lo = 0xffffffffu, hi = 0u;
#pragma unroll
  for (int j = 0; j < kItems; ++j) {
    key[j] = score_key(raw[j]);
    kept[j] = forced.is(base + j);
    valid[j] = base + j < num_pages && !kept[j];
    if (valid[j]) lo = min(lo, key[j]), hi = max(hi, key[j]);
  }
  lo = wave_min(lo);
  hi = wave_max(hi);
  if (lane == 0) range[wave][0] = lo, range[wave][1] = hi;
  __syncthreads();
#pragma unroll
  for (int w = 0; w < kWaves; ++w) lo = min(lo, range[w][0]), hi = max(hi, range[w][1]);
  lo = __builtin_amdgcn_readfirstlane(lo);
  hi = __builtin_amdgcn_readfirstlane(hi);

  // ---- radix select on (key - lo), shifted left so that the range's leading bit is
  // bit 31: the first digit already spreads the row over the histogram, and only
  // ceil(bits / 8) digits exist.  Monotone and one-to-one on the row's keys, so order
  // and ties are those of the scores.  Invariant: the selection is every key greater
  // than `prefix` on the bits decided so far, plus `need` of the keys that match it.
  const int bits = hi > lo ? 32 - __builtin_clz(hi - lo) : 0;
  const int align = 32 - bits;  // 32 when all keys are equal: nothing to decide
#pragma unroll
  for (int j = 0; j < kItems; ++j) key[j] = bits ? (key[j] - lo) << align : 0u;
  const int n_pass = (bits + 7) >> 3;
  uint32_t prefix = 0u;
  int need = K - forced.count;  // the forced pages are in the list for certain
  int decided_shift = 32;       // bits [decided_shift, 32) of the threshold are known
#pragma unroll
  for (int pass = 0; pass < 4; ++pass) {
    if (pass >= n_pass) break;
    const int shift = 24 - 8 * pass;
    const uint32_t high_mask = pass == 0 ? 0u : (0xffffffffu << (shift + 8));
    uint32_t* hp = pass == 0 ? hist[lane & (kCopies0 - 1)] : hist[kCopies0 - 1 + pass];
#pragma unroll
    for (int j = 0; j < kItems; ++j) {
      const bool act = valid[j] && (key[j] & high_mask) == prefix;
      const uint32_t digit = (key[j] >> shift) & 255u;
      if (pass == 0) {
        // a row with outliers puts nearly all keys into one bin here: the lanes that
        // carry lane 0's digit are counted by lane 0 alone (one atomic per lane at most,
        // all lanes are active)
        const uint32_t dd = act ? digit : 0xffffffffu;
        const uint32_t d0 = __builtin_amdgcn_readfirstlane(dd);
        const uint32_t n_same = (uint32_t)__popcll(__ballot(dd == d0));
        const bool go = lane == 0 ? act : (act && dd != d0);
        if (go) atomicAdd(&hp[digit], lane == 0 ? n_same : 1u);
      } else if (act) {
        atomicAdd(&hp[digit], 1u);
      }
    }
    __syncthreads();
    const BinHit hit = pass == 0 ? find_bin<kCopies0>(hist[0], need, lane)
                                 : find_bin(hp, need, lane);
    prefix |= (uint32_t)hit.bin << shift;
    need -= hit.above;
    decided_shift = shift;
    if (need == hit.count) break;  // the whole bin is selected: no need to split it further
  }

  // ---- emit in page order.  key > bin: selected; key in bin: the first `need`.
  const uint32_t T = decided_shift < 32 ? prefix >> decided_shift : 0u;
  int n_gt = 0, n_eq = 0;
  bool gt[kItems], eq[kItems];
#pragma unroll
  for (int j = 0; j < kItems; ++j) {
    const uint32_t kd = decided_shift < 32 ? key[j] >> decided_shift : 0u;
    gt[j] = (valid[j] && kd > T) || kept[j];
    eq[j] = valid[j] && kd == T;
    n_gt += gt[j];
    n_eq += eq[j];
  }
  const int packed = n_gt | (n_eq << 16);  // rows handled here have fewer than 2^16 pages
  const int incl = wave_incl_scan(packed, lane);
  if (lane == kWave - 1) wave_tot[wave] = incl;
  __syncthreads();
  int before = incl - packed;
  for (int w = 0; w < kWaves; ++w)
    if (w < wave) before += wave_tot[w];
  int gt_before = (uint32_t)before & 0xffffu, eq_before = (uint32_t)before >> 16;
#pragma unroll
  for (int j = 0; j < kItems; ++j) {
    const bool sel = gt[j] || (eq[j] && eq_before < need);
    if (sel) put(gt_before + min(eq_before, need), base + j, j, raw[j]);
    gt_before += gt[j];
    eq_before += eq[j];
  }
}

// The list goes to memory.
template <int kThreads, int kItems>
__device__ __forceinline__ void topk_block(TopkShared<kThreads>& sm, const float* __restrict__ row,
                                           const int32_t* __restrict__ seq_len_ptr, int max_pages,
                                           int k_pages, int32_t* __restrict__ out,
                                           int32_t* __restrict__ k_eff_slot, int page_shift,
                                           int policy) {
  topk_block_put<kThreads, kItems>(
      sm, row, seq_len_ptr, max_pages, k_pages, [out](int pos, int page, int, float) { out[pos] = page; },
      k_eff_slot, WholeRow{page_shift, policy}, [] {});
}

#endif  // __HIPCC__

}  // namespace quest
