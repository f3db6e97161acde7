// Device-side core of the criticality estimate (attention half of Algorithm 1,
// Section 3.4 of arXiv 2406.10774).
#pragma once

#include "quest_common.h"

namespace quest {

#if defined(__HIPCC__)

constexpr int kEstIters = 4;                     // wave-wide load pairs per wave (large tables)
constexpr int kEstPagesPerWave = 4 * kEstIters;  // 16

// kAppend: the wave that owns the newest token's page first performs the
// insertion half of Algorithm 1 for it (store k/v into the slot, fold k into
// the page's min/max, write the entry back) on the registers it scores from.
struct EstimateArgs {
  char* meta;
  const char* q;
  const int32_t* page_table;
  const int32_t* seq_lens;
  float* scores;
  int num_heads, max_pages;  // num_heads: KV heads (rows of meta, pools, scores)
  int group;                 // query heads per KV head: q has num_heads * group heads
  int64_t num_phys_pages;
  const char* k_new;  // kAppend only
  const char* v_new;
  char* k_pool;
  char* v_pool;
  int k_pool_write;
  int page_shift;  // log2(tokens per page)
};

// One wave scores the 4 * kIters logical pages starting at `base` of (sequence b,
// head h): DPP row g takes pages base + kIters*g .. + kIters - 1, one per
// wave-wide load pair.
template <bool kAppend, int kIters = kEstIters>
__device__ __forceinline__ void estimate_wave(const EstimateArgs& a, int b, int h, int base) {
  char* __restrict__ meta = a.meta;
  const char* __restrict__ q = a.q;
  const int32_t* __restrict__ page_table = a.page_table;
  const int32_t* __restrict__ seq_lens = a.seq_lens;
  float* __restrict__ scores = a.scores;
  const int num_heads = a.num_heads, max_pages = a.max_pages;
  const char* __restrict__ k_new = a.k_new;
  const char* __restrict__ v_new = a.v_new;
  char* __restrict__ k_pool = a.k_pool;
  char* __restrict__ v_pool = a.v_pool;
  const int k_pool_write = a.k_pool_write;
  const int lane = lane_id();
  const int grp = lane >> 4;  // DPP row: pages base + kIters*grp + it
  const int c = lane & 15;    // channels 8c..8c+7
  const size_t bh = (size_t)b * num_heads + h;

  // page-table entries are fetched before seq_lens is known (rows have
  // max_pages entries); whether a page holds tokens is decided afterwards
  const int32_t* pt = page_table + (size_t)b * max_pages;
  const int seq_len = seq_lens[b];
  int phys[kIters];
#pragma unroll
  for (int it = 0; it < kIters; ++it) {
    const int p = base + kIters * grp + it;
    phys[it] = p < max_pages ? pt[p] : 0;
  }
  const int group = a.group;
  const uint4 qv = ld16(q + bh * group * (kHeadDim * 2) + c * 16);  // first query head of the group
  const int page_shift = a.page_shift;
  const int num_pages = (seq_len + (1 << page_shift) - 1) >> page_shift;
  if (base >= num_pages) return;

  uint4 mn[kIters], mx[kIters];
#pragma unroll
  for (int it = 0; it < kIters; ++it) {
    const int p = base + kIters * grp + it;
    mn[it] = make_uint4(0, 0, 0, 0);
    mx[it] = make_uint4(0, 0, 0, 0);
    if (p < num_pages) {
      const char* entry = meta + meta_offset(a.num_phys_pages, phys[it], h) + c * 16;
      mn[it] = ld16_stream(entry);
      mx[it] = ld16_stream(entry + kHeadDim * 2);
    }
  }

  if (kAppend) {
    const int pos = seq_len - 1;
    const int last = pos >> page_shift;
    if (last >= base && last < base + 4 * kIters) {  // wave-uniform
      const int slot = pos - (last << page_shift);
      const uint4 kn = ld16(k_new + bh * (kHeadDim * 2) + c * 16);
      const uint4 key = order_key8(kn);
#pragma unroll
      for (int it = 0; it < kIters; ++it) {
        if (base + kIters * grp + it == last) {
          const size_t ph = (size_t)phys[it] * num_heads + h;
          if (k_pool_write) {
            const size_t off = ((ph << page_shift) + slot) * kRowBytes + c * 16;
            st16(k_pool + off, kn);
            st16(v_pool + off, ld16(v_new + bh * (kHeadDim * 2) + c * 16));
          }
          if (slot == 0) {
            mn[it] = kn;
            mx[it] = kn;
          } else {
            mn[it] = order_key8(key_min8(order_key8(mn[it]), key));
            mx[it] = order_key8(key_max8(order_key8(mx[it]), key));
          }
          char* entry = meta + meta_offset(a.num_phys_pages, phys[it], h) + c * 16;
          st16(entry, mn[it]);
          st16(entry + kHeadDim * 2, mx[it]);
        }
      }
    }
  }

  // One query head against the pages this wave holds: lane c of a row keeps the
  // score of the row's c-th page.
  auto score_pages = [&](const uint4 qh) {
    // per half: 0xffff where q is negative (min row wins), 0 elsewhere (max row wins)
    uint4 neg;
    neg.x = __builtin_bit_cast(uint32_t, __builtin_bit_cast(short2_t, qh.x) >> 15);
    neg.y = __builtin_bit_cast(uint32_t, __builtin_bit_cast(short2_t, qh.y) >> 15);
    neg.z = __builtin_bit_cast(uint32_t, __builtin_bit_cast(short2_t, qh.z) >> 15);
    neg.w = __builtin_bit_cast(uint32_t, __builtin_bit_cast(short2_t, qh.w) >> 15);
    float mine = 0.f;
#pragma unroll
    for (int it = 0; it < kIters; ++it) {
      uint4 sel;
      sel.x = (mn[it].x & neg.x) | (mx[it].x & ~neg.x);
      sel.y = (mn[it].y & neg.y) | (mx[it].y & ~neg.y);
      sel.z = (mn[it].z & neg.z) | (mx[it].z & ~neg.z);
      sel.w = (mn[it].w & neg.w) | (mx[it].w & ~neg.w);
      const float s = row16_sum(dot8(qh, sel, 0.f));
      if (c == it) mine = s;
    }
    return mine;
  };
  // The page's score for the KV head: the largest of its query heads' scores
  // (one query head per KV head in the paper's models: no further round).
  float keep = score_pages(qv);
  for (int g = 1; g < group; ++g)
    keep = fmaxf(keep, score_pages(ld16(q + (bh * group + g) * (kHeadDim * 2) + c * 16)));
  // lanes c < 4 of each row hold 4 consecutive pages: 16 consecutive floats per wave
  const int p = base + kIters * grp + c;
  if (c < kIters && p < num_pages) scores[bh * max_pages + p] = keep;
}

#endif  // __HIPCC__

}  // namespace quest
