// Query-aware page criticality (attention half of Algorithm 1, Section 3.4 of
// arXiv 2406.10774):  score[p] = sum_i max(q_i * m_{p,i}, q_i * M_{p,i}).
//
// Since m <= M per channel, max(q m, q M) is q * (q >= 0 ? M : m) exactly: the
// sign of q picks the row, done once per wave as a bit mask, and the products
// go through v_dot2_f32_f16 (fp16 products are exact in fp32, fp32 sum).
//
// One wavefront owns (head, block of 16 consecutive logical pages).  A 16-lane
// DPP row reads one metadata entry: 16 B per lane of the min row, then 16 B per
// lane of the max row (two 256 B segments, 512 B contiguous), so one wave-wide
// load instruction covers four pages; the 128-channel sum is a reduction inside
// the DPP row.  All eight loads of a wave are issued before the first use.
#include "quest_common.h"

namespace quest {

namespace {

constexpr int kEstWaves = 4;
constexpr int kEstIters = 4;                         // wave-wide load pairs per wave
constexpr int kEstPagesPerWave = 4 * kEstIters;      // 16
constexpr int kEstPagesPerGroup = kEstWaves * kEstPagesPerWave;

// kAppend: the wave that owns the newest token's page first performs the
// insertion half of Algorithm 1 for it (store k/v into the slot, fold k into
// the page's min/max, write the entry back) on the registers it scores from.
template <bool kAppend>
__global__ __launch_bounds__(kEstWaves* kWave) void estimate_kernel(
    char* __restrict__ meta, const char* __restrict__ q, const int32_t* __restrict__ page_table,
    const int32_t* __restrict__ seq_lens, float* __restrict__ scores, int num_heads, int max_pages,
    const char* __restrict__ k_new, const char* __restrict__ v_new, char* __restrict__ k_pool,
    char* __restrict__ v_pool, int k_pool_write) {
  const int b = blockIdx.z;
  const int h = blockIdx.y;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = lane_id();
  const int grp = lane >> 4;  // DPP row: pages base + 4*grp + it
  const int c = lane & 15;    // channels 8c..8c+7
  const int base = (blockIdx.x * kEstWaves + wave) * kEstPagesPerWave;
  const size_t bh = (size_t)b * num_heads + h;

  // page-table entries are fetched before seq_lens is known (rows have
  // max_pages entries); whether a page holds tokens is decided afterwards
  const int32_t* pt = page_table + (size_t)b * max_pages;
  const int seq_len = seq_lens[b];
  int phys[kEstIters];
#pragma unroll
  for (int it = 0; it < kEstIters; ++it) {
    const int p = base + 4 * grp + it;
    phys[it] = p < max_pages ? pt[p] : 0;
  }
  const uint4 qv = ld16(q + bh * (kHeadDim * 2) + c * 16);
  const int num_pages = (seq_len + kPageSize - 1) / kPageSize;
  if (base >= num_pages) return;

  uint4 mn[kEstIters], mx[kEstIters];
#pragma unroll
  for (int it = 0; it < kEstIters; ++it) {
    const int p = base + 4 * grp + it;
    mn[it] = make_uint4(0, 0, 0, 0);
    mx[it] = make_uint4(0, 0, 0, 0);
    if (p < num_pages) {
      const char* entry = meta + ((size_t)phys[it] * num_heads + h) * kMetaBytes + c * 16;
      mn[it] = ld16(entry);
      mx[it] = ld16(entry + kHeadDim * 2);
    }
  }

  if (kAppend) {
    const int pos = seq_len - 1;
    const int last = pos / kPageSize;
    if (last >= base && last < base + kEstPagesPerWave) {  // wave-uniform
      const int slot = pos - last * kPageSize;
      const uint4 kn = ld16(k_new + bh * (kHeadDim * 2) + c * 16);
      const uint4 key = order_key8(kn);
#pragma unroll
      for (int it = 0; it < kEstIters; ++it) {
        if (base + 4 * grp + it == last) {
          const size_t ph = (size_t)phys[it] * num_heads + h;
          if (k_pool_write) {
            const size_t off = ph * kBlockBytes + (size_t)slot * (kHeadDim * 2) + c * 16;
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
          char* entry = meta + ph * kMetaBytes + c * 16;
          st16(entry, mn[it]);
          st16(entry + kHeadDim * 2, mx[it]);
        }
      }
    }
  }

  // per half: 0xffff where q is negative (min row wins), 0 elsewhere (max row wins)
  uint4 neg;
  neg.x = __builtin_bit_cast(uint32_t, __builtin_bit_cast(short2_t, qv.x) >> 15);
  neg.y = __builtin_bit_cast(uint32_t, __builtin_bit_cast(short2_t, qv.y) >> 15);
  neg.z = __builtin_bit_cast(uint32_t, __builtin_bit_cast(short2_t, qv.z) >> 15);
  neg.w = __builtin_bit_cast(uint32_t, __builtin_bit_cast(short2_t, qv.w) >> 15);

  float keep = 0.f;
#pragma unroll
  for (int it = 0; it < kEstIters; ++it) {
    uint4 sel;
    sel.x = (mn[it].x & neg.x) | (mx[it].x & ~neg.x);
    sel.y = (mn[it].y & neg.y) | (mx[it].y & ~neg.y);
    sel.z = (mn[it].z & neg.z) | (mx[it].z & ~neg.z);
    sel.w = (mn[it].w & neg.w) | (mx[it].w & ~neg.w);
    const float s = row16_sum(dot8(qv, sel, 0.f));
    if (c == it) keep = s;
  }
  // lanes c < 4 of each row hold 4 consecutive pages: 16 consecutive floats per wave
  const int p = base + 4 * grp + c;
  if (c < kEstIters && p < num_pages) scores[bh * max_pages + p] = keep;
}

}  // namespace

int launch_estimate(const quest_cache& c, const void* q, float* scores, hipStream_t s) {
  dim3 grid((c.max_pages_per_seq + kEstPagesPerGroup - 1) / kEstPagesPerGroup, c.num_heads, c.batch);
  hipLaunchKernelGGL(estimate_kernel<false>, grid, dim3(kEstWaves * kWave), 0, s, (char*)c.meta,
                     (const char*)q, c.page_table, c.seq_lens, scores, c.num_heads,
                     c.max_pages_per_seq, nullptr, nullptr, nullptr, nullptr, 0);
  return check_launch("quest_estimate");
}

int launch_append_estimate(const quest_cache& c, const void* k_new, const void* v_new,
                           int k_pool_write, const void* q, float* scores, hipStream_t s) {
  dim3 grid((c.max_pages_per_seq + kEstPagesPerGroup - 1) / kEstPagesPerGroup, c.num_heads, c.batch);
  hipLaunchKernelGGL(estimate_kernel<true>, grid, dim3(kEstWaves * kWave), 0, s, (char*)c.meta,
                     (const char*)q, c.page_table, c.seq_lens, scores, c.num_heads,
                     c.max_pages_per_seq, (const char*)k_new, (const char*)v_new, (char*)c.k_pool,
                     (char*)c.v_pool, k_pool_write);
  return check_launch("quest_append_estimate");
}

}  // namespace quest
