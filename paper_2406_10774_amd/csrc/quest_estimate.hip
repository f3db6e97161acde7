// Query-aware page criticality (attention half of Algorithm 1, Section 3.4 of
// arXiv 2406.10774):  score[p] = sum_i max(q_i * m_{p,i}, q_i * M_{p,i}).
//
// Since m <= M per channel, max(q m, q M) is q * (q >= 0 ? M : m) exactly: the
// sign of q picks the row, done once per wave as a bit mask, and the products
// go through v_dot2_f32_f16 (fp16 products are exact in fp32, fp32 sum).
//
// One wavefront owns (head, block of 8 or 16 consecutive logical pages).  A 16-lane
// DPP row reads one metadata entry: 16 B per lane of the min row, then 16 B per
// lane of the max row (two 256 B segments, 512 B contiguous), so one wave-wide
// load instruction covers four pages; the 128-channel sum is a reduction inside
// the DPP row.  All loads of a wave are issued before the first use.
#include "quest_common.h"
#include "quest_estimate_core.h"

namespace quest {

namespace {

constexpr int kEstWaves = 4;

// Grid: x = blocks of pages, y = sequence, z = head.  The metadata table is head-major
// over the physical pages, so with the sequences' pages laid out one after the other
// consecutive work-groups walk memory in order (6.05 TB/s against 5.5 TB/s with the
// heads in y, at 16 sequences of 32k tokens).
template <bool kAppend, int kIters>
__global__ __launch_bounds__(kEstWaves* kWave) void estimate_kernel(const EstimateArgs a) {
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  estimate_wave<kAppend, kIters>(a, blockIdx.y, blockIdx.z,
                                 (blockIdx.x * kEstWaves + wave) * (4 * kIters));
}

// Pages per wave: 16 (eight wave-wide loads in flight) once the table is large; a small
// table (one sequence of 32 heads at 32k tokens is 32 MiB, a few microseconds) is scanned
// faster by twice as many waves of half the size: 7.6 us against 7.9 us there, 8.7 us
// with 32 pages per wave.
int est_iters(const quest_cache& c) {
  return (long)c.batch * kv_heads(c) * c.max_pages_per_seq <= (1l << 17) ? 2 : kEstIters;
}

template <bool kAppend>
void launch(const quest_cache& c, const EstimateArgs& a, hipStream_t s) {
  const int iters = est_iters(c);
  const int per_group = kEstWaves * 4 * iters;
  dim3 grid((c.max_pages_per_seq + per_group - 1) / per_group, c.batch, kv_heads(c));
  if (iters == 2)
    hipLaunchKernelGGL((estimate_kernel<kAppend, 2>), grid, dim3(kEstWaves * kWave), 0, s, a);
  else
    hipLaunchKernelGGL((estimate_kernel<kAppend, kEstIters>), grid, dim3(kEstWaves * kWave), 0, s, a);
}

}  // namespace

namespace {
EstimateArgs make_args(const quest_cache& c, const void* q, float* scores) {
  EstimateArgs a;
  a.meta = (char*)c.meta;
  a.q = (const char*)q;
  a.page_table = c.page_table;
  a.seq_lens = c.seq_lens;
  a.scores = scores;
  a.num_heads = kv_heads(c);
  a.group = group_size(c);
  a.max_pages = c.max_pages_per_seq;
  a.num_phys_pages = c.num_phys_pages;
  a.page_shift = page_shift_of(c.page_size);
  a.k_new = a.v_new = nullptr;
  a.k_pool = a.v_pool = nullptr;
  a.k_pool_write = 0;
  return a;
}
}  // namespace

int launch_estimate(const quest_cache& c, const void* q, float* scores, hipStream_t s) {
  launch<false>(c, make_args(c, q, scores), s);
  return check_launch("quest_estimate");
}

int launch_append_estimate(const quest_cache& c, const void* k_new, const void* v_new,
                           int k_pool_write, const void* q, float* scores, hipStream_t s) {
  EstimateArgs a = make_args(c, q, scores);
  a.k_new = (const char*)k_new;
  a.v_new = (const char*)v_new;
  a.k_pool = (char*)c.k_pool;
  a.v_pool = (char*)c.v_pool;
  a.k_pool_write = k_pool_write;
  launch<true>(c, a, s);
  return check_launch("quest_append_estimate");
}

}  // namespace quest
