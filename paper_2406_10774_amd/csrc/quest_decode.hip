// Sparse paged decode attention (Figure 5 stage 2 / Section 3.4 of arXiv
// 2406.10774): ordinary softmax attention of one query per (sequence, head)
// over the tokens of the selected pages only.  With no page list it runs over
// every page: the dense baseline the paper compares against (Section 3.1).
//
// Split-K flash-decoding.  One work-group per (sequence, head, split); each work-group of
// four waves owns a contiguous slice of the head's page list, its waves take
// the slice's pages round-robin.  A wave streams one unit (up to 16 tokens of one
// page: 4 KiB of keys and 4 KiB of values = 4 + 4 wave-wide 16-byte loads; pages
// of 32 or 64 tokens are 2 or 4 units, pages of 8 tokens units of 2 + 2 loads) per
// step, double-buffered in registers so the next unit's loads are in flight while
// the current one is reduced.  Lane l holds channels 8*(l%16)..+7 of tokens
// l/16 + 4r; q.k is a v_dot2_f32_f16 chain plus a reduction inside the 16-lane
// DPP row; each DPP row keeps its own online softmax state (running max,
// denominator, 8 accumulator channels per lane) in fp32, in the log2 domain.
// Rows, waves and finally splits are merged with the usual (max, sum,
// accumulator) rescaling; the split that finishes last merges the partial
// results of all splits of its head.  With grouped-query attention a work-group
// of the dense path serves several query heads of one KV head per page load.
//
// Single-query attention is a matrix-vector product (about one flop per byte
// read), far below the machine balance, so there is no MFMA here: the kernel is
// bound by how fast HBM delivers the 8 KiB per selected (page, head).
#include "quest_common.h"
#include "quest_decode_core.h"
#include "quest_team.h"
#include "quest_topk_core.h"

#include <cmath>
#include <type_traits>

namespace quest {

namespace {

constexpr int kComputeUnits = 256;  // MI355X; only used to decide how finely to split
constexpr int kDecWaves = 4;
constexpr int kDecThreads = kDecWaves * kWave;
// With the selection done in the same launch (see decode_split_kernel): 8 waves, the size
// the selection is fastest at, and room in LDS for a page list of this many entries.
constexpr int kSelWaves = 8;
constexpr int kSelListCap = 2048;

// The same value in a register that no load is outstanding for: the compiler waits for
// `v` here, once, instead of before every later use it cannot order against other loads.
__device__ __forceinline__ int settled(int v) {
  int r;
  asm volatile("v_mov_b32 %0, %1" : "=v"(r) : "v"(v));
  return r;
}

struct DecodeArgs {
  const char* k_pool;
  const char* v_pool;
  const char* q;
  const int32_t* page_table;
  const int32_t* seq_lens;
  const int32_t* topk_idx;  // nullptr: all pages (or: selected inside the launch, see scores)
  const float* scores;      // selection inside the launch: scores [B][kv heads][max_pages] ...
  int32_t* topk_out;        // ... the list is also written here [B][kv heads][k_pages] ...
  int32_t* k_eff;           // ... and K_b here (nullable)
  int policy;               // QUEST_FLAG_KEEP_* bits
  float* part_acc;          // [B*H*splits][D]   un-normalised accumulators
  float* part_ml;           // [B*H*splits][2]   running max (log2 domain), denominator
  void* out;
  float* lse;
  uint64_t* counters;       // [B*H] arrival counters, one per 256-byte slot (quest_team.h); zero between launches
  int batch, num_heads, max_pages, k_pages, splits, out_is_fp16;
  int list_len;             // entries of the page list the splits divide: k_pages, or max_pages
  int per_split;            // ceil(list_len / splits)
  int device_fences;        // QUEST_FLAG_DEVICE_FENCES: fences around the exchange as well
  int kv_heads, group;      // KV heads; query heads per KV head (num_heads = kv_heads * group)
  int page_shift;           // log2(tokens per page)
  int unit_shift;           // log2(streaming units per page): 0 up to 16 tokens, 1 for 32, 2 for 64
  float scale_log2;         // sm_scale * log2(e)
};

// All splits of one (sequence, head) get work-group ids that are equal modulo 8
// (grid.x is a multiple of 8), so under the usual round-robin placement they run on
// one die and their traffic stays in one L2.  Nothing depends on that: partial results
// are handed over with device-scope stores and loads (quest_team.h), correct wherever
// the splits run; the split that finishes last merges them, without a second launch.
// kLoads: wave-wide 16-byte loads per unit of keys (and of values): 4, or 2 for 8-token
// pages.  kG: query heads served by one work-group (they share the KV head, so a page is
// loaded once for all of them): 1 unless grouped-query attention; a group of G heads is
// served by G / kG work-groups per split.
//
// kSelItems > 0: the page list does not exist yet.  Every work-group first selects the
// pages of its head itself from the scores (the same selection as quest_topk, kSelItems
// scores per thread), keeps the list in LDS and uses its own slice; split 0 also writes
// the list out.  The selection is repeated by every split of a head, which costs nothing
// that matters (the compute units would idle meanwhile) and saves a launch and the trip
// of the list through memory.
template <int kLoads, int kG, int kWaves, int kSelItems>
__global__ __launch_bounds__(kWaves* kWave) void decode_split_kernel(const DecodeArgs a) {
  constexpr int kDecWaves = kWaves;
  __shared__ float sm_acc[kDecWaves][kG][kHeadDim];
  __shared__ float sm_m[kDecWaves][kG], sm_l[kDecWaves][kG];
  __shared__ uint32_t sm_before;
  // the selection's LDS only where there is a selection; the list as (logical page,
  // physical page) pairs
  __shared__ typename std::conditional<(kSelItems > 0), TopkShared<kWaves * kWave>, char>::type sm_topk;
  __shared__ int2 sm_list[kSelItems > 0 ? kSelListCap : 1];

  // blockIdx.x = slot + 8 * split, blockIdx.y = group of 8 items: the linear work-group
  // id is slot + 8 * (split + splits * blockIdx.y).  The usual shapes (one sequence, one
  // work-group per KV head) are taken apart without integer divisions: they sit in
  // front of the first load of every work-group.
  const int slot = blockIdx.x & 7;
  const int split = blockIdx.x >> 3;
  const int item = blockIdx.y * 8 + slot;  // (sequence, KV head, kG query heads of its group)
  const int subs = a.group / kG;           // work-groups per KV head and split: 1 without groups
  const int per_seq = a.kv_heads * subs;
  if (item >= a.batch * per_seq) return;
  const int b = a.batch == 1 ? 0 : item / per_seq;
  const int in_seq = item - b * per_seq;
  const int hk = subs == 1 ? in_seq : in_seq / subs;  // the KV head: its pages, its page list
  const int h = hk * a.group + (in_seq - hk * subs) * kG;  // first query head served here
  const size_t bh = (size_t)b * a.num_heads + h;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = lane_id();
  const int grp = lane >> 4;
  const int c = lane & 15;
  uint32_t* arrivals = reinterpret_cast<uint32_t*>(a.counters + bh * kTeamWordStride);

  // This wave's share of the page list: positions begin + wave + 4 i.  The list
  // length used for the split (k_pages, or max_pages without a list) is known
  // on the host, so list entries and page-table entries are fetched without
  // waiting for seq_lens; entries past the valid pages are dropped afterwards.
  const int begin = split * a.per_split;
  const int end = min(a.list_len, begin + a.per_split);
  const int iters = (a.per_split + kDecWaves - 1) / kDecWaves;
  const int32_t* idx_row =
      a.topk_idx ? a.topk_idx + ((size_t)b * a.kv_heads + hk) * a.k_pages : nullptr;
  const int32_t* pt = a.page_table + (size_t)b * a.max_pages;
  int seq_len;
  uint4 qv[kG];
  if constexpr (kSelItems > 0) {
    const size_t row = (size_t)b * a.kv_heads + hk;
    const bool writer = split == 0 && h == hk * a.group;  // one work-group per list writes it out
    int32_t* out_row = a.topk_out + row * a.k_pages;
    // Behind the loads of the scores (loads complete in order, so nothing may be in front
    // of what the selection waits for): the page-table entries of this thread's pages,
    // which travel with their scores so that the list needs no look-up afterwards, and
    // what the attention needs besides the pages.
    int my_phys[kSelItems];
    auto more_loads = [&] {
#pragma unroll
      for (int j = 0; j < kSelItems; ++j)
        my_phys[j] = pt[min((int)threadIdx.x * kSelItems + j, a.max_pages - 1)];
      seq_len = a.seq_lens[b];
#pragma unroll
      for (int g = 0; g < kG; ++g) qv[g] = ld16(a.q + (bh + g) * (kHeadDim * 2) + c * 16);
    };
    topk_block_put<kWaves * kWave, kSelItems>(
        sm_topk, a.scores + row * a.max_pages, a.seq_lens + b, a.max_pages, a.k_pages,
        [&](int pos, int page, int j, float) {
          int phys = 0;
          if (j >= 0) {
#pragma unroll
            for (int jj = 0; jj < kSelItems; ++jj)
              if (jj == j) phys = my_phys[jj];
          } else if (page >= 0) {
            phys = pt[page];
          }
          sm_list[pos] = make_int2(page, phys);
          if (writer) out_row[pos] = page;
        },
        (writer && hk == 0 && a.k_eff != nullptr) ? a.k_eff + b : nullptr,
        WholeRow{a.page_shift, a.policy}, more_loads);
    __syncthreads();
  } else {
    seq_len = a.seq_lens[b];
#pragma unroll
    for (int g = 0; g < kG; ++g) qv[g] = ld16(a.q + (bh + g) * (kHeadDim * 2) + c * 16);
  }

  Softmax st[kG];
#pragma unroll
  for (int g = 0; g < kG; ++g) {
    st[g].m = kNegBig;
    st[g].l = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) st[g].acc[j] = 0.f;
  }

  // A page is streamed as 1 << unit_shift units of up to 16 tokens; lane i of a
  // round holds unit i of this wave: list entry i >> unit_shift, unit i & mask.
  const int units = iters << a.unit_shift;
  const int num_pages = (seq_len + (1 << a.page_shift) - 1) >> a.page_shift;
  for (int chunk = 0; chunk < units; chunk += kWave) {
    const int u = chunk + lane;
    const int e = u >> a.unit_shift;
    const int un_v = u & ((1 << a.unit_shift) - 1);
    const int pos = begin + wave + kDecWaves * e;
    int lp_v = -1, ph_v = 0;
    if constexpr (kSelItems > 0) {
      if (e < iters && pos < end) {
        const int2 entry = sm_list[pos];
        lp_v = entry.x, ph_v = entry.y;
      }
    } else {
      if (e < iters && pos < end) lp_v = idx_row ? idx_row[pos] : pos;
      if (lp_v >= 0 && lp_v < a.max_pages) ph_v = pt[lp_v];
    }
    if (lp_v >= num_pages) lp_v = -1;

#define QUEST_LOAD_UNIT(regs, i)                                                               \
  load_unit<kLoads>(regs, a.k_pool, a.v_pool, a.kv_heads, hk, seq_len, __builtin_amdgcn_readlane(lp_v, i), \
                    __builtin_amdgcn_readlane(ph_v, i), __builtin_amdgcn_readlane(un_c, i),    \
                    a.page_shift, lane)
#define QUEST_FOLD(regs)                                  \
  do {                                                    \
    if (kG == 1)                                          \
      fold_page(st[0], regs, qv[0], a.scale_log2, grp);   \
    else                                                  \
      fold_group(st, regs, qv, a.scale_log2, grp);        \
  } while (0)
    // The units to stream are moved to the first n lanes (lists from the selection are
    // ascending and padded at the end, so normally they are there already; a caller's
    // list may have negative or out-of-range entries anywhere: those are skipped).
    // Two units in flight per wave: the next one is requested before the current one is
    // folded.  Every load inside the loop is unconditional and the index registers are
    // detached from the loads that produced them (one wait here), so the compiler's
    // wait counts inside the loop are exact: a conditional load, or an index still
    // marked as in flight, makes it wait for everything outstanding at every step,
    // which leaves a single unit in flight.
    const unsigned long long live = __ballot(lp_v >= 0);
    const int n = __popcll(live);
    int un_c = un_v;
    if (live & (live + 1)) {  // not a prefix of the lanes: compact (wave-uniform branch)
      const int to = lp_v >= 0 ? (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(live >> 32),
                                      __builtin_amdgcn_mbcnt_lo((uint32_t)live, 0u)) : kWave - 1;
      // a dead lane's target is lane 63, which no live lane can have unless all 64 are
      // live (then this branch is not taken); its value there is never used (63 >= n)
      lp_v = __builtin_amdgcn_ds_permute(to * 4, lp_v);
      ph_v = __builtin_amdgcn_ds_permute(to * 4, ph_v);
      un_c = __builtin_amdgcn_ds_permute(to * 4, un_v);
    }
    lp_v = settled(lp_v);
    ph_v = settled(ph_v);
    PageRegsT<kLoads> ra, rb;
    if (n > 0) {
      QUEST_LOAD_UNIT(ra, 0);
      int j = 0;
      for (; j + 2 < n; j += 2) {
        QUEST_LOAD_UNIT(rb, j + 1);
        QUEST_FOLD(ra);
        QUEST_LOAD_UNIT(ra, j + 2);
        QUEST_FOLD(rb);
      }
      if (j + 1 < n) {
        QUEST_LOAD_UNIT(rb, j + 1);
        QUEST_FOLD(ra);
        QUEST_FOLD(rb);
      } else {
        QUEST_FOLD(ra);
      }
    }
#undef QUEST_LOAD_UNIT
#undef QUEST_FOLD
  }

  // the four DPP rows of the wave, then the four waves of the group
#pragma unroll
  for (int g = 0; g < kG; ++g) {
    merge_rows(st[g]);
    if (lane < 16) {
#pragma unroll
      for (int j = 0; j < 8; ++j) sm_acc[wave][g][c * 8 + j] = st[g].acc[j];
      if (lane == 0) {
        sm_m[wave][g] = st[g].m;
        sm_l[wave][g] = st[g].l;
      }
    }
  }
  __syncthreads();
  const int t = threadIdx.x;
  // ---- this split's result per query head: written out if it is the only split, else
  // published as a partial; the split that arrives last merges
#pragma unroll
  for (int g = 0; g < kG; ++g) {
    float m_tot = sm_m[0][g];
#pragma unroll
    for (int w = 1; w < kDecWaves; ++w) m_tot = fmaxf(m_tot, sm_m[w][g]);
    float l_tot = 0.f, acc = 0.f;
#pragma unroll
    for (int w = 0; w < kDecWaves; ++w) {
      const float f = __builtin_amdgcn_exp2f(sm_m[w][g] - m_tot);
      l_tot += sm_l[w][g] * f;
      acc += sm_acc[w][g][t & (kHeadDim - 1)] * f;
    }
    if (a.splits == 1) {
      if (t < kHeadDim) {
        store_out(a.out, a.out_is_fp16, (bh + g) * kHeadDim + t, acc / l_tot);
        if (t == 0 && a.lse) a.lse[bh + g] = (m_tot + __builtin_amdgcn_logf(l_tot)) * kLn2;
      }
    } else {
      const size_t ps = (bh + g) * a.splits + split;
      if (t < kHeadDim) dev_st(a.part_acc + ps * kHeadDim + t, acc);
      if (t == 0) {
        dev_st(a.part_ml + ps * 2 + 0, m_tot);
        dev_st(a.part_ml + ps * 2 + 1, l_tot);
      }
    }
  }
  if (a.splits == 1) return;
  wait_stores();
  __syncthreads();
  if (t == 0) sm_before = team_arrive(arrivals, a.device_fences);
  __syncthreads();
  if (__builtin_amdgcn_readfirstlane(sm_before) != (uint32_t)a.splits - 1) return;
  team_acquire(a.device_fences);
  if (t == 0) team_reset(arrivals);

  // one pass over the splits in chunks of 8, all loads of a chunk in flight at once, with
  // a running maximum (the same rescaling as between pages); always in split order, so the
  // result does not depend on which split arrived last
  if (t >= kHeadDim) return;
#pragma unroll 1
  for (int g = 0; g < kG; ++g) {
    const float* ml = a.part_ml + (bh + g) * a.splits * 2;
    const float* pacc = a.part_acc + (bh + g) * a.splits * kHeadDim + t;
    float mx = kNegBig, l_all = 0.f, o = 0.f;
    for (int s0 = 0; s0 < a.splits; s0 += 8) {
      float2 pml[8];
      float pa[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int sidx = min(s0 + i, a.splits - 1);
        pml[i] = dev_ld2(ml + 2 * sidx);
        pa[i] = dev_ld(pacc + (size_t)sidx * kHeadDim);
      }
      float cm = mx;
#pragma unroll
      for (int i = 0; i < 8; ++i) cm = fmaxf(cm, pml[i].x);
      const float rescale = __builtin_amdgcn_exp2f(mx - cm);
      l_all *= rescale;
      o *= rescale;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float f = s0 + i < a.splits ? __builtin_amdgcn_exp2f(pml[i].x - cm) : 0.f;
        l_all += pml[i].y * f;
        o += pa[i] * f;
      }
      mx = cm;
    }
    store_out(a.out, a.out_is_fp16, (bh + g) * kHeadDim + t, o / l_all);
    if (t == 0 && a.lse) a.lse[bh + g] = (mx + __builtin_amdgcn_logf(l_all)) * kLn2;
  }
}

}  // namespace

// Number of splits of a head's page list.  A split holds at least 256 tokens (sixteen
// pages of 16: four per wave, two in flight at a time), and the whole launch stays within
// the ~1000 work-groups that are resident at once, so that all splits of a head
// start together and the merge reads few partial results.
namespace {
// Query heads one work-group serves.  Heads of a group share a KV head, so its pages can
// be loaded once for several of them: that pays on the dense path (4x less traffic; 47 us
// against 88 us at 32 query / 8 KV heads, 32k tokens).  With a short page list it does not:
// fewer, heavier work-groups and a merge over more partials (13.9 us against 10.1 us), so
// there every query head keeps its own work-groups and the later heads of a group find
// the pages in L2.
int heads_per_group(const quest_cache& c, int k_pages) {
  if (k_pages > 0) return 1;
  const int g = group_size(c);
  return g % 4 == 0 ? 4 : g % 2 == 0 ? 2 : 1;
}
struct SplitPlan {
  int list_len, per_split, splits;
};
SplitPlan plan_splits(const quest_cache& c, int k_pages) {
  constexpr int pages_per_split = 16;
  SplitPlan p;
  p.list_len = k_pages > 0 ? (k_pages < c.max_pages_per_seq ? k_pages : c.max_pages_per_seq)
                           : c.max_pages_per_seq;
  const long bh = (long)c.batch * c.num_heads / heads_per_group(c, k_pages);  // work items per split
  // the knob is in pages of 16 tokens: the same bytes per split for every page size
  const int shift = page_shift_of(c.page_size);
  const long pps = shift >= 0 && ((long)pages_per_split << 4 >> shift) > 0
                       ? ((long)pages_per_split << 4 >> shift)
                       : 1;
  long splits = (p.list_len + pps - 1) / pps;
  // few (sequence, head) items: shorter splits, down to one unit of 16 tokens per wave,
  // until there is a work-group for every compute unit
  const long unit = kDecWaves << 4 >> shift > 0 ? (long)(kDecWaves << 4 >> shift) : 1;
  const long fill = (kComputeUnits + bh - 1) / bh;
  const long finest = (p.list_len + unit - 1) / unit;
  if (splits < fill) splits = fill < finest ? fill : finest;
  const long qh = (long)c.batch * c.num_heads;  // a work-group's weight grows with its heads
  // Work-groups in all: two per compute unit stream best once there is enough work
  // (deeper streams per wave, fewer partial results to merge: 58 us against 62 us per
  // step at 4 sequences of 32 heads, 104 against 109 at 8); a single sequence of 32 heads
  // is faster with four (dense path: 100 us against 105 us).
  const long max_groups = qh <= 32 ? 4 * kComputeUnits : 2 * kComputeUnits;
  const long cap = max_groups / qh > 0 ? max_groups / qh : 1;
  if (splits > cap) splits = cap;
  if (splits < 1) splits = 1;
  if (splits > kMaxTeamSize) splits = kMaxTeamSize;
  p.per_split = (int)((p.list_len + splits - 1) / splits);
  p.splits = (p.list_len + p.per_split - 1) / p.per_split;  // no empty split
  return p;
}
// One arrival counter per (sequence, head), each in a 256-byte slot of its own.
size_t counter_bytes(const quest_cache& c) {
  return (size_t)c.batch * c.num_heads * kTeamWordStride * sizeof(uint64_t);
}
}  // namespace

size_t decode_counter_bytes(const quest_cache& c) { return counter_bytes(c); }

int decode_num_splits(const quest_cache& c, int k_pages) { return plan_splits(c, k_pages).splits; }

size_t decode_workspace_bytes(const quest_cache& c, int k_pages) {
  const size_t splits = plan_splits(c, k_pages).splits;
  if (splits == 1) return 0;
  return counter_bytes(c) + (size_t)c.batch * c.num_heads * splits * (kHeadDim + 2) * sizeof(float);
}

namespace {
// scores != nullptr: select inside the launch (topk_out, k_eff receive the list and K_b);
// the caller has checked select_decode_supported.
int launch_decode(const quest_cache& c, const void* q, const int32_t* topk_idx, const float* scores,
                  int32_t* topk_out, int32_t* k_eff, int k_pages, float sm_scale, void* out,
                  int out_is_fp16, float* lse, void* workspace, hipStream_t s) {
  const bool select = scores != nullptr;
  DecodeArgs a;
  a.k_pool = (const char*)c.k_pool;
  a.v_pool = (const char*)c.v_pool;
  a.q = (const char*)q;
  a.page_table = c.page_table;
  a.seq_lens = c.seq_lens;
  a.topk_idx = topk_idx;
  a.scores = scores;
  a.topk_out = topk_out;
  a.k_eff = k_eff;
  a.policy = c.flags;
  a.batch = c.batch;
  a.num_heads = c.num_heads;
  a.kv_heads = kv_heads(c);
  a.group = group_size(c);
  a.max_pages = c.max_pages_per_seq;
  a.k_pages = (topk_idx || select) ? k_pages : 0;
  const SplitPlan p = plan_splits(c, a.k_pages);
  a.splits = p.splits;
  a.list_len = p.list_len;
  a.per_split = p.per_split;
  a.device_fences = (c.flags & QUEST_FLAG_DEVICE_FENCES) != 0;
  a.out = out;
  a.out_is_fp16 = out_is_fp16;
  a.lse = lse;
  a.scale_log2 = sm_scale * kLog2e;
  a.page_shift = page_shift_of(c.page_size);
  a.unit_shift = a.page_shift > 4 ? a.page_shift - 4 : 0;
  const size_t n_part = (size_t)c.batch * c.num_heads * a.splits;
  a.counters = (uint64_t*)workspace;
  a.part_acc = workspace ? (float*)((char*)workspace + counter_bytes(c)) : nullptr;
  a.part_ml = a.part_acc ? a.part_acc + n_part * kHeadDim : nullptr;
  const int kg = heads_per_group(c, a.k_pages);
  const long items8 = ((long)c.batch * c.num_heads / kg + 7) / 8;
  if (items8 > 65535) {
    set_error("quest_sparse_decode: batch * heads = %ld exceeds the launch limit", items8 * 8);
    return QUEST_ERR_SHAPE;
  }
  const dim3 grid((unsigned)(8 * a.splits), (unsigned)items8);
  if (select) {
    const int mp = c.max_pages_per_seq;
    const dim3 block(kSelWaves * kWave);
#define QUEST_SELECT_CASE(I)                                                                 \
  if (mp <= kSelWaves * kWave * (I)) {                                                       \
    if (c.page_size == 8)                                                                    \
      hipLaunchKernelGGL((decode_split_kernel<2, 1, kSelWaves, I>), grid, block, 0, s, a);   \
    else                                                                                     \
      hipLaunchKernelGGL((decode_split_kernel<4, 1, kSelWaves, I>), grid, block, 0, s, a);   \
    return check_launch("quest_select_decode");                                              \
  }
    QUEST_SELECT_CASE(2)
    QUEST_SELECT_CASE(5)
    QUEST_SELECT_CASE(8)
#undef QUEST_SELECT_CASE
    set_error("quest_select_decode: internal: no selecting kernel for max_pages_per_seq = %d", mp);
    return QUEST_ERR_SHAPE;
  }
#define QUEST_DECODE_LAUNCH(L, G) \
  hipLaunchKernelGGL((decode_split_kernel<L, G, kDecWaves, 0>), grid, dim3(kDecThreads), 0, s, a)
  if (c.page_size == 8) {
    if (kg == 4) QUEST_DECODE_LAUNCH(2, 4);
    else if (kg == 2) QUEST_DECODE_LAUNCH(2, 2);
    else QUEST_DECODE_LAUNCH(2, 1);
  } else {
    if (kg == 4) QUEST_DECODE_LAUNCH(4, 4);
    else if (kg == 2) QUEST_DECODE_LAUNCH(4, 2);
    else QUEST_DECODE_LAUNCH(4, 1);
  }
#undef QUEST_DECODE_LAUNCH
  return check_launch("quest_sparse_decode");
}
}  // namespace

int launch_sparse_decode(const quest_cache& c, const void* q, const int32_t* topk_idx, int k_pages,
                         float sm_scale, void* out, int out_is_fp16, float* lse, void* workspace,
                         hipStream_t s) {
  return launch_decode(c, q, topk_idx, nullptr, nullptr, nullptr, k_pages, sm_scale, out, out_is_fp16,
                       lse, workspace, s);
}

// Selection and attention in one launch: while a row of scores fits the in-register
// selection of 512 threads with at most 8 keys each and the list fits in LDS.  Every
// split of a head repeats the selection, so for longer rows (measured at 4097 pages:
// 34.9 us against 34.2 us) the separate Top-K launch is the faster form.
bool select_decode_supported(const quest_cache& c, int k_pages) {
  return !(c.flags & QUEST_FLAG_SEPARATE_LAUNCHES) &&
         c.max_pages_per_seq <= kSelWaves * kWave * 8 && k_pages <= kSelListCap;
}

int launch_select_decode(const quest_cache& c, const void* q, const float* scores, int k_pages,
                         float sm_scale, int32_t* topk_idx, int32_t* k_eff, void* out,
                         int out_is_fp16, float* lse, void* workspace, hipStream_t s) {
  if (select_decode_supported(c, k_pages))
    return launch_decode(c, q, nullptr, scores, topk_idx, k_eff, k_pages, sm_scale, out, out_is_fp16,
                         lse, workspace, s);
  // very long rows: selection in two stages, candidates behind the attention's workspace
  const int r = topk_scratch_bytes(c, k_pages) > 0
                    ? launch_topk_chunked(c, scores, k_pages, topk_idx, k_eff,
                                          (char*)workspace + decode_workspace_bytes(c, k_pages), s)
                    : launch_topk(c, scores, k_pages, topk_idx, k_eff, s);
  if (r != QUEST_OK) return r;
  return launch_sparse_decode(c, q, topk_idx, k_pages, sm_scale, out, out_is_fp16, lse, workspace, s);
}

}  // namespace quest
