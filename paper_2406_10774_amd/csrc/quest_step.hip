// One decode step of Quest in a single launch: insertion of the new token,
// criticality estimate, Top-K selection and sparse attention (Algorithm 1 and
// Figure 5 of arXiv 2406.10774) chained inside one persistent kernel instead of
// three or four launches.  Same arithmetic as the stand-alone kernels (the
// device cores are shared), so metadata, scores and the page list are bit-equal
// to theirs.
//
// Why: at 32 heads / 32k context each streaming phase moves 32 MiB, about 4 us
// at HBM speed, while a kernel boundary costs 1.6 us plus the drain and ramp of
// the machine, and the dependent phases of different heads cannot overlap across
// launches.  Here the phases of a head are chained by per-head counters.
//
// Scheme.  A (sequence, head) pair is an "item"; item i belongs to die i % 8.
// Each die has a queue (one ticket counter) of tasks in a fixed order: first
// every estimate task of its items (64 or 128 pages each), then
// every attention task (a slice of the selected-page list).  Work-groups are
// persistent: a work-group reads the id of the die it really runs on and
// serves that die's queue until it is empty.  Everything the work-groups of an
// item hand to each other (scores, page list, split partials) therefore stays
// inside one die, whose L2 is coherent: plain stores, a wait for the stores, an
// L2 atomic, device-scope loads -- no device-wide cache maintenance.
//   * the work-group that finishes the last estimate task of an item runs the
//     Top-K selection for it and then raises the item's "list ready" flag;
//   * an attention task first waits for that flag;
//   * the work-group that finishes the last attention task of an item merges
//     the item's split partials and writes the output.
// No deadlock by construction: a work-group only ever waits (for the flag)
// while holding an attention task, and a queue hands out attention tasks only
// after all its estimate tasks have been handed out to work-groups that are
// running and never wait; so the flag is always on its way.  The wait is
// bounded anyway and raises a status word instead of hanging.
// The last work-group to leave checks that every queue was served (a die that
// got no work-group at all would leave its items undone: status word) and
// re-arms all counters for the next launch.
#include "quest_common.h"
#include "quest_decode_core.h"
#include "quest_estimate_core.h"
#include "quest_team.h"
#include "quest_topk_core.h"

#include <cstdlib>

namespace quest {

namespace {

constexpr int kStepThreads = 512;
constexpr int kStepWaves = kStepThreads / kWave;              // 8
constexpr int kNumDies = 8;
constexpr int kSlotWords = 64;  // 256-byte slots of uint32 words
// workspace words: slot 0 = {leavers, status}; slots 1..8 = die queues;
// slots 9.. = one per item {estimate tasks done, list ready, attention tasks done}
constexpr int kItemSlot0 = 1 + kNumDies;
constexpr uint32_t kSpinLimit = 1u << 20;  // about a second; the flag normally arrives within microseconds

enum : uint32_t { kStatusDieNotServed = 1, kStatusWaitTimedOut = 2 };

struct StepArgs {
  EstimateArgs est;
  const char* k_pool;
  const char* v_pool;
  int32_t* topk_idx;
  int32_t* k_eff;
  void* out;
  float* lse;
  uint32_t* words;   // counters (see above)
  float* part_acc;   // [items * dec_tasks][D]
  float* part_ml;    // [items * dec_tasks][2]
  int batch, k_pages, out_is_fp16;
  int est_iters;     // pages per DPP row in an estimate task (2 or 4): a task covers 32 * est_iters pages
  int est_tasks;     // E: estimate tasks per item = ceil(max_pages / (32 * est_iters))
  int dec_tasks;     // Dn: attention tasks per item
  int pages_per_wave;  // list positions per wave in an attention task (<= 64)
  float scale_log2;
#ifdef QUEST_STEP_TRACE
  unsigned long long* trace;
#endif
};

__device__ __forceinline__ uint32_t word_add(uint32_t* p, uint32_t v) {
  return __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint32_t word_load(const uint32_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void word_set(uint32_t* p, uint32_t v) {
  __hip_atomic_exchange(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

#ifdef QUEST_STEP_TRACE
#define STEP_TRACE(slot)                                                              \
  do {                                                                                \
    if (threadIdx.x == 0 && a.trace && a.trace[(size_t)blockIdx.x * 16 + (slot)] == 0) \
      a.trace[(size_t)blockIdx.x * 16 + (slot)] = wall_clock64();                     \
  } while (0)
#else
#define STEP_TRACE(slot) \
  do {                   \
  } while (0)
#endif

struct StepShared {
  TopkShared<kStepThreads> topk;
  float acc[kStepWaves][kHeadDim];
  float m[kStepWaves], l[kStepWaves];
  uint32_t u[4];
};

// ---- attention task: slice `chunk` of the item's page list
__device__ __forceinline__ void attention_task(const StepArgs& a, StepShared& sm, int item, int chunk,
                                               uint32_t* state) {
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = lane_id();
  const int grp = lane >> 4;
  const int c = lane & 15;
  const int num_heads = a.est.num_heads, max_pages = a.est.max_pages;
  const int b = item / num_heads;
  const int h = item - b * num_heads;

  // the page list must be complete
  if (tid == 0) {
    uint32_t spins = 0;
    while (word_load(state + 1) == 0u) {
      __builtin_amdgcn_s_sleep(1);
      if (++spins > kSpinLimit) {
        word_set(a.words + 1, kStatusWaitTimedOut);
        break;
      }
    }
  }
  __syncthreads();
  STEP_TRACE(6);

  const int list_len = a.k_pages < max_pages ? a.k_pages : max_pages;
  const int begin = chunk * kStepWaves * a.pages_per_wave;
  const int32_t* idx_row = a.topk_idx + (size_t)item * a.k_pages;
  const int32_t* pt = a.est.page_table + (size_t)b * max_pages;
  const int seq_len = a.est.seq_lens[b];
  const uint4 qv = ld16(a.est.q + (size_t)item * (kHeadDim * 2) + c * 16);

  // lane i: i-th list entry of this wave (positions begin + wave + 8 i)
  const int pos = begin + wave + kStepWaves * lane;
  int lp_v = -1;
  if (lane < a.pages_per_wave && pos < list_len) lp_v = team_ld(idx_row + pos);
  int ph_v = 0;
  if (lp_v >= 0 && lp_v < max_pages) ph_v = pt[lp_v];
  const int num_pages = (seq_len + kPageSize - 1) / kPageSize;
  if (lp_v >= num_pages) lp_v = -1;

  Softmax st;
  st.m = kNegBig;
  st.l = 0.f;
#pragma unroll
  for (int j = 0; j < 8; ++j) st.acc[j] = 0.f;

  {
    const int n_here = a.pages_per_wave;
    PageRegs ra, rb;
    int j = 0;
    int lp = __builtin_amdgcn_readlane(lp_v, 0);
    if (lp >= 0)
      load_page(ra, a.k_pool, a.v_pool, num_heads, h, seq_len, lp, __builtin_amdgcn_readlane(ph_v, 0),
                lane);
    while (lp >= 0) {
      int lp_b = -1;
      if (j + 1 < n_here) lp_b = __builtin_amdgcn_readlane(lp_v, j + 1);
      if (lp_b >= 0)
        load_page(rb, a.k_pool, a.v_pool, num_heads, h, seq_len, lp_b,
                  __builtin_amdgcn_readlane(ph_v, j + 1), lane);
      fold_page(st, ra, qv, a.scale_log2, grp);
      if (lp_b < 0) break;
      j += 2;
      lp = -1;
      if (j < n_here) lp = __builtin_amdgcn_readlane(lp_v, j);
      if (lp >= 0)
        load_page(ra, a.k_pool, a.v_pool, num_heads, h, seq_len, lp,
                  __builtin_amdgcn_readlane(ph_v, j), lane);
      fold_page(st, rb, qv, a.scale_log2, grp);
    }
  }

  STEP_TRACE(7);
  merge_lanes(st, 16);
  merge_lanes(st, 32);
  if (lane < 16) {
#pragma unroll
    for (int j = 0; j < 8; ++j) sm.acc[wave][c * 8 + j] = st.acc[j];
    if (lane == 0) {
      sm.m[wave] = st.m;
      sm.l[wave] = st.l;
    }
  }
  __syncthreads();
  float m_tot = sm.m[0];
#pragma unroll
  for (int w = 1; w < kStepWaves; ++w) m_tot = fmaxf(m_tot, sm.m[w]);
  float l_tot = 0.f, acc = 0.f;
#pragma unroll
  for (int w = 0; w < kStepWaves; ++w) {
    const float f = __builtin_amdgcn_exp2f(sm.m[w] - m_tot);
    l_tot += sm.l[w] * f;
    acc += sm.acc[w][tid & (kHeadDim - 1)] * f;
  }
  if (a.dec_tasks == 1) {
    if (tid < kHeadDim) {
      store_out(a.out, a.out_is_fp16, (size_t)item * kHeadDim + tid, acc / l_tot);
      if (tid == 0 && a.lse) a.lse[item] = (m_tot + __builtin_amdgcn_logf(l_tot)) * kLn2;
    }
    __syncthreads();  // sm is reused by the next task
    return;
  }

  // publish the partial; the task that arrives last merges
  const size_t ps = (size_t)item * a.dec_tasks + chunk;
  if (tid < kHeadDim) a.part_acc[ps * kHeadDim + tid] = acc;
  if (tid == 0) {
    a.part_ml[ps * 2 + 0] = m_tot;
    a.part_ml[ps * 2 + 1] = l_tot;
  }
  wait_stores();
  __syncthreads();
  if (tid == 0) sm.u[1] = word_add(state + 2, 1u);
  __syncthreads();
  const bool last = __builtin_amdgcn_readfirstlane(sm.u[1]) == (uint32_t)a.dec_tasks - 1;
  STEP_TRACE(8);
  __syncthreads();
  if (!last || tid >= kHeadDim) return;

  const float* ml = a.part_ml + (size_t)item * a.dec_tasks * 2;
  const float* pacc = a.part_acc + (size_t)item * a.dec_tasks * kHeadDim + tid;
  float mx = kNegBig, l_all = 0.f, o = 0.f;
  for (int s0 = 0; s0 < a.dec_tasks; s0 += 16) {
    float pm[16], pl[16], pa[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int sidx = min(s0 + i, a.dec_tasks - 1);
      pm[i] = team_ld(ml + 2 * sidx);
      pl[i] = team_ld(ml + 2 * sidx + 1);
      pa[i] = team_ld(pacc + (size_t)sidx * kHeadDim);
    }
    float cm = mx;
#pragma unroll
    for (int i = 0; i < 16; ++i) cm = fmaxf(cm, pm[i]);
    const float rescale = __builtin_amdgcn_exp2f(mx - cm);
    l_all *= rescale;
    o *= rescale;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float f = s0 + i < a.dec_tasks ? __builtin_amdgcn_exp2f(pm[i] - cm) : 0.f;
      l_all += pl[i] * f;
      o += pa[i] * f;
    }
    mx = cm;
  }
  store_out(a.out, a.out_is_fp16, (size_t)item * kHeadDim + tid, o / l_all);
  if (tid == 0 && a.lse) a.lse[item] = (mx + __builtin_amdgcn_logf(l_all)) * kLn2;
  STEP_TRACE(9);
}

template <int kItems, bool kAppend>
__global__ __launch_bounds__(kStepThreads, 4) void step_kernel(const StepArgs a) {
  __shared__ StepShared sm;
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int die = xcc_id() & (kNumDies - 1);
  const int num_heads = a.est.num_heads, max_pages = a.est.max_pages;
  const int items = a.batch * num_heads;
  const int my_items = items > die ? (items - die + kNumDies - 1) / kNumDies : 0;
  const uint32_t n_est = (uint32_t)my_items * a.est_tasks;
  const uint32_t total = n_est + (uint32_t)my_items * a.dec_tasks;
  uint32_t* queue = a.words + (1 + die) * kSlotWords;
  STEP_TRACE(0);

  for (;;) {
    if (tid == 0) sm.u[0] = word_add(queue, 1u);
    __syncthreads();
    // the value is the same in every lane; say so, or the loop counts as divergent
    // and the barriers inside it stop being reached by whole waves together
    const uint32_t ticket = __builtin_amdgcn_readfirstlane(sm.u[0]);
    __syncthreads();
    if (ticket >= total) break;
    if (ticket < n_est) {
      STEP_TRACE(1);
      // ---- estimate task (with the insertion of the new token where it falls)
      const int item = (int)(ticket / a.est_tasks) * kNumDies + die;
      const int chunk = (int)(ticket % a.est_tasks);
      const int b = item / num_heads;
      const int h = item - b * num_heads;
      uint32_t* state = a.words + (size_t)(kItemSlot0 + item) * kSlotWords;
      if (a.est_iters == 2)
        estimate_wave<kAppend, 2>(a.est, b, h, (chunk * kStepWaves + wave) * 8);
      else
        estimate_wave<kAppend, 4>(a.est, b, h, (chunk * kStepWaves + wave) * 16);
      wait_stores();
      STEP_TRACE(2);
      __syncthreads();
      if (tid == 0) sm.u[1] = word_add(state, 1u);
      __syncthreads();
      const bool last = __builtin_amdgcn_readfirstlane(sm.u[1]) == (uint32_t)a.est_tasks - 1;
      STEP_TRACE(3);
      __syncthreads();
      if (last) {
        topk_block<kStepThreads, kItems, true>(
            sm.topk, a.est.scores + (size_t)item * max_pages, a.est.seq_lens + b, max_pages,
            a.k_pages, a.topk_idx + (size_t)item * a.k_pages,
            (h == 0 && a.k_eff != nullptr) ? a.k_eff + b : nullptr);
        wait_stores();
        __syncthreads();
        if (tid == 0) word_set(state + 1, 1u);
        STEP_TRACE(4);
        // Every single-lane section in this loop is closed by a barrier before the
        // back-edge.  Without it the compiler may sink the section into the next
        // iteration's single-lane ticket draw and let the other lanes of wave 0 run
        // ahead to the next barrier alone; the hardware barrier counts waves, not
        // lanes, so the work-group would then loop on a stale ticket for ever.
        __syncthreads();
      }
    } else {
      STEP_TRACE(5);
      const uint32_t t = ticket - n_est;
      const int item = (int)(t / a.dec_tasks) * kNumDies + die;
      const int chunk = (int)(t % a.dec_tasks);
      attention_task(a, sm, item, chunk, a.words + (size_t)(kItemSlot0 + item) * kSlotWords);
      __syncthreads();
    }
  }

  STEP_TRACE(10);
  // ---- leave; the last one out checks the queues and re-arms every counter
  if (tid == 0) sm.u[2] = word_add(a.words, 1u);
  __syncthreads();
  if (__builtin_amdgcn_readfirstlane(sm.u[2]) != gridDim.x - 1) return;
  if (tid < kNumDies) {
    const int cnt = items > tid ? (items - tid + kNumDies - 1) / kNumDies : 0;
    const uint32_t want = (uint32_t)cnt * (a.est_tasks + a.dec_tasks);
    uint32_t* qd = a.words + (1 + tid) * kSlotWords;
    // a served queue ends above `want`: each of its work-groups drew one "empty" ticket
    if (want != 0 && word_load(qd) <= want) word_set(a.words + 1, kStatusDieNotServed);
    word_set(qd, 0u);
  }
  for (int i = tid; i < items * 3; i += kStepThreads)
    word_set(a.words + (size_t)(kItemSlot0 + i / 3) * kSlotWords + i % 3, 0u);
  if (tid == 0) word_set(a.words, 0u);
}

int env_int(const char* name, int fallback) {
  const char* v = std::getenv(name);
  return (v && *v) ? std::atoi(v) : fallback;
}

struct StepPlan {
  int groups, est_iters, est_tasks, dec_tasks, pages_per_wave;
  bool fused;
};

StepPlan plan_step(const quest_cache& c, int k_pages) {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess)
      cus = n;
    else
      cus = -1;
    (void)hipGetLastError();
  }
  StepPlan p;
  // The persistent kernel is opt-in, and its die-queue scheme is laid out for the
  // full MI355X (8 dies x 32 CUs); any other device shape, or rows too long for
  // the in-register selection, takes the three-launch path.
  p.fused = (c.flags & QUEST_FLAG_PERSISTENT_STEP) && cus == 256 &&
            c.max_pages_per_seq <= kStepThreads * 16;
  p.groups = 2 * 256;
  // Estimate tasks of 64 pages: with the queue in item order, the work-groups of
  // a die first all work on its first items and then on the rest, so the
  // selection of the first items overlaps with the estimate of the others.
  static const int est_iters = env_int("QUEST_STEP_EST_ITERS", 2);
  p.est_iters = est_iters == 4 ? 4 : 2;
  const int est_pages = kStepWaves * 4 * p.est_iters;
  p.est_tasks = (c.max_pages_per_seq + est_pages - 1) / est_pages;
  const long items = (long)c.batch * c.num_heads;
  const long list_len = k_pages < c.max_pages_per_seq ? k_pages : c.max_pages_per_seq;
  long ppw = (items * list_len + (long)kStepWaves * p.groups - 1) / ((long)kStepWaves * p.groups);
  if (ppw < 1) ppw = 1;
  if (ppw > 64) ppw = 64;
  p.pages_per_wave = (int)ppw;
  p.dec_tasks = (int)((list_len + kStepWaves * ppw - 1) / (kStepWaves * ppw));
  return p;
}

size_t step_counter_bytes(const quest_cache& c) {
  return (size_t)(kItemSlot0 + (size_t)c.batch * c.num_heads) * kSlotWords * sizeof(uint32_t);
}

template <int kItems>
int launch_step_items(const StepArgs& a, bool append, int groups, hipStream_t s) {
  if (append)
    hipLaunchKernelGGL((step_kernel<kItems, true>), dim3(groups), dim3(kStepThreads), 0, s, a);
  else
    hipLaunchKernelGGL((step_kernel<kItems, false>), dim3(groups), dim3(kStepThreads), 0, s, a);
  return check_launch("quest_decode_step");
}

}  // namespace

size_t step_workspace_bytes(const quest_cache& c, int k_pages) {
  const StepPlan p = plan_step(c, k_pages);
  const size_t fused = step_counter_bytes(c) + (size_t)c.batch * c.num_heads * p.dec_tasks *
                                                   (kHeadDim + 2) * sizeof(float);
  const size_t unfused = decode_workspace_bytes(c, k_pages);
  return fused > unfused ? fused : unfused;
}

int launch_decode_step(const quest_cache& c, const void* k_new, const void* v_new, int k_pool_write,
                       const void* q, int k_pages, float sm_scale, float* scores, int32_t* topk_idx,
                       int32_t* k_eff, void* out, int out_is_fp16, float* lse, void* workspace,
                       hipStream_t s) {
  const StepPlan p = plan_step(c, k_pages);
  if (!p.fused) {
    int r = k_new ? launch_append_estimate(c, k_new, v_new, k_pool_write, q, scores, s)
                  : launch_estimate(c, q, scores, s);
    if (r != QUEST_OK) return r;
    r = launch_topk(c, scores, k_pages, topk_idx, k_eff, s);
    if (r != QUEST_OK) return r;
    return launch_sparse_decode(c, q, topk_idx, k_pages, sm_scale, out, out_is_fp16, lse, workspace,
                                s);
  }
  StepArgs a;
  a.est.meta = (char*)c.meta;
  a.est.q = (const char*)q;
  a.est.page_table = c.page_table;
  a.est.seq_lens = c.seq_lens;
  a.est.scores = scores;
  a.est.num_heads = c.num_heads;
  a.est.max_pages = c.max_pages_per_seq;
  a.est.num_phys_pages = c.num_phys_pages;
  a.est.k_new = (const char*)k_new;
  a.est.v_new = (const char*)v_new;
  a.est.k_pool = (char*)c.k_pool;
  a.est.v_pool = (char*)c.v_pool;
  a.est.k_pool_write = k_pool_write;
  a.k_pool = (const char*)c.k_pool;
  a.v_pool = (const char*)c.v_pool;
  a.topk_idx = topk_idx;
  a.k_eff = k_eff;
  a.out = out;
  a.lse = lse;
  a.words = (uint32_t*)workspace;
  a.part_acc = (float*)((char*)workspace + step_counter_bytes(c));
  a.part_ml = a.part_acc + (size_t)c.batch * c.num_heads * p.dec_tasks * kHeadDim;
  a.batch = c.batch;
  a.k_pages = k_pages;
  a.out_is_fp16 = out_is_fp16;
  a.est_iters = p.est_iters;
  a.est_tasks = p.est_tasks;
  a.dec_tasks = p.dec_tasks;
  a.pages_per_wave = p.pages_per_wave;
  a.scale_log2 = sm_scale * kLog2e;
#ifdef QUEST_STEP_TRACE
  a.trace = std::getenv("QUEST_STEP_TRACE_PTR")
                ? (unsigned long long*)std::strtoull(std::getenv("QUEST_STEP_TRACE_PTR"), nullptr, 16)
                : nullptr;
#endif
  const bool append = k_new != nullptr;
  const int mp = c.max_pages_per_seq;
#define QUEST_STEP_CASE(I) \
  if (mp <= kStepThreads * (I)) return launch_step_items<I>(a, append, p.groups, s)
  QUEST_STEP_CASE(1);
  QUEST_STEP_CASE(2);
  QUEST_STEP_CASE(3);
  QUEST_STEP_CASE(4);
  QUEST_STEP_CASE(5);
  QUEST_STEP_CASE(6);
  QUEST_STEP_CASE(8);
  QUEST_STEP_CASE(10);
  QUEST_STEP_CASE(12);
  QUEST_STEP_CASE(16);
#undef QUEST_STEP_CASE
  set_error("quest_decode_step: internal: no kernel for max_pages_per_seq = %d", mp);
  return QUEST_ERR_SHAPE;
}

}  // namespace quest
