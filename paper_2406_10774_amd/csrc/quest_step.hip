// One decode step of Quest in a single launch: insertion of the new token,
// criticality estimate, Top-K selection and sparse attention (Algorithm 1 and
// Figure 5 of arXiv 2406.10774) chained inside one kernel instead of three
// launches.  Same arithmetic as the stand-alone kernels (the device cores are
// shared), so metadata, scores and the page list are bit-equal to theirs.
//
// Why: at 32 heads / 32k context each streaming phase moves 32 MiB, about 4 us
// at HBM speed, while a kernel boundary costs 1.6 us plus the drain and ramp of
// the machine.
//
// Scheme.  Every (sequence, head) has a team of M work-groups (8 waves each),
// laid out on one die (quest_team.h).  Member m
//   1. scores its slice of the head's pages (and inserts the new token if it
//      falls into the slice), publishes; the member that arrives last selects
//      the head's pages and raises the head's "list ready" flag;
//   2. waits for the flag, runs attention over its slice of the selected-page
//      list, publishes its partial; the member that arrives last merges, writes
//      the output and re-arms the head's counters for the next launch.
// A member only waits after finishing its own estimate, and the flag is raised
// by whichever member finishes its estimate last, so the wait cannot deadlock as
// long as the members of a team get to run; the host keeps the grid within what
// is resident at once, and the wait is bounded anyway (status word instead of a
// hang).  Exchanges between members go through the die's L2 when the whole team
// is known to share a die, through device-scope fences otherwise.
#include "quest_common.h"
#include "quest_decode_core.h"
#include "quest_estimate_core.h"
#include "quest_team.h"
#include "quest_topk_core.h"

#include <cstdlib>

namespace quest {

namespace {

constexpr int kStepThreads = 512;
constexpr int kStepWaves = kStepThreads / kWave;  // 8
constexpr int kSlotBytes = 256;                   // per (sequence, head): team word, flag, arrivals
constexpr uint32_t kSpinLimit = 1u << 20;  // about a second; the flag normally arrives within microseconds

enum : uint32_t { kStatusWaitTimedOut = 2 };

struct StepArgs {
  EstimateArgs est;
  const char* k_pool;
  const char* v_pool;
  int32_t* topk_idx;
  int32_t* k_eff;
  void* out;
  float* lse;
  char* slots;        // [items] 256-byte slots: u64 team word, u32 list-ready flag, u32 attention arrivals
  uint32_t* status;   // sticky: non-zero = a launch left work undone
  float* part_acc;    // [items * members][D]
  float* part_ml;     // [items * members][2]
  int batch, k_pages, out_is_fp16, force_device_fences;
  int policy;         // QUEST_FLAG_KEEP_* bits of the cache
  int members;        // M: work-groups per (sequence, head)
  int est_calls;      // blocks of 32 * kIters pages a member scores one after the other
  int list_per_member;  // selected-list positions per member
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
#define STEP_TRACE(slot)                                                                  \
  do {                                                                                    \
    if (threadIdx.x == 0 && a.trace) a.trace[(size_t)blockIdx.x * 16 + (slot)] = wall_clock64(); \
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

// In every barrier-separated section below, values read from LDS that steer
// control flow go through readfirstlane and every single-lane section is closed
// by a barrier: otherwise the compiler may let part of wave 0 run ahead to the
// next s_barrier alone (the hardware barrier counts waves, not lanes).
template <int kItems, int kIters, bool kAppend>
__global__ __launch_bounds__(kStepThreads, 4) void step_kernel(const StepArgs a) {
  __shared__ StepShared sm;
  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lane = lane_id();
  const int grp = lane >> 4;
  const int c = lane & 15;
  const int num_heads = a.est.num_heads, max_pages = a.est.max_pages;
  const int M = a.members;

  const int slot = blockIdx.x & 7;
  const int rank = blockIdx.x >> 3;
  const int member = rank % M;
  const int item = (rank / M) * 8 + slot;
  if (item >= a.batch * num_heads) return;
  const int b = item / num_heads;
  const int h = item - b * num_heads;
  const uint32_t die = xcc_id();
  char* st_slot = a.slots + (size_t)item * kSlotBytes;
  uint64_t* team_word = reinterpret_cast<uint64_t*>(st_slot);
  uint32_t* flag = reinterpret_cast<uint32_t*>(st_slot + 8);
  uint32_t* arrivals = reinterpret_cast<uint32_t*>(st_slot + 12);
  if (M > 1 && tid == 0) team_checkin(team_word, die);
  STEP_TRACE(0);

  // ---- 1. estimate (and insertion) over this member's slice of the pages
  {
    constexpr int kWavePages = 4 * kIters;
    const int span = kStepWaves * kWavePages * a.est_calls;
    for (int call = 0; call < a.est_calls; ++call)
      estimate_wave<kAppend, kIters>(a.est, b, h,
                                     member * span + (call * kStepWaves + wave) * kWavePages);
  }
  uint64_t seen = 0;
  if (M > 1 && tid == 0) seen = team_load(team_word);
  wait_stores();
  STEP_TRACE(1);
  __syncthreads();
  bool fenced = false, last_est = true;
  if (M > 1) {
    if (tid == 0) {
      const uint64_t before = team_publish(team_word, seen, M, die, a.force_device_fences);
      sm.u[0] = (uint32_t)before;
      sm.u[1] = (uint32_t)(before >> 32);
    }
    __syncthreads();
    const uint64_t before = (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane(sm.u[0]) |
                            ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane(sm.u[1]) << 32);
    // definitive when true: all M members have started and share this die
    fenced = a.force_device_fences || !team_on_one_die(before, M, die);
    last_est = team_is_last(before, M);
    __syncthreads();
  }
  STEP_TRACE(2);

  // ---- 2. the member that finished the head's estimate selects its pages
  if (last_est) {
    if (fenced) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    topk_block<kStepThreads, kItems, true>(
        sm.topk, a.est.scores + (size_t)item * max_pages, a.est.seq_lens + b, max_pages, a.k_pages,
        a.topk_idx + (size_t)item * a.k_pages, (h == 0 && a.k_eff != nullptr) ? a.k_eff + b : nullptr,
        a.est.page_shift, a.policy
#ifdef QUEST_STEP_TRACE
        ,
        a.trace ? a.trace + (size_t)blockIdx.x * 16 + 8 : nullptr
#endif
    );
    wait_stores();
    __syncthreads();
    if (M > 1 && tid == 0) {
      if (fenced) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
      word_set(flag, 1u);
    }
    __syncthreads();
    STEP_TRACE(3);
  }

  // ---- 3. attention over this member's slice of the selected-page list
  if (M > 1) {
    if (tid == 0) {
      uint32_t spins = 0;
      while (word_load(flag) == 0u) {
        __builtin_amdgcn_s_sleep(1);
        if (++spins > kSpinLimit) {
          word_set(a.status, kStatusWaitTimedOut);
          break;
        }
      }
    }
    __syncthreads();
    if (fenced) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
  }
  STEP_TRACE(4);

  const int list_len = a.k_pages < max_pages ? a.k_pages : max_pages;
  const int begin = member * a.list_per_member;
  const int end = min(list_len, begin + a.list_per_member);
  const int n_here = (a.list_per_member + kStepWaves - 1) / kStepWaves;  // <= 64 (host)
  const int32_t* idx_row = a.topk_idx + (size_t)item * a.k_pages;
  const int32_t* pt = a.est.page_table + (size_t)b * max_pages;
  const int seq_len = a.est.seq_lens[b];
  const uint4 qv = ld16(a.est.q + (size_t)item * (kHeadDim * 2) + c * 16);

  // lane i: i-th list entry of this wave (positions begin + wave + 8 i)
  const int pos = begin + wave + kStepWaves * lane;
  int lp_v = -1;
  if (lane < n_here && pos < end) lp_v = team_ld(idx_row + pos);
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
  STEP_TRACE(5);

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
  if (M == 1) {
    if (tid < kHeadDim) {
      store_out(a.out, a.out_is_fp16, (size_t)item * kHeadDim + tid, acc / l_tot);
      if (tid == 0 && a.lse) a.lse[item] = (m_tot + __builtin_amdgcn_logf(l_tot)) * kLn2;
    }
    return;
  }

  // publish the partial; the member that arrives last merges and re-arms
  const size_t ps = (size_t)item * M + member;
  if (tid < kHeadDim) a.part_acc[ps * kHeadDim + tid] = acc;
  if (tid == 0) {
    a.part_ml[ps * 2 + 0] = m_tot;
    a.part_ml[ps * 2 + 1] = l_tot;
  }
  wait_stores();
  __syncthreads();
  if (tid == 0) {
    if (fenced) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    sm.u[2] = word_add(arrivals, 1u);
  }
  __syncthreads();
  const bool last = __builtin_amdgcn_readfirstlane(sm.u[2]) == (uint32_t)M - 1;
  STEP_TRACE(6);
  if (!last) return;
  if (fenced) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
  if (tid == 0) {  // every member has passed all its waits: re-arm for the next launch
    team_reset(team_word);
    word_set(flag, 0u);
    word_set(arrivals, 0u);
  }
  if (tid >= kHeadDim) return;

  const float* ml = a.part_ml + (size_t)item * M * 2;
  const float* pacc = a.part_acc + (size_t)item * M * kHeadDim + tid;
  float mx = kNegBig, l_all = 0.f, o = 0.f;
  for (int s0 = 0; s0 < M; s0 += 16) {
    float pm[16], pl[16], pa[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int sidx = min(s0 + i, M - 1);
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
      const float f = s0 + i < M ? __builtin_amdgcn_exp2f(pm[i] - cm) : 0.f;
      l_all += pl[i] * f;
      o += pa[i] * f;
    }
    mx = cm;
  }
  store_out(a.out, a.out_is_fp16, (size_t)item * kHeadDim + tid, o / l_all);
  if (tid == 0 && a.lse) a.lse[item] = (mx + __builtin_amdgcn_logf(l_all)) * kLn2;
  STEP_TRACE(7);
}

int env_int(const char* name, int fallback) {
  const char* v = std::getenv(name);
  return (v && *v) ? std::atoi(v) : fallback;
}

struct StepPlan {
  bool fused;
  int iters, est_calls, members, list_per_member;
};

// Work-groups of this kernel that can be resident at once on the device.
int resident_capacity() {
  static int cap = 0;
  if (cap == 0) {
    int dev = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess &&
        hipOccupancyMaxActiveBlocksPerMultiprocessor(
            &per_cu, reinterpret_cast<const void*>(&step_kernel<5, 5, true>), kStepThreads, 0) ==
            hipSuccess)
      cap = cus * per_cu;
    else
      cap = -1;
    (void)hipGetLastError();
  }
  return cap;
}

StepPlan plan_step(const quest_cache& c, int k_pages) {
  StepPlan p = {};
  const long items = (long)c.batch * c.num_heads;
  const int cap = resident_capacity();
  // opt-in, 16-token pages, one KV head per query head, rows within the in-register selection,
  // every team resident at once
  p.fused = (c.flags & QUEST_FLAG_PERSISTENT_STEP) && c.page_size == kPageSize &&
            group_size(c) == 1 && cap > 0 &&
            items <= cap && c.max_pages_per_seq <= kStepThreads * 16;
  if (!p.fused) return p;
  const int mp = c.max_pages_per_seq;
  static const int force_iters = env_int("QUEST_STEP_EST_ITERS", 0);
  const int choices[4] = {4, 5, 6, 8};
  p.iters = 8;
  p.est_calls = 1;
  bool found = false;
  for (int i = 0; i < 4 && !found; ++i) {
    if (force_iters && choices[i] != force_iters) continue;
    const int span = kStepWaves * 4 * choices[i];
    const long m = (mp + span - 1) / span;
    if (items * m <= cap) {
      p.iters = choices[i];
      p.members = (int)m;
      found = true;
    }
  }
  if (!found) {  // several blocks per member, 256 pages each
    const long per_item = cap / items;  // >= 1
    const int span1 = kStepWaves * 4 * 8;
    p.est_calls = (int)(((mp + span1 - 1) / span1 + per_item - 1) / per_item);
    p.members = (mp + span1 * p.est_calls - 1) / (span1 * p.est_calls);
  }
  if (p.members > kMaxTeamSize) {
    p.fused = false;
    return p;
  }
  const int list_len = k_pages < mp ? k_pages : mp;
  p.list_per_member = (list_len + p.members - 1) / p.members;
  if ((p.list_per_member + kStepWaves - 1) / kStepWaves > kWave) p.fused = false;  // one lane per entry
  return p;
}

size_t slots_bytes(const quest_cache& c) { return (size_t)c.batch * c.num_heads * kSlotBytes; }

template <int kItems, int kIters>
int launch_variant(const StepArgs& a, bool append, unsigned groups, hipStream_t s) {
  if (append)
    hipLaunchKernelGGL((step_kernel<kItems, kIters, true>), dim3(groups), dim3(kStepThreads), 0, s, a);
  else
    hipLaunchKernelGGL((step_kernel<kItems, kIters, false>), dim3(groups), dim3(kStepThreads), 0, s, a);
  return check_launch("quest_decode_step");
}

template <int kItems>
int launch_items(const StepArgs& a, int iters, bool append, unsigned groups, hipStream_t s) {
  switch (iters) {
    case 4: return launch_variant<kItems, 4>(a, append, groups, s);
    case 5: return launch_variant<kItems, 5>(a, append, groups, s);
    case 6: return launch_variant<kItems, 6>(a, append, groups, s);
    default: return launch_variant<kItems, 8>(a, append, groups, s);
  }
}

}  // namespace

// Layout: [items] 256-byte slots | split partials | 256-byte status slot (last).
size_t step_workspace_bytes(const quest_cache& c, int k_pages) {
  // size for the largest team the plan can choose (one member per 128 pages), so
  // that the size does not depend on flags or on the device
  const size_t max_members = (c.max_pages_per_seq + 127) / 128;
  const size_t fused = slots_bytes(c) +
                       (size_t)c.batch * c.num_heads * max_members * (kHeadDim + 2) * sizeof(float) +
                       kSlotBytes;
  const size_t unfused = decode_workspace_bytes(c, k_pages) + kSlotBytes;
  return fused > unfused ? fused : unfused;
}

int launch_decode_step(const quest_cache& c, const void* k_new, const void* v_new, int k_pool_write,
                       const void* q, int k_pages, float sm_scale, float* scores, int32_t* topk_idx,
                       int32_t* k_eff, void* out, int out_is_fp16, float* lse, void* workspace,
                       size_t workspace_bytes, hipStream_t s) {
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
  static const int force_fences = env_int("QUEST_FORCE_DEVICE_FENCES", 0);
  StepArgs a;
  a.est.meta = (char*)c.meta;
  a.est.q = (const char*)q;
  a.est.page_table = c.page_table;
  a.est.seq_lens = c.seq_lens;
  a.est.scores = scores;
  a.est.num_heads = c.num_heads;
  a.est.max_pages = c.max_pages_per_seq;
  a.est.num_phys_pages = c.num_phys_pages;
  a.est.page_shift = page_shift_of(c.page_size);
  a.est.group = 1;
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
  a.slots = (char*)workspace;
  (void)workspace_bytes;  // checked by the caller; the status slot sits at the end of the required size
  a.status = (uint32_t*)((char*)workspace + step_workspace_bytes(c, k_pages) - kSlotBytes);
  a.part_acc = (float*)((char*)workspace + slots_bytes(c));
  a.part_ml = a.part_acc + (size_t)c.batch * c.num_heads * p.members * kHeadDim;
  a.batch = c.batch;
  a.k_pages = k_pages;
  a.out_is_fp16 = out_is_fp16;
  a.policy = c.flags;
  a.force_device_fences = force_fences || (c.flags & QUEST_FLAG_DEVICE_FENCES) != 0;
  a.members = p.members;
  a.est_calls = p.est_calls;
  a.list_per_member = p.list_per_member;
  a.scale_log2 = sm_scale * kLog2e;
#ifdef QUEST_STEP_TRACE
  a.trace = std::getenv("QUEST_STEP_TRACE_PTR")
                ? (unsigned long long*)std::strtoull(std::getenv("QUEST_STEP_TRACE_PTR"), nullptr, 16)
                : nullptr;
#endif
  const bool append = k_new != nullptr;
  const long items8 = ((long)c.batch * c.num_heads + 7) / 8 * 8;
  const unsigned groups = (unsigned)(items8 * p.members);
  const int mp = c.max_pages_per_seq;
#define QUEST_STEP_CASE(I) \
  if (mp <= kStepThreads * (I)) return launch_items<I>(a, p.iters, append, groups, s)
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
