// Top-K page selection (Section 3.4 of arXiv 2406.10774: "choose the top K
// pages as critical").  One work-group per (sequence, head).
//
// Scores are mapped to unsigned 32-bit keys whose integer order equals the
// order of the float values (-0 folded onto +0).  An MSB-first radix select
// (four 8-bit digits, LDS histogram per digit) finds the key T of the K-th
// largest score and how many keys equal to T still fit.  A final pass in page
// order emits every page with key > T plus the first `need` pages with
// key == T, each at the position given by a block-wide prefix count, so the
// output is ascending and the lowest page index wins among equal scores.
#include "quest_common.h"

namespace quest {

namespace {

__device__ __forceinline__ uint32_t score_key(float s) {
  uint32_t u = __builtin_bit_cast(uint32_t, s);
  if (u == 0x80000000u) u = 0;  // -0 ranks equal to +0
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ int wave_incl_scan(int v, int lane) {
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    const int o = __shfl_up(v, d);
    if (lane >= d) v += o;
  }
  return v;
}

// LDS: hist[256] | wave_gt[16] | wave_eq[16] | bcast[2] | keys[max_pages] (kLdsKeys only)
constexpr int kTopkLdsHeaderWords = 256 + 16 + 16 + 2 + 6;  // padded to 296 words

template <int kThreads, bool kLdsKeys>
__global__ __launch_bounds__(kThreads) void topk_kernel(
    const float* __restrict__ scores, const int32_t* __restrict__ seq_lens,
    int32_t* __restrict__ topk_idx, int32_t* __restrict__ k_eff, int num_heads, int max_pages,
    int k_pages) {
  extern __shared__ uint32_t smem[];
  uint32_t* hist = smem;
  int* wave_gt = reinterpret_cast<int*>(smem + 256);
  int* wave_eq = reinterpret_cast<int*>(smem + 272);
  int* bcast = reinterpret_cast<int*>(smem + 288);
  uint32_t* keys = smem + kTopkLdsHeaderWords;

  const int h = blockIdx.x;
  const int b = blockIdx.y;
  const int tid = threadIdx.x;
  const int lane = lane_id();
  const int wave = tid >> 6;
  constexpr int kWaves = kThreads / kWave;

  const int num_pages = (seq_lens[b] + kPageSize - 1) / kPageSize;
  const int K = min(k_pages, num_pages);
  const float* row = scores + ((size_t)b * num_heads + h) * max_pages;
  int32_t* out = topk_idx + ((size_t)b * num_heads + h) * k_pages;
  if (h == 0 && tid == 0 && k_eff != nullptr) k_eff[b] = K;

  if (K == num_pages) {  // everything is selected: identity list, padded with -1
    for (int i = tid; i < k_pages; i += kThreads) out[i] = i < K ? i : -1;
    return;
  }

  auto key_at = [&](int i) -> uint32_t { return kLdsKeys ? keys[i] : score_key(row[i]); };

  if (kLdsKeys)
    for (int i = tid; i < num_pages; i += kThreads) keys[i] = score_key(row[i]);
  if (tid < 256) hist[tid] = 0;
  __syncthreads();

  // ---- radix select: after the loop `prefix` is the K-th largest key and
  // `need` (>= 1) the number of keys equal to it that belong to the selection
  uint32_t prefix = 0;
  int need = K;
#pragma unroll
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    const uint32_t high_mask = pass == 0 ? 0u : (0xffffffffu << (shift + 8));
    for (int i = tid; i < num_pages; i += kThreads) {
      const uint32_t key = key_at(i);
      if ((key & high_mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (wave == 0) {
      // lane l owns bins 255-4l .. 252-4l (descending), scan from the top bin down
      const int top = 255 - 4 * lane;
      const int c0 = hist[top], c1 = hist[top - 1], c2 = hist[top - 2], c3 = hist[top - 3];
      hist[top] = 0;
      hist[top - 1] = 0;
      hist[top - 2] = 0;
      hist[top - 3] = 0;
      const int tot = c0 + c1 + c2 + c3;
      const int incl = wave_incl_scan(tot, lane);
      const int excl = incl - tot;
      if (excl < need && need <= incl) {
        int bin = top, above = excl;
        if (need > above + c0) {
          above += c0;
          bin = top - 1;
          if (need > above + c1) {
            above += c1;
            bin = top - 2;
            if (need > above + c2) {
              above += c2;
              bin = top - 3;
            }
          }
        }
        bcast[0] = bin;
        bcast[1] = above;
      }
    }
    __syncthreads();
    prefix |= (uint32_t)bcast[0] << shift;
    need -= bcast[1];
  }
  const uint32_t T = prefix;

  // ---- emit in page order: thread t owns the contiguous chunk [t*items, (t+1)*items)
  const int items = (num_pages + kThreads - 1) / kThreads;
  const int begin = min(tid * items, num_pages);
  const int end = min(begin + items, num_pages);
  int n_gt = 0, n_eq = 0;
  for (int i = begin; i < end; ++i) {
    const uint32_t key = key_at(i);
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
    const uint32_t key = key_at(i);
    if (key > T) {
      out[gt_before + min(eq_before, need)] = i;
      ++gt_before;
    } else if (key == T) {
      if (eq_before < need) out[gt_before + eq_before] = i;
      ++eq_before;
    }
  }
}

template <int kThreads, bool kLdsKeys>
int launch_one(const quest_cache& c, const float* scores, int k_pages, int32_t* topk_idx,
               int32_t* k_eff, size_t lds_bytes, hipStream_t s) {
  auto kern = topk_kernel<kThreads, kLdsKeys>;
  if (lds_bytes > 64 * 1024) {
    // opt in to a large dynamic LDS allocation (gfx950 has 160 KiB per CU)
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (e != hipSuccess) {
      (void)hipGetLastError();
      return 1;  // caller falls back to keys re-read from global memory
    }
  }
  hipLaunchKernelGGL(kern, dim3(c.num_heads, c.batch), dim3(kThreads), lds_bytes, s, scores,
                     c.seq_lens, topk_idx, k_eff, c.num_heads, c.max_pages_per_seq, k_pages);
  return check_launch("quest_topk");
}

}  // namespace

int launch_topk(const quest_cache& c, const float* scores, int k_pages, int32_t* topk_idx,
                int32_t* k_eff, hipStream_t s) {
  const size_t header = kTopkLdsHeaderWords * sizeof(uint32_t);
  const size_t with_keys = header + (size_t)c.max_pages_per_seq * sizeof(uint32_t);
  constexpr size_t kLdsLimit = 160 * 1024;
  if (c.max_pages_per_seq <= 4096)
    return launch_one<256, true>(c, scores, k_pages, topk_idx, k_eff, with_keys, s);
  if (with_keys <= kLdsLimit) {
    int r = launch_one<1024, true>(c, scores, k_pages, topk_idx, k_eff, with_keys, s);
    if (r <= 0) return r;
  }
  return launch_one<1024, false>(c, scores, k_pages, topk_idx, k_eff, header, s);
}

}  // namespace quest
