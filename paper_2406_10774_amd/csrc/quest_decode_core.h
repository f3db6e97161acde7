// Device-side pieces of the paged decode attention (Figure 5 stage 2 of arXiv
// 2406.10774): streaming one (page, head) block of keys and values through a
// wave with an online softmax.  See quest_decode.hip for the scheme.
#pragma once

#include "quest_common.h"

namespace quest {

#if defined(__HIPCC__)

constexpr float kNegBig = -1.0e30f;  // "no token yet": finite, so exp2(m - m) never sees inf - inf
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Registers of one unit of streaming: up to 16 consecutive tokens of one (page,
// head): kLoads = 4 wave-wide 16-byte loads of keys and 4 of values (2 and 2 for
// pages of 8 tokens).  Pages of 32 or 64 tokens are walked as 2 or 4 such units.
template <int kLoads>  // 2 or 4
struct PageRegsT {
  uint4 k[kLoads], v[kLoads];
  int n_valid;
};

__device__ __forceinline__ float lo(uint32_t h2) {
  return (float)__builtin_bit_cast(half2_t, h2)[0];
}
__device__ __forceinline__ float hi(uint32_t h2) {
  return (float)__builtin_bit_cast(half2_t, h2)[1];
}

struct Softmax {
  float m, l, acc[8];
};

// Unit `unit` (tokens [unit * 4 kLoads, (unit + 1) * 4 kLoads)) of logical page
// `logical_page`, stored in physical page `phys`; pages hold 1 << page_shift tokens.
template <int kLoads>
__device__ __forceinline__ void load_unit(PageRegsT<kLoads>& r, const char* __restrict__ k_pool,
                                          const char* __restrict__ v_pool, int num_heads, int h,
                                          int seq_len, int logical_page, int phys, int unit,
                                          int page_shift, int lane) {
  const size_t row = (((size_t)phys * num_heads + h) << page_shift) + (size_t)unit * (4 * kLoads);
  const size_t off = row * kRowBytes + lane * 16;
#pragma unroll
  for (int i = 0; i < kLoads; ++i) r.k[i] = ld16_stream(k_pool + off + i * 1024);
#pragma unroll
  for (int i = 0; i < kLoads; ++i) r.v[i] = ld16_stream(v_pool + off + i * 1024);
  r.n_valid = min(4 * kLoads, seq_len - (logical_page << page_shift) - unit * (4 * kLoads));
}

// n_valid may be anything up to 4 kLoads, also <= 0 (a unit past the end of a
// partial page): such tokens contribute nothing.
template <int kLoads>
__device__ __forceinline__ void fold_page(Softmax& st, PageRegsT<kLoads>& r, const uint4 qv,
                                          float scale_log2, int grp) {
  float z[kLoads];
#pragma unroll
  for (int i = 0; i < kLoads; ++i) z[i] = row16_sum(dot8(qv, r.k[i], 0.f)) * scale_log2;
  if (r.n_valid < 4 * kLoads) {  // partial last page: stale slots contribute nothing
#pragma unroll
    for (int i = 0; i < kLoads; ++i) {
      if (grp + 4 * i >= r.n_valid) {
        z[i] = -INFINITY;
        r.v[i] = make_uint4(0, 0, 0, 0);
      }
    }
  }
  float m_new = st.m;
#pragma unroll
  for (int i = 0; i < kLoads; ++i) m_new = fmaxf(m_new, z[i]);
  const float alpha = __builtin_amdgcn_exp2f(st.m - m_new);
  float p[kLoads];
#pragma unroll
  for (int i = 0; i < kLoads; ++i) p[i] = __builtin_amdgcn_exp2f(z[i] - m_new);
  float p_sum = p[0] + p[1];
  if (kLoads == 4) p_sum += p[kLoads - 2] + p[kLoads - 1];
  st.l = st.l * alpha + p_sum;
#pragma unroll
  for (int j = 0; j < 8; ++j) st.acc[j] *= alpha;
#pragma unroll
  for (int i = 0; i < kLoads; ++i) {
    st.acc[0] += p[i] * lo(r.v[i].x);
    st.acc[1] += p[i] * hi(r.v[i].x);
    st.acc[2] += p[i] * lo(r.v[i].y);
    st.acc[3] += p[i] * hi(r.v[i].y);
    st.acc[4] += p[i] * lo(r.v[i].z);
    st.acc[5] += p[i] * hi(r.v[i].z);
    st.acc[6] += p[i] * lo(r.v[i].w);
    st.acc[7] += p[i] * hi(r.v[i].w);
  }
  st.m = m_new;
}

// The same unit against kG query heads that share the KV head (grouped-query
// attention): keys and values are loaded once, the values converted to fp32
// once, and every head keeps its own online-softmax state.
template <int kLoads, int kG>
__device__ __forceinline__ void fold_group(Softmax (&st)[kG], PageRegsT<kLoads>& r,
                                           const uint4 (&qv)[kG], float scale_log2, int grp) {
  bool live[kLoads];
  float vf[kLoads][8];
#pragma unroll
  for (int i = 0; i < kLoads; ++i) {
    live[i] = grp + 4 * i < r.n_valid;  // stale slots of a partial page contribute nothing
    const uint4 v = live[i] ? r.v[i] : make_uint4(0, 0, 0, 0);
    vf[i][0] = lo(v.x), vf[i][1] = hi(v.x), vf[i][2] = lo(v.y), vf[i][3] = hi(v.y);
    vf[i][4] = lo(v.z), vf[i][5] = hi(v.z), vf[i][6] = lo(v.w), vf[i][7] = hi(v.w);
  }
#pragma unroll
  for (int g = 0; g < kG; ++g) {
    float z[kLoads];
    float m_new = st[g].m;
#pragma unroll
    for (int i = 0; i < kLoads; ++i) {
      z[i] = live[i] ? row16_sum(dot8(qv[g], r.k[i], 0.f)) * scale_log2 : -INFINITY;
      m_new = fmaxf(m_new, z[i]);
    }
    const float alpha = __builtin_amdgcn_exp2f(st[g].m - m_new);
    float p[kLoads];
#pragma unroll
    for (int i = 0; i < kLoads; ++i) p[i] = __builtin_amdgcn_exp2f(z[i] - m_new);
    float p_sum = p[0] + p[1];
    if (kLoads == 4) p_sum += p[kLoads - 2] + p[kLoads - 1];
    st[g].l = st[g].l * alpha + p_sum;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float acc = st[g].acc[j] * alpha;
#pragma unroll
      for (int i = 0; i < kLoads; ++i) acc += p[i] * vf[i][j];
      st[g].acc[j] = acc;
    }
    st[g].m = m_new;
  }
}

// Merge the online-softmax states of the wave's four DPP rows (lanes 16 apart, then lanes
// 32 apart); every lane ends up with the merged state of its channels.
__device__ __forceinline__ float as_f(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t as_u(float f) { return __builtin_bit_cast(uint32_t, f); }
template <bool kAcross32>
__device__ __forceinline__ void merge_rows_step(Softmax& st) {
  auto pair = [](float v) { return kAcross32 ? pair_across32(as_u(v)) : pair_across16(as_u(v)); };
  const LanePair m = pair(st.m), l = pair(st.l);
  const float m_n = fmaxf(as_f(m.first), as_f(m.second));
  const float a = __builtin_amdgcn_exp2f(as_f(m.first) - m_n);
  const float b = __builtin_amdgcn_exp2f(as_f(m.second) - m_n);
  st.l = as_f(l.first) * a + as_f(l.second) * b;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const LanePair p = pair(st.acc[j]);
    st.acc[j] = as_f(p.first) * a + as_f(p.second) * b;
  }
  st.m = m_n;
}
__device__ __forceinline__ void merge_rows(Softmax& st) {
  merge_rows_step<false>(st);
  merge_rows_step<true>(st);
}

__device__ __forceinline__ void store_out(void* out, int out_is_fp16, size_t idx, float v) {
  if (out_is_fp16)
    reinterpret_cast<_Float16*>(out)[idx] = (_Float16)v;
  else
    reinterpret_cast<float*>(out)[idx] = v;
}

#endif  // __HIPCC__

}  // namespace quest
