// Device-side pieces of the paged decode attention (Figure 5 stage 2 of arXiv
// 2406.10774): streaming one (page, head) block of keys and values through a
// wave with an online softmax.  Shared by the stand-alone kernel and the
// single-launch decode step.  See quest_decode.hip for the scheme.
#pragma once

#include "quest_common.h"

namespace quest {

#if defined(__HIPCC__)

constexpr float kNegBig = -1.0e30f;  // "no token yet": finite, so exp2(m - m) never sees inf - inf
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

struct PageRegs {
  uint4 k[4], v[4];
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

__device__ __forceinline__ void load_page(PageRegs& r, const char* __restrict__ k_pool,
                                          const char* __restrict__ v_pool, int num_heads, int h,
                                          int seq_len, int logical_page, int phys, int lane) {
  const size_t off = ((size_t)phys * num_heads + h) * kBlockBytes + lane * 16;
#pragma unroll
  for (int i = 0; i < 4; ++i) r.k[i] = ld16(k_pool + off + i * 1024);
#pragma unroll
  for (int i = 0; i < 4; ++i) r.v[i] = ld16(v_pool + off + i * 1024);
  r.n_valid = min(kPageSize, seq_len - logical_page * kPageSize);
}

__device__ __forceinline__ void fold_page(Softmax& st, PageRegs& r, const uint4 qv, float scale_log2,
                                          int grp) {
  float z[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) z[i] = row16_sum(dot8(qv, r.k[i], 0.f)) * scale_log2;
  if (r.n_valid < kPageSize) {  // partial last page: stale slots contribute nothing
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (grp + 4 * i >= r.n_valid) {
        z[i] = -INFINITY;
        r.v[i] = make_uint4(0, 0, 0, 0);
      }
    }
  }
  const float m_new = fmaxf(fmaxf(st.m, fmaxf(z[0], z[1])), fmaxf(z[2], z[3]));
  const float alpha = __builtin_amdgcn_exp2f(st.m - m_new);
  float p[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) p[i] = __builtin_amdgcn_exp2f(z[i] - m_new);
  st.l = st.l * alpha + ((p[0] + p[1]) + (p[2] + p[3]));
#pragma unroll
  for (int j = 0; j < 8; ++j) st.acc[j] *= alpha;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
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

// merge the state held by lane ^ mask into this lane's
__device__ __forceinline__ void merge_lanes(Softmax& st, int mask) {
  const float m_o = __shfl_xor(st.m, mask);
  const float l_o = __shfl_xor(st.l, mask);
  const float m_n = fmaxf(st.m, m_o);
  const float a = __builtin_amdgcn_exp2f(st.m - m_n);
  const float b = __builtin_amdgcn_exp2f(m_o - m_n);
  st.l = st.l * a + l_o * b;
#pragma unroll
  for (int j = 0; j < 8; ++j) st.acc[j] = st.acc[j] * a + __shfl_xor(st.acc[j], mask) * b;
  st.m = m_n;
}

__device__ __forceinline__ void store_out(void* out, int out_is_fp16, size_t idx, float v) {
  if (out_is_fp16)
    reinterpret_cast<_Float16*>(out)[idx] = (_Float16)v;
  else
    reinterpret_cast<float*>(out)[idx] = v;
}

#endif  // __HIPCC__

}  // namespace quest
