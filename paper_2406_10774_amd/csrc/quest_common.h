// Shared device helpers and host-side launch plumbing for the Quest kernels.
// gfx950 only: 64-lane wavefronts, DPP row operations, packed 16-bit integer
// min/max, v_dot2_f32_f16.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/quest.h"

namespace quest {

constexpr int kHeadDim = 128;   // D: channels per head
constexpr int kWave = 64;
constexpr int kRowBytes = kHeadDim * 2;  // one token's key (or value) of one head

// Supported page sizes: 8, 16, 32, 64 tokens (the sweep of Figure 8 of arXiv
// 2406.10774 covers these); kernels take log2(S).  Returns -1 for others.
inline int page_shift_of(int page_size) {
  return page_size == 8 ? 3 : page_size == 16 ? 4 : page_size == 32 ? 5 : page_size == 64 ? 6 : -1;
}
// One (page, head) block of keys (or of values) is S*D fp16 (4 KiB at S = 16 = 4
// wave-wide 16-byte loads); one metadata entry (min row + max row) is kMetaBytes.  The metadata
// table is head-major, [H][num_phys_pages]: the estimate scans every page of a
// head, and consecutive physical pages of one head are then contiguous (with
// page-major entries the same scan touches 512 B every 16 KiB, measured 25 %
// slower on MI355X).
constexpr int kMetaBytes = 2 * kHeadDim * 2;

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef short short2_t __attribute__((ext_vector_type(2)));

// KV heads and query heads per KV head of a cache (grouped-query attention).
inline int kv_heads(const quest_cache& c) { return c.num_kv_heads > 0 ? c.num_kv_heads : c.num_heads; }
inline int group_size(const quest_cache& c) { return c.num_heads / kv_heads(c); }

// ---------------------------------------------------------------- host side
void set_error(const char* fmt, ...);
int check_cache(const quest_cache* c, const char* who);
int check_launch(const char* who);

// Launchers (one per kernel family); each validates nothing, quest_api.hip does.
int launch_build_meta(const quest_cache& c, hipStream_t s);
int launch_append_meta(const quest_cache& c, const void* k_new, const void* v_new,
                       int k_pool_write, hipStream_t s);
int launch_estimate(const quest_cache& c, const void* q, float* scores, hipStream_t s);
int launch_append_estimate(const quest_cache& c, const void* k_new, const void* v_new,
                           int k_pool_write, const void* q, float* scores, hipStream_t s);
int launch_topk(const quest_cache& c, const float* scores, int k_pages, int32_t* topk_idx,
                int32_t* k_eff, hipStream_t s);
// Scratch for the two-stage selection of very long rows (0: not used for this shape), and
// the selection itself; the scratch need not be initialised.
size_t topk_scratch_bytes(const quest_cache& c, int k_pages);
int launch_topk_chunked(const quest_cache& c, const float* scores, int k_pages, int32_t* topk_idx,
                        int32_t* k_eff, void* scratch, hipStream_t s);
int decode_num_splits(const quest_cache& c, int k_pages);
size_t decode_workspace_bytes(const quest_cache& c, int k_pages);
int launch_sparse_decode(const quest_cache& c, const void* q, const int32_t* topk_idx, int k_pages,
                         float sm_scale, void* out, int out_is_fp16, float* lse, void* workspace,
                         hipStream_t s);

bool select_decode_supported(const quest_cache& c, int k_pages);
int launch_select_decode(const quest_cache& c, const void* q, const float* scores, int k_pages,
                         float sm_scale, int32_t* topk_idx, int32_t* k_eff, void* out,
                         int out_is_fp16, float* lse, void* workspace, hipStream_t s);

size_t step_workspace_bytes(const quest_cache& c, int k_pages);
// Leading part of a decode workspace: the arrival counters (must be zero before a launch).
size_t decode_counter_bytes(const quest_cache& c);
int launch_decode_step(const quest_cache& c, const void* k_new, const void* v_new, int k_pool_write,
                       const void* q, int k_pages, float sm_scale, float* scores, int32_t* topk_idx,
                       int32_t* k_eff, void* out, int out_is_fp16, float* lse, void* workspace,
                       size_t workspace_bytes, hipStream_t s);
int launch_decode_step_static(const quest_cache& c, const void* k_new, const void* v_new,
                              int k_pool_write, const void* q, int k_pages, float sm_scale,
                              float* scores, int32_t* topk_idx, int32_t* k_eff, void* out,
                              int out_is_fp16, float* lse, hipStream_t s);

// -------------------------------------------------------------- device side
#if defined(__HIPCC__)

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

// 16-byte global load / store (global_load_dwordx4).
__device__ __forceinline__ uint4 ld16(const void* p) { return *reinterpret_cast<const uint4*>(p); }
__device__ __forceinline__ void st16(void* p, uint4 v) { *reinterpret_cast<uint4*>(p) = v; }
// The same load marked non-temporal, for data a launch touches once (metadata entries,
// K/V pages): measured on MI355X, 32 MiB scanned in 6.1 us against 6.5 us, the dense
// attention over 512 MiB in 88 us against 100 us.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 ld16_stream(const void* p) {
  const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

// x + (x rotated right by N lanes inside its 16-lane DPP row).
template <int N>
__device__ __forceinline__ float row_ror_add(float x) {
  int v = __builtin_bit_cast(int, x);
  v = __builtin_amdgcn_update_dpp(0, v, 0x120 + N, 0xf, 0xf, false);
  return x + __builtin_bit_cast(float, v);
}

// Sum over the 16 lanes of a DPP row; every lane of the row gets the same bits
// (rotations by 8, 4, 2, 1: each step adds two already-identical partial sums
// in commuted order, so the result does not depend on the lane).
__device__ __forceinline__ float row16_sum(float x) {
  x = row_ror_add<8>(x);
  x = row_ror_add<4>(x);
  x = row_ror_add<2>(x);
  x = row_ror_add<1>(x);
  return x;
}

// fp16 pair dot product accumulated in fp32 (v_dot2_f32_f16).
__device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float acc) {
  return __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, a), __builtin_bit_cast(half2_t, b), acc,
                                false);
}

// 8-channel fp16 dot product of two 16-byte vectors, fp32 accumulate.
__device__ __forceinline__ float dot8(uint4 a, uint4 b, float acc) {
  acc = dot2(a.x, b.x, acc);
  acc = dot2(a.y, b.y, acc);
  acc = dot2(a.z, b.z, acc);
  acc = dot2(a.w, b.w, acc);
  return acc;
}

// fp16 bit pattern <-> signed 16-bit key whose integer order is "by value,
// -0 below +0": non-negative halves map to themselves, negative ones get their
// magnitude bits flipped.  The map is its own inverse.  Two halves per dword.
__device__ __forceinline__ uint32_t order_key2(uint32_t h2) {
  short2_t v = __builtin_bit_cast(short2_t, h2);
  v = v ^ ((v >> 15) & (short)0x7fff);
  return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ uint32_t key_min2(uint32_t a, uint32_t b) {
  return __builtin_bit_cast(
      uint32_t, __builtin_elementwise_min(__builtin_bit_cast(short2_t, a), __builtin_bit_cast(short2_t, b)));
}
__device__ __forceinline__ uint32_t key_max2(uint32_t a, uint32_t b) {
  return __builtin_bit_cast(
      uint32_t, __builtin_elementwise_max(__builtin_bit_cast(short2_t, a), __builtin_bit_cast(short2_t, b)));
}
__device__ __forceinline__ uint4 order_key8(uint4 v) {
  return make_uint4(order_key2(v.x), order_key2(v.y), order_key2(v.z), order_key2(v.w));
}
__device__ __forceinline__ uint4 key_min8(uint4 a, uint4 b) {
  return make_uint4(key_min2(a.x, b.x), key_min2(a.y, b.y), key_min2(a.z, b.z), key_min2(a.w, b.w));
}
__device__ __forceinline__ uint4 key_max8(uint4 a, uint4 b) {
  return make_uint4(key_max2(a.x, b.x), key_max2(a.y, b.y), key_max2(a.z, b.z), key_max2(a.w, b.w));
}

// The value of the lane 16 (32) lanes away next to this lane's own, without going through
// LDS: v_permlane16_swap / v_permlane32_swap exchange the odd rows (the upper half) of
// one register with the even rows (the lower half) of another.  With both registers
// holding v, the pair (first, second) is (v of the even row / lower half, v of the odd row
// / upper half) in every lane of the two: a commutative op(first, second) is the
// reduction over the pair, the same bits in both lanes.
struct LanePair {
  uint32_t first, second;
};
__device__ __forceinline__ LanePair pair_across16(uint32_t v) {
  const auto r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
  return {r[0], r[1]};
}
__device__ __forceinline__ LanePair pair_across32(uint32_t v) {
  const auto r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
  return {r[0], r[1]};
}
// min / max over the four DPP rows of packed 16-bit order keys; every lane gets the result
__device__ __forceinline__ uint32_t rows_key_min2(uint32_t v) {
  LanePair p = pair_across16(v);
  p = pair_across32(key_min2(p.first, p.second));
  return key_min2(p.first, p.second);
}
__device__ __forceinline__ uint32_t rows_key_max2(uint32_t v) {
  LanePair p = pair_across16(v);
  p = pair_across32(key_max2(p.first, p.second));
  return key_max2(p.first, p.second);
}
__device__ __forceinline__ uint4 rows_key_min8(uint4 v) {
  return make_uint4(rows_key_min2(v.x), rows_key_min2(v.y), rows_key_min2(v.z), rows_key_min2(v.w));
}
__device__ __forceinline__ uint4 rows_key_max8(uint4 v) {
  return make_uint4(rows_key_max2(v.x), rows_key_max2(v.y), rows_key_max2(v.z), rows_key_max2(v.w));
}

__device__ __forceinline__ int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Byte offset of the metadata entry of (physical page, head).
__device__ __forceinline__ size_t meta_offset(int64_t num_phys_pages, int phys, int h) {
  return ((size_t)h * (size_t)num_phys_pages + (size_t)phys) * kMetaBytes;
}

#endif  // __HIPCC__

}  // namespace quest
