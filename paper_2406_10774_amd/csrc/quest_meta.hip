// Per-page channel-wise min/max key metadata: bulk build after prefill and the
// per-token update (Section 3.4 and the insertion half of Algorithm 1 of
// arXiv 2406.10774).
//
// Both kernels compare fp16 values through a signed 16-bit key whose integer
// order is "by value, -0 below +0" (order_key2), with packed 16-bit min/max.
// Integer min/max are associative and commutative, so any reduction tree gives
// the same bits as a sequential scan.
#include "quest_common.h"

namespace quest {

namespace {

constexpr int kBuildWaves = 4;          // waves per work-group
constexpr int kBuildLoads = 16;         // wave-wide 16-byte loads a wave issues up front (16 KiB)

constexpr uint32_t kKeyMax2 = 0x7fff7fffu;  // identity of min
constexpr uint32_t kKeyMin2 = 0x80008000u;  // identity of max

// One wave reduces kBuildLoads / (kS / 4) key blocks of kS tokens each (4 blocks of
// 4 KiB at the paper's page size of 16).  Lane l holds channels 8*(l%16)..+7 of
// tokens l/16 + 4r (r = 0..kS/4-1): load r of a block is its contiguous 1 KiB
// [r*1024, r*1024+1024), 16 bytes per lane.  The (page, head) blocks are walked in
// memory order: the pools are page-major, so consecutive heads of one page are
// contiguous, a wave's loads cover one run of 16 KiB and work-groups follow each other
// through the pool (59 us against 61 us with a work-group per (head, 16 pages), one
// sequence of 32 heads at 32k tokens).
template <int kS>
__global__ __launch_bounds__(kBuildWaves* kWave) void build_meta_kernel(
    const char* __restrict__ k_pool, char* __restrict__ meta, const int32_t* __restrict__ page_table,
    const int32_t* __restrict__ seq_lens, int num_heads, int max_pages, int64_t num_phys_pages) {
  constexpr int kLoads = kS / 4;                        // per block
  constexpr int kUnitsPerWave = kBuildLoads / kLoads;   // (page, head) blocks per wave: 8, 4, 2, 1
  const int b = blockIdx.y;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = lane_id();
  const int grp = lane >> 4;
  const int seq_len = seq_lens[b];
  const int num_pages = (seq_len + kS - 1) / kS;
  const long units = (long)num_pages * num_heads;       // unit = page * H + head
  const long u0 = ((long)blockIdx.x * kBuildWaves + wave) * kUnitsPerWave;
  if (u0 >= units) return;

  uint4 buf[kUnitsPerWave][kLoads];
  int phys[kUnitsPerWave], page[kUnitsPerWave], head[kUnitsPerWave];
#pragma unroll
  for (int u = 0; u < kUnitsPerWave; ++u) {
    const long unit = u0 + u < units ? u0 + u : u0;     // past the end: re-read the first, skipped below
    page[u] = (int)(unit / num_heads);
    head[u] = (int)(unit - (long)page[u] * num_heads);
    phys[u] = page_table[(size_t)b * max_pages + page[u]];
  }
#pragma unroll
  for (int u = 0; u < kUnitsPerWave; ++u) {
    const char* blk = k_pool + ((size_t)phys[u] * num_heads + head[u]) * (kS * kRowBytes);
#pragma unroll
    for (int r = 0; r < kLoads; ++r) buf[u][r] = ld16_stream(blk + r * 1024 + lane * 16);
  }
#pragma unroll
  for (int u = 0; u < kUnitsPerWave; ++u) {
    if (u0 + u >= units) break;
    const int n_valid = min(kS, seq_len - page[u] * kS);
    uint4 mn = make_uint4(kKeyMax2, kKeyMax2, kKeyMax2, kKeyMax2);
    uint4 mx = make_uint4(kKeyMin2, kKeyMin2, kKeyMin2, kKeyMin2);
#pragma unroll
    for (int r = 0; r < kLoads; ++r) {
      if (grp + 4 * r < n_valid) {  // stale slots of a partial page never take part
        const uint4 key = order_key8(buf[u][r]);
        mn = key_min8(mn, key);
        mx = key_max8(mx, key);
      }
    }
    mn = rows_key_min8(mn);
    mx = rows_key_max8(mx);
    char* entry = meta + meta_offset(num_phys_pages, phys[u], head[u]);
    if (lane < 32) st16(entry + lane * 16, order_key8(grp == 0 ? mn : mx));
  }
}

// 16 lanes per (sequence, head): lane c owns channels 8c..8c+7 of the new token.
__global__ __launch_bounds__(256) void append_meta_kernel(
    char* __restrict__ k_pool, char* __restrict__ v_pool, char* __restrict__ meta,
    const int32_t* __restrict__ page_table, const int32_t* __restrict__ seq_lens,
    const char* __restrict__ k_new, const char* __restrict__ v_new, int batch, int num_heads,
    int max_pages, int k_pool_write, int64_t num_phys_pages, int page_shift) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  const int bh = t >> 4;
  const int c = t & 15;
  if (bh >= batch * num_heads) return;
  const int b = bh / num_heads;
  const int h = bh - b * num_heads;
  const int pos = seq_lens[b] - 1;
  const int page = pos >> page_shift;
  const int slot = pos - (page << page_shift);
  const int phys = page_table[(size_t)b * max_pages + page];
  const size_t ph = (size_t)phys * num_heads + h;

  const uint4 k = ld16(k_new + (size_t)bh * (kHeadDim * 2) + c * 16);
  if (k_pool_write) {
    const size_t off = ((ph << page_shift) + slot) * kRowBytes + c * 16;
    st16(k_pool + off, k);
    st16(v_pool + off, ld16(v_new + (size_t)bh * (kHeadDim * 2) + c * 16));
  }
  char* entry = meta + meta_offset(num_phys_pages, phys, h) + c * 16;
  if (slot == 0) {  // first token of a page: min = max = k
    st16(entry, k);
    st16(entry + kHeadDim * 2, k);
  } else {
    const uint4 key = order_key8(k);
    const uint4 mn = key_min8(order_key8(ld16(entry)), key);
    const uint4 mx = key_max8(order_key8(ld16(entry + kHeadDim * 2)), key);
    st16(entry, order_key8(mn));
    st16(entry + kHeadDim * 2, order_key8(mx));
  }
}

}  // namespace

template <int kS>
int launch_build_meta_for(const quest_cache& c, hipStream_t s) {
  constexpr int kUnitsPerGroup = kBuildWaves * (kBuildLoads / (kS / 4));
  const long units = (long)c.max_pages_per_seq * kv_heads(c);
  dim3 grid((unsigned)((units + kUnitsPerGroup - 1) / kUnitsPerGroup), c.batch);
  hipLaunchKernelGGL(build_meta_kernel<kS>, grid, dim3(kBuildWaves * kWave), 0, s,
                     (const char*)c.k_pool, (char*)c.meta, c.page_table, c.seq_lens, kv_heads(c),
                     c.max_pages_per_seq, c.num_phys_pages);
  return check_launch("quest_build_meta");
}

int launch_build_meta(const quest_cache& c, hipStream_t s) {
  switch (c.page_size) {
    case 8: return launch_build_meta_for<8>(c, s);
    case 32: return launch_build_meta_for<32>(c, s);
    case 64: return launch_build_meta_for<64>(c, s);
    default: return launch_build_meta_for<16>(c, s);
  }
}

int launch_append_meta(const quest_cache& c, const void* k_new, const void* v_new, int k_pool_write,
                       hipStream_t s) {
  const int threads = c.batch * kv_heads(c) * 16;
  hipLaunchKernelGGL(append_meta_kernel, dim3((threads + 255) / 256), dim3(256), 0, s,
                     (char*)c.k_pool, (char*)c.v_pool, (char*)c.meta, c.page_table, c.seq_lens,
                     (const char*)k_new, (const char*)v_new, c.batch, kv_heads(c),
                     c.max_pages_per_seq, k_pool_write, c.num_phys_pages,
                     page_shift_of(c.page_size));
  return check_launch("quest_append_meta");
}

}  // namespace quest
