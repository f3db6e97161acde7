// Yardsticks for the benchmark only (their own library, not part of the Quest C ABI):
// what the machine does on the access patterns of the decode step with no arithmetic
// at all, so that a kernel's time can be read against "as fast as these bytes move here"
// next to the published peak.
//   yardstick_empty   one empty work-group: the floor of a launch in a replayed graph
//   yardstick_read    sequential 16-byte-per-lane reads of one or two ranges (the
//                     metadata scan of the estimate; K and V of the dense attention)
//   yardstick_gather  4 KiB blocks of two pools fetched through a list of block ids (the
//                     selected K/V pages of sparse attention), in the attention's launch
//                     shape: a work-group of 8 waves per 16 list entries, 2 per wave
// All pointers are device pointers; calls only enqueue on `stream`.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

template <bool kNt>
__device__ __forceinline__ u32x4_t load16(const char* p) {
  const u32x4_t* q = reinterpret_cast<const u32x4_t*>(p);
  if constexpr (kNt)
    return __builtin_nontemporal_load(q);
  else
    return *q;
}

__global__ void empty_kernel(uint32_t* sink) {
  if (sink != nullptr && threadIdx.x == 0xffff) *sink = 1u;
}

// Each wave reads kLoads consecutive KiB once; waves cover [0, bytes_a) of a, then
// [0, bytes_b) of b.  A range whose size is not a multiple of kLoads KiB loses its tail.
constexpr int kLoads = 8;
template <bool kNt>
__global__ __launch_bounds__(256) void read_kernel(const char* __restrict__ a, size_t chunks_a,
                                                   const char* __restrict__ b, size_t chunks_b,
                                                   uint32_t* __restrict__ sink) {
  const size_t wave = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int lane = threadIdx.x & 63;
  if (wave >= chunks_a + chunks_b) return;
  const char* p = wave < chunks_a ? a + wave * (kLoads * 1024) : b + (wave - chunks_a) * (kLoads * 1024);
  u32x4_t r[kLoads];
#pragma unroll
  for (int j = 0; j < kLoads; ++j) r[j] = load16<kNt>(p + j * 1024 + lane * 16);
  uint32_t acc = 0;
#pragma unroll
  for (int j = 0; j < kLoads; ++j) acc ^= r[j].x ^ r[j].y ^ r[j].z ^ r[j].w;
  if (acc == 0x12345678u && sink != nullptr) sink[0] = acc;  // keeps the loads alive
}

// Work-group g of 8 waves takes list entries [16 g, 16 g + 16): wave w entries w and w + 8,
// both requested at once: 4 KiB of k_pool and 4 KiB of v_pool at block id * 4096.
template <bool kNt>
__global__ __launch_bounds__(512) void gather_kernel(const char* __restrict__ k_pool,
                                                     const char* __restrict__ v_pool,
                                                     const int32_t* __restrict__ list, int n,
                                                     uint32_t* __restrict__ sink) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  u32x4_t r[2][8];
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    const int e = blockIdx.x * 16 + wave + 8 * p;
    const size_t off = (size_t)list[e < n ? e : n - 1] * 4096 + lane * 16;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      r[p][j] = load16<kNt>(k_pool + off + j * 1024);
      r[p][4 + j] = load16<kNt>(v_pool + off + j * 1024);
    }
  }
  uint32_t acc = 0;
#pragma unroll
  for (int p = 0; p < 2; ++p)
#pragma unroll
    for (int j = 0; j < 8; ++j) acc ^= r[p][j].x ^ r[p][j].y ^ r[p][j].z ^ r[p][j].w;
  if (acc == 0x12345678u && sink != nullptr) sink[0] = acc;
}

int launched() { return hipGetLastError() == hipSuccess ? 0 : -1; }

}  // namespace

extern "C" {

int yardstick_empty(void* stream) {
  hipLaunchKernelGGL(empty_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, (uint32_t*)nullptr);
  return launched();
}

// Reads bytes_a of a and bytes_b of b (b may be NULL with bytes_b == 0); sizes are taken
// down to multiples of 8 KiB.  sink: 4 writable bytes (never written in practice).
int yardstick_read(const void* a, size_t bytes_a, const void* b, size_t bytes_b, int nontemporal,
                   void* sink, void* stream) {
  const size_t ca = bytes_a / (kLoads * 1024), cb = b ? bytes_b / (kLoads * 1024) : 0;
  if (a == nullptr || ca + cb == 0) return -1;
  const size_t groups = (ca + cb + 3) / 4;
  if (groups > 0x7fffffffu) return -1;
  if (nontemporal)
    hipLaunchKernelGGL(read_kernel<true>, dim3((unsigned)groups), dim3(256), 0, (hipStream_t)stream,
                       (const char*)a, ca, (const char*)b, cb, (uint32_t*)sink);
  else
    hipLaunchKernelGGL(read_kernel<false>, dim3((unsigned)groups), dim3(256), 0, (hipStream_t)stream,
                       (const char*)a, ca, (const char*)b, cb, (uint32_t*)sink);
  return launched();
}

// list: n block ids (int32, device), every id * 4096 + 4096 <= the size of each pool.
int yardstick_gather(const void* k_pool, const void* v_pool, const int32_t* list, int n,
                     int nontemporal, void* sink, void* stream) {
  if (k_pool == nullptr || v_pool == nullptr || list == nullptr || n < 1) return -1;
  const unsigned groups = (unsigned)((n + 15) / 16);
  if (nontemporal)
    hipLaunchKernelGGL(gather_kernel<true>, dim3(groups), dim3(512), 0, (hipStream_t)stream,
                       (const char*)k_pool, (const char*)v_pool, list, n, (uint32_t*)sink);
  else
    hipLaunchKernelGGL(gather_kernel<false>, dim3(groups), dim3(512), 0, (hipStream_t)stream,
                       (const char*)k_pool, (const char*)v_pool, list, n, (uint32_t*)sink);
  return launched();
}

}  // extern "C"
