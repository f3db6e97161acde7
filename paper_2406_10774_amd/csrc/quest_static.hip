// quest_decode_step for callers that cannot bring a workspace (code under HIP graph
// capture in a harness that forbids allocations, tight serving loops): the same
// launches as quest_decode_step, with the decode workspace (arrival counters and
// split-K partial results, for very long rows also the candidates of the two-stage
// selection) in a static device array of this library instead of caller memory.
#include "quest_common.h"

#include <mutex>

namespace quest {

namespace {

// Every GPU the library runs on holds its own copy of this array until the process
// ends.  Counters and split-K partial results never need more than about 0.8 MiB (the
// launch keeps batch * heads * splits within ~1000 work-groups); the rest is for the
// candidates of the two-stage selection of rows from 16384 pages on (batch * KV heads *
// chunks * k_pages * 8 bytes: 0.6 MiB for one sequence of 32 heads at 512k tokens with a
// budget of 4096 tokens).
constexpr size_t kScratchBytes = 4u << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_lock;
void* g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on each device

// `scratch` names the array in device code only; host code must ask the runtime for its
// address, once per device, with that device current.
int scratch_pointer(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    set_error("quest_decode_step_static: no usable current device (%s, device %d)",
              hipGetErrorString(e), dev);
    return QUEST_ERR_HIP;
  }
  std::lock_guard<std::mutex> guard(g_lock);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || p == nullptr) {
      set_error("quest_decode_step_static: hipGetSymbolAddress failed on device %d: %s", dev,
                hipGetErrorString(e));
      return QUEST_ERR_HIP;
    }
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return QUEST_OK;
}

// The arrival counters must be zero when a launch starts.  Every launch leaves them so,
// but the array is shared by all calls on the device and a call that was aborted (or a
// different cache shape before it) must not be able to poison the next: clear them with a
// kernel (a memset node in a captured graph is not reliable on every runtime).
__global__ void clear_words_kernel(uint32_t* p, size_t n) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
}

}  // namespace

int launch_decode_step_static(const quest_cache& c, const void* k_new, const void* v_new,
                              int k_pool_write, const void* q, int k_pages, float sm_scale,
                              float* scores, int32_t* topk_idx, int32_t* k_eff, void* out,
                              int out_is_fp16, float* lse, hipStream_t s) {
  const size_t need = step_workspace_bytes(c, k_pages);
  if (need > kScratchBytes) {
    set_error("quest_decode_step_static: this shape needs %zu bytes of scratch, the static buffer "
              "holds %zu; use quest_decode_step with a workspace", need, kScratchBytes);
    return QUEST_ERR_WORKSPACE;
  }
  void* ws = nullptr;
  int r = scratch_pointer(&ws);
  if (r != QUEST_OK) return r;
  // counters exist when the attention runs in several splits; they are then the first
  // bytes of its workspace (<= need <= kScratchBytes)
  const size_t words = decode_workspace_bytes(c, k_pages) ? decode_counter_bytes(c) / sizeof(uint32_t) : 0;
  if (need > 0 && words > 0) {
    hipLaunchKernelGGL(clear_words_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, s,
                       (uint32_t*)ws, words);
    r = check_launch("quest_decode_step_static");
    if (r != QUEST_OK) return r;
  }
  return launch_decode_step(c, k_new, v_new, k_pool_write, q, k_pages, sm_scale, scores, topk_idx,
                            k_eff, out, out_is_fp16, lse, ws, need, s);
}

}  // namespace quest
