// Exchange of results between the work-groups of one launch ("a team": the
// splits of one head) without a second kernel.
//
// MI355X has eight accelerator dies (XCCs), each with its own L2, and the L2s
// are not kept coherent with each other inside a launch.  What one member hands
// to another is therefore written with device-scope stores (written through to
// the point all dies share) and read with device-scope loads (which do not hit
// a die's private copy).  The hand-over itself is a counter:
//
//   writer:  device-scope stores of its result
//            wait until they have completed (s_waitcnt vmcnt(0)), work-group barrier
//            one device-scope atomic add on the team's counter
//   reader:  the member whose add returned n - 1 is the last to arrive; every other
//            member's stores completed before its add did, so device-scope loads
//            now return them
//
// No cache write-back or invalidate is needed because no shared datum ever sits
// in a die-private cache line.  With QUEST_FLAG_DEVICE_FENCES the members
// additionally issue device-scope release / acquire fences around the counter
// (the textbook form; slower, same results), which keeps that path tested.
//
// One 32-bit counter per team, in a 256-byte slot of its own, zero between
// launches: the last member re-arms it.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace quest {

constexpr int kTeamWordStride = 32;  // uint64 words between two team counters (256 B)
constexpr int kMaxTeamSize = 8191;

#if defined(__HIPCC__)

__device__ __forceinline__ void dev_st(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void dev_st(uint32_t* p, uint32_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float dev_ld(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// two adjacent floats at an 8-byte aligned address, as one access
__device__ __forceinline__ float2 dev_ld2(const float* p) {
  const uint64_t bits =
      __hip_atomic_load(reinterpret_cast<const uint64_t*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return make_float2(__builtin_bit_cast(float, (uint32_t)bits), __builtin_bit_cast(float, (uint32_t)(bits >> 32)));
}

// Wait until this wave's global stores have completed.
__device__ __forceinline__ void wait_stores() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// To be called by ONE thread after every wave of the work-group that stored a part of
// the result has waited for its stores and the work-group has passed a barrier.
// Returns how many members had arrived before: n - 1 means this member is the last.
__device__ __forceinline__ uint32_t team_arrive(uint32_t* counter, bool fences) {
  if (fences) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
  return __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// For the last member, by every thread that is going to read the others' results.
__device__ __forceinline__ void team_acquire(bool fences) {
  if (fences) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
}

// The last member re-arms the counter for the next launch.
__device__ __forceinline__ void team_reset(uint32_t* counter) { dev_st(counter, 0u); }

#endif  // __HIPCC__

}  // namespace quest
