// Exchange of results between the work-groups of one launch ("a team": e.g. the
// splits of one head) without a second kernel and without device-wide cache
// maintenance in the common case.
//
// MI355X has eight accelerator dies (XCCs), each with its own L2.  Inside a die
// the L2 is the coherence point: a completed global store is in the L2 (the
// per-CU vector cache is write-through) and a device-scope load bypasses the
// vector cache, so two work-groups on the same die can hand data to each other
// through plain stores, a wait for the stores, an L2 atomic and device-scope
// loads.  The L2s of different dies are not kept coherent with each other
// inside a launch: that needs a write-back of the writer's L2 and an invalidate
// of the reader's (device-scope release / acquire fences), which cost many
// microseconds.
//
// Work-groups are dealt to the dies round-robin by their linear id, with a
// rotation that differs from launch to launch, so work-groups whose ids are
// equal modulo 8 run on the same die.  Teams are laid out that way, but
// nothing here *relies* on it: every member checks in with the id of the die it
// really runs on, and a member that cannot prove that the whole team shares its
// die takes the fenced path.  Correct under any placement, fast under the
// usual one.
//
// One 64-bit word per team (in its own 256-byte slot, zero between launches):
//   bits  0..13  tickets: members that have published their result
//   bits 14..27  check-ins: members that have started
//   bits 28..44  sum of the members' die ids
//   bits 45..63  sum of the squares of the members' die ids
// All members run on die x  <=>  check-ins == n, sum == n x, sum of squares ==
// n x^2 (the sum of (x_i - x)^2 is then zero).  Team size is limited to 8191.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace quest {

constexpr int kTeamWordStride = 32;  // uint64 words between two team words (256 B)
constexpr int kMaxTeamSize = 8191;

#if defined(__HIPCC__)

__device__ __forceinline__ uint32_t xcc_id() {
  uint32_t x;
  asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(x));
  return x & 0xf;
}

__device__ __forceinline__ uint64_t team_checkin_value(uint32_t die) {
  return (1ull << 14) | ((uint64_t)die << 28) | ((uint64_t)(die * die) << 45);
}

// Called by one thread when the work-group starts; the result is not needed,
// so the atomic costs no latency.
__device__ __forceinline__ void team_checkin(uint64_t* word, uint32_t die) {
  __hip_atomic_fetch_add(word, team_checkin_value(die), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// True if `w` proves that all n members have started and all run on `die`.
__device__ __forceinline__ bool team_on_one_die(uint64_t w, uint32_t n, uint32_t die) {
  const uint32_t checkins = (uint32_t)(w >> 14) & 0x3fffu;
  const uint32_t sum = (uint32_t)(w >> 28) & 0x1ffffu;
  const uint32_t sq = (uint32_t)(w >> 45);
  return checkins == n && sum == n * die && sq == n * die * die;
}

__device__ __forceinline__ uint64_t team_load(const uint64_t* word) {
  return __hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Publish: to be called by ONE thread after every wave of the work-group has
// waited for its own result stores (s_waitcnt vmcnt(0)) and the work-group has
// passed a barrier.  `seen` is the team word as loaded (team_load) by the same
// thread any time after the launch's check-ins can have landed -- typically
// issued together with the result stores so that its latency hides behind
// theirs; it only decides whether this die's L2 has to be written back first
// (unless the whole team is known to share the die).  Returns the word as it was
// before this member's ticket: the member is the last one iff its ticket field
// equals n - 1.
__device__ __forceinline__ uint64_t team_publish(uint64_t* word, uint64_t seen, uint32_t n,
                                                 uint32_t die, bool force_fences) {
  if (force_fences || !team_on_one_die(seen, n, die))
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
  return __hip_atomic_fetch_add(word, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ bool team_is_last(uint64_t before, uint32_t n) {
  return ((uint32_t)before & 0x3fffu) == n - 1;
}

// For the last member, by every thread that is going to read the others'
// results: if the team spans dies, drop this die's stale L2 lines first.  The
// reads themselves must be device-scope loads (team_ld).  `before` is what
// team_publish returned: by then every member has checked in.
__device__ __forceinline__ void team_acquire(uint64_t before, uint32_t n, uint32_t die,
                                             bool force_fences) {
  if (force_fences || !team_on_one_die(before, n, die))
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
}

// The last member re-arms the word for the next launch.
__device__ __forceinline__ void team_reset(uint64_t* word) {
  __hip_atomic_exchange(word, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ float team_ld(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int team_ld(const int* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Wait until this wave's global stores have completed (reached the L2).
__device__ __forceinline__ void wait_stores() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

#endif  // __HIPCC__

}  // namespace quest
