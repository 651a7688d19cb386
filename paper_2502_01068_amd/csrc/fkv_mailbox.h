// Cross-block exchange inside one launch: mailbox slots in device memory and bounded polling.
#pragma once

#include "fkv_internal.h"

namespace fkv {

// Cross-block exchange through mailboxes.  A mailbox slot is ONE atomic object (64 bits for a
// (max, sum) partial, 32 bits for a log-sum-exp) that carries its own "not posted yet" state: the
// all-ones pattern, which no posted value has.  The producer posts with a relaxed agent-scope
// atomic exchange, the single consumer polls with relaxed agent-scope atomic loads and puts the
// empty pattern back once it has the value.  Since the value itself is the signal, nothing has
// to be ordered against anything else: no fences, no counters, no second location that could
// become visible before the first (agent-scope fences would write back / invalidate a whole L2
// on this multi-XCD part, tens of microseconds).  Each slot has one producer and one consumer per
// launch; the empty pattern the consumer leaves behind is ordered before the next launch by the
// kernel boundary.  Slots are touched by nothing else.
constexpr unsigned long long kEmpty64 = ~0ull;
constexpr unsigned kEmpty32 = ~0u;

__device__ __forceinline__ void box_post(float2 *slot, float2 v) {
  unsigned long long bits;
  __builtin_memcpy(&bits, &v, sizeof bits);
  if (bits == kEmpty64) bits = 0x7FC000007FC00000ull;  // a NaN pair with that payload is posted as plain NaNs
  (void)__hip_atomic_exchange(reinterpret_cast<unsigned long long *>(slot), bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long box_peek(const float2 *slot) {
  return __hip_atomic_load(reinterpret_cast<const unsigned long long *>(slot), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void box_clear(float2 *slot) {
  __hip_atomic_store(reinterpret_cast<unsigned long long *>(slot), kEmpty64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void box_post(float *slot, float v) {
  unsigned bits = __float_as_uint(v);
  if (bits == kEmpty32) bits = 0x7FC00000u;
  (void)__hip_atomic_exchange(reinterpret_cast<unsigned *>(slot), bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned box_peek(const float *slot) {
  return __hip_atomic_load(reinterpret_cast<const unsigned *>(slot), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void box_clear(float *slot) {
  __hip_atomic_store(reinterpret_cast<unsigned *>(slot), kEmpty32, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Time limit of a polling loop.  Reading the clock costs a round trip through the scalar memory path
// (comparable to the poll itself), so it is read only every 64th round, the first time to start
// the interval; limits below 1 ms (how tests force the failure path) are checked on every round,
// from a start time taken before the first poll.  Wave-uniform.
struct BoundedWait {
  unsigned long long t0, limit;
  unsigned round;
  bool strict;
  __device__ __forceinline__ explicit BoundedWait(unsigned long long limit_ticks)
      : t0(0), limit(limit_ticks), round(0), strict(limit_ticks < 100000ull) {
    if (strict) t0 = wall_clock64();
  }
  // Call after a poll that did not complete; true once the limit has passed.
  __device__ __forceinline__ bool expired() {
    ++round;
    if (strict) return wall_clock64() - t0 > limit;
    if ((round & 63u) != 0u) return false;
    const unsigned long long now = wall_clock64();
    if (round == 64u) { t0 = now; return false; }
    return now - t0 > limit;
  }
};

// Tagged mailbox word for one-to-many exchanges: the launch's epoch in the high half, 32 bits of payload
// in the low half, written by one block with a single 64-bit atomic and read by any number of
// blocks, which poll until the high half is the epoch they expect.  As with the self-clearing slots
// the value is its own signal, so nothing has to be ordered against anything else; nobody clears a
// word, the next launch's epoch makes it stale.  Epoch 0 is never used (the words start as zero).
__device__ __forceinline__ void tag_post(unsigned long long *slot, unsigned epoch, unsigned payload) {
  (void)__hip_atomic_exchange(slot, ((unsigned long long)epoch << 32) | payload, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long tag_peek(const unsigned long long *slot) {
  return __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ bool tag_is(unsigned long long word, unsigned epoch) { return (unsigned)(word >> 32) == epoch; }

}  // namespace fkv
