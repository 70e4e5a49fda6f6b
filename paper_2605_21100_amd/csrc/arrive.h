// Last-arriver protocol of the fused tile reduction: the tiles of one (shard, kv head) publish their partials to
// the workspace, count themselves at a per-segment counter, and the workgroup that counts last reads all partials
// and reduces them -- inside the same launch, across workgroups on different XCDs (whose L2 caches are not coherent
// with each other for ordinary accesses).
//
// What makes a partial visible to the reducer, step by step:
//   producer  (1) every partial word is written with a device-scope store (st_dev, st_dev2: relaxed atomic store, agent scope
//                 -> a store that is performed at the device's point of coherence, not left dirty in this XCD's L2);
//             (2) every thread waits until all its stores have been acknowledged (s_waitcnt vmcnt(0)); for a
//                 device-scope store the acknowledgement means it has been performed at that point of coherence.
//                 A workgroup-scope release fence alone emits no such wait on this target (one CU, one L1);
//             (3) workgroup barrier: all threads of the workgroup have passed (2);
//             (4) one thread counts the arrival with a device-scope atomic add (performed at the same point of
//                 coherence, so it cannot be observed before the stores of (1), which completed before it issued).
//   reducer   (5) the thread that reads n_parts - 1 from the counter is the last arriver: all other producers
//                 have passed (4), hence (1)-(3).  The counter RMW is an acquire at agent scope: loads that follow
//                 it in program order cannot be satisfied before it;
//             (6) its result reaches the workgroup through LDS and a barrier, and the branch on it is a control
//                 dependency: no partial load is issued before the count is known (the hardware issues a
//                 wavefront's memory instructions in order and does not speculate past the branch);
//             (7) the partials are read with device-scope loads (ld_dev, ld_dev2), each served from the point of coherence,
//                 never from a stale line of this XCD's L2 or the CU's L1.
// What the compiler may move: the relaxed atomics are not reordered with each other across the inline-asm wait,
// the fence and the barrier (all three are compiler barriers for memory operations); ordinary loads/stores of
// other data may move, but none of them touches the partials.
// No cache-wide write-back or invalidate is issued on the producer side (a device-scope release fence there cost
// twice the kernel's run time when it was measured), which is why (1) and (7) use per-access device scope instead.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace nanocp {

__device__ inline void st_dev(float* ptr, float v) {
  __hip_atomic_store(ptr, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline float ld_dev(const float* ptr) {
  return __hip_atomic_load(ptr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// the same for two floats at once (8-byte device-scope accesses; `ptr` 8-byte aligned)
__device__ inline void st_dev2(float* ptr, float a, float b) {
  const uint64_t w = (uint64_t)__float_as_uint(a) | ((uint64_t)__float_as_uint(b) << 32);
  __hip_atomic_store((uint64_t*)ptr, w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void ld_dev2(const float* ptr, float& a, float& b) {
  const uint64_t w = __hip_atomic_load((const uint64_t*)ptr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  a = __uint_as_float((uint32_t)w);
  b = __uint_as_float((uint32_t)(w >> 32));
}

// Steps (2)-(6).  Call from every thread of the workgroup after its st_dev stores; `flag` is an int in LDS.
// Returns true in every thread of the workgroup that delivered the last of the n_parts partials.
__device__ inline bool arrive_is_last(int32_t* counter, int n_parts, int* flag) {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __syncthreads();
  if (threadIdx.x == 0) {
#ifdef NANOCP_ARRIVE_RELAXED
    *flag = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#else
    *flag = __hip_atomic_fetch_add(counter, 1, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT);
#endif
  }
  __syncthreads();
  return *flag == n_parts - 1;
}

// after the reduction: re-arm the counter for the next launch (one thread)
__device__ inline void arrive_reset(int32_t* counter) {
  __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace nanocp
