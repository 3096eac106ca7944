// Flags in LDS between the waves of one workgroup (lccrf_lane.hip, lccrf_lane_max.hip).
#pragma once
#include <hip/hip_runtime.h>

namespace lccrf {

// Flags in LDS.  What orders a flag against the data it guards is the hardware: the LDS instructions of a wave
// execute in the order they were issued, and LDS has no cache between the waves of a workgroup, so a wave that
// reads the new flag and then reads the data finds what the writer stored before it stored the flag.  The
// compiler only has to keep that order in the instruction stream (a signal fence).  A fence of the memory
// model would add waits that the chain cannot afford: s_waitcnt lgkmcnt(0) on every step, and, without an
// address space, vmcnt(0), which drains every global load and store the wave has in flight.
__device__ __forceinline__ int lds_load_acquire(const int* p) {
    const int v = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    return v;
}
__device__ __forceinline__ void lds_store_release(int* p, int v) {
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
__device__ __forceinline__ unsigned long long lds_load_acquire(const unsigned long long* p) {
    const unsigned long long v = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    return v;
}
__device__ __forceinline__ void lds_store_release(unsigned long long* p, unsigned long long v) {
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

}  // namespace lccrf
