// Host-side launch entry points of the kernel translation units (internal to the library).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace lccrf {

// Sum-product chains, position by position.  op 0: logZ only; op 1: marginals (+ logZ if
// non-null).  dtype 0: float, 1: bfloat16.  ua/ub: [B][N][T] floats, Oa/Ob: [B][N] doubles of
// scratch.  Enqueues on `st`; returns the launch status.
// `between`, if non-null, is recorded on `st` after the first pass.
hipError_t launch_sequential_sum(int op, int dtype, const void* phi, const int32_t* lengths, int B, int N, int T,
                                 float* ua, float* ub, double* Oa, double* Ob, float* logZ, float* mu,
                                 hipStream_t st, hipEvent_t between = nullptr);

// Max-plus chain with back-pointers and back-trace.  bp: [B][N][T] bytes of scratch.
hipError_t launch_sequential_max(int dtype, const void* phi, const int32_t* lengths, int B, int N, int T,
                                 uint8_t* bp, float* best_score, int32_t* tags, hipStream_t st);

}  // namespace lccrf
