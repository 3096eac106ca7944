// Host-side launch entry points of the kernel translation units (internal to the library).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace lccrf {

// Sum-product chains, position by position.  op 0: logZ only; op 1: marginals (+ logZ if
// non-null).  dtype 0: float, 1: bfloat16.  ua/ub: [B][N][T] floats, Oa/Ob: [B][N] doubles of
// scratch.  Enqueues on `st`; returns the launch status.
// `between`, if non-null, is recorded on `st` after the first pass.  exact_only: skip the
// speculative uniform-shift step and run the exact step at every position.
// mail / failed: scratch of the paired second pass (pair_mail_words(B) 8-byte words and B ints),
// or null to always use one workgroup per chain.
hipError_t launch_sequential_sum(int op, int dtype, const void* phi, const int32_t* lengths, int B, int N, int T,
                                 float* ua, float* ub, double* Oa, double* Ob, float* logZ, float* mu,
                                 hipStream_t st, hipEvent_t between = nullptr, bool exact_only = false,
                                 unsigned long long* mail = nullptr, int* failed = nullptr);

// Paired second pass (two workgroups per chain; lccrf_pair.hip).
size_t pair_mail_words(int B);
bool pair_supported(int T);
hipError_t launch_pair_reset(unsigned long long* mail, int B, int* failed, hipStream_t st);
hipError_t launch_pair_marginals(int dtype, const void* phi, const int32_t* lengths, int B, int N, int T,
                                 const float* ua, const float* ub, const double* Oa, const double* Ob,
                                 float* logZ, float* mu, unsigned long long* mail, int* failed, hipStream_t st);

// Max-plus chain with back-pointers and back-trace.  bp: [B][N][T] bytes of scratch.
hipError_t launch_sequential_max(int dtype, const void* phi, const int32_t* lengths, int B, int N, int T,
                                 uint8_t* bp, float* best_score, int32_t* tags, hipStream_t st);

}  // namespace lccrf
