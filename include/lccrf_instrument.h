/*
 * lccrf_instrument.h - benchmark instrumentation of the linear-chain CRF library.
 *
 * Not part of the query interface (include/lccrf.h): what is declared here exists so that a
 * benchmark can time the two passes of lccrf_marginals separately on the launch stream.
 */
#ifndef LCCRF_INSTRUMENT_H
#define LCCRF_INSTRUMENT_H

#include "lccrf.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * lccrf_marginals_algo (section "Computing Marginals" of the paper, Eq. 3-4) with three
 * caller-created hipEvent_t handles (passed as void*, any may be NULL) recorded on `stream`
 * before the first kernel, between the two passes of the sequential schedule (after every
 * matrix has been read once and the half-way vectors are stored; before the pass that
 * re-reads phi and writes the marginals), and after the last kernel.  Lets a caller time the
 * passes separately with hipEventElapsedTime.  Same results and errors as lccrf_marginals_algo.
 */
int lccrf_marginals_timed(const void* phi, lccrf_dtype dt, const int32_t* lengths,
                          int B, int N, int T, float* logZ, float* marginals,
                          void* workspace, size_t workspace_bytes, void* stream, lccrf_algo algo,
                          void* ev_begin, void* ev_between, void* ev_end);

/*
 * Streaming probe: `workgroups` workgroups of 1024 threads each read a contiguous share of in[0 .. bytes)
 * in 16-byte accesses with four loads in flight per thread, the access pattern of the chain kernels
 * (one workgroup per chain, one tile per position), and, if `out` is non-NULL, write every vector to
 * the same place in out.  Timed by the caller, it gives the bandwidth that many workgroups can draw:
 * the practical ceiling for a batch with that many chains, beside the datasheet peak.
 *   in, out   device buffers of `bytes` bytes, 16-byte aligned (out may be NULL: read only)
 *   sink      one device float (keeps the reads alive; never written for real data)
 * The bytes actually covered are lccrf_stream_probe_bytes(bytes, workgroups) (whole rounds of 64 KiB per
 * workgroup; 0 if bytes is too small for one round each, which lccrf_stream_probe refuses with
 * LCCRF_EINVAL).  Enqueues one kernel on `stream`; errors as the queries.
 */
int lccrf_stream_probe(const void* in, void* out, size_t bytes, int workgroups, float* sink, void* stream);
size_t lccrf_stream_probe_bytes(size_t bytes, int workgroups);

#ifdef __cplusplus
}
#endif
#endif /* LCCRF_INSTRUMENT_H */
