// Streaming probe (declared in include/lccrf_instrument.h): what G workgroups of this chip can read,
// or read and write, from HBM when each streams a contiguous region of its own in 16-byte accesses with
// several loads in flight per thread, which is the access pattern of the chain kernels (one workgroup per
// chain, one tile per position).  It gives the practical ceilings the kernels are compared with beside the
// datasheet peak: a batch of B sequences has only 2B chains, and that many workgroups cannot draw the
// bandwidth of the whole chip.  Instrumentation for benchmarks, not a query.
#include "../../include/lccrf_instrument.h"

#include <hip/hip_runtime.h>

namespace {

typedef float probe_vec4 __attribute__((ext_vector_type(4)));

constexpr int kProbeInFlight = 4;   // 16-byte loads a thread keeps in flight
constexpr int kProbeThreads = 1024;

// Workgroup g covers vectors [g * per, (g + 1) * per) of `in` (per a multiple of kProbeThreads * kProbeInFlight):
// rounds of kProbeInFlight coalesced 16-byte loads per thread, each round issued before the previous one
// is consumed.  WRITE: every vector is stored (changed) to `out`; otherwise the values are summed and
// kept alive by a store that never happens for real data.
template <bool WRITE>
__global__ __launch_bounds__(kProbeThreads) void stream_probe_kernel(const probe_vec4* __restrict__ in,
                                                                     probe_vec4* __restrict__ out, size_t per,
                                                                     float* __restrict__ sink) {
    const probe_vec4* p = in + (size_t)blockIdx.x * per + threadIdx.x;
    probe_vec4* q = out + (size_t)blockIdx.x * per + threadIdx.x;
    const size_t rounds = per / ((size_t)kProbeThreads * kProbeInFlight);
    probe_vec4 cur[kProbeInFlight], nxt[kProbeInFlight];
    float acc = 0.f;
#pragma unroll
    for (int k = 0; k < kProbeInFlight; ++k) cur[k] = __builtin_nontemporal_load(p + (size_t)k * kProbeThreads);
    for (size_t r = 0; r < rounds; ++r) {
        const size_t ahead = (r + 1 < rounds ? r + 1 : r) * kProbeInFlight * kProbeThreads;  // the last round is loaded twice
#pragma unroll
        for (int k = 0; k < kProbeInFlight; ++k) nxt[k] = __builtin_nontemporal_load(p + ahead + (size_t)k * kProbeThreads);
#pragma unroll
        for (int k = 0; k < kProbeInFlight; ++k) {
            if (WRITE) {
                probe_vec4 o = cur[k];
                o[0] += 1.f;
                __builtin_nontemporal_store(o, q + (r * kProbeInFlight + k) * kProbeThreads);
            } else {
                acc += (cur[k][0] + cur[k][1]) + (cur[k][2] + cur[k][3]);
            }
            cur[k] = nxt[k];
        }
    }
    if (!WRITE && acc == 12345.678f) sink[0] = acc;
}

}  // namespace

extern "C" int lccrf_stream_probe(const void* in, void* out, size_t bytes, int workgroups, float* sink, void* stream) {
    if (!in || !sink) return LCCRF_ENULL;
    const size_t unit = (size_t)kProbeThreads * kProbeInFlight * sizeof(probe_vec4);  // bytes of one round of one workgroup
    if (workgroups < 1 || workgroups > (1 << 20) || bytes < unit * (size_t)workgroups) return LCCRF_EINVAL;
    if (reinterpret_cast<uintptr_t>(in) % 16 || reinterpret_cast<uintptr_t>(out) % 16) return LCCRF_EALIGN;
    const size_t per = bytes / unit / (size_t)workgroups * (unit / sizeof(probe_vec4));  // vectors per workgroup
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (out)
        hipLaunchKernelGGL(stream_probe_kernel<true>, dim3(workgroups), dim3(kProbeThreads), 0, st,
                           static_cast<const probe_vec4*>(in), static_cast<probe_vec4*>(out), per, sink);
    else
        hipLaunchKernelGGL(stream_probe_kernel<false>, dim3(workgroups), dim3(kProbeThreads), 0, st,
                           static_cast<const probe_vec4*>(in), static_cast<probe_vec4*>(nullptr), per, sink);
    return hipGetLastError() == hipSuccess ? LCCRF_OK : LCCRF_ELAUNCH;
}

extern "C" size_t lccrf_stream_probe_bytes(size_t bytes, int workgroups) {
    const size_t unit = (size_t)kProbeThreads * kProbeInFlight * sizeof(probe_vec4);
    if (workgroups < 1 || bytes < unit * (size_t)workgroups) return 0;
    return bytes / unit / (size_t)workgroups * unit * (size_t)workgroups;
}
