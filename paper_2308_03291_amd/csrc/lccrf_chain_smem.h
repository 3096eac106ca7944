// Shared-memory state of one sum-product chain (one workgroup) and the small collective steps on it,
// shared by the chain kernels of lccrf_chain.hip and the row-batch kernels of lccrf_stream.hip.
#pragma once

#include "lccrf_chain_args.h"
#include "lccrf_device.h"

namespace lccrf {

template <typename G>
struct ChainSmem {
    alignas(16) float pmax[G::WAVES][G::TCAP];  // per-wave column maxima of x = ua(s) + phi2(s,t) ...
    alignas(16) float psum[G::WAVES][G::TCAP];  // ... and column sums of 2^(x - that maximum)
    alignas(16) float rvec[2][G::TCAP];         // un-normalised result vector of a step (double buffered)
    alignas(16) float wmax[2][16];              // per-wave maxima of rvec (normaliser = their maximum)
    alignas(16) float wtot[2][16];              // per-wave sums of the marginals written by a step
    alignas(16) float red[2][4];                // scratch for the mid-point log-sum-exp
    int bad[4];                                 // "speculative step n rejected", indexed by n & 3
};

template <typename G>
__device__ __forceinline__ void smem_init(ChainSmem<G>& sm, int tid) {
    for (int k = tid; k < 2 * G::TCAP; k += G::W) (&sm.rvec[0][0])[k] = LCCRF_NEG_INF;
    if (tid < 32) (&sm.wmax[0][0])[tid] = LCCRF_NEG_INF;
    if (tid < 32) (&sm.wtot[0][0])[tid] = 0.f;
    if (tid < 4) sm.bad[tid] = 0;
}


// Normaliser of the vector in rvec[buf]: its maximum (0 if the vector is all -inf).
template <typename G>
__device__ __forceinline__ float read_shift(const ChainSmem<G>& sm, int buf) {
    const float4 q0 = *reinterpret_cast<const float4*>(&sm.wmax[buf][0]);
    const float4 q1 = *reinterpret_cast<const float4*>(&sm.wmax[buf][4]);
    const float4 q2 = *reinterpret_cast<const float4*>(&sm.wmax[buf][8]);
    const float4 q3 = *reinterpret_cast<const float4*>(&sm.wmax[buf][12]);
    const float a = max3_raw(max3_raw(q0.x, q0.y, q0.z), q0.w, q1.x), b = max3_raw(max3_raw(q1.y, q1.z, q1.w), q2.x, q2.y);
    const float c = max3_raw(max3_raw(q2.z, q2.w, q3.x), q3.y, q3.z);
    return finite_or_zero(max3_raw(max3_raw(a, b, c), q3.w, q3.w));
}

// -log2 of the sum of the marginals the last step wrote (0 if nothing usable was written).
template <typename G>
__device__ __forceinline__ float read_drift(const ChainSmem<G>& sm, int buf) {
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < 16; w += 4) {
        const float4 q = *reinterpret_cast<const float4*>(&sm.wtot[buf][w]);
        tot += (q.x + q.y) + (q.z + q.w);
    }
    return (tot > 0.5f && tot < 2.0f) ? -lg2(tot) : 0.f;
}

// Publish r (one value per column thread, -inf for t >= T) as the next vector.
// r must be -inf in every lane that owns no column; the wave-wide exchange runs with all
// lanes of the (wave-uniformly selected) column waves active.
template <typename G>
__device__ __forceinline__ void publish_columns(ChainSmem<G>& sm, int nbuf, int tid, float r) {
    if ((tid >> 6) < G::COLWAVES) {
        if (tid < G::TCAP) sm.rvec[nbuf][tid] = r;
        const float wm = xor_max<1, 64>(r);
        if ((tid & 63) == 0) sm.wmax[nbuf][tid >> 6] = wm;
    }
}

// log2 Z from the two vectors stored for the meeting position h.  Every thread of the
// workgroup returns the same value.
template <typename G>
__device__ __forceinline__ double midpoint_log2z(ChainSmem<G>& sm, const ChainArgs& a, size_t vb, int h, int T, int tid) {
    float z = LCCRF_NEG_INF;
    if (tid < T) z = a.ua[(vb + h) * T + tid] + a.ub[(vb + h) * T + tid];
    if ((tid >> 6) < G::COLWAVES) {
        const float wm = xor_max<1, 64>(z);
        if ((tid & 63) == 0) sm.red[0][tid >> 6] = wm;
    }
    __syncthreads();
    float M = LCCRF_NEG_INF;
#pragma unroll
    for (int w = 0; w < G::COLWAVES; ++w) M = fmaxf(M, sm.red[0][w]);
    const float g = finite_or_zero(M);
    if ((tid >> 6) < G::COLWAVES) {
        const float ws = xor_sum<1, 64>(ex2(z - g));  // z = -inf outside the T columns: adds 0
        if ((tid & 63) == 0) sm.red[1][tid >> 6] = ws;
    }
    __syncthreads();
    float S = 0.f;
#pragma unroll
    for (int w = 0; w < G::COLWAVES; ++w) S += sm.red[1][w];
    return (double)(M + lg2(S)) + a.Oa[vb + h] + a.Ob[vb + h];
}

}  // namespace lccrf
