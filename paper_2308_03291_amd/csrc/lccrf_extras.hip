// Queries derived from the partition function (paper, sections "Computing Probability of a
// Structure and Partition Function" and "Entropy and KL Divergence"): the log-probability of
// a given tag path and the entropy of the distribution.  The heavy part of both is the
// first pass of the chain kernels; what is here only finishes them.
#include "lccrf_chain_args.h"
#include "lccrf_device.h"
#include "lccrf_launch.h"

namespace lccrf {

// log p(y) = phi[0][0][y_0] + sum_i phi[i][y_{i-1}][y_i] - logZ.  One workgroup per sequence; the
// score is summed in double precision (it and logZ are both of the size of the chain's total,
// their difference is not).  A tag outside [0, T) makes the result NaN.
constexpr int kPathThreads = 512;
template <typename TIN>
__global__ __launch_bounds__(kPathThreads) void path_log_prob_kernel(const TIN* __restrict__ phi, const int32_t* __restrict__ lengths,
                                                          const int32_t* __restrict__ tags, int N, int T,
                                                          const double* __restrict__ logZ64, float* __restrict__ out) {
    __shared__ double part[kPathThreads / 64];
    __shared__ int part_bad[kPathThreads / 64];
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int L = clamp_length(lengths, b, N);
    const int32_t* y = tags + (size_t)b * N;
    const TIN* phib = phi + (size_t)b * N * T * T;
    double acc = 0.0;
    bool bad = false;
    for (int i = tid; i < L; i += kPathThreads) {
        const int t = y[i], s = i > 0 ? y[i - 1] : 0;
        if (t < 0 || t >= T || s < 0 || s >= T) { bad = true; continue; }
        acc += (double)Elem<TIN>::get(phib + (size_t)i * T * T + (size_t)s * T + t);
    }
    acc += lane_xor<1>(acc);
    acc += lane_xor<2>(acc);
    acc += lane_xor<4>(acc);
    acc += lane_xor<8>(acc);
    acc += lane_xor<16>(acc);
    acc += lane_xor<32>(acc);
    const bool wave_bad = __builtin_amdgcn_ballot_w64(bad) != 0;
    if (lane == 0) {
        part[wave] = acc;
        part_bad[wave] = wave_bad ? 1 : 0;
    }
    __syncthreads();
    if (tid == 0) {
        double total = 0.0;
        int any_bad = 0;
        for (int w = 0; w < kPathThreads / 64; ++w) {
            total += part[w];
            any_bad |= part_bad[w];
        }
        out[b] = any_bad ? __builtin_nanf("") : (float)(total - logZ64[b]);
    }
}

hipError_t launch_path_log_prob(int dtype, const void* phi, const int32_t* lengths, const int32_t* tags, int B, int N,
                                int T, const double* logZ64, float* out, hipStream_t st) {
    if (dtype == 0)
        hipLaunchKernelGGL(path_log_prob_kernel<float>, dim3(B), dim3(kPathThreads), 0, st, static_cast<const float*>(phi), lengths,
                           tags, N, T, logZ64, out);
    else
        hipLaunchKernelGGL(path_log_prob_kernel<uint16_t>, dim3(B), dim3(kPathThreads), 0, st, static_cast<const uint16_t*>(phi),
                           lengths, tags, N, T, logZ64, out);
    return hipGetLastError();
}

// Entropy from what the two half chains leave at the meeting position h.  With the Markov
// property p(y) = p(y_h) p(y_<h | y_h) p(y_>h | y_h), so
//     H = H(y_h) + sum_t p(y_h = t) [ H(y_<h | y_h = t) + H(y_>h | y_h = t) ],
// the two conditional entropies being what the chains carried along (ha, hb, base 2) and
// p(y_h = t) the softmax of alpha_h + beta_h.  One wave per sequence.  No finite path: NaN.
__global__ __launch_bounds__(64) void entropy_combine_kernel(ChainArgs a, float* __restrict__ H) {
    const int b = blockIdx.x, lane = threadIdx.x;
    const int N = a.N, T = a.T;
    const int L = clamp_length(a.lengths, b, N);
    if (L == 0) {
        if (lane == 0) H[b] = 0.f;
        return;
    }
    const int h = meeting_point(0, L - 1);
    const size_t vb = (size_t)b * N;
    const float* ua = a.ua + (vb + h) * T;
    const float* ub = a.ub + (vb + h) * T;
    float m = LCCRF_NEG_INF;
    for (int t = lane; t < T; t += 64) m = fmaxf(m, ua[t] + ub[t]);
    m = xor_max<1, 64>(m);
    if (m == LCCRF_NEG_INF) {
        if (lane == 0) H[b] = __builtin_nanf("");
        return;
    }
    float S = 0.f;
    for (int t = lane; t < T; t += 64) S += ex2(ua[t] + ub[t] - m);
    S = xor_sum<1, 64>(S);
    const float lS = lg2(S);
    float acc = 0.f;
    for (int t = lane; t < T; t += 64) {
        const float z = ua[t] + ub[t] - m;  // log2 of p(y_h = t) S
        const float p = ex2(z) / S;
        if (p > 0.f) acc += p * (a.ha[(size_t)b * T + t] + a.hb[(size_t)b * T + t] - (z - lS));
    }
    acc = xor_sum<1, 64>(acc);
    if (lane == 0) H[b] = (float)((double)acc * kLn2);
}

static hipError_t launch_entropy_combine(const ChainArgs& a, float* H, hipStream_t st) {
    hipLaunchKernelGGL(entropy_combine_kernel, dim3(a.B), dim3(64), 0, st, a, H);
    return hipGetLastError();
}


// ---------------------------------------------------------------------------------------
// Expectations carried along the half chains: entropy first pass for T > 32 (the one-wave
// kernels carry it themselves for T <= 32), and the expected score difference behind the
// cross-entropy and the Kullback-Leibler divergence of two chains (any T).
//
// The same two half chains as chain_half_kernel, each carrying besides its normalised vector a
// second vector h: the conditional expectation, given the current tag, of a quantity summed over
// the path behind it.  With q(s|t) = 2^(ua(s) + phi2(s,t)) / S(t) on the forward chain
// (q(t|s) = 2^(phi2(s,t) + ub(t)) / S(s) on the backward chain):
//     MODE 0, entropy (base 2):   h_i(t) = sum_s q(s|t) [h_{i-1}(s) - log2 q(s|t)],
//                                 evaluated as U / S + log2 S with U = sum e (h - log2 e);
//     MODE 1, cross-entropy:      h_i(t) = sum_s q(s|t) [h_{i-1}(s) + psi_i(s,t)],
//     MODE 2, KL divergence:      h_i(t) = sum_s q(s|t) [h_{i-1}(s) + phi_i(s,t) - psi_i(s,t)],
// psi being the potentials of the second chain (natural units), read beside phi; an edge of
// weight zero contributes nothing whatever psi holds there.  In modes 1 and 2 a common shift of
// h (its largest finite entry) moves into a double-precision offset at every step, so the vector
// stays small however long the chain is.
// At 33 .. 128 tags every mode first tries every step with one shift for the whole matrix, the normaliser
// of the vector it starts from, as the chain kernels do (lccrf_chain.hip): U / S (+ log2 S) does not depend
// on the shift as long as no term that matters is flushed, which holds if every sum lies in
// [2^-60, 2^60]; otherwise the step is replayed exactly on the same registers.  The other geometries take
// plain exact steps (every sum against its own maximum): the forward step takes the column maxima
// through LDS first, then the sums.
template <typename G>
struct EntropySmem {
    alignas(16) float pmax[G::WAVES][G::TCAP];
    alignas(16) float psum[G::WAVES][G::TCAP];
    alignas(16) float pU[G::WAVES][G::TCAP];
    alignas(16) float rvec[2][G::TCAP];
    alignas(16) float hvec[2][G::TCAP];
    alignas(16) float wmax[2][16];
    int bad[4];  // "speculative step n rejected", indexed by n & 3
};

template <typename TIN, bool ALIGNED>
__device__ __forceinline__ void load_row4(const TIN* __restrict__ mat, int T, int c4, int s, float (&o)[4]) {
    const TIN* row = mat + (size_t)(s < T ? s : T - 1) * T;
    if (ALIGNED) {
        Elem<TIN>::get4(row + (c4 < T ? c4 : T - 4), o);
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) o[j] = Elem<TIN>::get(row + (c4 + j < T ? c4 + j : T - 1));
    }
}

__device__ __forceinline__ float expectation_of(float U, float S) { return S > 0.f ? U / S : 0.f; }

template <typename G, typename TIN, bool ALIGNED, int MODE>
__global__ __launch_bounds__(G::W) void entropy_half_kernel(ChainArgs a) {
    __shared__ EntropySmem<G> sm;
    constexpr int ITEMS = G::ITEMS, PF = 2;
    constexpr bool CROSS = MODE != 0;
    // the second tile travels through a ring of its own where registers allow (QRING); the
    // sixteen-wave geometries have 128 registers a thread: there its rows are fetched where they
    // are used
    constexpr bool LATE_PSI = CROSS && G::WAVES >= 16;
    constexpr bool QRING = CROSS && !LATE_PSI;
    constexpr int QITEMS = QRING ? ITEMS : 1, QPF = QRING ? PF : 1;
    constexpr bool SPEC = (ITEMS == 4 || ITEMS == 8) && G::LPR >= 16;  // speculative step first
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b = blockIdx.x >> 1, dir = blockIdx.x & 1;
    const int N = a.N, T = a.T;
    const int L = clamp_length(a.lengths, b, N);
    if (L == 0) return;
    const int e = L - 1, h = meeting_point(0, e);
    const int c4 = 4 * (tid % G::LPR), r0 = tid / G::LPR;
    const size_t TT = (size_t)T * T, vb = (size_t)b * N;
    const TIN* phib = static_cast<const TIN*>(a.phi) + (size_t)b * N * TT;
    const TIN* psib = CROSS ? static_cast<const TIN*>(a.psi) + (size_t)b * N * TT : phib;

    for (int k = tid; k < 2 * G::TCAP; k += G::W) {
        (&sm.rvec[0][0])[k] = LCCRF_NEG_INF;
        (&sm.hvec[0][0])[k] = 0.f;
    }
    if (tid < 32) (&sm.wmax[0][0])[tid] = LCCRF_NEG_INF;
    if (tid < 4) sm.bad[tid] = 0;
    int nstep = 0;
    __syncthreads();
    if (tid < T) {
        const float p0 = Elem<TIN>::get(phib + tid);
        sm.rvec[0][tid] = dir == 0 ? p0 * kLog2e : 0.f;
        if (CROSS && dir == 0 && p0 != LCCRF_NEG_INF) {  // the score of the first tag belongs to the forward chain
            const float q0 = Elem<TIN>::get(psib + tid);
            sm.hvec[0][tid] = MODE == 1 ? q0 : p0 - q0;
        }
    }
    __syncthreads();

    float ring[PF][ITEMS][4];
    float qring[QPF][QITEMS][4];
    auto load = [&](int i, int slot) {
        load_tile<G, TIN, ALIGNED>(phib + (size_t)i * TT, T, c4, r0, ring[slot], b != a.B - 1 || i != N - 1);
        if constexpr (QRING) load_tile<G, TIN, ALIGNED>(psib + (size_t)i * TT, T, c4, r0, qring[slot], b != a.B - 1 || i != N - 1);
    };
    // what an edge adds to the carried expectation (modes 1 and 2)
    auto edge_term = [&](int i, int slot, int k, const float (&x)[4], float (&f)[4]) {
        float qv[4];
        if constexpr (LATE_PSI) {
            load_row4<TIN, ALIGNED>(psib + (size_t)i * TT, T, c4, r0 + k * G::RPP, qv);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) qv[j] = qring[QRING ? slot : 0][QRING ? k : 0][j];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) f[j] = MODE == 1 ? qv[j] : x[j] - qv[j];
    };
    double O = 0.0, Hoff = 0.0;
    int buf = 0;
    auto shift = [&]() {  // normaliser of the vector in rvec[buf]: its maximum, by every thread
        float d = LCCRF_NEG_INF;
        for (int t = lane; t < T; t += 64) d = fmaxf(d, sm.rvec[buf][t]);
        return finite_or_zero(xor_max<1, 64>(d));
    };
    auto hshift = [&]() {  // largest finite entry of hvec[buf] (0 if there is none), by every thread
        float d = LCCRF_NEG_INF;
        for (int t = lane; t < T; t += 64) {
            const float g = sm.hvec[buf][t];
            if (fabsf(g) < __builtin_huge_valf()) d = fmaxf(d, g);
        }
        return finite_or_zero(xor_max<1, 64>(d));
    };

    if (dir == 0) {
        walk<PF>(1, h, +1, load, [&](int i, int slot) {
            float (&x)[ITEMS][4] = ring[slot];
            settle_tile<G, ALIGNED>(x, T, c4);
            if constexpr (QRING) settle_tile<G, ALIGNED>(qring[slot], T, c4);
            const float d = shift();
            O += (double)d;
            float c = 0.f;
            if (CROSS) {
                c = hshift();
                Hoff += (double)c;
            }
            float ua[ITEMS], hin[ITEMS], lm[4] = {LCCRF_NEG_INF, LCCRF_NEG_INF, LCCRF_NEG_INF, LCCRF_NEG_INF};
#pragma unroll
            for (int k = 0; k < ITEMS; ++k) {
                const int s = r0 + k * G::RPP;
                ua[k] = (s < T) ? sm.rvec[buf][s] - d : LCCRF_NEG_INF;
                hin[k] = (s < T) ? sm.hvec[buf][s] - c : 0.f;
            }
            if constexpr (SPEC) {
                // one shift for the whole matrix: the normaliser d predicts this step's growth
                const int flag = nstep & 3;
                if (tid == 0) sm.bad[(nstep + 1) & 3] = 0;
                float ls[4] = {0.f, 0.f, 0.f, 0.f}, lu[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int k = 0; k < ITEMS; ++k) {
                    const float uac = ua[k] - d;
                    float f[4] = {0.f, 0.f, 0.f, 0.f};
                    if constexpr (CROSS) edge_term(i, slot, k, x[k], f);
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float arg = __builtin_fmaf(x[k][j], kLog2e, uac);
                        const float ex = ex2(arg);
                        ls[j] += ex;
                        if (CROSS) lu[j] += ex > 0.f ? ex * (hin[k] + f[j]) : 0.f;
                        else lu[j] = __builtin_fmaf(ex, hin[k] - log2_term(arg), lu[j]);
                    }
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    ls[j] = xor_sum<G::LPR, 64>(ls[j]);
                    lu[j] = xor_sum<G::LPR, 64>(lu[j]);
                }
                if (lane < G::LPR) {
                    *reinterpret_cast<float4*>(&sm.psum[wave][c4]) = make_float4(ls[0], ls[1], ls[2], ls[3]);
                    *reinterpret_cast<float4*>(&sm.pU[wave][c4]) = make_float4(lu[0], lu[1], lu[2], lu[3]);
                }
                __syncthreads();
                if (wave < G::COLWAVES) {
                    bool good = true;
                    if (tid < T) {
                        float S = 0.f, U = 0.f;
#pragma unroll
                        for (int w = 0; w < G::WAVES; ++w) {
                            S += sm.psum[w][tid];
                            U += sm.pU[w][tid];
                        }
                        good = sum_in_range(S);
                        sm.rvec[buf ^ 1][tid] = d + lg2(S);
                        sm.hvec[buf ^ 1][tid] = CROSS ? expectation_of(U, S) : entropy_of(U, S);
                    }
                    if (!__all(good) && lane == 0) sm.bad[flag] = 1;
                }
                __syncthreads();
                ++nstep;
                if (sm.bad[flag] == 0) {
                    buf ^= 1;
                    return;
                }
                __syncthreads();  // nobody still reads the flag or the rejected vectors
            }
#pragma unroll
            for (int k = 0; k < ITEMS; ++k) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float xs = __builtin_fmaf(x[k][j], kLog2e, ua[k]);
                    if (!CROSS) x[k][j] = xs;  // the raw potential is needed again in mode 2
                    lm[j] = fmaxf(lm[j], xs);
                }
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) lm[j] = xor_max<G::LPR, 64>(lm[j]);
            if (lane < G::LPR) *reinterpret_cast<float4*>(&sm.pmax[wave][c4]) = make_float4(lm[0], lm[1], lm[2], lm[3]);
            __syncthreads();
            float M[4], ls[4] = {0.f, 0.f, 0.f, 0.f}, lu[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                M[j] = LCCRF_NEG_INF;
#pragma unroll
                for (int w = 0; w < G::WAVES; ++w) M[j] = fmaxf(M[j], sm.pmax[w][c4 + j]);
                M[j] = finite_or_zero(M[j]);
            }
#pragma unroll
            for (int k = 0; k < ITEMS; ++k) {
                float f[4] = {0.f, 0.f, 0.f, 0.f};
                if constexpr (CROSS) edge_term(i, slot, k, x[k], f);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float arg = (CROSS ? __builtin_fmaf(x[k][j], kLog2e, ua[k]) : x[k][j]) - M[j];
                    const float ex = ex2(arg);
                    ls[j] += ex;
                    if (CROSS) lu[j] += ex > 0.f ? ex * (hin[k] + f[j]) : 0.f;
                    else lu[j] = __builtin_fmaf(ex, hin[k] - log2_term(arg), lu[j]);
                }
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                ls[j] = xor_sum<G::LPR, 64>(ls[j]);
                lu[j] = xor_sum<G::LPR, 64>(lu[j]);
            }
            if (lane < G::LPR) {
                *reinterpret_cast<float4*>(&sm.psum[wave][c4]) = make_float4(ls[0], ls[1], ls[2], ls[3]);
                *reinterpret_cast<float4*>(&sm.pU[wave][c4]) = make_float4(lu[0], lu[1], lu[2], lu[3]);
            }
            __syncthreads();
            if (tid < T) {
                float S = 0.f, U = 0.f, Mt = LCCRF_NEG_INF;
#pragma unroll
                for (int w = 0; w < G::WAVES; ++w) {
                    S += sm.psum[w][tid];
                    U += sm.pU[w][tid];
                    Mt = fmaxf(Mt, sm.pmax[w][tid]);
                }
                sm.rvec[buf ^ 1][tid] = Mt + lg2(S);  // Mt = -inf gives S = 0: -inf
                sm.hvec[buf ^ 1][tid] = CROSS ? expectation_of(U, S) : entropy_of(U, S);
            }
            __syncthreads();
            buf ^= 1;
        });
    } else {
        walk<PF>(e, h + 1, -1, load, [&](int i, int slot) {
            float (&y)[ITEMS][4] = ring[slot];
            settle_tile<G, ALIGNED>(y, T, c4);
            if constexpr (QRING) settle_tile<G, ALIGNED>(qring[slot], T, c4);
            const float d = shift();
            O += (double)d;
            float c = 0.f;
            if (CROSS) {
                c = hshift();
                Hoff += (double)c;
            }
            float ub[4], hin[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                ub[j] = (c4 + j < T) ? sm.rvec[buf][c4 + j] - d : LCCRF_NEG_INF;
                hin[j] = (c4 + j < T) ? sm.hvec[buf][c4 + j] - c : 0.f;
            }
            if constexpr (SPEC) {
                const int flag = nstep & 3;
                if (tid == 0) sm.bad[(nstep + 1) & 3] = 0;
                float Sl[ITEMS], Ul[ITEMS];
#pragma unroll
                for (int k = 0; k < ITEMS; ++k) {
                    Sl[k] = 0.f;
                    Ul[k] = 0.f;
                    float f[4] = {0.f, 0.f, 0.f, 0.f};
                    if constexpr (CROSS) edge_term(i, slot, k, y[k], f);
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float arg = __builtin_fmaf(y[k][j], kLog2e, ub[j] - d);
                        const float ex = ex2(arg);
                        Sl[k] += ex;
                        if (CROSS) Ul[k] += ex > 0.f ? ex * (hin[j] + f[j]) : 0.f;
                        else Ul[k] = __builtin_fmaf(ex, hin[j] - log2_term(arg), Ul[k]);
                    }
                }
                // four rows at a time: each lane ends up with the complete sums of one of them
                const int kk = 2 * (lane & 1) + ((lane >> 1) & 1);
                bool good = true;
#pragma unroll
                for (int k0 = 0; k0 < ITEMS; k0 += 4) {
                    const float S = reduce4_over_lanes<G::LPR>(Sl[k0], Sl[k0 + 1], Sl[k0 + 2], Sl[k0 + 3], lane);
                    const float U = reduce4_over_lanes<G::LPR>(Ul[k0], Ul[k0 + 1], Ul[k0 + 2], Ul[k0 + 3], lane);
                    const int s = r0 + (k0 + kk) * G::RPP;
                    if ((tid % G::LPR) < 4 && s < T) {
                        sm.rvec[buf ^ 1][s] = d + lg2(S);
                        sm.hvec[buf ^ 1][s] = CROSS ? expectation_of(U, S) : entropy_of(U, S);
                    }
                    good = good && (s >= T || sum_in_range(S));
                }
                if (!__all(good) && lane == 0) sm.bad[flag] = 1;
                __syncthreads();
                ++nstep;
                if (sm.bad[flag] == 0) {
                    buf ^= 1;
                    return;
                }
                __syncthreads();  // nobody still reads the flag or the rejected vectors
            }
#pragma unroll
            for (int k = 0; k < ITEMS; ++k) {
                float f[4] = {0.f, 0.f, 0.f, 0.f};
                if constexpr (CROSS) edge_term(i, slot, k, y[k], f);
#pragma unroll
                for (int j = 0; j < 4; ++j) y[k][j] = __builtin_fmaf(y[k][j], kLog2e, ub[j]);
                const float m = xor_max<1, G::LPR>(fmaxf(fmaxf(y[k][0], y[k][1]), fmaxf(y[k][2], y[k][3])));
                const float g = finite_or_zero(m);
                float Sl = 0.f, Ul = 0.f;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float arg = y[k][j] - g;
                    const float ex = ex2(arg);
                    Sl += ex;
                    if (CROSS) Ul += ex > 0.f ? ex * (hin[j] + f[j]) : 0.f;
                    else Ul = __builtin_fmaf(ex, hin[j] - log2_term(arg), Ul);
                }
                const float S = xor_sum<1, G::LPR>(Sl), U = xor_sum<1, G::LPR>(Ul);
                const int s = r0 + k * G::RPP;
                if (c4 == 0 && s < T) {
                    sm.rvec[buf ^ 1][s] = m + lg2(S);
                    sm.hvec[buf ^ 1][s] = CROSS ? expectation_of(U, S) : entropy_of(U, S);
                }
            }
            __syncthreads();
            buf ^= 1;
        });
    }
    // the vectors of the meeting position
    const float d = shift();
    O += (double)d;
    if (tid < T) {
        (dir == 0 ? a.ua : a.ub)[(vb + h) * T + tid] = sm.rvec[buf][tid] - d;
        (dir == 0 ? a.ha : a.hb)[(size_t)b * T + tid] = sm.hvec[buf][tid];
    }
    if (tid == 0) (dir == 0 ? a.Oa : a.Ob)[vb + h] = O;
    if (CROSS && tid == 0) a.hoff[2 * b + dir] = Hoff;
}

template <typename TIN, bool ALIGNED, int MODE>
static hipError_t launch_entropy_T(const ChainArgs& a, hipStream_t st) {
    const dim3 grid(2 * a.B);
    if (a.T <= 16)
        hipLaunchKernelGGL((entropy_half_kernel<Geo<4, 1, 1>, TIN, ALIGNED, MODE>), grid, dim3(64), 0, st, a);
    else if (a.T <= 32)
        hipLaunchKernelGGL((entropy_half_kernel<Geo<8, 4, 1>, TIN, ALIGNED, MODE>), grid, dim3(256), 0, st, a);
    else if (a.T <= 64)
        hipLaunchKernelGGL((entropy_half_kernel<Geo<16, 4, 4>, TIN, ALIGNED, MODE>), grid, dim3(256), 0, st, a);
    else if (a.T <= 128) {
        if constexpr (MODE == 0)
            hipLaunchKernelGGL((entropy_half_kernel<Geo<32, 16, 4>, TIN, ALIGNED, MODE>), grid, dim3(1024), 0, st, a);
        else  // two tiles in flight: eight waves, so that a thread has the registers for both rings
            hipLaunchKernelGGL((entropy_half_kernel<Geo<32, 8, 8>, TIN, ALIGNED, MODE>), grid, dim3(512), 0, st, a);
    } else
        return hipErrorInvalidValue;  // larger tag sets take the row-batch kernel (launch_stream_expect)
    return hipGetLastError();
}
template <int MODE>
static hipError_t launch_entropy_mode(int dtype, const ChainArgs& a, hipStream_t st) {
    if (stream_supported(a.T)) return launch_stream_expect(MODE, dtype, a, st);
    const bool aligned = (a.T % 4) == 0;
    if (dtype == 0) return aligned ? launch_entropy_T<float, true, MODE>(a, st) : launch_entropy_T<float, false, MODE>(a, st);
    return aligned ? launch_entropy_T<uint16_t, true, MODE>(a, st) : launch_entropy_T<uint16_t, false, MODE>(a, st);
}

// H(p) [B] for every sequence: first pass in entropy mode, then the combination at the meeting point.
hipError_t launch_entropy(int dtype, const void* phi, const int32_t* lengths, int B, int N, int T, float* ua, float* ub,
                          double* Oa, double* Ob, float* ha, float* hb, float* H, hipStream_t st) {
    ChainArgs a{phi, lengths, B, N, T, ua, ub, Oa, Ob, nullptr, nullptr, 0, nullptr, 0, 1, nullptr, nullptr, nullptr, nullptr};
    a.ha = ha;
    a.hb = hb;
    const hipError_t e = wave_supported(T) ? launch_wave_pass(false, dtype, a, st) : launch_entropy_mode<0>(dtype, a, st);
    if (e != hipSuccess) return e;
    return launch_entropy_combine(a, H, st);
}

// Entropy from the per-wave sums of conditional edge entropies the second pass leaves in entropy
// mode (chunked schedule): H = ln 2 * sum over the chunks of the sequence, both directions.  One
// wave per sequence.  logZ: what the run has found for log Z ([B] floats): -inf means no finite
// path, the entropy is NaN then.
__global__ __launch_bounds__(64) void entropy_reduce_kernel(const float* __restrict__ ent, const int32_t* __restrict__ lengths,
                                                            const float* __restrict__ logZ, int N, int chunk, int C,
                                                            float* __restrict__ H) {
    const int b = blockIdx.x, lane = threadIdx.x;
    const int L = clamp_length(lengths, b, N);
    if (L == 0) {
        if (lane == 0) H[b] = 0.f;
        return;
    }
    const int Cb = (L + chunk - 1) / chunk;
    double acc = 0.0;
    for (int k = lane; k < 2 * Cb; k += 64) acc += (double)ent[2 * (size_t)b * C + k];
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) acc += __shfl_xor(acc, off, 64);
    if (lane == 0) H[b] = logZ[b] == LCCRF_NEG_INF ? __builtin_nanf("") : (float)(acc * kLn2);
}

hipError_t launch_entropy_reduce(const float* ent, const int32_t* lengths, const float* logZ, int B, int N, int chunk,
                                 float* H, hipStream_t st) {
    const int C = (N + chunk - 1) / chunk;
    hipLaunchKernelGGL(entropy_reduce_kernel, dim3(B), dim3(64), 0, st, ent, lengths, logZ, N, chunk, C, H);
    return hipGetLastError();
}

// The same sum over the chunks for the expectations of a second chain's potentials (natural units):
// cross-entropy logZq - E, or with kl the divergence logZq - logZp - E for E the expectation of the
// difference of the potentials.  No finite path under the chain itself (logZp = -inf): NaN.
__global__ __launch_bounds__(64) void cross_reduce_kernel(const float* __restrict__ ent, const int32_t* __restrict__ lengths,
                                                          const double* __restrict__ logZq, const double* __restrict__ logZp,
                                                          int N, int chunk, int C, int kl, float* __restrict__ out) {
    const int b = blockIdx.x, lane = threadIdx.x;
    const int L = clamp_length(lengths, b, N);
    if (L == 0) {
        if (lane == 0) out[b] = 0.f;
        return;
    }
    const int Cb = (L + chunk - 1) / chunk;
    double acc = 0.0;
    for (int k = lane; k < 2 * Cb; k += 64) acc += (double)ent[2 * (size_t)b * C + k];
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) acc += __shfl_xor(acc, off, 64);
    if (lane == 0) {
        const double lzp = logZp[b];
        out[b] = lzp == -__builtin_huge_val() ? __builtin_nanf("") : (float)(logZq[b] - (kl ? lzp : 0.0) - acc);
    }
}

hipError_t launch_cross_reduce(bool kl, const float* ent, const int32_t* lengths, const double* logZq, const double* logZp,
                               int B, int N, int chunk, float* out, hipStream_t st) {
    const int C = (N + chunk - 1) / chunk;
    hipLaunchKernelGGL(cross_reduce_kernel, dim3(B), dim3(64), 0, st, ent, lengths, logZq, logZp, N, chunk, C, kl ? 1 : 0, out);
    return hipGetLastError();
}

// Cross-entropy H(p, q) = log Z_q - E_p[score_q(y)] (kl = false) or Kullback-Leibler divergence
// KL(p || q) = E_p[score_p(y) - score_q(y)] - log Z_p + log Z_q (kl = true) of two chains over the
// same sequences: the expectation from the half chains of p at their meeting position (as the
// entropy above), log Z_p from the same vectors, log Z_q handed in (double precision, natural
// logarithm).  No finite path under p: NaN.  One wave per sequence.
__global__ __launch_bounds__(64) void cross_combine_kernel(ChainArgs a, const double* __restrict__ logZq, float* __restrict__ out,
                                                           int kl) {
    const int b = blockIdx.x, lane = threadIdx.x;
    const int N = a.N, T = a.T;
    const int L = clamp_length(a.lengths, b, N);
    if (L == 0) {
        if (lane == 0) out[b] = 0.f;
        return;
    }
    const int h = meeting_point(0, L - 1);
    const size_t vb = (size_t)b * N;
    const float* ua = a.ua + (vb + h) * T;
    const float* ub = a.ub + (vb + h) * T;
    float m = LCCRF_NEG_INF;
    for (int t = lane; t < T; t += 64) m = fmaxf(m, ua[t] + ub[t]);
    m = xor_max<1, 64>(m);
    if (m == LCCRF_NEG_INF) {
        if (lane == 0) out[b] = __builtin_nanf("");
        return;
    }
    float S = 0.f;
    for (int t = lane; t < T; t += 64) S += ex2(ua[t] + ub[t] - m);
    S = xor_sum<1, 64>(S);
    float acc = 0.f;
    for (int t = lane; t < T; t += 64) {
        const float p = ex2(ua[t] + ub[t] - m) / S;
        if (p > 0.f) acc += p * (a.ha[(size_t)b * T + t] + a.hb[(size_t)b * T + t]);
    }
    acc = xor_sum<1, 64>(acc);
    if (lane == 0) {
        const double E = (double)acc + a.hoff[2 * b] + a.hoff[2 * b + 1];
        const double lzp = (a.Oa[vb + h] + a.Ob[vb + h] + (double)m + (double)lg2(S)) * kLn2;
        out[b] = (float)(kl ? E - lzp + logZq[b] : logZq[b] - E);
    }
}

hipError_t launch_cross(bool kl, int dtype, const void* phi_p, const void* phi_q, const int32_t* lengths, int B, int N,
                        int T, float* ua, float* ub, double* Oa, double* Ob, float* ha, float* hb, double* hoff,
                        const double* logZq, float* out, hipStream_t st) {
    ChainArgs a{phi_p, lengths, B, N, T, ua, ub, Oa, Ob, nullptr, nullptr, 0, nullptr, 0, 1, nullptr, nullptr, nullptr, nullptr};
    a.ha = ha;
    a.hb = hb;
    a.hoff = hoff;
    a.psi = phi_q;
    const hipError_t e = kl ? launch_entropy_mode<2>(dtype, a, st) : launch_entropy_mode<1>(dtype, a, st);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(cross_combine_kernel, dim3(B), dim3(64), 0, st, a, logZq, out, kl ? 1 : 0);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Backward sweep of forward-filtering backward-sampling (paper, section "Sampling a Structure"):
// y_{L-1} ~ exp(alpha_{L-1}(t)), then y_i ~ exp(alpha_i(s) + phi_{i+1}(s, y_{i+1})) going down.
// The randomness is an input: uniforms[b][i] decides position i by inversion of the cumulative
// weights over ascending tags (the smallest tag whose cumulative weight exceeds u * total; the
// last tag of positive weight if rounding leaves none).
//
// With the uniforms fixed, position i is a MAP from the tag above it to its own tag, and that map
// does not depend on any other position: F_i[t] = the tag drawn for y_i if y_{i+1} = t.  So the
// sweep splits into a pass that is parallel over all positions and reads phi once
// (sample_map_kernel: all T columns of every matrix, T^2 work a position like a forward step) and
// a walk through the table of maps that touches one byte a position (sample_walk_kernel), instead
// of N dependent column gathers from HBM.  The total weight of column t is alpha_{i+1}(t), which
// the forward pass has stored, so one sweep over the rows of a column finds where the running sum
// crosses u (weights relative to that total; it equals the sum up to the rounding of the forward
// step, which matters only for a draw closer than that to the edge of a tag's interval).

// Where the uniforms come from: the caller's array, or (given == null) the counter-based generator
// Philox4x32-10 (Salmon, Moraes, Dror and Shaw, "Parallel random numbers: as easy as 1, 2, 3", 2011) keyed
// by the caller's 64-bit seed: the uniform of position i of sequence b is the first output word of the
// counter (b N + i, 0) under that key, its upper 24 bits times 2^-24.  A draw is a function of (seed, b, i)
// alone, so a call is reproducible whatever the launch shape, and any draw can be regenerated on its own.
struct Uniforms {
    const float* given;
    unsigned long long seed;
    __device__ __forceinline__ float at(size_t idx) const {
        if (given) return given[idx];
        unsigned c0 = (unsigned)(idx & 0xffffffffull), c1 = (unsigned)(idx >> 32), c2 = 0u, c3 = 0u;
        unsigned k0 = (unsigned)(seed & 0xffffffffull), k1 = (unsigned)(seed >> 32);
#pragma unroll
        for (int round = 0; round < 10; ++round) {
            const unsigned hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
            const unsigned hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
            c0 = hi1 ^ c1 ^ k0;
            c1 = lo1;
            c2 = hi0 ^ c3 ^ k1;
            c3 = lo0;
            k0 += 0x9E3779B9u;
            k1 += 0xBB67AE85u;
        }
        return (float)(c0 >> 8) * 0x1p-24f;
    }
};

// LPP lanes serve one position (16, 32 or 64: the tag count rounded up), CPT columns a lane (more
// than one only above 64 tags); a wave serves 64 / LPP positions, a workgroup four waves.
template <typename TIN, int LPP, int CPT>
__global__ __launch_bounds__(256) void sample_map_kernel(const TIN* __restrict__ phi, const int32_t* __restrict__ lengths,
                                                         const float* __restrict__ ua, const double* __restrict__ Oa,
                                                         const Uniforms uniforms, int B, int N, int T,
                                                         uint8_t* __restrict__ F) {
    constexpr int PPW = 64 / LPP, TCAP = LPP * CPT;
    __shared__ float alds[4][PPW][TCAP];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int pl = lane / LPP, tl = lane % LPP;
    const long long unit = ((long long)blockIdx.x * 4 + wave) * PPW + pl;  // (b, i), i = 0 .. N-2
    if (unit >= (long long)B * (N - 1)) return;
    const int b = (int)(unit / (N - 1)), i = (int)(unit % (N - 1));
    const int L = clamp_length(lengths, b, N);
    if (i >= L - 1) return;
    const size_t TT = (size_t)T * T, vb = (size_t)b * N;
    const TIN* mat = phi + (vb + i + 1) * TT;  // phi_{i+1}
    const float dO = (float)(Oa[vb + i] - Oa[vb + i + 1]);
    const float u = uniforms.at(vb + i);
    float base[CPT], cum[CPT];
    int first[CPT], last[CPT], col[CPT];
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
        const int t = tl + c * LPP;
        col[c] = t < T ? t : T - 1;
        base[c] = t < T ? dO - ua[(vb + i + 1) * T + t] : LCCRF_NEG_INF;  // an unreachable tag above: +inf, no weight
        if (!(base[c] < __builtin_huge_valf())) base[c] = LCCRF_NEG_INF;
        alds[wave][pl][t] = t < T ? ua[(vb + i) * T + t] : LCCRF_NEG_INF;
        cum[c] = 0.f;
        first[c] = -1;
        last[c] = -1;
    }
    const float* arow = alds[wave][pl];
#pragma unroll 4
    for (int s = 0; s < T; ++s) {
        const float as = arow[s];
        const TIN* row = mat + (size_t)s * T;
#pragma unroll
        for (int c = 0; c < CPT; ++c) {
            const float w = ex2(__builtin_fmaf(Elem<TIN>::get(row + col[c]), kLog2e, base[c]) + as);
            cum[c] += w;
            last[c] = w > 0.f ? s : last[c];
            first[c] = (first[c] < 0 && cum[c] > u) ? s : first[c];
        }
    }
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
        const int t = tl + c * LPP;
        const int pick = first[c] >= 0 ? first[c] : (last[c] >= 0 ? last[c] : 0);
        if (t < T) F[(vb + i) * T + t] = (uint8_t)pick;
    }
}

constexpr int kWalkWindow = 16384;  // bytes of the table of maps held in LDS at a time

// The tag of the last position: inversion over exp(alpha_{L-1}) by one wave, K tags a lane (lane l owns
// tags l K .. l K + K - 1, so that lane-wise prefix sums keep the tag order).  -1: no finite path.
template <int K>
__device__ __forceinline__ int draw_last_tag(const float* __restrict__ alpha_last, float u, int T, int lane) {
    float w[K], m = LCCRF_NEG_INF;
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int s = lane * K + k;
        w[k] = s < T ? alpha_last[s] : LCCRF_NEG_INF;
        m = fmaxf(m, w[k]);
    }
    m = xor_max<1, 64>(m);
    if (m == LCCRF_NEG_INF) return -1;
    float part = 0.f;
#pragma unroll
    for (int k = 0; k < K; ++k) {
        w[k] = ex2(w[k] - m);
        part += w[k];
    }
    float incl = part;  // inclusive prefix sum over lanes (ascending lane = ascending tag)
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const float v = __shfl_up(incl, off, 64);
        if (lane >= off) incl += v;
    }
    const float target = u * __shfl(incl, 63, 64);
    float cum = incl - part;
    int first_over = 0x7fffffff, last_pos = -1;
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int s = lane * K + k;
        cum += w[k];
        if (w[k] > 0.f) last_pos = s;
        if (first_over == 0x7fffffff && cum > target && s < T) first_over = s;
    }
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        first_over = min(first_over, __shfl_xor(first_over, off, 64));
        last_pos = max(last_pos, __shfl_xor(last_pos, off, 64));
    }
    return first_over != 0x7fffffff ? first_over : last_pos;
}

// The maps of positions lo .. lo + np - 1 of a sequence (Fb: its rows of the table) into LDS.
__device__ __forceinline__ void load_window(uint8_t* win, const uint8_t* __restrict__ Fb, int lo, int np, int T, int lane) {
    const uint8_t* src = Fb + (size_t)lo * T;
    const int nbytes = np * T;
    if (((reinterpret_cast<uintptr_t>(src) | (uintptr_t)nbytes) & 15) == 0) {
        for (int k = lane; k < nbytes / 16; k += 64)
            reinterpret_cast<uint4*>(win)[k] = reinterpret_cast<const uint4*>(src)[k];
    } else {
        for (int k = lane; k < nbytes; k += 64) win[k] = src[k];
    }
}

// A long window is cut into 64 segments: lane l composes the maps of segment l for all T possible
// tags above it (independent look-ups, so they overlap) into segmap[l][.].
__device__ __forceinline__ void compose_segments(const uint8_t* win, uint8_t* segmap, int np, int T, int lane, int& bot, int& top) {
    const int seg = (np + 63) / 64;
    bot = lane * seg < np ? lane * seg : np;  // window-relative
    top = bot + seg < np ? bot + seg : np;
    for (int c0 = 0; c0 < T; c0 += 4) {
        int t0 = c0, t1 = c0 + 1 < T ? c0 + 1 : c0, t2 = c0 + 2 < T ? c0 + 2 : c0, t3 = c0 + 3 < T ? c0 + 3 : c0;
        for (int r = top - 1; r >= bot; --r) {
            const uint8_t* row = win + r * T;
            t0 = row[t0]; t1 = row[t1]; t2 = row[t2]; t3 = row[t3];
        }
        segmap[lane * T + c0] = (uint8_t)t0;
        if (c0 + 1 < T) segmap[lane * T + c0 + 1] = (uint8_t)t1;
        if (c0 + 2 < T) segmap[lane * T + c0 + 2] = (uint8_t)t2;
        if (c0 + 3 < T) segmap[lane * T + c0 + 3] = (uint8_t)t3;
    }
}

// Positions lo .. lo + np - 1 (their maps in win) from the tag `cur` above them, tags written to y;
// returns the tag of position lo.  A short window is walked by one lane; a long one (small tag sets)
// segment by segment: every lane composes its segment, one lane passes the actual tag down through
// the 64 segment maps, and every lane walks its segment from the tag it was handed.
__device__ __forceinline__ int walk_window(const uint8_t* win, uint8_t* segmap, uint8_t* entry, int lo, int np, int T,
                                           int lane, int cur, int32_t* __restrict__ y) {
    if (np <= 128) {
        if (lane == 0) {
            for (int r = np - 1; r >= 0; --r) {
                cur = win[r * T + cur];
                y[lo + r] = cur;
            }
            entry[64] = (uint8_t)cur;
        }
    } else {
        int bot, top;
        compose_segments(win, segmap, np, T, lane, bot, top);
        __syncthreads();
        if (lane == 0) {
            for (int l = 63; l >= 0; --l) {
                entry[l] = (uint8_t)cur;
                cur = segmap[l * T + cur];
            }
            entry[64] = (uint8_t)cur;
        }
        __syncthreads();
        int t = entry[lane];
        for (int r = top - 1; r >= bot; --r) {
            t = win[r * T + t];
            y[lo + r] = t;
        }
    }
    __syncthreads();
    return entry[64];
}

// One wave per sequence: draws y_{L-1} from alpha_{L-1}, then follows the maps down through LDS
// windows of the table, one after the other.
template <int K>
__global__ __launch_bounds__(64) void sample_walk_kernel(const int32_t* __restrict__ lengths, const float* __restrict__ ua,
                                                         const Uniforms uniforms, const uint8_t* __restrict__ F,
                                                         int N, int T, int32_t* __restrict__ tags) {
    __shared__ __attribute__((aligned(16))) uint8_t win[kWalkWindow];
    __shared__ uint8_t segmap[64 * 256];
    __shared__ uint8_t entry[65];
    const int b = blockIdx.x, lane = threadIdx.x;
    const int L = clamp_length(lengths, b, N);
    int32_t* y = tags + (size_t)b * N;
    for (int i = L + lane; i < N; i += 64) y[i] = -1;
    if (L == 0) return;
    const size_t vb = (size_t)b * N;
    int cur = draw_last_tag<K>(ua + (vb + L - 1) * T, uniforms.at(vb + L - 1), T, lane);
    if (cur < 0) {  // no finite path: all tags 0
        for (int i = lane; i < L; i += 64) y[i] = 0;
        return;
    }
    if (lane == 0) y[L - 1] = cur;
    const int wp = kWalkWindow / T;  // positions a window (T <= 256: at least 64)
    int hi = L - 1;                  // positions [0, hi) still to walk
    while (hi > 0) {
        const int lo = hi - wp > 0 ? hi - wp : 0;
        load_window(win, F + vb * T, lo, hi - lo, T, lane);
        __syncthreads();
        cur = walk_window(win, segmap, entry, lo, hi - lo, T, lane, cur, y);
        hi = lo;
    }
}

// Long sequences, all windows at once (W windows a sequence, counted from the top: window w holds the
// positions below L - 1 - w wp).  First every window's maps are composed into one map of the tag above
// the window to the tag of its lowest position (winmap [B][W][T] bytes) ...
__global__ __launch_bounds__(64) void sample_window_map_kernel(const int32_t* __restrict__ lengths,
                                                               const uint8_t* __restrict__ F, int N, int T, int W,
                                                               uint8_t* __restrict__ winmap) {
    __shared__ __attribute__((aligned(16))) uint8_t win[kWalkWindow];
    __shared__ uint8_t segmap[64 * 256];
    const int b = blockIdx.x / W, w = blockIdx.x % W, lane = threadIdx.x;
    const int L = clamp_length(lengths, b, N);
    const int wp = kWalkWindow / T;
    const int hi = L - 1 - w * wp;
    if (hi <= 0) return;
    const int lo = hi - wp > 0 ? hi - wp : 0, np = hi - lo;
    load_window(win, F + (size_t)b * N * T, lo, np, T, lane);
    __syncthreads();
    uint8_t* out = winmap + ((size_t)b * W + w) * T;
    if (np <= 128) {
        for (int t = lane; t < T; t += 64) {
            int cur = t;
            for (int r = np - 1; r >= 0; --r) cur = win[r * T + cur];
            out[t] = (uint8_t)cur;
        }
    } else {
        int bot, top;
        compose_segments(win, segmap, np, T, lane, bot, top);
        __syncthreads();
        for (int t = lane; t < T; t += 64) {
            int cur = t;
            for (int l = 63; l >= 0; --l) cur = segmap[l * T + cur];
            out[t] = (uint8_t)cur;
        }
    }
}

// ... then every window finds the tag above it by passing the tag of the last position through the
// maps of the windows above (at most W look-ups in LDS) and walks its own positions.
template <int K>
__global__ __launch_bounds__(64) void sample_window_walk_kernel(const int32_t* __restrict__ lengths, const float* __restrict__ ua,
                                                                const Uniforms uniforms, const uint8_t* __restrict__ F,
                                                                int N, int T, int W, const uint8_t* __restrict__ winmap,
                                                                int32_t* __restrict__ tags) {
    __shared__ __attribute__((aligned(16))) uint8_t win[kWalkWindow];
    __shared__ uint8_t segmap[64 * 256];  // first the maps of the windows above (W T <= 16384 bytes)
    __shared__ uint8_t entry[65];
    const int b = blockIdx.x / W, w = blockIdx.x % W, lane = threadIdx.x;
    const int L = clamp_length(lengths, b, N);
    int32_t* y = tags + (size_t)b * N;
    if (w == 0)
        for (int i = L + lane; i < N; i += 64) y[i] = -1;
    if (L == 0) return;
    const size_t vb = (size_t)b * N;
    const int wp = kWalkWindow / T;
    const int hi = L - 1 - w * wp;
    const int lo = hi - wp > 0 ? hi - wp : 0;
    int cur = draw_last_tag<K>(ua + (vb + L - 1) * T, uniforms.at(vb + L - 1), T, lane);
    if (cur < 0) {  // no finite path: all tags 0
        if (w == 0 && lane == 0) y[L - 1] = 0;
        for (int i = lo + lane; i < hi; i += 64) y[i] = 0;
        return;
    }
    if (w == 0 && lane == 0) y[L - 1] = cur;
    if (hi <= 0) return;
    load_window(win, F + vb * T, lo, hi - lo, T, lane);
    const uint8_t* above = winmap + (size_t)b * W * T;
    for (int k = lane; k < w * T; k += 64) segmap[k] = above[k];
    __syncthreads();
    for (int v = 0; v < w; ++v) cur = segmap[v * T + cur];
    __syncthreads();
    walk_window(win, segmap, entry, lo, hi - lo, T, lane, cur, y);
}

template <typename TIN>
static hipError_t launch_sample_T(const TIN* phi, const int32_t* lengths, const float* ua, const double* Oa,
                                  const Uniforms uniforms, int B, int N, int T, uint8_t* F, uint8_t* winmap, int32_t* tags,
                                  hipStream_t st) {
    if (N > 1) {
        const long long units = (long long)B * (N - 1);
        auto blocks = [&](int ppw) { return dim3((unsigned)((units + 4 * ppw - 1) / (4 * ppw))); };
        if (T <= 16)
            hipLaunchKernelGGL((sample_map_kernel<TIN, 16, 1>), blocks(4), dim3(256), 0, st, phi, lengths, ua, Oa, uniforms, B, N, T, F);
        else if (T <= 32)
            hipLaunchKernelGGL((sample_map_kernel<TIN, 32, 1>), blocks(2), dim3(256), 0, st, phi, lengths, ua, Oa, uniforms, B, N, T, F);
        else if (T <= 64)
            hipLaunchKernelGGL((sample_map_kernel<TIN, 64, 1>), blocks(1), dim3(256), 0, st, phi, lengths, ua, Oa, uniforms, B, N, T, F);
        else if (T <= 128)
            hipLaunchKernelGGL((sample_map_kernel<TIN, 64, 2>), blocks(1), dim3(256), 0, st, phi, lengths, ua, Oa, uniforms, B, N, T, F);
        else
            hipLaunchKernelGGL((sample_map_kernel<TIN, 64, 4>), blocks(1), dim3(256), 0, st, phi, lengths, ua, Oa, uniforms, B, N, T, F);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    // Several windows a sequence: all of them at once, two launches, if their maps fit the LDS staging.
    const int wp = kWalkWindow / T, W = N > 1 ? (N - 1 + wp - 1) / wp : 1;
    if (W >= 2 && (size_t)W * T <= 64 * 256 && winmap) {
        hipLaunchKernelGGL(sample_window_map_kernel, dim3(B * W), dim3(64), 0, st, lengths, F, N, T, W, winmap);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        const dim3 grid(B * W);
        if (T <= 64) hipLaunchKernelGGL(sample_window_walk_kernel<1>, grid, dim3(64), 0, st, lengths, ua, uniforms, F, N, T, W, winmap, tags);
        else if (T <= 128) hipLaunchKernelGGL(sample_window_walk_kernel<2>, grid, dim3(64), 0, st, lengths, ua, uniforms, F, N, T, W, winmap, tags);
        else hipLaunchKernelGGL(sample_window_walk_kernel<4>, grid, dim3(64), 0, st, lengths, ua, uniforms, F, N, T, W, winmap, tags);
        return hipGetLastError();
    }
    if (T <= 64) hipLaunchKernelGGL(sample_walk_kernel<1>, dim3(B), dim3(64), 0, st, lengths, ua, uniforms, F, N, T, tags);
    else if (T <= 128) hipLaunchKernelGGL(sample_walk_kernel<2>, dim3(B), dim3(64), 0, st, lengths, ua, uniforms, F, N, T, tags);
    else hipLaunchKernelGGL(sample_walk_kernel<4>, dim3(B), dim3(64), 0, st, lengths, ua, uniforms, F, N, T, tags);
    return hipGetLastError();
}

// ua, Oa: alpha of every position from the forward pass ([B][N][T] normalised vectors, [B][N] offsets);
// F: [B][N][T] bytes of scratch for the maps; winmap: sample_winmap_bytes(B, N, T) bytes of scratch for
// the composed maps of the windows of long sequences (null: windows are walked one after the other).
size_t sample_winmap_bytes(int B, int N, int T) {
    const int wp = kWalkWindow / T;
    return (size_t)B * ((N + wp - 1) / wp + 1) * T;
}

hipError_t launch_backward_sample(int dtype, const void* phi, const int32_t* lengths, const float* ua, const double* Oa,
                                  const float* uniforms, unsigned long long seed, int B, int N, int T, uint8_t* F,
                                  uint8_t* winmap, int32_t* tags, hipStream_t st) {
    const Uniforms us{uniforms, seed};
    if (dtype == 0)
        return launch_sample_T(static_cast<const float*>(phi), lengths, ua, Oa, us, B, N, T, F, winmap, tags, st);
    return launch_sample_T(static_cast<const uint16_t*>(phi), lengths, ua, Oa, us, B, N, T, F, winmap, tags, st);
}

}  // namespace lccrf
