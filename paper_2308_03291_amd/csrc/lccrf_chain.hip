// Sequential (position-by-position) log-semiring chains for the linear-chain CRF.
//
// The paper computes logZ with the forward algorithm (section "Sequence Tagging") and
// obtains marginals as the gradient of logZ (section "Computing Marginals", Eq. 4), i.e.
// by replaying the recursion backwards.  Here both recursions are written by hand and each
// sequence is served by TWO chains that run at the same time and meet in the middle:
//
//   pass 1 (chain_half_kernel):  a forward workgroup computes alpha_0 .. alpha_h and a
//       backward workgroup computes beta_{L-1} .. beta_h (h = L / 2); both store their
//       normalised vectors.  Together they read every matrix once.
//   pass 2 (chain_marginal_kernel):  the forward workgroup continues over h+1 .. L-1 and
//       now has beta_i (stored by pass 1) when it reads phi_i, so it writes the marginals
//       mu_i = exp(alpha_{i-1} + phi_i + beta_i - logZ) in the same sweep; the backward
//       workgroup does the same over h .. 1 with the stored alpha_{i-1}.  Together they
//       read every matrix a second time and write every marginal once.
//
// That is the minimum traffic of forward-backward (two reads of phi, one write of mu) at
// half the serial depth and with twice as many workgroups streaming from HBM.
//
// Memory pipeline: every thread keeps a ring of PF tiles of phi in registers; the slot of
// the tile just consumed is refilled with the tile PF steps ahead as soon as its last
// register has been read, before the step's reductions and barriers, so PF - 1 whole tiles
// per workgroup are always in flight while the chain waits on its exchanges.
//
// Numerics: vectors are kept as u = alpha - O with a double-precision running offset O and
// max(u) = 0 after every step, so magnitudes stay small however long the chain is; every
// log-sum-exp is shifted by an exact maximum (partial sums carry their own maximum and are
// rescaled when merged); -inf entries are neutral.  The marginals of
// a position must sum to one; the sum actually written at one step is fed back as a
// correction (kappa) to the next, so rounding drift between the forward and the backward
// offsets (a random walk over thousands of float32 steps) never builds up in the output.
#include "lccrf_device.h"
#include "lccrf_launch.h"

namespace lccrf {

template <typename G>
struct ChainSmem {
    alignas(16) float pmax[G::WAVES][G::TCAP];  // per-wave column maxima of x = ua(s) + phi2(s,t) ...
    alignas(16) float psum[G::WAVES][G::TCAP];  // ... and column sums of 2^(x - that maximum)
    alignas(16) float rvec[2][G::TCAP];         // un-normalised result vector of a step (double buffered)
    alignas(16) float wmax[2][16];              // per-wave maxima of rvec (normaliser = their maximum)
    alignas(16) float wtot[2][16];              // per-wave sums of the marginals written by a step
    alignas(16) float red[2][4];                // scratch for the mid-point log-sum-exp
};

template <typename G>
__device__ __forceinline__ void smem_init(ChainSmem<G>& sm, int tid) {
    for (int k = tid; k < 2 * G::TCAP; k += G::W) (&sm.rvec[0][0])[k] = LCCRF_NEG_INF;
    if (tid < 32) (&sm.wmax[0][0])[tid] = LCCRF_NEG_INF;
    if (tid < 32) (&sm.wtot[0][0])[tid] = 0.f;
}

// Normaliser of the vector in rvec[buf]: its maximum (0 if the vector is all -inf).
template <typename G>
__device__ __forceinline__ float read_shift(const ChainSmem<G>& sm, int buf) {
    float d = LCCRF_NEG_INF;
#pragma unroll
    for (int w = 0; w < 16; w += 4) {
        const float4 q = *reinterpret_cast<const float4*>(&sm.wmax[buf][w]);
        d = fmaxf(fmaxf(d, fmaxf(q.x, q.y)), fmaxf(q.z, q.w));
    }
    return finite_or_zero(d);
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

// One exact forward step: r(t) = log2 sum_s 2^(ua(s) + phi2(s,t)).
//
// Single sweep with thread-local shifts: each thread takes the maximum of its own ITEMS rows
// per column, exponentiates against it, and the (maximum, sum) pairs are merged exactly -
// first across the row groups of the wave, then across waves by one thread per column.  Two
// barriers per step, and nothing a thread writes depends on another thread's data.
//
// WITH_MU: also writes mu(s,t) = 2^(ua(s) + phi2(s,t) + ubK(t)), ubK = beta_i(t) + (offsets - logZ),
// to `mu_out` and leaves the sum of what it wrote in wtot.
// `refill` is called once the tile's registers (reused for x) are free again.
template <typename G, bool WITH_MU, bool ALIGNED, typename Refill>
__device__ __forceinline__ void fwd_step(ChainSmem<G>& sm, int buf, int tid, int c4, int r0, int T,
                                         float (&v)[G::ITEMS][4], const float (&ua)[G::ITEMS],
                                         const float (&ubK)[4], float* __restrict__ mu_out, Refill refill) {
    constexpr int ITEMS = G::ITEMS;
    const int lane = tid & 63, wave = tid >> 6;
    mask_tile<G>(v, T, c4, r0);
    float (&x)[ITEMS][4] = v;  // the tile is turned into x = ua(s) + phi2(s,t) in place
    float lm[4] = {LCCRF_NEG_INF, LCCRF_NEG_INF, LCCRF_NEG_INF, LCCRF_NEG_INF};
#pragma unroll
    for (int k = 0; k < ITEMS; ++k)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            x[k][j] = __builtin_fmaf(v[k][j], kLog2e, ua[k]);
            lm[j] = fmaxf(lm[j], x[k][j]);
        }
    float g[4], ls[4] = {0.f, 0.f, 0.f, 0.f}, gm[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < 4; ++j) g[j] = finite_or_zero(lm[j]);
    if (WITH_MU) {
#pragma unroll
        for (int j = 0; j < 4; ++j) gm[j] = ex2(g[j] + ubK[j]);
    }
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) {
        float e[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            e[j] = ex2(x[k][j] - g[j]);
            ls[j] += e[j];
        }
        if (WITH_MU) {
            const int s = r0 + k * G::RPP;
            if (s < T && c4 < T) {
                float* p = mu_out + (size_t)s * T + c4;
                if (ALIGNED) {
                    *reinterpret_cast<float4*>(p) = make_float4(e[0] * gm[0], e[1] * gm[1], e[2] * gm[2], e[3] * gm[3]);
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (c4 + j < T) p[j] = e[j] * gm[j];
                }
            }
        }
    }
    refill();
    if (WITH_MU) {
        float tot = (ls[0] * gm[0] + ls[1] * gm[1]) + (ls[2] * gm[2] + ls[3] * gm[3]);
        tot = xor_sum<1, 64>(tot);
        if (lane == 0) sm.wtot[buf ^ 1][wave] = tot;
    }
    // merge the (max, sum) pairs of the wave's row groups
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float M = xor_max<G::LPR, 64>(lm[j]);
        if (G::LPR < 64) ls[j] = xor_sum<G::LPR, 64>(ls[j] * ex2(lm[j] - finite_or_zero(M)));
        lm[j] = M;
    }
    if (lane < G::LPR) {
        *reinterpret_cast<float4*>(&sm.pmax[wave][c4]) = make_float4(lm[0], lm[1], lm[2], lm[3]);
        *reinterpret_cast<float4*>(&sm.psum[wave][c4]) = make_float4(ls[0], ls[1], ls[2], ls[3]);
    }
    __syncthreads();
    float r = LCCRF_NEG_INF;
    if (tid < G::TCAP) {
        float mw[G::WAVES];
        float M = LCCRF_NEG_INF;
#pragma unroll
        for (int w = 0; w < G::WAVES; ++w) { mw[w] = sm.pmax[w][tid]; M = fmaxf(M, mw[w]); }
        const float gM = finite_or_zero(M);
        float S = 0.f;
#pragma unroll
        for (int w = 0; w < G::WAVES; ++w) S = __builtin_fmaf(sm.psum[w][tid], ex2(mw[w] - gM), S);
        r = M + lg2(S);  // M = -inf gives S = 0: -inf + -inf = -inf
    }
    publish_columns<G>(sm, buf ^ 1, tid, r);
    __syncthreads();
}

// One exact backward step: r(s) = log2 sum_t 2^(phi2(s,t) + ub(t)).
// The LPR lanes of a row sit in one wave: the row maximum and the row sum are all-reduced
// across them with LDS-free lane exchanges, so the step needs a single barrier.
// WITH_MU: also writes mu(s,t) = 2^(uaK(s) + phi2(s,t) + ub(t)), uaK = alpha_{i-1}(s) + (offsets - logZ).
template <typename G, bool WITH_MU, bool ALIGNED, typename Refill>
__device__ __forceinline__ void bwd_step(ChainSmem<G>& sm, int buf, int tid, int c4, int r0, int T,
                                         float (&v)[G::ITEMS][4], const float (&ub)[4],
                                         const float (&uaK)[G::ITEMS], float* __restrict__ mu_out, Refill refill) {
    constexpr int ITEMS = G::ITEMS;
    const int lane = tid & 63, wave = tid >> 6;
    mask_tile<G>(v, T, c4, r0);
    float (&y)[ITEMS][4] = v;  // the tile is turned into y = phi2(s,t) + ub(t) in place
    float m[ITEMS];
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) {
#pragma unroll
        for (int j = 0; j < 4; ++j) y[k][j] = __builtin_fmaf(v[k][j], kLog2e, ub[j]);
        m[k] = fmaxf(fmaxf(y[k][0], y[k][1]), fmaxf(y[k][2], y[k][3]));
    }
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) m[k] = xor_max<1, G::LPR>(m[k]);
    float S[ITEMS];
    float tot = 0.f;
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) {
        const float g = finite_or_zero(m[k]);
        float e[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) e[j] = ex2(y[k][j] - g);
        S[k] = (e[0] + e[1]) + (e[2] + e[3]);
        if (WITH_MU) {
            const int s = r0 + k * G::RPP;
            const float f = ex2(g + uaK[k]);
            if (s < T && c4 < T) {
                float* p = mu_out + (size_t)s * T + c4;
                if (ALIGNED) {
                    *reinterpret_cast<float4*>(p) = make_float4(e[0] * f, e[1] * f, e[2] * f, e[3] * f);
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (c4 + j < T) p[j] = e[j] * f;
                }
            }
            tot += S[k] * f;
        }
    }
    refill();
    float wm = LCCRF_NEG_INF;
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) {
        const float r = m[k] + lg2(xor_sum<1, G::LPR>(S[k]));
        const int s = r0 + k * G::RPP;
        if (c4 == 0 && s < T) sm.rvec[buf ^ 1][s] = r;
        wm = fmaxf(wm, r);
    }
    wm = xor_max<G::LPR, 64>(wm);  // every lane of a row already holds the row's r
    if (lane == 0) sm.wmax[buf ^ 1][wave] = wm;
    if (WITH_MU) {
        tot = xor_sum<1, 64>(tot);
        if (lane == 0) sm.wtot[buf ^ 1][wave] = tot;
    }
    __syncthreads();
}

struct ChainArgs {
    const void* phi;
    const int32_t* lengths;
    int B, N, T;
    float* ua;   // [B][N][T] normalised forward vectors (base-2 logs)
    float* ub;   // [B][N][T] normalised backward vectors
    double* Oa;  // [B][N] forward offsets:  alpha_i = (ua_i + Oa_i) * ln 2
    double* Ob;  // [B][N] backward offsets
    float* logZ;
    float* mu;
};

// Walks positions first, first+dir, ..., last (dir = +1 or -1) with a ring of PF tiles.
// `load(i, slot)` fills ring slot `slot` with position i's data, `step(i, slot, refill)`
// consumes it and must call refill() once the slot's registers are free.
template <int PF, typename Load, typename Step>
__device__ __forceinline__ void walk(int first, int last, int dir, Load load, Step step) {
    const int n = (last - first) * dir + 1;  // number of positions (<= 0: nothing to do)
    if (n <= 0) return;
#pragma unroll
    for (int p = 0; p < PF; ++p)
        if (p < n) load(first + p * dir, p);
    int done = 0;
    while (true) {
#pragma unroll
        for (int p = 0; p < PF; ++p) {
            const int i = first + done * dir;
            const bool more = done + PF < n;
            step(i, p, [&]() { if (more) load(i + PF * dir, p); });
            if (++done >= n) return;
        }
    }
}

// ---------------------------------------------------------------------------------------
// Pass 1: both half chains, vectors stored, nothing else written.
template <typename G, typename TIN, bool ALIGNED, int PF>
__global__ __launch_bounds__(G::W) void chain_half_kernel(ChainArgs a) {
    __shared__ ChainSmem<G> sm;
    constexpr int ITEMS = G::ITEMS;
    const int tid = threadIdx.x;
    const int b = blockIdx.x >> 1, dir = blockIdx.x & 1;
    const int N = a.N, T = a.T;
    const int L = clamp_length(a.lengths, b, N);
    if (L == 0) return;
    const int h = L / 2;
    const int c4 = 4 * (tid % G::LPR), r0 = tid / G::LPR;
    const TIN* phib = static_cast<const TIN*>(a.phi) + (size_t)b * N * T * T;
    const size_t TT = (size_t)T * T;
    const size_t vb = (size_t)b * N;

    smem_init<G>(sm, tid);
    __syncthreads();
    float ring[PF][ITEMS][4];
    const float dummy4[4] = {0.f, 0.f, 0.f, 0.f};
    float dummyI[ITEMS];
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) dummyI[k] = 0.f;
    double O = 0.0;
    int buf = 0;
    auto load = [&](int i, int slot) { load_tile<G, TIN, ALIGNED>(phib + (size_t)i * TT, T, c4, r0, ring[slot]); };

    if (dir == 0) {
        publish_columns<G>(sm, 0, tid, (tid < T) ? Elem<TIN>::get(phib + tid) * kLog2e : LCCRF_NEG_INF);
        __syncthreads();
        walk<PF>(1, h, +1, load, [&](int i, int slot, auto refill) {
            const float d = read_shift<G>(sm, buf);
            O += (double)d;
            float ua[ITEMS];
#pragma unroll
            for (int k = 0; k < ITEMS; ++k) {
                const int s = r0 + k * G::RPP;
                ua[k] = (s < T) ? sm.rvec[buf][s] - d : LCCRF_NEG_INF;
            }
            if (tid < T) a.ua[(vb + i - 1) * T + tid] = sm.rvec[buf][tid] - d;
            if (tid == 0) a.Oa[vb + i - 1] = O;
            fwd_step<G, false, ALIGNED>(sm, buf, tid, c4, r0, T, ring[slot], ua, dummy4, nullptr, refill);
            buf ^= 1;
        });
        const float d = read_shift<G>(sm, buf);
        O += (double)d;
        if (tid < T) a.ua[(vb + h) * T + tid] = sm.rvec[buf][tid] - d;
        if (tid == 0) a.Oa[vb + h] = O;
    } else {
        publish_columns<G>(sm, 0, tid, (tid < T) ? 0.f : LCCRF_NEG_INF);
        __syncthreads();
        walk<PF>(L - 1, h + 1, -1, load, [&](int i, int slot, auto refill) {
            const float d = read_shift<G>(sm, buf);
            O += (double)d;
            const float4 q = *reinterpret_cast<const float4*>(&sm.rvec[buf][c4]);
            const float ub[4] = {q.x - d, q.y - d, q.z - d, q.w - d};
            if (tid < T) a.ub[(vb + i) * T + tid] = sm.rvec[buf][tid] - d;
            if (tid == 0) a.Ob[vb + i] = O;
            bwd_step<G, false, ALIGNED>(sm, buf, tid, c4, r0, T, ring[slot], ub, dummyI, nullptr, refill);
            buf ^= 1;
        });
        const float d = read_shift<G>(sm, buf);
        O += (double)d;
        if (tid < T) a.ub[(vb + h) * T + tid] = sm.rvec[buf][tid] - d;
        if (tid == 0) a.Ob[vb + h] = O;
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

// ---------------------------------------------------------------------------------------
// Pass 2: both chains continue past the meeting point and write the marginals.
template <typename G, typename TIN, bool ALIGNED, int PF>
__global__ __launch_bounds__(G::W) void chain_marginal_kernel(ChainArgs a) {
    __shared__ ChainSmem<G> sm;
    constexpr int ITEMS = G::ITEMS;
    const int tid = threadIdx.x;
    const int b = blockIdx.x >> 1, dir = blockIdx.x & 1;
    const int N = a.N, T = a.T;
    const int L = clamp_length(a.lengths, b, N);
    const size_t TT = (size_t)T * T;
    const size_t vb = (size_t)b * N;
    float* mub = a.mu + (size_t)b * N * TT;

    if (dir == 0) {
        // positions past the end carry no edge: their marginals are zero
        const size_t z0 = (size_t)L * TT, z1 = (size_t)N * TT;
        if (ALIGNED) {
            float4* p = reinterpret_cast<float4*>(mub);
            for (size_t k = z0 / 4 + tid; k < z1 / 4; k += G::W) p[k] = make_float4(0.f, 0.f, 0.f, 0.f);
        } else {
            for (size_t k = z0 + tid; k < z1; k += G::W) mub[k] = 0.f;
        }
    }
    if (L == 0) {
        if (dir == 0 && tid == 0 && a.logZ) a.logZ[b] = 0.f;
        return;
    }
    const int h = L / 2;
    const int c4 = 4 * (tid % G::LPR), r0 = tid / G::LPR;
    const TIN* phib = static_cast<const TIN*>(a.phi) + (size_t)b * N * TT;

    smem_init<G>(sm, tid);
    const double lz2 = midpoint_log2z<G>(sm, a, vb, h, T, tid);
    const bool feasible = lz2 > -1.0e300;  // false: no path has a finite score, marginals are 0
    if (dir == 0 && tid == 0 && a.logZ) a.logZ[b] = (float)(lz2 * kLn2);

    float ring[PF][ITEMS][4];
    int buf = 0;
    float kappa = 0.f;  // running correction that keeps each position's marginals summing to one

    if (dir == 0) {
        double O = a.Oa[vb + h];
        publish_columns<G>(sm, 0, tid, (tid < T) ? a.ua[(vb + h) * T + tid] : LCCRF_NEG_INF);
        __syncthreads();
        float aux[PF][4];
        double ob[PF];
        auto load = [&](int i, int slot) {
            load_tile<G, TIN, ALIGNED>(phib + (size_t)i * TT, T, c4, r0, ring[slot]);
#pragma unroll
            for (int j = 0; j < 4; ++j) aux[slot][j] = (c4 + j < T) ? a.ub[(vb + i) * T + c4 + j] : LCCRF_NEG_INF;
            ob[slot] = a.Ob[vb + i];
        };
        walk<PF>(h + 1, L - 1, +1, load, [&](int i, int slot, auto refill) {
            const float d = read_shift<G>(sm, buf);
            kappa += read_drift<G>(sm, buf);
            O += (double)d;
            float ua[ITEMS];
#pragma unroll
            for (int k = 0; k < ITEMS; ++k) {
                const int s = r0 + k * G::RPP;
                ua[k] = (s < T) ? sm.rvec[buf][s] - d : LCCRF_NEG_INF;
            }
            const float K = feasible ? (float)(O + ob[slot] - lz2) + kappa : LCCRF_NEG_INF;
            const float ubK[4] = {aux[slot][0] + K, aux[slot][1] + K, aux[slot][2] + K, aux[slot][3] + K};
            fwd_step<G, true, ALIGNED>(sm, buf, tid, c4, r0, T, ring[slot], ua, ubK, mub + (size_t)i * TT, refill);
            buf ^= 1;
        });
    } else {
        double O = a.Ob[vb + h];
        publish_columns<G>(sm, 0, tid, (tid < T) ? a.ub[(vb + h) * T + tid] : LCCRF_NEG_INF);
        __syncthreads();
        float aux[PF][ITEMS];
        double oa[PF];
        auto load = [&](int i, int slot) {
            load_tile<G, TIN, ALIGNED>(phib + (size_t)i * TT, T, c4, r0, ring[slot]);
#pragma unroll
            for (int k = 0; k < ITEMS; ++k) {
                const int s = r0 + k * G::RPP;
                aux[slot][k] = (s < T) ? a.ua[(vb + i - 1) * T + s] : LCCRF_NEG_INF;
            }
            oa[slot] = a.Oa[vb + i - 1];
        };
        walk<PF>(h, 1, -1, load, [&](int i, int slot, auto refill) {
            const float d = read_shift<G>(sm, buf);
            kappa += read_drift<G>(sm, buf);
            O += (double)d;
            const float4 q = *reinterpret_cast<const float4*>(&sm.rvec[buf][c4]);
            const float ub[4] = {q.x - d, q.y - d, q.z - d, q.w - d};
            const float K = feasible ? (float)(oa[slot] + O - lz2) + kappa : LCCRF_NEG_INF;
            float uaK[ITEMS];
#pragma unroll
            for (int k = 0; k < ITEMS; ++k) uaK[k] = aux[slot][k] + K;
            bwd_step<G, true, ALIGNED>(sm, buf, tid, c4, r0, T, ring[slot], ub, uaK, mub + (size_t)i * TT, refill);
            buf ^= 1;
        });
        // position 0: p(y_0 = t) = softmax_t(alpha_0(t) + beta_0(t)) in row 0, zeros elsewhere
        for (int k = T + tid; k < (int)TT; k += G::W) mub[k] = 0.f;
        if (tid < 64) {
            float m = LCCRF_NEG_INF;
            for (int t = tid; t < T; t += 64) m = fmaxf(m, a.ua[vb * T + t] + sm.rvec[buf][t]);
            m = xor_max<1, 64>(m);
            float S = 0.f;
            for (int t = tid; t < T; t += 64) S += ex2(a.ua[vb * T + t] + sm.rvec[buf][t] - finite_or_zero(m));
            S = xor_sum<1, 64>(S);
            const float c = (feasible && S > 0.f) ? 1.0f / S : 0.f;
            for (int t = tid; t < T; t += 64)
                mub[t] = c * ex2(a.ua[vb * T + t] + sm.rvec[buf][t] - finite_or_zero(m));
        }
    }
}

// logZ alone: combine the two stored mid-point vectors.  One wave per sequence.
__global__ __launch_bounds__(64) void logz_combine_kernel(ChainArgs a) {
    const int b = blockIdx.x, lane = threadIdx.x;
    const int N = a.N, T = a.T;
    const int L = clamp_length(a.lengths, b, N);
    if (L == 0) {
        if (lane == 0) a.logZ[b] = 0.f;
        return;
    }
    const int h = L / 2;
    const size_t vb = (size_t)b * N;
    const float* ua = a.ua + (vb + h) * T;
    const float* ub = a.ub + (vb + h) * T;
    float m = LCCRF_NEG_INF;
    for (int t = lane; t < T; t += 64) m = fmaxf(m, ua[t] + ub[t]);
    m = xor_max<1, 64>(m);
    const float g = finite_or_zero(m);
    float S = 0.f;
    for (int t = lane; t < T; t += 64) S += ex2(ua[t] + ub[t] - g);
    S = xor_sum<1, 64>(S);
    if (lane == 0) a.logZ[b] = (float)(((double)(m + lg2(S)) + a.Oa[vb + h] + a.Ob[vb + h]) * kLn2);
}

// ---------------------------------------------------------------------------------------
// Host-side dispatch.
template <typename G, typename TIN, bool ALIGNED, int PF1, int PF2>
static hipError_t launch_geo(int op, const ChainArgs& a, hipStream_t st, hipEvent_t between) {
    hipLaunchKernelGGL((chain_half_kernel<G, TIN, ALIGNED, PF1>), dim3(2 * a.B), dim3(G::W), 0, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (between) {
        e = hipEventRecord(between, st);
        if (e != hipSuccess) return e;
    }
    if (op == 0) {
        hipLaunchKernelGGL(logz_combine_kernel, dim3(a.B), dim3(64), 0, st, a);
    } else {
        hipLaunchKernelGGL((chain_marginal_kernel<G, TIN, ALIGNED, PF2>), dim3(2 * a.B), dim3(G::W), 0, st, a);
    }
    return hipGetLastError();
}

template <typename TIN, bool ALIGNED>
static hipError_t launch_T(int op, const ChainArgs& a, hipStream_t st, hipEvent_t between) {
    const int T = a.T;
    if (T <= 4) return launch_geo<Geo<1, 1, 1>, TIN, ALIGNED, 4, 4>(op, a, st, between);
    if (T <= 8) return launch_geo<Geo<2, 1, 1>, TIN, ALIGNED, 4, 4>(op, a, st, between);
    if (T <= 16) return launch_geo<Geo<4, 1, 1>, TIN, ALIGNED, 4, 4>(op, a, st, between);
    if (T <= 32) return launch_geo<Geo<8, 4, 1>, TIN, ALIGNED, 4, 4>(op, a, st, between);
    if (T <= 64) return launch_geo<Geo<16, 4, 4>, TIN, ALIGNED, 4, 3>(op, a, st, between);
    if (T <= 128) return launch_geo<Geo<32, 16, 4>, TIN, ALIGNED, 4, 3>(op, a, st, between);
    return launch_geo<Geo<64, 16, 16>, TIN, ALIGNED, 1, 1>(op, a, st, between);
}

// op: 0 = logZ only, 1 = marginals (+ logZ).  Workspace pointers already carved by the caller.
hipError_t launch_sequential_sum(int op, int dtype, const void* phi, const int32_t* lengths, int B, int N, int T,
                                 float* ua, float* ub, double* Oa, double* Ob, float* logZ, float* mu,
                                 hipStream_t st, hipEvent_t between) {
    ChainArgs a{phi, lengths, B, N, T, ua, ub, Oa, Ob, logZ, mu};
    const bool aligned = (T % 4) == 0;
    if (dtype == 0)
        return aligned ? launch_T<float, true>(op, a, st, between) : launch_T<float, false>(op, a, st, between);
    return aligned ? launch_T<uint16_t, true>(op, a, st, between) : launch_T<uint16_t, false>(op, a, st, between);
}

}  // namespace lccrf
