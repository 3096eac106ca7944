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
// max(u) = 0 after every step, so magnitudes stay small however long the chain is; -inf
// entries are neutral.  Every step is first tried with ONE shift for the whole matrix, the
// previous step's normaliser (potentials of neighbouring positions are on the same scale,
// so it predicts this step's): one fma, one exp and one add per potential and plain sums to
// merge.  The step is accepted only if every sum it produced lies in [2^-60, 2^60] - then no
// term that matters can have overflowed or been flushed - and is otherwise replayed on the
// same registers by the exact step, whose every log-sum-exp is shifted by its own maximum
// (partial sums carry their maximum and are rescaled when merged).  The marginals of
// a position must sum to one; the sum actually written at one step is fed back as a
// correction (kappa) to the next, so rounding drift between the forward and the backward
// offsets (a random walk over thousands of float32 steps) never builds up in the output.
#include "lccrf_chain_args.h"
#include "lccrf_chain_smem.h"
#include "lccrf_device.h"
#include "lccrf_launch.h"

namespace lccrf {

// Tiles arrive with clamped addresses: entries outside the T x T matrix hold finite copies of
// in-range data.  They never reach a result: rows s >= T carry ua = -inf (forward) or are
// dropped when the row result is published (backward); columns t >= T carry ub = -inf
// (backward) or are dropped by the column thread (forward); their marginals are not stored
// and enter the marginal sum with weight 0.

// ----- forward: r(t) = log2 sum_s 2^(ua(s) + phi2(s,t)) ----------------------------------

// Speculative step with the uniform shift c.  Leaves v untouched.  Sets sm.bad[flag] if a
// column sum left the accepted range.
template <typename G, bool WITH_MU, bool ALIGNED>
__device__ __forceinline__ void fwd_fast(ChainSmem<G>& sm, int buf, int flag, int tid, int c4, int r0, int T,
                                         const float (&v)[G::ITEMS][4], const float (&ua)[G::ITEMS], float c,
                                         const float (&ubK)[4], float* __restrict__ mu_out) {
    constexpr int ITEMS = G::ITEMS;
    const int lane = tid & 63, wave = tid >> 6;
    float ls[4] = {0.f, 0.f, 0.f, 0.f}, gm[4] = {0.f, 0.f, 0.f, 0.f};
    if (WITH_MU) {
#pragma unroll
        for (int j = 0; j < 4; ++j) gm[j] = ex2(c + ubK[j]);
    }
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) {
        const float uac = ua[k] - c;
        float e[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            e[j] = ex2(__builtin_fmaf(v[k][j], kLog2e, uac));
            ls[j] += e[j];
        }
        if (WITH_MU) store4<ALIGNED, (G::TCAP > 64)>(mu_out, T, r0 + k * G::RPP, c4, e[0] * gm[0], e[1] * gm[1], e[2] * gm[2], e[3] * gm[3]);
    }
    if (WITH_MU) {
        float tot = (ls[0] * gm[0] + ls[1] * gm[1]) + (ls[2] * gm[2] + ls[3] * gm[3]);
        tot = xor_sum<1, 64>(tot);
        if (lane == 0) sm.wtot[buf ^ 1][wave] = tot;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) ls[j] = xor_sum<G::LPR, 64>(ls[j]);
    if (lane < G::LPR) *reinterpret_cast<float4*>(&sm.psum[wave][c4]) = make_float4(ls[0], ls[1], ls[2], ls[3]);
    __syncthreads();
    if (wave < G::COLWAVES) {
        float r = LCCRF_NEG_INF;
        bool ok = true;
        if (tid < T) {
            float S = 0.f;
#pragma unroll
            for (int w = 0; w < G::WAVES; ++w) S += sm.psum[w][tid];
            r = c + lg2(S);
            ok = sum_in_range(S);
        }
        if (tid < G::TCAP) sm.rvec[buf ^ 1][tid] = r;
        const float wm = xor_max<1, 64>(r);
        if (lane == 0) sm.wmax[buf ^ 1][wave] = wm;
        if (!__all(ok) && lane == 0) sm.bad[flag] = 1;
    }
    __syncthreads();
}

// Exact step: a single sweep with thread-local shifts.  Each thread takes the maximum of its
// own ITEMS rows per column and exponentiates against it; the (maximum, sum) pairs are merged
// exactly, first across the row groups of the wave, then across waves by one thread per
// column.  Turns the tile into x = ua(s) + phi2(s,t) in place.
template <typename G, bool WITH_MU, bool ALIGNED>
__device__ __forceinline__ void fwd_exact(ChainSmem<G>& sm, int buf, int tid, int c4, int r0, int T,
                                          float (&v)[G::ITEMS][4], const float (&ua)[G::ITEMS],
                                          const float (&ubK)[4], float* __restrict__ mu_out) {
    constexpr int ITEMS = G::ITEMS;
    const int lane = tid & 63, wave = tid >> 6;
    float (&x)[ITEMS][4] = v;
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
        if (WITH_MU) store4<ALIGNED, (G::TCAP > 64)>(mu_out, T, r0 + k * G::RPP, c4, e[0] * gm[0], e[1] * gm[1], e[2] * gm[2], e[3] * gm[3]);
    }
    if (WITH_MU) {
        float tot = (ls[0] * gm[0] + ls[1] * gm[1]) + (ls[2] * gm[2] + ls[3] * gm[3]);
        tot = xor_sum<1, 64>(tot);
        if (lane == 0) sm.wtot[buf ^ 1][wave] = tot;
    }
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
    if (wave < G::COLWAVES) {
        float r = LCCRF_NEG_INF;
        if (tid < T) {
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
        if (tid < G::TCAP) sm.rvec[buf ^ 1][tid] = r;
        const float wm = xor_max<1, 64>(r);
        if (lane == 0) sm.wmax[buf ^ 1][wave] = wm;
    }
    __syncthreads();
}

// ----- backward: r(s) = log2 sum_t 2^(phi2(s,t) + ub(t)) ---------------------------------
// The LPR lanes of a row sit in one wave: row sums (and, in the exact step, row maxima) are
// all-reduced across them with LDS-free lane exchanges, so a step needs a single barrier.

template <typename G, bool WITH_MU, bool ALIGNED>
__device__ __forceinline__ void bwd_fast(ChainSmem<G>& sm, int buf, int flag, int tid, int c4, int r0, int T,
                                         const float (&v)[G::ITEMS][4], const float (&ub)[4], float c,
                                         const float (&uaK)[G::ITEMS], float* __restrict__ mu_out) {
    constexpr int ITEMS = G::ITEMS;
    const int lane = tid & 63, wave = tid >> 6;
    const float ubc[4] = {ub[0] - c, ub[1] - c, ub[2] - c, ub[3] - c};
    float S[ITEMS];
    float tot = 0.f;
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) {
        float e[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) e[j] = ex2(__builtin_fmaf(v[k][j], kLog2e, ubc[j]));
        S[k] = (e[0] + e[1]) + (e[2] + e[3]);
        if (WITH_MU) {
            const float f = ex2(c + uaK[k]);
            store4<ALIGNED, (G::TCAP > 64)>(mu_out, T, r0 + k * G::RPP, c4, e[0] * f, e[1] * f, e[2] * f, e[3] * f);
            tot += S[k] * f;
        }
    }
    float wm = LCCRF_NEG_INF;
    bool ok = true;
    if constexpr (ITEMS % 4 == 0 && G::LPR >= 16) {
        // four rows at a time: each lane ends up with the complete sum of one of them
        const int kk = 2 * (lane & 1) + ((lane >> 1) & 1);
#pragma unroll
        for (int k0 = 0; k0 < ITEMS; k0 += 4) {
            const float Sk = reduce4_over_lanes<G::LPR>(S[k0], S[k0 + 1], S[k0 + 2], S[k0 + 3], lane);
            const int s = r0 + (k0 + kk) * G::RPP;
            const float r = (s < T) ? c + lg2(Sk) : LCCRF_NEG_INF;
            if ((tid % G::LPR) < 4 && s < T) sm.rvec[buf ^ 1][s] = r;
            ok = ok && (s >= T || sum_in_range(Sk));
            wm = fmaxf(wm, r);
        }
        wm = xor_max<1, 4>(wm);
    } else {
#pragma unroll
        for (int k = 0; k < ITEMS; ++k) {
            const float Sk = xor_sum<1, G::LPR>(S[k]);
            const int s = r0 + k * G::RPP;
            const float r = (s < T) ? c + lg2(Sk) : LCCRF_NEG_INF;
            if (c4 == 0 && s < T) sm.rvec[buf ^ 1][s] = r;
            ok = ok && (s >= T || sum_in_range(Sk));
            wm = fmaxf(wm, r);
        }
    }
    wm = xor_max<G::LPR, 64>(wm);  // lanes of other row groups hold other rows' results
    if (lane == 0) sm.wmax[buf ^ 1][wave] = wm;
    if (!__all(ok) && lane == 0) sm.bad[flag] = 1;
    if (WITH_MU) {
        tot = xor_sum<1, 64>(tot);
        if (lane == 0) sm.wtot[buf ^ 1][wave] = tot;
    }
    __syncthreads();
}

// Exact step: row maximum first, then the sum against it.  Turns the tile into
// y = phi2(s,t) + ub(t) in place.
template <typename G, bool WITH_MU, bool ALIGNED>
__device__ __forceinline__ void bwd_exact(ChainSmem<G>& sm, int buf, int tid, int c4, int r0, int T,
                                          float (&v)[G::ITEMS][4], const float (&ub)[4],
                                          const float (&uaK)[G::ITEMS], float* __restrict__ mu_out) {
    constexpr int ITEMS = G::ITEMS;
    const int lane = tid & 63, wave = tid >> 6;
    float (&y)[ITEMS][4] = v;
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
            const float f = ex2(g + uaK[k]);
            store4<ALIGNED, (G::TCAP > 64)>(mu_out, T, r0 + k * G::RPP, c4, e[0] * f, e[1] * f, e[2] * f, e[3] * f);
            tot += S[k] * f;
        }
    }
    float wm = LCCRF_NEG_INF;
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) {
        const int s = r0 + k * G::RPP;
        const float r = (s < T) ? m[k] + lg2(xor_sum<1, G::LPR>(S[k])) : LCCRF_NEG_INF;
        if (c4 == 0 && s < T) sm.rvec[buf ^ 1][s] = r;
        wm = fmaxf(wm, r);
    }
    wm = xor_max<G::LPR, 64>(wm);
    if (lane == 0) sm.wmax[buf ^ 1][wave] = wm;
    if (WITH_MU) {
        tot = xor_sum<1, 64>(tot);
        if (lane == 0) sm.wtot[buf ^ 1][wave] = tot;
    }
    __syncthreads();
}

// One position of a forward chain: speculative step, exact replay if it was rejected.
template <typename G, bool WITH_MU, bool ALIGNED>
__device__ __forceinline__ void fwd_advance(ChainSmem<G>& sm, int& buf, int& nstep, bool exact_only, int tid, int c4,
                                            int r0, int T, float (&v)[G::ITEMS][4], const float (&ua)[G::ITEMS],
                                            float c, const float (&ubK)[4], float* __restrict__ mu_out) {
    // 64 potentials a thread and tile (T > 128), second pass: the speculative step would have to
    // keep the tile intact beside its own values and the marginals' factors for a possible replay,
    // which does not fit the registers; the exact step works in place.
    if constexpr (G::ITEMS >= 16 && WITH_MU) exact_only = true;
    bool replay = exact_only;
    if (!exact_only) {
        const int flag = nstep & 3;
        if (tid == 0) sm.bad[(nstep + 1) & 3] = 0;
        fwd_fast<G, WITH_MU, ALIGNED>(sm, buf, flag, tid, c4, r0, T, v, ua, c, ubK, mu_out);
        replay = sm.bad[flag] != 0;
    }
    if (replay) fwd_exact<G, WITH_MU, ALIGNED>(sm, buf, tid, c4, r0, T, v, ua, ubK, mu_out);
    buf ^= 1;
    ++nstep;
}

template <typename G, bool WITH_MU, bool ALIGNED>
__device__ __forceinline__ void bwd_advance(ChainSmem<G>& sm, int& buf, int& nstep, bool exact_only, int tid, int c4,
                                            int r0, int T, float (&v)[G::ITEMS][4], const float (&ub)[4], float c,
                                            const float (&uaK)[G::ITEMS], float* __restrict__ mu_out) {
    if constexpr (G::ITEMS >= 16 && WITH_MU) exact_only = true;  // as in fwd_advance
    bool replay = exact_only;
    if (!exact_only) {
        const int flag = nstep & 3;
        if (tid == 0) sm.bad[(nstep + 1) & 3] = 0;
        bwd_fast<G, WITH_MU, ALIGNED>(sm, buf, flag, tid, c4, r0, T, v, ub, c, uaK, mu_out);
        replay = sm.bad[flag] != 0;
    }
    if (replay) bwd_exact<G, WITH_MU, ALIGNED>(sm, buf, tid, c4, r0, T, v, ub, uaK, mu_out);
    buf ^= 1;
    ++nstep;
}

// ---------------------------------------------------------------------------------------
// Forward half chain for 32 < T <= 128 with the tile turned through LDS memory.
//
// With rows spread over all waves, the forward step has to merge the waves' partial column sums
// through LDS behind a second barrier while all but the column waves wait.  Here every tile is written
// to LDS as it arrives (coalesced rows, one position ahead of its use) and read back so that a wave
// owns 256 / LPR complete columns (8 of 128 with sixteen waves, 16 of 64 with four): the sum over rows
// never leaves the wave, the step has one barrier like the backward step, and the exact replay needs
// no cross-wave merge either.
// Lane l of wave w holds rows (l % LPR) + LPR k, k < 4, of columns (256 / LPR) w + 4 (l / LPR) + j, j < 4.
template <typename G, bool ALIGNED, int PF>
constexpr bool half_turns() {
    return ((G::LPR == 32 && G::WAVES == 16) || (G::LPR == 16 && G::WAVES == 4)) && G::ITEMS == 4 && PF == 4;
}
// LDS floats of the two turned tiles of geometry G: TCAP rows of TCAP + 4 floats each (the padding keeps 16-byte
// accesses free of bank conflicts).
template <typename G>
constexpr int turn_floats() { return 2 * G::TCAP * (G::TCAP + 4); }

template <typename G, typename TIN, int PF, bool ALIGNED>
__device__ __forceinline__ void forward_half_turned(ChainSmem<G>& sm, float* __restrict__ tiles, const ChainArgs& a,
                                                    const Span& sp, int tid) {
    static_assert(G::ITEMS == 4 && PF == 4 && G::LPR * 4 == G::TCAP && G::WAVES * (256 / G::LPR) == G::TCAP,
                  "a wave owns 256 / LPR whole columns, a lane four rows LPR apart");
    constexpr int LPR = G::LPR, ROWS = G::TCAP, STRIDE = G::TCAP + 4;
    const int lane = tid & 63, wave = tid >> 6;
    const int b = sp.b, N = a.N, T = a.T;
    const int p0 = sp.p0, h = forward_end(a, sp.p0, sp.e);
    const int c4 = 4 * (tid % LPR), r0 = tid / LPR;
    const size_t TT = (size_t)T * T, vb = (size_t)b * N;
    const TIN* phib = static_cast<const TIN*>(a.phi) + (size_t)b * N * TT;
    const bool exact_only = a.exact_only != 0;
    const int rowl = lane % LPR, colw = (256 / LPR) * wave + 4 * (lane / LPR);
    const int kk = 2 * (lane & 1) + ((lane >> 1) & 1);  // the column reduce4_over_lanes leaves in this lane

    double O = 0.0;
    {
        float v0 = LCCRF_NEG_INF;
        if (tid < T) v0 = sp.first ? Elem<TIN>::get(phib + tid) * kLog2e : a.Fv[((size_t)b * a.C + sp.c - 1) * T + tid];
        if (!sp.first) O = a.OF[(size_t)b * a.C + sp.c - 1];
        publish_columns<G>(sm, 0, tid, v0);
    }
    const int first = p0 + 1, n = h - p0;  // positions first .. h
    int buf = 0, nstep = 0;
    if (n > 0) {
        float ring[PF][4][4];
        auto load = [&](int i, int slot) { load_tile<G, TIN, ALIGNED>(phib + (size_t)i * TT, T, c4, r0, ring[slot], b != a.B - 1 || i != N - 1); };
        auto to_lds = [&](int slot, int wb) {
            settle_tile<G, ALIGNED>(ring[slot], T, c4);
#pragma unroll
            for (int k = 0; k < 4; ++k)
                *reinterpret_cast<float4*>(&tiles[(wb * ROWS + r0 + LPR * k) * STRIDE + c4]) =
                    make_float4(ring[slot][k][0], ring[slot][k][1], ring[slot][k][2], ring[slot][k][3]);
        };
#pragma unroll
        for (int p = 0; p < PF; ++p) load(first + (p < n ? p : n - 1), p);
        to_lds(0, 0);
        load(first + (PF < n ? PF : n - 1), 0);
        __syncthreads();
        int done = 0;
        bool running = true;
        while (running) {
#pragma unroll
            for (int p = 0; p < PF; ++p) {
                const int i = first + done;
                const int rb = p & 1, nslot = (p + 1) % PF;
                // this wave's columns of tile i, four rows at a time
                const float* mine = &tiles[(rb * ROWS + rowl) * STRIDE + colw];
                const float d = read_shift<G>(sm, buf);
                O += (double)d;
                float ua[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) ua[k] = sm.rvec[buf][rowl + LPR * k] - d;  // -inf for rows >= T
                if (tid < T) a.ua[(vb + i - 1) * T + tid] = sm.rvec[buf][tid] - d;
                if (tid == 0) a.Oa[vb + i - 1] = O;
                // tile i + 1 goes to the other LDS buffer; its ring slot takes tile i + 1 + PF
                to_lds(nslot, nslot & 1);
                {
                    const int ahead = done + 1 + PF;
                    load(first + (ahead < n ? ahead : n - 1), nslot);
                }
                const int flag = nstep & 3;
                if (tid == 0) sm.bad[(nstep + 1) & 3] = 0;
                if (!exact_only) {
                    float ls[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const float uac = ua[k] - d;  // shift c = d, the previous normaliser
                        const float4 q = *reinterpret_cast<const float4*>(mine + LPR * k * STRIDE);
                        ls[0] += ex2(__builtin_fmaf(q.x, kLog2e, uac));
                        ls[1] += ex2(__builtin_fmaf(q.y, kLog2e, uac));
                        ls[2] += ex2(__builtin_fmaf(q.z, kLog2e, uac));
                        ls[3] += ex2(__builtin_fmaf(q.w, kLog2e, uac));
                    }
                    const float S = reduce4_over_lanes<LPR>(ls[0], ls[1], ls[2], ls[3], lane);
                    const int col = colw + kk;
                    const float r = (col < T) ? d + lg2(S) : LCCRF_NEG_INF;
                    if (rowl < 4) sm.rvec[buf ^ 1][col] = r;
                    const float wm = xor_max<LPR, 64>(xor_max<1, 4>(r));
                    if (lane == 0) sm.wmax[buf ^ 1][wave] = wm;
                    const bool ok = col >= T || sum_in_range(S);
                    if (!__all(ok) && lane == 0) sm.bad[flag] = 1;
                    __syncthreads();
                }
                if (exact_only || sm.bad[flag] != 0) {
                    // exact step: every log-sum-exp against its own maximum, all inside the wave
                    float v[4][4];
                    float lm[4] = {LCCRF_NEG_INF, LCCRF_NEG_INF, LCCRF_NEG_INF, LCCRF_NEG_INF};
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const float4 q = *reinterpret_cast<const float4*>(mine + LPR * k * STRIDE);
                        v[k][0] = __builtin_fmaf(q.x, kLog2e, ua[k]);
                        v[k][1] = __builtin_fmaf(q.y, kLog2e, ua[k]);
                        v[k][2] = __builtin_fmaf(q.z, kLog2e, ua[k]);
                        v[k][3] = __builtin_fmaf(q.w, kLog2e, ua[k]);
#pragma unroll
                        for (int j = 0; j < 4; ++j) lm[j] = fmaxf(lm[j], v[k][j]);
                    }
                    float r[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float M = xor_max<1, LPR>(lm[j]);
                        const float g = finite_or_zero(M);
                        float Sl = 0.f;
#pragma unroll
                        for (int k = 0; k < 4; ++k) Sl += ex2(v[k][j] - g);
                        r[j] = (colw + j < T) ? M + lg2(xor_sum<1, LPR>(Sl)) : LCCRF_NEG_INF;
                    }
                    __syncthreads();  // nobody still reads the rejected vector
                    if (rowl == 0) *reinterpret_cast<float4*>(&sm.rvec[buf ^ 1][colw]) = make_float4(r[0], r[1], r[2], r[3]);
                    const float wm = xor_max<LPR, 64>(fmaxf(fmaxf(r[0], r[1]), fmaxf(r[2], r[3])));
                    if (lane == 0) sm.wmax[buf ^ 1][wave] = wm;
                    __syncthreads();
                }
                buf ^= 1;
                ++nstep;
                if (++done >= n) { running = false; break; }
            }
        }
    } else {
        __syncthreads();
    }
    const float d = read_shift<G>(sm, buf);
    O += (double)d;
    if (tid < T) a.ua[(vb + h) * T + tid] = sm.rvec[buf][tid] - d;
    if (tid == 0) a.Oa[vb + h] = O;
}

// The forward chain of the second pass in the same turned form (four-wave geometry, 32 < T <= 64):
// it continues alpha past the meeting point and writes the marginals of positions h + 1 .. e.  Measured on
// 128 ragged sequences of 48 tags this chain, with its second barrier a step, was what the second pass waited
// for (82 us alone against 65 us for the backward chain alone).  A lane writes the marginals of its four rows
// of four columns; the sixteen lanes of a column quad cover sixteen consecutive rows.
template <typename G, bool ALIGNED>
constexpr bool marginal_turns() { return G::LPR == 16 && G::WAVES == 4 && G::ITEMS == 4; }

template <typename G, typename TIN, bool ALIGNED>
__device__ __forceinline__ void forward_marginal_turned(ChainSmem<G>& sm, float* __restrict__ tiles, const ChainArgs& a,
                                                        const Span& sp, int tid, double lz2, bool feasible) {
    constexpr int PF = 4, LPR = G::LPR, ROWS = G::TCAP, STRIDE = G::TCAP + 4;
    static_assert(G::ITEMS == 4 && G::LPR * 4 == G::TCAP && G::WAVES * (256 / G::LPR) == G::TCAP, "as forward_half_turned");
    const int lane = tid & 63, wave = tid >> 6;
    const int b = sp.b, N = a.N, T = a.T;
    const int e = sp.e, h = meeting_point(sp.p0, sp.e);
    const int c4 = 4 * (tid % LPR), r0 = tid / LPR;
    const size_t TT = (size_t)T * T, vb = (size_t)b * N;
    const TIN* phib = static_cast<const TIN*>(a.phi) + (size_t)b * N * TT;
    float* mub = a.mu + (size_t)b * N * TT;
    const bool exact_only = a.exact_only != 0;
    const int rowl = lane % LPR, colw = (256 / LPR) * wave + 4 * (lane / LPR);
    const int colc = colw < T ? colw : (ALIGNED ? T - 4 : 0);  // (clamped: where the stored backward vector is read)
    const int kk = 2 * (lane & 1) + ((lane >> 1) & 1);  // the column reduce4_over_lanes leaves in this lane

    double O = a.Oa[vb + h];
    publish_columns<G>(sm, 0, tid, (tid < T) ? a.ua[(vb + h) * T + tid] : LCCRF_NEG_INF);
    const int first = h + 1, n = e - h;  // positions first .. e
    if (n <= 0) return;
    float kappa = 0.f;
    int buf = 0, nstep = 0;
    float ring[PF][4][4], aux[PF][4];
    double ob[PF];
    auto load = [&](int i, int slot) { load_tile<G, TIN, ALIGNED>(phib + (size_t)i * TT, T, c4, r0, ring[slot], b != a.B - 1 || i != N - 1); };
    auto load_aux = [&](int i, int slot) {  // beta_i of this lane's columns and its offset
        if constexpr (ALIGNED) {
            Elem<float>::get4(a.ub + (vb + i) * T + colc, aux[slot]);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) aux[slot][j] = a.ub[(vb + i) * T + (colc + j < T ? colc + j : colc)];
        }
        ob[slot] = a.Ob[vb + i];
    };
    auto to_lds = [&](int slot, int wb) {
        settle_tile<G, ALIGNED>(ring[slot], T, c4);
#pragma unroll
        for (int k = 0; k < 4; ++k)
            *reinterpret_cast<float4*>(&tiles[(wb * ROWS + r0 + LPR * k) * STRIDE + c4]) =
                make_float4(ring[slot][k][0], ring[slot][k][1], ring[slot][k][2], ring[slot][k][3]);
    };
#pragma unroll
    for (int p = 0; p < PF; ++p) {
        load(first + (p < n ? p : n - 1), p);
        load_aux(first + (p < n ? p : n - 1), p);
    }
    to_lds(0, 0);
    load(first + (PF < n ? PF : n - 1), 0);
    __syncthreads();
    int done = 0;
    bool running = true;
    while (running) {
#pragma unroll
        for (int p = 0; p < PF; ++p) {
            const int i = first + done;
            const int rb = p & 1, nslot = (p + 1) % PF;
            const float* mine = &tiles[(rb * ROWS + rowl) * STRIDE + colw];
            float* mu_out = mub + (size_t)i * TT;
            const float d = read_shift<G>(sm, buf);
            kappa += read_drift<G>(sm, buf);
            O += (double)d;
            float ua[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) ua[k] = sm.rvec[buf][rowl + LPR * k] - d;  // -inf for rows >= T
            const float K = feasible ? (float)(O + ob[p] - lz2) + kappa : LCCRF_NEG_INF;
            float ubK[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) ubK[j] = (colw + j < T) ? aux[p][j] + K : LCCRF_NEG_INF;
            {
                const int ahead = done + PF;
                load_aux(first + (ahead < n ? ahead : n - 1), p);
            }
            // tile i + 1 goes to the other LDS buffer; its ring slot takes tile i + 1 + PF
            to_lds(nslot, nslot & 1);
            {
                const int ahead = done + 1 + PF;
                load(first + (ahead < n ? ahead : n - 1), nslot);
            }
            const int flag = nstep & 3;
            if (tid == 0) sm.bad[(nstep + 1) & 3] = 0;
            if (!exact_only) {
                float ls[4] = {0.f, 0.f, 0.f, 0.f}, gm[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) gm[j] = ex2(d + ubK[j]);
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const float uac = ua[k] - d;  // shift c = d, the previous normaliser
                    const float4 q = *reinterpret_cast<const float4*>(mine + LPR * k * STRIDE);
                    const float e0 = ex2(__builtin_fmaf(q.x, kLog2e, uac)), e1 = ex2(__builtin_fmaf(q.y, kLog2e, uac));
                    const float e2 = ex2(__builtin_fmaf(q.z, kLog2e, uac)), e3 = ex2(__builtin_fmaf(q.w, kLog2e, uac));
                    ls[0] += e0; ls[1] += e1; ls[2] += e2; ls[3] += e3;
                    store4<ALIGNED, false>(mu_out, T, rowl + LPR * k, colw, e0 * gm[0], e1 * gm[1], e2 * gm[2], e3 * gm[3]);
                }
                float tot = (ls[0] * gm[0] + ls[1] * gm[1]) + (ls[2] * gm[2] + ls[3] * gm[3]);
                tot = xor_sum<1, 64>(tot);
                if (lane == 0) sm.wtot[buf ^ 1][wave] = tot;
                const float S = reduce4_over_lanes<LPR>(ls[0], ls[1], ls[2], ls[3], lane);
                const int col = colw + kk;
                const float r = (col < T) ? d + lg2(S) : LCCRF_NEG_INF;
                if (rowl < 4) sm.rvec[buf ^ 1][col] = r;
                const float wm = xor_max<LPR, 64>(xor_max<1, 4>(r));
                if (lane == 0) sm.wmax[buf ^ 1][wave] = wm;
                const bool ok = col >= T || sum_in_range(S);
                if (!__all(ok) && lane == 0) sm.bad[flag] = 1;
                __syncthreads();
            }
            if (exact_only || sm.bad[flag] != 0) {
                // exact step: every log-sum-exp against its own maximum, all inside the wave; the marginals again
                float v[4][4];
                float lm[4] = {LCCRF_NEG_INF, LCCRF_NEG_INF, LCCRF_NEG_INF, LCCRF_NEG_INF};
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const float4 q = *reinterpret_cast<const float4*>(mine + LPR * k * STRIDE);
                    v[k][0] = __builtin_fmaf(q.x, kLog2e, ua[k]);
                    v[k][1] = __builtin_fmaf(q.y, kLog2e, ua[k]);
                    v[k][2] = __builtin_fmaf(q.z, kLog2e, ua[k]);
                    v[k][3] = __builtin_fmaf(q.w, kLog2e, ua[k]);
#pragma unroll
                    for (int j = 0; j < 4; ++j) lm[j] = fmaxf(lm[j], v[k][j]);
                }
                float r[4], g[4], gx[4], Sl[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    lm[j] = xor_max<1, LPR>(lm[j]);
                    g[j] = finite_or_zero(lm[j]);
                    gx[j] = ex2(g[j] + ubK[j]);
                }
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    float ex[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        ex[j] = ex2(v[k][j] - g[j]);
                        Sl[j] += ex[j];
                    }
                    store4<ALIGNED, false>(mu_out, T, rowl + LPR * k, colw, ex[0] * gx[0], ex[1] * gx[1], ex[2] * gx[2], ex[3] * gx[3]);
                }
                float tot = (Sl[0] * gx[0] + Sl[1] * gx[1]) + (Sl[2] * gx[2] + Sl[3] * gx[3]);
                tot = xor_sum<1, 64>(tot);
#pragma unroll
                for (int j = 0; j < 4; ++j) r[j] = (colw + j < T) ? lm[j] + lg2(xor_sum<1, LPR>(Sl[j])) : LCCRF_NEG_INF;
                __syncthreads();  // nobody still reads the rejected vector
                if (rowl == 0) *reinterpret_cast<float4*>(&sm.rvec[buf ^ 1][colw]) = make_float4(r[0], r[1], r[2], r[3]);
                const float wm = xor_max<LPR, 64>(fmaxf(fmaxf(r[0], r[1]), fmaxf(r[2], r[3])));
                if (lane == 0) {
                    sm.wmax[buf ^ 1][wave] = wm;
                    sm.wtot[buf ^ 1][wave] = tot;
                }
                __syncthreads();
            }
            buf ^= 1;
            ++nstep;
            if (++done >= n) { running = false; break; }
        }
    }
}

// ---------------------------------------------------------------------------------------
// Pass 1: both half chains, vectors stored, nothing else written.
// STRUCT: potentials are trans + emit (float, T <= 128; a compile-time choice, see lccrf_wave.hip).
template <typename G, typename TIN, bool ALIGNED, int PF, bool STRUCT = false>
__global__ __launch_bounds__(G::W) void chain_half_kernel(ChainArgs a) {
    __shared__ ChainSmem<G> sm;
    constexpr int ITEMS = G::ITEMS;
    const int tid = threadIdx.x;
    const int dir = blockIdx.x & 1;
    const Span sp = make_span(a, blockIdx.x >> 1);
    const int b = sp.b;
    const int N = a.N, T = a.T;
    if (a.pair_mail && dir == 0) {  // the second pass finds its mailboxes and failure flag clean
        for (int k = tid; k < a.pair_words; k += G::W) a.pair_mail[(size_t)b * a.pair_words + k] = 0ull;
        if (tid == 0) a.pair_failed[b] = 0;
    }
    if (sp.empty) return;
    const int p0 = sp.p0, e = sp.e;
    const int h = forward_end(a, p0, e);
    if (a.full_forward && dir == 1) return;
    const int c4 = 4 * (tid % G::LPR), r0 = tid / G::LPR;
    const TIN* phib = static_cast<const TIN*>(a.phi) + (size_t)b * N * T * T;
    const size_t TT = (size_t)T * T;
    const size_t vb = (size_t)b * N;
    const bool exact_only = a.exact_only != 0;

    smem_init<G>(sm, tid);
    __syncthreads();
    if constexpr (half_turns<G, ALIGNED, PF>() && !STRUCT) {  // (structured tiles are formed in registers: nothing to turn)
        if (dir == 0) {
            extern __shared__ __attribute__((aligned(16))) float turn_tiles[];
            forward_half_turned<G, TIN, PF, ALIGNED>(sm, turn_tiles, a, sp, tid);
            return;
        }
    }
    float ring[PF][ITEMS][4];
    const float dummy4[4] = {0.f, 0.f, 0.f, 0.f};
    float dummyI[ITEMS];
#pragma unroll
    for (int k = 0; k < ITEMS; ++k) dummyI[k] = 0.f;
    double O = 0.0;
    int buf = 0, nstep = 0;
    // structured potentials (trans tile in registers, emissions streamed): geometries up to T = 128 only
    constexpr bool CAN_STRUCT = STRUCT;
    constexpr bool structured = STRUCT;
    const float* emb = structured ? a.emit + (size_t)b * N * T : nullptr;
    float tr[CAN_STRUCT ? ITEMS : 1][4];
    if constexpr (CAN_STRUCT) {
        load_tile<G, float, ALIGNED>(a.trans, T, c4, r0, tr);
        settle_tile<G, ALIGNED>(tr, T, c4);
    }
    auto load = [&](int i, int slot) {
        if constexpr (CAN_STRUCT) {
            load_emit4<ALIGNED>(emb + (size_t)i * T, T, c4, ring[slot][0], b != a.B - 1 || i != N - 1);
            return;
        }
        load_tile<G, TIN, ALIGNED>(phib + (size_t)i * TT, T, c4, r0, ring[slot], b != a.B - 1 || i != N - 1);
    };
    auto tile_ready = [&](int slot) {  // turns a slot that holds emissions into the tile
        if constexpr (CAN_STRUCT) {
            settle_emit4<ALIGNED>(ring[slot][0], T, c4);
            add_trans<ITEMS>(ring[slot], tr);
        } else {
            settle_tile<G, ALIGNED>(ring[slot], T, c4);
        }
    };

    if (dir == 0) {
        float v0 = LCCRF_NEG_INF;
        if (tid < T)
            v0 = !sp.first ? a.Fv[((size_t)b * a.C + sp.c - 1) * T + tid]
                 : (structured ? a.trans[tid] + emb[tid] : Elem<TIN>::get(phib + tid)) * kLog2e;
        if (!sp.first) O = a.OF[(size_t)b * a.C + sp.c - 1];
        publish_columns<G>(sm, 0, tid, v0);
        __syncthreads();
        walk<PF>(p0 + 1, h, +1, load, [&](int i, int slot) {
            tile_ready(slot);
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
            fwd_advance<G, false, ALIGNED>(sm, buf, nstep, exact_only, tid, c4, r0, T, ring[slot], ua, d, dummy4, nullptr);
        });
        const float d = read_shift<G>(sm, buf);
        O += (double)d;
        if (tid < T) a.ua[(vb + h) * T + tid] = sm.rvec[buf][tid] - d;
        if (tid == 0) a.Oa[vb + h] = O;
    } else {
        float v0 = LCCRF_NEG_INF;
        if (tid < T) v0 = sp.last ? 0.f : a.Gv[((size_t)b * a.C + sp.c) * T + tid];
        if (!sp.last) O = a.OG[(size_t)b * a.C + sp.c];
        publish_columns<G>(sm, 0, tid, v0);
        __syncthreads();
        walk<PF>(e, h + 1, -1, load, [&](int i, int slot) {
            tile_ready(slot);
            const float d = read_shift<G>(sm, buf);
            O += (double)d;
            const float4 q = *reinterpret_cast<const float4*>(&sm.rvec[buf][c4]);
            const float ub[4] = {q.x - d, q.y - d, q.z - d, q.w - d};
            if (tid < T) a.ub[(vb + i) * T + tid] = sm.rvec[buf][tid] - d;
            if (tid == 0) a.Ob[vb + i] = O;
            bwd_advance<G, false, ALIGNED>(sm, buf, nstep, exact_only, tid, c4, r0, T, ring[slot], ub, d, dummyI, nullptr);
        });
        const float d = read_shift<G>(sm, buf);
        O += (double)d;
        if (tid < T) a.ub[(vb + h) * T + tid] = sm.rvec[buf][tid] - d;
        if (tid == 0) a.Ob[vb + h] = O;
    }
}

// ---------------------------------------------------------------------------------------
// Pass 2: both chains continue past the meeting point and write the marginals.
template <typename G, typename TIN, bool ALIGNED, int PF, bool STRUCT = false>
__global__ __launch_bounds__(G::W) void chain_marginal_kernel(ChainArgs a) {
    __shared__ ChainSmem<G> sm;
    constexpr int ITEMS = G::ITEMS;
    const int tid = threadIdx.x;
    const int dir = blockIdx.x & 1;
    const Span sp = make_span(a, blockIdx.x >> 1);
    const int b = sp.b;
    const int N = a.N, T = a.T;
    const int L = sp.L;
    const size_t TT = (size_t)T * T;
    const size_t vb = (size_t)b * N;
    float* mub = a.mu + (size_t)b * N * TT;
    const bool exact_only = a.exact_only != 0;
    if (a.only_failed && a.only_failed[b] == 0) return;  // the paired pass has done this sequence

    if (dir == 0) {
        // positions past the end carry no edge: their marginals are zero (a chunk clears its own range)
        const int zfrom = a.chunk > 0 ? (sp.c * a.chunk > L ? sp.c * a.chunk : L) : L;
        const int zto = a.chunk > 0 ? ((sp.c + 1) * a.chunk < N ? (sp.c + 1) * a.chunk : N) : N;
        const size_t z0 = (size_t)zfrom * TT, z1 = (size_t)(zto > zfrom ? zto : zfrom) * TT;
        if (ALIGNED) {
            float4* p = reinterpret_cast<float4*>(mub);
            for (size_t k = z0 / 4 + tid; k < z1 / 4; k += G::W) p[k] = make_float4(0.f, 0.f, 0.f, 0.f);
        } else {
            for (size_t k = z0 + tid; k < z1; k += G::W) mub[k] = 0.f;
        }
    }
    if (L == 0) {
        if (dir == 0 && sp.c == 0 && tid == 0 && a.logZ) a.logZ[b] = 0.f;
        return;
    }
    if (sp.empty) return;
    const int p0 = sp.p0, e = sp.e;
    const int h = meeting_point(p0, e);
    const int c4 = 4 * (tid % G::LPR), r0 = tid / G::LPR;
    const TIN* phib = static_cast<const TIN*>(a.phi) + (size_t)b * N * TT;

    smem_init<G>(sm, tid);
    const double lz2 = midpoint_log2z<G>(sm, a, vb, h, T, tid);
    const bool feasible = lz2 > -1.0e300;  // false: no path has a finite score, marginals are 0
    if (dir == 0 && sp.c == 0 && tid == 0 && a.logZ) a.logZ[b] = (float)(lz2 * kLn2);

    if constexpr (marginal_turns<G, ALIGNED>() && !STRUCT) {
        if (dir == 0) {
            extern __shared__ __attribute__((aligned(16))) float turn_tiles[];
            forward_marginal_turned<G, TIN, ALIGNED>(sm, turn_tiles, a, sp, tid, lz2, feasible);
            return;
        }
    }
    float ring[PF][ITEMS][4];
    int buf = 0, nstep = 0;
    float kappa = 0.f;  // running correction that keeps each position's marginals summing to one
    constexpr bool CAN_STRUCT = STRUCT;
    constexpr bool structured = STRUCT;
    const float* emb = structured ? a.emit + (size_t)b * N * T : nullptr;
    float tr[CAN_STRUCT ? ITEMS : 1][4];
    if constexpr (CAN_STRUCT) {
        load_tile<G, float, ALIGNED>(a.trans, T, c4, r0, tr);
        settle_tile<G, ALIGNED>(tr, T, c4);
    }
    auto load_phi = [&](int i, int slot) {
        if constexpr (CAN_STRUCT) {
            load_emit4<ALIGNED>(emb + (size_t)i * T, T, c4, ring[slot][0], b != a.B - 1 || i != N - 1);
            return;
        }
        load_tile<G, TIN, ALIGNED>(phib + (size_t)i * TT, T, c4, r0, ring[slot], b != a.B - 1 || i != N - 1);
    };
    auto tile_ready = [&](int slot) {
        if constexpr (CAN_STRUCT) {
            settle_emit4<ALIGNED>(ring[slot][0], T, c4);
            add_trans<ITEMS>(ring[slot], tr);
        } else {
            settle_tile<G, ALIGNED>(ring[slot], T, c4);
        }
    };

    if (dir == 0) {
        double O = a.Oa[vb + h];
        publish_columns<G>(sm, 0, tid, (tid < T) ? a.ua[(vb + h) * T + tid] : LCCRF_NEG_INF);
        __syncthreads();
        float aux[PF][4];
        double ob[PF];
        auto load = [&](int i, int slot) {
            load_phi(i, slot);
#pragma unroll
            for (int j = 0; j < 4; ++j) aux[slot][j] = a.ub[(vb + i) * T + (c4 + j < T ? c4 + j : T - 1)];
            ob[slot] = a.Ob[vb + i];
        };
        walk<PF>(h + 1, e, +1, load, [&](int i, int slot) {
            tile_ready(slot);
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
            float ubK[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) ubK[j] = (c4 + j < T) ? aux[slot][j] + K : LCCRF_NEG_INF;
            fwd_advance<G, true, ALIGNED>(sm, buf, nstep, exact_only, tid, c4, r0, T, ring[slot], ua, d, ubK,
                                          mub + (size_t)i * TT);
        });
    } else {
        double O = a.Ob[vb + h];
        publish_columns<G>(sm, 0, tid, (tid < T) ? a.ub[(vb + h) * T + tid] : LCCRF_NEG_INF);
        __syncthreads();
        float aux[PF][ITEMS];
        double oa[PF];
        auto load = [&](int i, int slot) {
            load_phi(i, slot);
#pragma unroll
            for (int k = 0; k < ITEMS; ++k) {
                const int s = r0 + k * G::RPP;
                aux[slot][k] = a.ua[(vb + i - 1) * T + (s < T ? s : T - 1)];
            }
            oa[slot] = a.Oa[vb + i - 1];
        };
        walk<PF>(h, p0 + 1, -1, load, [&](int i, int slot) {
            tile_ready(slot);
            const float d = read_shift<G>(sm, buf);
            kappa += read_drift<G>(sm, buf);
            O += (double)d;
            const float4 q = *reinterpret_cast<const float4*>(&sm.rvec[buf][c4]);
            const float ub[4] = {q.x - d, q.y - d, q.z - d, q.w - d};
            const float K = feasible ? (float)(oa[slot] + O - lz2) + kappa : LCCRF_NEG_INF;
            float uaK[ITEMS];
#pragma unroll
            for (int k = 0; k < ITEMS; ++k) uaK[k] = (r0 + k * G::RPP < T) ? aux[slot][k] + K : LCCRF_NEG_INF;
            bwd_advance<G, true, ALIGNED>(sm, buf, nstep, exact_only, tid, c4, r0, T, ring[slot], ub, d, uaK,
                                          mub + (size_t)i * TT);
        });
        // position 0: p(y_0 = t) = softmax_t(alpha_0(t) + beta_0(t)) in row 0, zeros elsewhere
        if (!sp.first) return;
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
        if (lane == 0 && a.logZ) a.logZ[b] = 0.f;
        if (lane == 0 && a.logZ64) a.logZ64[b] = 0.0;
        return;
    }
    const int h = meeting_point(0, L - 1);
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
    const double lz = ((double)(m + lg2(S)) + a.Oa[vb + h] + a.Ob[vb + h]) * kLn2;
    if (lane == 0 && a.logZ) a.logZ[b] = (float)lz;
    if (lane == 0 && a.logZ64) a.logZ64[b] = lz;
}

// ---------------------------------------------------------------------------------------
// Host-side dispatch.
struct PairPlan {
    unsigned long long* mail;
    int* failed;
    int dtype;
    int poll_limit;
};

template <typename G, typename TIN, bool ALIGNED, int PF1, int PF2>
static hipError_t launch_geo(int op, ChainArgs a, hipStream_t st, hipEvent_t between, const PairPlan& pair) {
    hipError_t e = hipSuccess;
    size_t turn_bytes = 0;
    if constexpr (half_turns<G, ALIGNED, PF1>()) {
        turn_bytes = turn_floats<G>() * sizeof(float);
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&chain_half_kernel<G, TIN, ALIGNED, PF1>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)turn_bytes);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((chain_half_kernel<G, TIN, ALIGNED, PF1>), dim3(2 * a.B * a.C), dim3(G::W), turn_bytes, st, a);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (between) {
        e = hipEventRecord(between, st);
        if (e != hipSuccess) return e;
    }
    if (op == 2) return hipSuccess;  // first pass only
    if (op == 0) {
        hipLaunchKernelGGL(logz_combine_kernel, dim3(a.B), dim3(64), 0, st, a);
        return hipGetLastError();
    }
    if (pair.mail) {
        // two workgroups per chain, speculative steps only; whatever they flag as failed is redone below
        // (the first pass above has cleared the mailboxes and the flags: a.pair_mail)
        e = launch_pair_marginals(pair.dtype, a.phi, a.lengths, a.B, a.N, a.T, a.ua, a.ub, a.Oa, a.Ob, a.logZ, a.mu,
                                  pair.mail, pair.failed, pair.poll_limit, st);
        if (e != hipSuccess) return e;
        a.only_failed = pair.failed;
    }
    size_t turn2_bytes = 0;
    if constexpr (marginal_turns<G, ALIGNED>()) {
        turn2_bytes = turn_floats<G>() * sizeof(float);
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&chain_marginal_kernel<G, TIN, ALIGNED, PF2>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)turn2_bytes);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((chain_marginal_kernel<G, TIN, ALIGNED, PF2>), dim3(2 * a.B * a.C), dim3(G::W), turn2_bytes, st, a);
    return hipGetLastError();
}

// Structured potentials at 32 < T <= 128 (G: the geometry of the dense kernels for that tag count).
template <typename G, bool ALIGNED, int PF2>
static hipError_t launch_structured_geo(int op, const ChainArgs& a, hipStream_t st, hipEvent_t between) {
    hipLaunchKernelGGL((chain_half_kernel<G, float, ALIGNED, 4, true>), dim3(2 * a.B * a.C), dim3(G::W), 0, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (between) {
        e = hipEventRecord(between, st);
        if (e != hipSuccess) return e;
    }
    if (op == 0) {
        hipLaunchKernelGGL(logz_combine_kernel, dim3(a.B), dim3(64), 0, st, a);
        return hipGetLastError();
    }
    hipLaunchKernelGGL((chain_marginal_kernel<G, float, ALIGNED, PF2, true>), dim3(2 * a.B * a.C), dim3(G::W), 0, st, a);
    return hipGetLastError();
}
template <bool ALIGNED>
static hipError_t launch_structured_sum(int op, const ChainArgs& a, hipStream_t st, hipEvent_t between) {
    if (a.T <= 64) return launch_structured_geo<Geo<16, 4, 4>, ALIGNED, 3>(op, a, st, between);
    return launch_structured_geo<Geo<32, 16, 4>, ALIGNED, 2>(op, a, st, between);
}

template <typename TIN, bool ALIGNED>
static hipError_t launch_T(int op, const ChainArgs& a, hipStream_t st, hipEvent_t between, const PairPlan& pair) {
    const int T = a.T;  // T <= 32 is served by the one-wave kernels (launch_wave)
    if (T <= 64) return launch_geo<Geo<16, 4, 4>, TIN, ALIGNED, 4, 3>(op, a, st, between, pair);
    if (T <= 128) return launch_geo<Geo<32, 16, 4>, TIN, ALIGNED, 4, 2>(op, a, st, between, pair);
    return hipErrorInvalidValue;  // larger tag sets take the row-batch kernels (launch_stream)
}

// Both passes with one wave per chain (T <= 32).
static hipError_t launch_wave(int op, int dtype, const ChainArgs& a, hipStream_t st, hipEvent_t between) {
    hipError_t e = launch_wave_pass(false, dtype, a, st);
    if (e != hipSuccess) return e;
    if (between) {
        e = hipEventRecord(between, st);
        if (e != hipSuccess) return e;
    }
    if (op == 2) return hipSuccess;  // first pass only
    if (op == 0) {
        hipLaunchKernelGGL(logz_combine_kernel, dim3(a.B), dim3(64), 0, st, a);
        return hipGetLastError();
    }
    return launch_wave_pass(true, dtype, a, st);
}

// Both passes in row batches (128 < T <= 256).
static hipError_t launch_stream(int op, int dtype, const ChainArgs& a, hipStream_t st, hipEvent_t between) {
    hipError_t e = launch_stream_pass(false, dtype, a, st);
    if (e != hipSuccess) return e;
    if (between) {
        e = hipEventRecord(between, st);
        if (e != hipSuccess) return e;
    }
    if (op == 2) return hipSuccess;  // first pass only
    if (op == 0) {
        hipLaunchKernelGGL(logz_combine_kernel, dim3(a.B), dim3(64), 0, st, a);
        return hipGetLastError();
    }
    return launch_stream_pass(true, dtype, a, st);
}

bool structured_supported(int T) { return T >= 1 && T <= 128; }
bool lane_chains_supported(int T) { return lane_supported(T); }

// Forward chains over whole sequences, every alpha stored (ua, Oa): the first pass of sampling.
hipError_t launch_full_forward(int dtype, const void* phi, const int32_t* lengths, int B, int N, int T, float* ua,
                               float* ub, double* Oa, double* Ob, hipStream_t st) {
    ChainArgs a{phi, lengths, B, N, T, ua, ub, Oa, Ob, nullptr, nullptr, 0, nullptr, 0, 1, nullptr, nullptr, nullptr, nullptr};
    a.full_forward = 1;
    if (wave_supported(T)) return launch_wave(2, dtype, a, st, nullptr);
    if (stream_supported(T)) return launch_stream(2, dtype, a, st, nullptr);
    const PairPlan pair{nullptr, nullptr, dtype, 0};
    const bool aligned = (T % 4) == 0;
    if (dtype == 0)
        return aligned ? launch_T<float, true>(2, a, st, nullptr, pair) : launch_T<float, false>(2, a, st, nullptr, pair);
    return aligned ? launch_T<uint16_t, true>(2, a, st, nullptr, pair) : launch_T<uint16_t, false>(2, a, st, nullptr, pair);
}

hipError_t launch_chunked_full_forward(int dtype, const void* phi, const int32_t* lengths, int B, int N, int T,
                                       float* ua, float* ub, double* Oa, double* Ob, int chunk, const float* Fv,
                                       const double* OF, hipStream_t st) {
    if (!wave_supported(T)) return hipErrorInvalidValue;
    const int C = (N + chunk - 1) / chunk;
    ChainArgs a{phi, lengths, B, N, T, ua, ub, Oa, Ob, nullptr, nullptr, 0, nullptr, chunk, C, Fv, OF, nullptr, nullptr};
    a.full_forward = 1;
    return launch_wave(2, dtype, a, st, nullptr);
}

// op: 0 = logZ only, 1 = marginals (+ logZ).  Workspace pointers already carved by the caller.
hipError_t launch_sequential_sum(int op, int dtype, const void* phi, const int32_t* lengths, int B, int N, int T,
                                 float* ua, float* ub, double* Oa, double* Ob, float* logZ, float* mu,
                                 hipStream_t st, hipEvent_t between, bool exact_only, unsigned long long* mail,
                                 int* failed, double* logZ64, const float* emit, const float* trans, int pair_poll_limit,
                                 int cus, bool lanes, int lane_poll_limit) {
    ChainArgs a{phi, lengths, B, N, T, ua, ub, Oa, Ob, logZ, mu, exact_only ? 1 : 0, nullptr, 0, 1, nullptr, nullptr, nullptr, nullptr};
    a.logZ64 = logZ64;
    a.emit = emit;
    a.trans = trans;
    if (emit && T > 128) return hipErrorInvalidValue;  // the caller checks structured_supported(T) first
    if (lanes) {
        if (exact_only || !lane_supported(T)) return hipErrorInvalidValue;
        hipError_t e = launch_lane_pass(false, dtype, a, op == 0, lane_poll_limit, st);
        if (e != hipSuccess) return e;
        if (between) {
            e = hipEventRecord(between, st);
            if (e != hipSuccess) return e;
        }
        if (op == 0) {
            hipLaunchKernelGGL(logz_combine_kernel, dim3(a.B), dim3(64), 0, st, a);
            return hipGetLastError();
        }
        return launch_lane_pass(true, dtype, a, false, lane_poll_limit, st);
    }
    if (wave_supported(T) && op == 1 && !emit && wave_chunks_fused(N - 1)) {
        // Short sequences: both passes in one launch, the vectors in LDS (as for the chunks of the scan).
        if (between) {
            const hipError_t e = hipEventRecord(between, st);
            if (e != hipSuccess) return e;
        }
        return launch_wave_chunks(dtype, a, st);
    }
    if (wave_supported(T) && op == 0 && !emit) {
        if (between) {
            const hipError_t e = hipEventRecord(between, st);
            if (e != hipSuccess) return e;
        }
        return launch_wave_logz(dtype, a, st);
    }
    if (wave_supported(T)) return launch_wave(op, dtype, a, st, between);
    if (emit) return (T % 4) == 0 ? launch_structured_sum<true>(op, a, st, between) : launch_structured_sum<false>(op, a, st, between);
    if (stream_supported(T)) return launch_stream(op, dtype, a, st, between);
    // Pairs pay off when one workgroup per chain would leave at least half of the chip idle.
    const bool use_pairs = op == 1 && !exact_only && mail && failed && pair_supported(T) && 4 * B <= cus;
    const PairPlan pair{use_pairs ? mail : nullptr, failed, dtype, pair_poll_limit};
    if (use_pairs) {
        a.pair_mail = mail;
        a.pair_failed = failed;
        a.pair_words = (int)pair_mail_words(1);
    }
    const bool aligned = (T % 4) == 0;
    if (dtype == 0)
        return aligned ? launch_T<float, true>(op, a, st, between, pair) : launch_T<float, false>(op, a, st, between, pair);
    return aligned ? launch_T<uint16_t, true>(op, a, st, between, pair)
                   : launch_T<uint16_t, false>(op, a, st, between, pair);
}

// Marginals of every chunk of every sequence from the boundary vectors of the scan: the same two
// passes, one pair of workgroups per chunk.  logZ is not written here (the scan has it already).
hipError_t launch_chunked_marginals(int dtype, const void* phi, const int32_t* lengths, int B, int N, int T,
                                    float* ua, float* ub, double* Oa, double* Ob, float* mu, int chunk,
                                    const float* Fv, const double* OF, const float* Gv, const double* OG,
                                    hipStream_t st, hipEvent_t between, bool exact_only, float* ent, const void* psi,
                                    bool difference, const float* emit, const float* trans) {
    const int C = (N + chunk - 1) / chunk;
    ChainArgs a{phi, lengths, B, N, T, ua, ub, Oa, Ob, nullptr, mu, exact_only ? 1 : 0, nullptr, chunk, C, Fv, OF, Gv, OG};
    a.ent = ent;  // entropy or expectation mode of the second pass (one-wave kernels only: the scan's tag sets)
    a.ent_kind = !ent ? 0 : !psi ? 1 : difference ? 3 : 2;
    if (ent) a.psi = psi;  // (only the second pass of the one-wave kernels looks at it)
    if (ent && !wave_supported(T)) return hipErrorInvalidValue;
    if (emit) {  // structured potentials: the two passes as separate launches, T <= 64 (the scan's tag sets)
        if (ent || dtype != 0 || !trans || T > 64) return hipErrorInvalidValue;
        a.emit = emit;
        a.trans = trans;
        if (wave_supported(T)) return launch_wave(1, dtype, a, st, between);
        return (T % 4) == 0 ? launch_structured_sum<true>(1, a, st, between) : launch_structured_sum<false>(1, a, st, between);
    }
    if (wave_supported(T) && wave_chunks_fused(chunk)) {
        if (between) {  // (the boundary phases lie before it, both passes of the chunks after it)
            const hipError_t e = hipEventRecord(between, st);
            if (e != hipSuccess) return e;
        }
        return launch_wave_chunks(dtype, a, st);
    }
    if (wave_supported(T)) return launch_wave(1, dtype, a, st, between);
    const PairPlan pair{nullptr, nullptr, dtype, 0};
    const bool aligned = (T % 4) == 0;
    if (dtype == 0)
        return aligned ? launch_T<float, true>(1, a, st, between, pair) : launch_T<float, false>(1, a, st, between, pair);
    return aligned ? launch_T<uint16_t, true>(1, a, st, between, pair) : launch_T<uint16_t, false>(1, a, st, between, pair);
}

}  // namespace lccrf
