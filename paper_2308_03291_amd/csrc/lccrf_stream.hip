// Sum-product chains for tag sets of 129 .. 256: the matrix of a position streams through registers in
// row batches.
//
// Same two passes, same two chains per sequence and same workspace as lccrf_chain.hip (section
// "Sequence Tagging" of the paper for the forward recursion, "Computing Marginals" Eq. 3-4 for what the
// second pass writes).  A matrix of up to 256 x 256 potentials is 64 numbers a thread of a 1024-thread
// workgroup; held as one tile it spills (a tile, its exponentials and the marginals' factors do not fit
// 128 registers), and nothing in a step needs it whole: the speculative step (one shift for the whole
// matrix, see lccrf_chain.hip) only adds up exponentials.  So a matrix is taken as four batches of 64 rows,
// four rows a thread, through a ring of four batch slots that is refilled across position boundaries: the
// loads of the next position are in flight while this position's sums are merged.
//
//   lane l of wave w holds, of batch q, rows 64 q + 4 w + k (k < 4), columns 4 l .. 4 l + 3:
//   a wave reads four whole rows (16-byte loads, 1 KB contiguous each).
//   forward (sum over rows): per-thread column sums over all batches, then across the 16 waves through LDS;
//   backward (sum over columns): a row is complete inside its wave and batch: four rows at a time by the
//   packed lane reduction, results straight into the next vector.
//
// A rejected speculative step is replayed exactly by streaming the same matrix again from memory (it is in
// the cache: it was read microseconds ago): thread-local maxima in a first sweep, exponentials against
// them in a second (forward), or row maximum and row sum batch by batch (backward).
#include "lccrf_chain_args.h"
#include "lccrf_chain_smem.h"
#include "lccrf_device.h"
#include "lccrf_launch.h"

namespace lccrf {

namespace {

using SG = Geo<64, 16, 16>;     // shape of the shared-memory state: 256 columns, 16 waves
constexpr int kBatchRows = 64;
// Batches in flight per thread.  Two slots are 128 KB a workgroup, more than a compute unit's share of the memory
// system holds in flight (about 50 GB/s at 2 us); a third keeps loads in flight across the merge at the end of a
// position (first pass).  The second pass also carries the marginals' factors and spills with three:
// 1024 threads leave 128 registers a thread.
template <bool WITH_MU>
constexpr int kStreamRing = WITH_MU ? 2 : 3;

struct BatchSlot {
    float v[4][4];  // potentials: rows row0 .. row0 + 3, columns c4 .. c4 + 3
    float ax[4];    // second pass: the stored vector of the other direction at this position (forward chain: four
                    // columns of beta_i; backward chain: alpha_{i-1} of the four rows) ...
    double o;       // ... and its offset
};

// This thread's part of rows row0 .. row0 + 3 of one matrix, addresses clamped into the matrix.
// (A tag count that is no multiple of four: see load_row4_anywhere; `followed`: another matrix of the tensor lies
// behind this one, the same for the whole workgroup.  settle_batch() has to come before the values are used.)
template <typename TIN, bool ALIGNED>
__device__ __forceinline__ void load_batch(const TIN* __restrict__ mat, int T, int row0, int c4, float (&v)[4][4],
                                           bool followed = false) {
    if (ALIGNED) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int s = row0 + k;
            const TIN* row = mat + (size_t)(s < T ? s : T - 1) * T;
            Elem<TIN>::get4_stream(row + (c4 < T ? c4 : T - 4), v[k]);
        }
    } else if (followed) {  // (more than 128 tags here)
#pragma unroll
        for (int k = 0; k < 4; ++k) load_row4_anywhere<TIN, true>(mat, T, row0 + k, c4, v[k]);
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) load_row4_anywhere<TIN, false>(mat, T, row0 + k, c4, v[k]);
    }
}
template <bool ALIGNED>
__device__ __forceinline__ void settle_batch(float (&v)[4][4], int T, int c4) {
    if constexpr (!ALIGNED) {
#pragma unroll
        for (int k = 0; k < 4; ++k) settle_row4(v[k], T, c4);
    }
}

// Four consecutive floats of a stored vector starting at entry e0 (clamped into the T entries).
template <bool ALIGNED>
__device__ __forceinline__ void load_vec4(const float* __restrict__ vec, int T, int e0, float (&o)[4]) {
    if (ALIGNED) {
        Elem<float>::get4(vec + (e0 < T ? e0 : T - 4), o);
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) o[j] = vec[e0 + j < T ? e0 + j : T - 1];
    }
}

}  // namespace

// WITH_MU false: pass 1 (both half chains, vectors stored); true: pass 2 (both chains continue past the
// meeting point and write the marginals).
template <typename TIN, bool ALIGNED, bool WITH_MU>
__global__ __launch_bounds__(1024) void stream_chain_kernel(ChainArgs a) {
    __shared__ ChainSmem<SG> sm;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int dir = blockIdx.x & 1;
    const int b = blockIdx.x >> 1;
    const int N = a.N, T = a.T;
    const int L = clamp_length(a.lengths, b, N);
    const size_t TT = (size_t)T * T;
    const size_t vb = (size_t)b * N;
    const TIN* phib = static_cast<const TIN*>(a.phi) + (size_t)b * N * TT;
    float* mub = WITH_MU ? a.mu + (size_t)b * N * TT : nullptr;
    const bool exact_only = a.exact_only != 0;
    const int NBq = (T + kBatchRows - 1) / kBatchRows;  // batches a matrix: 3 or 4
    const int c4 = 4 * lane;

    if (WITH_MU && dir == 0) {  // positions past the end carry no edge: their marginals are zero
        const size_t z0 = (size_t)L * TT, z1 = (size_t)N * TT;
        if (ALIGNED) {
            float4* p = reinterpret_cast<float4*>(mub);
            for (size_t k = z0 / 4 + tid; k < z1 / 4; k += 1024) p[k] = make_float4(0.f, 0.f, 0.f, 0.f);
        } else {
            for (size_t k = z0 + tid; k < z1; k += 1024) mub[k] = 0.f;
        }
    }
    if (L == 0) {
        if (WITH_MU && dir == 0 && tid == 0 && a.logZ) a.logZ[b] = 0.f;
        return;
    }
    const int e = L - 1;
    const int h = WITH_MU ? meeting_point(0, e) : forward_end(a, 0, e);
    if (!WITH_MU && a.full_forward && dir == 1) return;

    smem_init<SG>(sm, tid);
    double lz2 = 0.0;
    bool feasible = true;
    if constexpr (WITH_MU) {
        lz2 = midpoint_log2z<SG>(sm, a, vb, h, T, tid);
        feasible = lz2 > -1.0e300;  // false: no path has a finite score, marginals are 0
        if (dir == 0 && tid == 0 && a.logZ) a.logZ[b] = (float)(lz2 * kLn2);
    } else {
        __syncthreads();
    }

    // the vector the chain starts from, and the positions it walks
    double O = 0.0;
    int first, n;
    {
        float v0 = LCCRF_NEG_INF;
        if (!WITH_MU) {
            if (dir == 0) {
                if (tid < T) v0 = Elem<TIN>::get(phib + tid) * kLog2e;
                first = 1; n = h;
            } else {
                if (tid < T) v0 = 0.f;
                first = e; n = e - h;
            }
        } else {
            if (dir == 0) {
                if (tid < T) v0 = a.ua[(vb + h) * T + tid];
                O = a.Oa[vb + h];
                first = h + 1; n = e - h;
            } else {
                if (tid < T) v0 = a.ub[(vb + h) * T + tid];
                O = a.Ob[vb + h];
                first = h; n = h;
            }
        }
        publish_columns<SG>(sm, 0, tid, v0);
        __syncthreads();
    }

    int buf = 0, nstep = 0;
    float kappa = 0.f;  // running correction that keeps each position's marginals summing to one
    // state of the position in progress
    float d = 0.f, K = 0.f, tot = 0.f, wm = LCCRF_NEG_INF;
    float ls[4] = {0.f, 0.f, 0.f, 0.f};
    float gm[4] = {0.f, 0.f, 0.f, 0.f}, ubc[4] = {0.f, 0.f, 0.f, 0.f};
    float ubK[4] = {LCCRF_NEG_INF, LCCRF_NEG_INF, LCCRF_NEG_INF, LCCRF_NEG_INF};  // second pass, forward: beta_i + K of the thread's columns
    bool ok = true;

    BatchSlot ring[kStreamRing<WITH_MU>];
    // unit u = batch u % NBq of the matrix of position first +- u / NBq; one loader per direction, so that
    // neither holds a branch around its loads
    auto load_forward = [&](int u, int slot) {
        const int pos = first + u / NBq, q = u % NBq;
        load_batch<TIN, ALIGNED>(phib + (size_t)pos * TT, T, kBatchRows * q + 4 * wave, c4, ring[slot].v, b != a.B - 1 || pos != N - 1);
        if constexpr (WITH_MU) {
            load_vec4<ALIGNED>(a.ub + (vb + pos) * T, T, c4, ring[slot].ax);
            ring[slot].o = a.Ob[vb + pos];
        }
    };
    auto load_backward = [&](int u, int slot) {
        const int pos = first - u / NBq, q = u % NBq;
        const int row0 = kBatchRows * q + 4 * wave;
        load_batch<TIN, ALIGNED>(phib + (size_t)pos * TT, T, row0, c4, ring[slot].v, b != a.B - 1 || pos != N - 1);
        if constexpr (WITH_MU) {
            load_vec4<ALIGNED>(a.ua + (vb + pos - 1) * T, T, row0, ring[slot].ax);
            ring[slot].o = a.Oa[vb + pos - 1];
        }
    };

    // ---- exact replays: the matrix of position i again, straight from memory
    auto forward_exact = [&](int i) {
        const TIN* mat = phib + (size_t)i * TT;
        float lm[4] = {LCCRF_NEG_INF, LCCRF_NEG_INF, LCCRF_NEG_INF, LCCRF_NEG_INF};
        for (int q = 0; q < NBq; ++q) {
            const int row0 = kBatchRows * q + 4 * wave;
            float v[4][4];
            load_batch<TIN, ALIGNED>(mat, T, row0, c4, v, b != a.B - 1 || i != N - 1);
            settle_batch<ALIGNED>(v, T, c4);
            const float4 r4 = *reinterpret_cast<const float4*>(&sm.rvec[buf][row0]);
            const float ua[4] = {r4.x - d, r4.y - d, r4.z - d, r4.w - d};  // -inf for rows >= T
#pragma unroll
            for (int k = 0; k < 4; ++k)
#pragma unroll
                for (int j = 0; j < 4; ++j) lm[j] = fmaxf(lm[j], __builtin_fmaf(v[k][j], kLog2e, ua[k]));
        }
        float g[4], gx[4] = {0.f, 0.f, 0.f, 0.f}, es[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < 4; ++j) g[j] = finite_or_zero(lm[j]);
        if constexpr (WITH_MU) {
#pragma unroll
            for (int j = 0; j < 4; ++j) gx[j] = ex2(g[j] + ubK[j]);
        }
        for (int q = 0; q < NBq; ++q) {
            const int row0 = kBatchRows * q + 4 * wave;
            float v[4][4];
            load_batch<TIN, ALIGNED>(mat, T, row0, c4, v, b != a.B - 1 || i != N - 1);
            settle_batch<ALIGNED>(v, T, c4);
            const float4 r4 = *reinterpret_cast<const float4*>(&sm.rvec[buf][row0]);
            const float ua[4] = {r4.x - d, r4.y - d, r4.z - d, r4.w - d};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                float ex[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    ex[j] = ex2(__builtin_fmaf(v[k][j], kLog2e, ua[k]) - g[j]);
                    es[j] += ex[j];
                }
                if constexpr (WITH_MU)
                    store4<ALIGNED, true>(mub + (size_t)i * TT, T, row0 + k, c4, ex[0] * gx[0], ex[1] * gx[1], ex[2] * gx[2], ex[3] * gx[3]);
            }
        }
        if constexpr (WITH_MU) {
            float t = (es[0] * gx[0] + es[1] * gx[1]) + (es[2] * gx[2] + es[3] * gx[3]);
            t = xor_sum<1, 64>(t);
            if (lane == 0) sm.wtot[buf ^ 1][wave] = t;
        }
        *reinterpret_cast<float4*>(&sm.pmax[wave][c4]) = make_float4(lm[0], lm[1], lm[2], lm[3]);
        *reinterpret_cast<float4*>(&sm.psum[wave][c4]) = make_float4(es[0], es[1], es[2], es[3]);
        __syncthreads();
        if (wave < SG::COLWAVES) {
            float r = LCCRF_NEG_INF;
            if (tid < T) {
                float M = LCCRF_NEG_INF;
#pragma unroll
                for (int w = 0; w < 16; ++w) M = fmaxf(M, sm.pmax[w][tid]);
                const float gM = finite_or_zero(M);
                float S = 0.f;
#pragma unroll
                for (int w = 0; w < 16; ++w) S = __builtin_fmaf(sm.psum[w][tid], ex2(sm.pmax[w][tid] - gM), S);
                r = M + lg2(S);  // M = -inf gives S = 0: -inf + -inf = -inf
            }
            sm.rvec[buf ^ 1][tid] = r;
            const float m = xor_max<1, 64>(r);
            if (lane == 0) sm.wmax[buf ^ 1][wave] = m;
        }
        __syncthreads();
    };
    auto backward_exact = [&](int i) {
        const TIN* mat = phib + (size_t)i * TT;
        const float4 q4 = *reinterpret_cast<const float4*>(&sm.rvec[buf][c4]);
        const float ub[4] = {q4.x - d, q4.y - d, q4.z - d, q4.w - d};  // -inf for columns >= T
        float t = 0.f, m_all = LCCRF_NEG_INF;
        for (int q = 0; q < NBq; ++q) {
            const int row0 = kBatchRows * q + 4 * wave;
            float v[4][4], uaK[4] = {0.f, 0.f, 0.f, 0.f};
            load_batch<TIN, ALIGNED>(mat, T, row0, c4, v, b != a.B - 1 || i != N - 1);
            settle_batch<ALIGNED>(v, T, c4);
            if constexpr (WITH_MU) {
                float ax[4];
                load_vec4<ALIGNED>(a.ua + (vb + i - 1) * T, T, row0, ax);
#pragma unroll
                for (int k = 0; k < 4; ++k) uaK[k] = (row0 + k < T) ? ax[k] + K : LCCRF_NEG_INF;
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                float y[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) y[j] = __builtin_fmaf(v[k][j], kLog2e, ub[j]);
                const float m = xor_max<1, 64>(fmaxf(fmaxf(y[0], y[1]), fmaxf(y[2], y[3])));
                const float g = finite_or_zero(m);
                float ex[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) ex[j] = ex2(y[j] - g);
                const float Sk = (ex[0] + ex[1]) + (ex[2] + ex[3]);
                if constexpr (WITH_MU) {
                    const float f = ex2(g + uaK[k]);
                    store4<ALIGNED, true>(mub + (size_t)i * TT, T, row0 + k, c4, ex[0] * f, ex[1] * f, ex[2] * f, ex[3] * f);
                    t += Sk * f;
                }
                const int s = row0 + k;
                const float r = (s < T) ? m + lg2(xor_sum<1, 64>(Sk)) : LCCRF_NEG_INF;
                if (lane == 0 && s < T) sm.rvec[buf ^ 1][s] = r;
                m_all = fmaxf(m_all, r);
            }
        }
        if (lane == 0) sm.wmax[buf ^ 1][wave] = m_all;
        if constexpr (WITH_MU) {
            t = xor_sum<1, 64>(t);
            if (lane == 0) sm.wtot[buf ^ 1][wave] = t;
        }
        __syncthreads();
    };

    if (dir == 0) {
        // ---------------- forward chain ----------------
        walk<kStreamRing<WITH_MU>>(0, n * NBq - 1, +1, load_forward, [&](int u, int slot) {
            settle_batch<ALIGNED>(ring[slot].v, T, c4);
            const int i = first + u / NBq, q = u % NBq;
            const int row0 = kBatchRows * q + 4 * wave;
            if (q == 0) {
                d = read_shift<SG>(sm, buf);
                if constexpr (WITH_MU) kappa += read_drift<SG>(sm, buf);
                O += (double)d;
                if constexpr (!WITH_MU) {
                    if (tid < T) a.ua[(vb + i - 1) * T + tid] = sm.rvec[buf][tid] - d;
                    if (tid == 0) a.Oa[vb + i - 1] = O;
                } else {
                    K = feasible ? (float)(O + ring[slot].o - lz2) + kappa : LCCRF_NEG_INF;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        ubK[j] = (c4 + j < T) ? ring[slot].ax[j] + K : LCCRF_NEG_INF;
                        gm[j] = ex2(d + ubK[j]);
                    }
                }
                if (tid == 0) sm.bad[(nstep + 1) & 3] = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j) ls[j] = 0.f;
            }
            const float4 r4 = *reinterpret_cast<const float4*>(&sm.rvec[buf][row0]);
            const float uac[4] = {r4.x - d - d, r4.y - d - d, r4.z - d - d, r4.w - d - d};  // ua - c, shift c = d; -inf for rows >= T
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                float ex[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    ex[j] = ex2(__builtin_fmaf(ring[slot].v[k][j], kLog2e, uac[k]));
                    ls[j] += ex[j];
                }
                if constexpr (WITH_MU)
                    store4<ALIGNED, true>(mub + (size_t)i * TT, T, row0 + k, c4, ex[0] * gm[0], ex[1] * gm[1], ex[2] * gm[2], ex[3] * gm[3]);
            }
            if (q == NBq - 1) {
                const int flag = nstep & 3;
                if constexpr (WITH_MU) {
                    float t = (ls[0] * gm[0] + ls[1] * gm[1]) + (ls[2] * gm[2] + ls[3] * gm[3]);
                    t = xor_sum<1, 64>(t);
                    if (lane == 0) sm.wtot[buf ^ 1][wave] = t;
                }
                *reinterpret_cast<float4*>(&sm.psum[wave][c4]) = make_float4(ls[0], ls[1], ls[2], ls[3]);
                __syncthreads();
                if (wave < SG::COLWAVES) {
                    float r = LCCRF_NEG_INF;
                    bool good = true;
                    if (tid < T) {
                        float S = 0.f;
#pragma unroll
                        for (int w = 0; w < 16; ++w) S += sm.psum[w][tid];
                        r = d + lg2(S);
                        good = sum_in_range(S);
                    }
                    sm.rvec[buf ^ 1][tid] = r;
                    const float m = xor_max<1, 64>(r);
                    if (lane == 0) sm.wmax[buf ^ 1][wave] = m;
                    if (!__all(good) && lane == 0) sm.bad[flag] = 1;
                }
                __syncthreads();
                if (exact_only || sm.bad[flag] != 0) forward_exact(i);
                buf ^= 1;
                ++nstep;
            }
        });
        if constexpr (!WITH_MU) {
            const float dl = read_shift<SG>(sm, buf);
            O += (double)dl;
            if (tid < T) a.ua[(vb + h) * T + tid] = sm.rvec[buf][tid] - dl;
            if (tid == 0) a.Oa[vb + h] = O;
        }
    } else {
        // ---------------- backward chain ----------------
        walk<kStreamRing<WITH_MU>>(0, n * NBq - 1, +1, load_backward, [&](int u, int slot) {
            settle_batch<ALIGNED>(ring[slot].v, T, c4);
            const int i = first - u / NBq, q = u % NBq;
            const int row0 = kBatchRows * q + 4 * wave;
            if (q == 0) {
                d = read_shift<SG>(sm, buf);
                if constexpr (WITH_MU) kappa += read_drift<SG>(sm, buf);
                O += (double)d;
                const float4 q4 = *reinterpret_cast<const float4*>(&sm.rvec[buf][c4]);
                ubc[0] = q4.x - d - d; ubc[1] = q4.y - d - d; ubc[2] = q4.z - d - d; ubc[3] = q4.w - d - d;  // ub - c, c = d
                if constexpr (!WITH_MU) {
                    if (tid < T) a.ub[(vb + i) * T + tid] = sm.rvec[buf][tid] - d;
                    if (tid == 0) a.Ob[vb + i] = O;
                } else {
                    K = feasible ? (float)(ring[slot].o + O - lz2) + kappa : LCCRF_NEG_INF;
                }
                if (tid == 0) sm.bad[(nstep + 1) & 3] = 0;
                tot = 0.f;
                wm = LCCRF_NEG_INF;
                ok = true;
            }
            float S[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                float ex[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) ex[j] = ex2(__builtin_fmaf(ring[slot].v[k][j], kLog2e, ubc[j]));
                S[k] = (ex[0] + ex[1]) + (ex[2] + ex[3]);
                if constexpr (WITH_MU) {
                    const float f = (row0 + k < T) ? ex2(d + ring[slot].ax[k] + K) : 0.f;
                    store4<ALIGNED, true>(mub + (size_t)i * TT, T, row0 + k, c4, ex[0] * f, ex[1] * f, ex[2] * f, ex[3] * f);
                    tot += S[k] * f;
                }
            }
            {   // four rows at a time: each lane ends up with the complete sum of one of them
                const int kk = 2 * (lane & 1) + ((lane >> 1) & 1);
                const float Sk = reduce4_over_lanes<64>(S[0], S[1], S[2], S[3], lane);
                const int s = row0 + kk;
                const float r = (s < T) ? d + lg2(Sk) : LCCRF_NEG_INF;
                if (lane < 4 && s < T) sm.rvec[buf ^ 1][s] = r;
                ok = ok && (s >= T || sum_in_range(Sk));
                wm = fmaxf(wm, r);
            }
            if (q == NBq - 1) {
                const int flag = nstep & 3;
                const float m = xor_max<1, 4>(wm);
                if (lane == 0) sm.wmax[buf ^ 1][wave] = m;
                if (!__all(ok) && lane == 0) sm.bad[flag] = 1;
                if constexpr (WITH_MU) {
                    const float t = xor_sum<1, 64>(tot);
                    if (lane == 0) sm.wtot[buf ^ 1][wave] = t;
                }
                __syncthreads();
                if (exact_only || sm.bad[flag] != 0) backward_exact(i);
                buf ^= 1;
                ++nstep;
            }
        });
        if constexpr (!WITH_MU) {
            const float dl = read_shift<SG>(sm, buf);
            O += (double)dl;
            if (tid < T) a.ub[(vb + h) * T + tid] = sm.rvec[buf][tid] - dl;
            if (tid == 0) a.Ob[vb + h] = O;
        } else {
            // position 0: p(y_0 = t) = softmax_t(alpha_0(t) + beta_0(t)) in row 0, zeros elsewhere
            for (int k = T + tid; k < (int)TT; k += 1024) mub[k] = 0.f;
            if (tid < 64) {
                float m = LCCRF_NEG_INF;
                for (int t = tid; t < T; t += 64) m = fmaxf(m, a.ua[vb * T + t] + sm.rvec[buf][t]);
                m = xor_max<1, 64>(m);
                float S = 0.f;
                for (int t = tid; t < T; t += 64) S += ex2(a.ua[vb * T + t] + sm.rvec[buf][t] - finite_or_zero(m));
                S = xor_sum<1, 64>(S);
                const float c = (feasible && S > 0.f) ? 1.0f / S : 0.f;
                for (int t = tid; t < T; t += 64) mub[t] = c * ex2(a.ua[vb * T + t] + sm.rvec[buf][t] - finite_or_zero(m));
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// Expectations carried along the half chains at 129 .. 256 tags, in row batches: the first pass of the
// entropy (MODE 0), of the cross-entropy (MODE 1) and of the KL divergence (MODE 2); the recursions and what
// the chains leave for the meeting position are those of entropy_half_kernel (lccrf_extras.hip, section
// "Entropy and KL Divergence" of the paper).  Beside its vector a chain carries h, the conditional
// expectation given the current tag of a quantity summed over the path behind it; a step forms
// S = sum e and U = sum e (h - log2 e) (entropy) or U = sum e (h + f) (f the edge's term: psi, or phi - psi)
// from the same shifted exponentials e, and the new h is U / S (+ log2 S).  Neither depends on the shift,
// so the speculative step (one shift for the whole matrix) serves here as well; a rejected step streams
// the matrix again: column maxima through LDS first, then the sums against them (forward); row maximum
// and row sums batch by batch (backward).  In modes 1 and 2 the largest finite entry of h moves into a
// double-precision offset at every step.
template <typename TIN, bool ALIGNED, int MODE>
__global__ __launch_bounds__(1024) void stream_expect_kernel(ChainArgs a) {
    constexpr bool CROSS = MODE != 0;
    constexpr int RING = CROSS ? 2 : 3;
    __shared__ ChainSmem<SG> sm;
    __shared__ __attribute__((aligned(16))) float hvec[2][SG::TCAP];
    __shared__ __attribute__((aligned(16))) float pU[16][SG::TCAP];
    __shared__ __attribute__((aligned(16))) float hmaxw[2][16];  // per-wave largest finite entries of hvec
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int dir = blockIdx.x & 1, b = blockIdx.x >> 1;
    const int N = a.N, T = a.T;
    const int L = clamp_length(a.lengths, b, N);
    if (L == 0) return;
    const size_t TT = (size_t)T * T, vb = (size_t)b * N;
    const TIN* phib = static_cast<const TIN*>(a.phi) + (size_t)b * N * TT;
    const TIN* psib = CROSS ? static_cast<const TIN*>(a.psi) + (size_t)b * N * TT : phib;
    const bool exact_only = a.exact_only != 0;
    const int NBq = (T + kBatchRows - 1) / kBatchRows;
    const int c4 = 4 * lane;
    const int e = L - 1, h = meeting_point(0, e);
    const int first = dir == 0 ? 1 : e, n = dir == 0 ? h : e - h;

    smem_init<SG>(sm, tid);
    for (int k = tid; k < 2 * SG::TCAP; k += 1024) (&hvec[0][0])[k] = 0.f;
    if (tid < 32) (&hmaxw[0][0])[tid] = LCCRF_NEG_INF;
    __syncthreads();
    {
        float v0 = LCCRF_NEG_INF, h0 = 0.f;
        if (tid < T) {
            const float p0 = Elem<TIN>::get(phib + tid);
            v0 = dir == 0 ? p0 * kLog2e : 0.f;
            if (CROSS && dir == 0 && p0 != LCCRF_NEG_INF) {  // the score of the first tag belongs to the forward chain
                const float q0 = Elem<TIN>::get(psib + tid);
                h0 = MODE == 1 ? q0 : p0 - q0;
            }
        }
        publish_columns<SG>(sm, 0, tid, v0);
        if (wave < SG::COLWAVES) {
            hvec[0][tid] = h0;
            const float hm = xor_max<1, 64>((tid < T && fabsf(h0) < __builtin_huge_valf()) ? h0 : LCCRF_NEG_INF);
            if (lane == 0) hmaxw[0][wave] = hm;
        }
        __syncthreads();
    }
    auto read_hshift = [&](int bf) {  // largest finite entry of hvec[bf] (0 if there is none)
        const float4 q0 = *reinterpret_cast<const float4*>(&hmaxw[bf][0]), q1 = *reinterpret_cast<const float4*>(&hmaxw[bf][4]);
        const float4 q2 = *reinterpret_cast<const float4*>(&hmaxw[bf][8]), q3 = *reinterpret_cast<const float4*>(&hmaxw[bf][12]);
        const float x = max3_raw(max3_raw(q0.x, q0.y, q0.z), q0.w, q1.x), y = max3_raw(max3_raw(q1.y, q1.z, q1.w), q2.x, q2.y);
        const float z = max3_raw(max3_raw(q2.z, q2.w, q3.x), q3.y, q3.z);
        return finite_or_zero(max3_raw(max3_raw(x, y, z), q3.w, q3.w));
    };
    const auto finite_or_ninf = [](float g) { return fabsf(g) < __builtin_huge_valf() ? g : LCCRF_NEG_INF; };
    // what an edge adds to the carried expectation (modes 1 and 2); x: the potential, qv: the second chain's
    const auto edge_term = [](float x, float qv) { return MODE == 1 ? qv : x - qv; };

    int buf = 0, nstep = 0;
    double O = 0.0, Hoff = 0.0;
    float d = 0.f, c = 0.f, wm = LCCRF_NEG_INF, hm = LCCRF_NEG_INF;
    float ls[4] = {0.f, 0.f, 0.f, 0.f}, lu[4] = {0.f, 0.f, 0.f, 0.f};
    float ubc[4] = {0.f, 0.f, 0.f, 0.f}, hcol[4] = {0.f, 0.f, 0.f, 0.f};
    bool ok = true;

    float ring[RING][4][4];
    float qring[CROSS ? RING : 1][4][4];
    auto load = [&](int u, int slot) {
        const int pos = dir == 0 ? first + u / NBq : first - u / NBq, q = u % NBq;
        load_batch<TIN, ALIGNED>(phib + (size_t)pos * TT, T, kBatchRows * q + 4 * wave, c4, ring[slot], b != a.B - 1 || pos != N - 1);
        if constexpr (CROSS) load_batch<TIN, ALIGNED>(psib + (size_t)pos * TT, T, kBatchRows * q + 4 * wave, c4, qring[slot], b != a.B - 1 || pos != N - 1);
    };
    // publishes the column threads' results of a forward step (r, hv: this thread's column, or -inf / 0)
    auto publish_forward = [&](float r, float hv) {
        sm.rvec[buf ^ 1][tid] = r;
        hvec[buf ^ 1][tid] = hv;
        const float m = xor_max<1, 64>(r);
        const float g = xor_max<1, 64>(tid < T ? finite_or_ninf(hv) : LCCRF_NEG_INF);
        if (lane == 0) {
            sm.wmax[buf ^ 1][wave] = m;
            hmaxw[buf ^ 1][wave] = g;
        }
    };

    auto forward_exact = [&](int i) {
        const TIN* mat = phib + (size_t)i * TT;
        const TIN* qmat = psib + (size_t)i * TT;
        float lm[4] = {LCCRF_NEG_INF, LCCRF_NEG_INF, LCCRF_NEG_INF, LCCRF_NEG_INF};
        for (int q = 0; q < NBq; ++q) {
            const int row0 = kBatchRows * q + 4 * wave;
            float v[4][4];
            load_batch<TIN, ALIGNED>(mat, T, row0, c4, v, b != a.B - 1 || i != N - 1);
            settle_batch<ALIGNED>(v, T, c4);
            const float4 r4 = *reinterpret_cast<const float4*>(&sm.rvec[buf][row0]);
            const float ua[4] = {r4.x - d, r4.y - d, r4.z - d, r4.w - d};  // -inf for rows >= T
#pragma unroll
            for (int k = 0; k < 4; ++k)
#pragma unroll
                for (int j = 0; j < 4; ++j) lm[j] = fmaxf(lm[j], __builtin_fmaf(v[k][j], kLog2e, ua[k]));
        }
        *reinterpret_cast<float4*>(&sm.pmax[wave][c4]) = make_float4(lm[0], lm[1], lm[2], lm[3]);
        __syncthreads();
        float g[4], es[4] = {0.f, 0.f, 0.f, 0.f}, eu[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float M = LCCRF_NEG_INF;
#pragma unroll
            for (int w = 0; w < 16; ++w) M = fmaxf(M, sm.pmax[w][c4 + j]);
            g[j] = finite_or_zero(M);
        }
        for (int q = 0; q < NBq; ++q) {
            const int row0 = kBatchRows * q + 4 * wave;
            float v[4][4], qv[4][4];
            load_batch<TIN, ALIGNED>(mat, T, row0, c4, v, b != a.B - 1 || i != N - 1);
            settle_batch<ALIGNED>(v, T, c4);
            if constexpr (CROSS) {
                load_batch<TIN, ALIGNED>(qmat, T, row0, c4, qv, b != a.B - 1 || i != N - 1);
                settle_batch<ALIGNED>(qv, T, c4);
            }
            const float4 r4 = *reinterpret_cast<const float4*>(&sm.rvec[buf][row0]);
            const float4 h4 = *reinterpret_cast<const float4*>(&hvec[buf][row0]);
            const float ua[4] = {r4.x - d, r4.y - d, r4.z - d, r4.w - d};
            const float hin[4] = {h4.x - c, h4.y - c, h4.z - c, h4.w - c};
#pragma unroll
            for (int k = 0; k < 4; ++k)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float arg = __builtin_fmaf(v[k][j], kLog2e, ua[k]) - g[j];
                    const float ex = ex2(arg);
                    es[j] += ex;
                    if (CROSS) eu[j] += ex > 0.f ? ex * (hin[k] + edge_term(v[k][j], qv[k][j])) : 0.f;
                    else eu[j] = __builtin_fmaf(ex, hin[k] - log2_term(arg), eu[j]);
                }
        }
        *reinterpret_cast<float4*>(&sm.psum[wave][c4]) = make_float4(es[0], es[1], es[2], es[3]);
        *reinterpret_cast<float4*>(&pU[wave][c4]) = make_float4(eu[0], eu[1], eu[2], eu[3]);
        __syncthreads();
        if (wave < SG::COLWAVES) {
            float r = LCCRF_NEG_INF, hv = 0.f;
            if (tid < T) {
                float S = 0.f, U = 0.f, M = LCCRF_NEG_INF;
#pragma unroll
                for (int w = 0; w < 16; ++w) {
                    S += sm.psum[w][tid];
                    U += pU[w][tid];
                    M = fmaxf(M, sm.pmax[w][tid]);
                }
                r = M + lg2(S);  // M = -inf gives S = 0: -inf
                hv = CROSS ? (S > 0.f ? U / S : 0.f) : entropy_of(U, S);
            }
            publish_forward(r, hv);
        }
        __syncthreads();
    };
    auto backward_exact = [&](int i) {
        const TIN* mat = phib + (size_t)i * TT;
        const TIN* qmat = psib + (size_t)i * TT;
        const float4 q4 = *reinterpret_cast<const float4*>(&sm.rvec[buf][c4]);
        const float ub[4] = {q4.x - d, q4.y - d, q4.z - d, q4.w - d};  // -inf for columns >= T
        float m_all = LCCRF_NEG_INF, h_all = LCCRF_NEG_INF;
        for (int q = 0; q < NBq; ++q) {
            const int row0 = kBatchRows * q + 4 * wave;
            float v[4][4], qv[4][4];
            load_batch<TIN, ALIGNED>(mat, T, row0, c4, v, b != a.B - 1 || i != N - 1);
            settle_batch<ALIGNED>(v, T, c4);
            if constexpr (CROSS) {
                load_batch<TIN, ALIGNED>(qmat, T, row0, c4, qv, b != a.B - 1 || i != N - 1);
                settle_batch<ALIGNED>(qv, T, c4);
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                float y[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) y[j] = __builtin_fmaf(v[k][j], kLog2e, ub[j]);
                const float m = xor_max<1, 64>(fmaxf(fmaxf(y[0], y[1]), fmaxf(y[2], y[3])));
                const float g = finite_or_zero(m);
                float Sk = 0.f, Uk = 0.f;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float arg = y[j] - g;
                    const float ex = ex2(arg);
                    Sk += ex;
                    if (CROSS) Uk += ex > 0.f ? ex * (hcol[j] + edge_term(v[k][j], qv[k][j])) : 0.f;
                    else Uk = __builtin_fmaf(ex, hcol[j] - log2_term(arg), Uk);
                }
                const float S = xor_sum<1, 64>(Sk), U = xor_sum<1, 64>(Uk);
                const int s = row0 + k;
                const float r = (s < T) ? m + lg2(S) : LCCRF_NEG_INF;
                const float hv = CROSS ? (S > 0.f ? U / S : 0.f) : entropy_of(U, S);
                if (lane == 0 && s < T) {
                    sm.rvec[buf ^ 1][s] = r;
                    hvec[buf ^ 1][s] = hv;
                }
                m_all = fmaxf(m_all, r);
                if (s < T) h_all = fmaxf(h_all, finite_or_ninf(hv));
            }
        }
        if (lane == 0) {
            sm.wmax[buf ^ 1][wave] = m_all;
            hmaxw[buf ^ 1][wave] = h_all;
        }
        __syncthreads();
    };

    if (dir == 0) {
        walk<RING>(0, n * NBq - 1, +1, load, [&](int u, int slot) {
            settle_batch<ALIGNED>(ring[slot], T, c4);
            if constexpr (CROSS) settle_batch<ALIGNED>(qring[slot], T, c4);
            const int i = first + u / NBq, q = u % NBq;
            const int row0 = kBatchRows * q + 4 * wave;
            if (q == 0) {
                d = read_shift<SG>(sm, buf);
                O += (double)d;
                if constexpr (CROSS) {
                    c = read_hshift(buf);
                    Hoff += (double)c;
                }
                if (tid == 0) sm.bad[(nstep + 1) & 3] = 0;
#pragma unroll
                for (int j = 0; j < 4; ++j) ls[j] = lu[j] = 0.f;
            }
            const float4 r4 = *reinterpret_cast<const float4*>(&sm.rvec[buf][row0]);
            const float4 h4 = *reinterpret_cast<const float4*>(&hvec[buf][row0]);
            const float uac[4] = {r4.x - d - d, r4.y - d - d, r4.z - d - d, r4.w - d - d};  // ua - c, shift c = d; -inf for rows >= T
            const float hin[4] = {h4.x - c, h4.y - c, h4.z - c, h4.w - c};
#pragma unroll
            for (int k = 0; k < 4; ++k)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float arg = __builtin_fmaf(ring[slot][k][j], kLog2e, uac[k]);
                    const float ex = ex2(arg);
                    ls[j] += ex;
                    if (CROSS) lu[j] += ex > 0.f ? ex * (hin[k] + edge_term(ring[slot][k][j], qring[CROSS ? slot : 0][k][j])) : 0.f;
                    else lu[j] = __builtin_fmaf(ex, hin[k] - log2_term(arg), lu[j]);
                }
            if (q == NBq - 1) {
                const int flag = nstep & 3;
                *reinterpret_cast<float4*>(&sm.psum[wave][c4]) = make_float4(ls[0], ls[1], ls[2], ls[3]);
                *reinterpret_cast<float4*>(&pU[wave][c4]) = make_float4(lu[0], lu[1], lu[2], lu[3]);
                __syncthreads();
                if (wave < SG::COLWAVES) {
                    float r = LCCRF_NEG_INF, hv = 0.f;
                    bool good = true;
                    if (tid < T) {
                        float S = 0.f, U = 0.f;
#pragma unroll
                        for (int w = 0; w < 16; ++w) {
                            S += sm.psum[w][tid];
                            U += pU[w][tid];
                        }
                        r = d + lg2(S);
                        hv = CROSS ? (S > 0.f ? U / S : 0.f) : entropy_of(U, S);
                        good = sum_in_range(S);
                    }
                    publish_forward(r, hv);
                    if (!__all(good) && lane == 0) sm.bad[flag] = 1;
                }
                __syncthreads();
                if (exact_only || sm.bad[flag] != 0) forward_exact(i);
                buf ^= 1;
                ++nstep;
            }
        });
    } else {
        walk<RING>(0, n * NBq - 1, +1, load, [&](int u, int slot) {
            settle_batch<ALIGNED>(ring[slot], T, c4);
            if constexpr (CROSS) settle_batch<ALIGNED>(qring[slot], T, c4);
            const int i = first - u / NBq, q = u % NBq;
            const int row0 = kBatchRows * q + 4 * wave;
            if (q == 0) {
                d = read_shift<SG>(sm, buf);
                O += (double)d;
                if constexpr (CROSS) {
                    c = read_hshift(buf);
                    Hoff += (double)c;
                }
                const float4 q4 = *reinterpret_cast<const float4*>(&sm.rvec[buf][c4]);
                const float4 h4 = *reinterpret_cast<const float4*>(&hvec[buf][c4]);
                ubc[0] = q4.x - d - d; ubc[1] = q4.y - d - d; ubc[2] = q4.z - d - d; ubc[3] = q4.w - d - d;  // ub - c, c = d
                hcol[0] = h4.x - c; hcol[1] = h4.y - c; hcol[2] = h4.z - c; hcol[3] = h4.w - c;
                if (tid == 0) sm.bad[(nstep + 1) & 3] = 0;
                wm = LCCRF_NEG_INF;
                hm = LCCRF_NEG_INF;
                ok = true;
            }
            float Sl[4], Ul[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                Sl[k] = 0.f;
                Ul[k] = 0.f;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float arg = __builtin_fmaf(ring[slot][k][j], kLog2e, ubc[j]);
                    const float ex = ex2(arg);
                    Sl[k] += ex;
                    if (CROSS) Ul[k] += ex > 0.f ? ex * (hcol[j] + edge_term(ring[slot][k][j], qring[CROSS ? slot : 0][k][j])) : 0.f;
                    else Ul[k] = __builtin_fmaf(ex, hcol[j] - log2_term(arg), Ul[k]);
                }
            }
            {   // four rows at a time: each lane ends up with the complete sums of one of them
                const int kk = 2 * (lane & 1) + ((lane >> 1) & 1);
                const float S = reduce4_over_lanes<64>(Sl[0], Sl[1], Sl[2], Sl[3], lane);
                const float U = reduce4_over_lanes<64>(Ul[0], Ul[1], Ul[2], Ul[3], lane);
                const int s = row0 + kk;
                const float r = (s < T) ? d + lg2(S) : LCCRF_NEG_INF;
                const float hv = CROSS ? (S > 0.f ? U / S : 0.f) : entropy_of(U, S);
                if (lane < 4 && s < T) {
                    sm.rvec[buf ^ 1][s] = r;
                    hvec[buf ^ 1][s] = hv;
                }
                ok = ok && (s >= T || sum_in_range(S));
                wm = fmaxf(wm, r);
                if (s < T) hm = fmaxf(hm, finite_or_ninf(hv));
            }
            if (q == NBq - 1) {
                const int flag = nstep & 3;
                const float m = xor_max<1, 4>(wm), g = xor_max<1, 4>(hm);
                if (lane == 0) {
                    sm.wmax[buf ^ 1][wave] = m;
                    hmaxw[buf ^ 1][wave] = g;
                }
                if (!__all(ok) && lane == 0) sm.bad[flag] = 1;
                __syncthreads();
                if (exact_only || sm.bad[flag] != 0) backward_exact(i);
                buf ^= 1;
                ++nstep;
            }
        });
    }
    // the vectors of the meeting position
    const float dl = read_shift<SG>(sm, buf);
    O += (double)dl;
    if (tid < T) {
        (dir == 0 ? a.ua : a.ub)[(vb + h) * T + tid] = sm.rvec[buf][tid] - dl;
        (dir == 0 ? a.ha : a.hb)[(size_t)b * T + tid] = hvec[buf][tid];
    }
    if (tid == 0) (dir == 0 ? a.Oa : a.Ob)[vb + h] = O;
    if (CROSS && tid == 0) a.hoff[2 * b + dir] = Hoff;
}

template <typename TIN, bool ALIGNED>
static hipError_t launch_stream_expect_t(int mode, const ChainArgs& a, hipStream_t st) {
    const dim3 grid(2 * a.B), block(1024);
    if (mode == 0) hipLaunchKernelGGL((stream_expect_kernel<TIN, ALIGNED, 0>), grid, block, 0, st, a);
    else if (mode == 1) hipLaunchKernelGGL((stream_expect_kernel<TIN, ALIGNED, 1>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((stream_expect_kernel<TIN, ALIGNED, 2>), grid, block, 0, st, a);
    return hipGetLastError();
}

hipError_t launch_stream_expect(int mode, int dtype, const ChainArgs& a, hipStream_t st) {
    if (!stream_supported(a.T) || a.chunk > 0 || a.emit || mode < 0 || mode > 2 || (mode != 0 && !a.psi)) return hipErrorInvalidValue;
    const bool aligned = (a.T % 4) == 0;
    if (dtype == 0) return aligned ? launch_stream_expect_t<float, true>(mode, a, st) : launch_stream_expect_t<float, false>(mode, a, st);
    return aligned ? launch_stream_expect_t<uint16_t, true>(mode, a, st) : launch_stream_expect_t<uint16_t, false>(mode, a, st);
}

template <typename TIN, bool ALIGNED>
static hipError_t launch_stream_t(bool second_pass, const ChainArgs& a, hipStream_t st) {
    if (second_pass)
        hipLaunchKernelGGL((stream_chain_kernel<TIN, ALIGNED, true>), dim3(2 * a.B), dim3(1024), 0, st, a);
    else
        hipLaunchKernelGGL((stream_chain_kernel<TIN, ALIGNED, false>), dim3(2 * a.B), dim3(1024), 0, st, a);
    return hipGetLastError();
}

bool stream_supported(int T) { return T > 128 && T <= 256; }

hipError_t launch_stream_pass(bool second_pass, int dtype, const ChainArgs& a, hipStream_t st) {
    if (!stream_supported(a.T) || a.chunk > 0 || a.emit) return hipErrorInvalidValue;
    const bool aligned = (a.T % 4) == 0;
    if (dtype == 0) return aligned ? launch_stream_t<float, true>(second_pass, a, st) : launch_stream_t<float, false>(second_pass, a, st);
    return aligned ? launch_stream_t<uint16_t, true>(second_pass, a, st) : launch_stream_t<uint16_t, false>(second_pass, a, st);
}

}  // namespace lccrf
