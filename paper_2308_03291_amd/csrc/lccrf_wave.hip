// Sum-product chains for small tag sets (T <= 32): one wave per chain, nothing but registers.
//
// Same schedule and arithmetic as lccrf_chain.hip (two chains per sequence or per chunk meeting
// in the middle, pass 1 stores the vectors, pass 2 writes the marginals; speculative
// uniform-shift step with exact replay; drift feedback), but a matrix of at most 32 x 32 fits one
// wave, so a step needs no LDS memory and no barrier: its latency is a handful of lane exchanges
// instead of two workgroup barriers.  That latency is what bounds these shapes (a step moves
// 1 to 8 KB), both for whole sequences and for the chunks of the scan.
//
// Lane mapping for the padded size TP (16 or 32): CG = TP / 4 lanes cover one row with four
// columns each (16-byte loads), the RG = 64 / CG row groups own R = TP / RG consecutive rows
// each: lane (rg, cg) holds phi[R rg + k][4 cg + j], k < R, j < 4.
//
// A vector of TP entries lives in registers in one of two forms:
//   column form: lane (rg, cg) holds entries 4 cg + j   (the same in every row group);
//   row form:    lane (rg, cg) holds entries R rg + k   (the same in every column group).
// The forward step takes alpha in row form and, after summing over the row groups, leaves the
// new alpha in column form; the backward step takes beta in column form and leaves the new beta
// in row form.  Turning one form into the other is a transpose of the 8 x 8 (4 x 16) lane grid:
// at most four ds_bpermute per step.
#include "lccrf_chain_args.h"
#include "lccrf_device.h"
#include "lccrf_launch.h"

#include <type_traits>

namespace lccrf {

template <int TP>
struct WGeo {
    static_assert(TP == 16 || TP == 32, "padded tag-set sizes served by one wave");
    static constexpr int CG = TP / 4;
    static constexpr int RG = 64 / CG;
    static constexpr int R = TP / RG;  // 1 or 4
};

__device__ __forceinline__ float lane_read(float x, int src_lane) {
    return __int_as_float(__builtin_amdgcn_ds_bpermute(src_lane << 2, __float_as_int(x)));
}

template <int TP>
__device__ __forceinline__ void col_to_row(const float (&vc)[4], float (&vr)[WGeo<TP>::R], int lane) {
    if constexpr (TP == 32) {
        // entries 4 rg + k are the four registers of any lane whose column group is rg
        const int src = (lane & ~7) | (lane >> 3);
#pragma unroll
        for (int k = 0; k < WGeo<TP>::R; ++k) vr[k] = lane_read(vc[k], src);
    } else {
        // entry rg is register rg % 4 of a lane whose column group is rg / 4; every lane offers
        // the register its own row group selects and is read by lanes of that same row group
        const int sel = (lane >> 2) & 3;
        const float pub = sel == 0 ? vc[0] : sel == 1 ? vc[1] : sel == 2 ? vc[2] : vc[3];
        vr[0] = lane_read(pub, (lane & ~3) | (lane >> 4));
    }
}

template <int TP>
__device__ __forceinline__ void row_to_col(const float (&vr)[WGeo<TP>::R], float (&vc)[4], int lane) {
    if constexpr (TP == 32) {
        // entries 4 cg + j are the four registers of any lane whose row group is cg
        const int src = ((lane & 7) << 3) | (lane >> 3);
#pragma unroll
        for (int j = 0; j < 4; ++j) vc[j] = lane_read(vr[j], src);
    } else {
        // entry 4 cg + j is the register of any lane whose row group is 4 cg + j
        const int cg = lane & 3;
#pragma unroll
        for (int j = 0; j < 4; ++j) vc[j] = lane_read(vr[0], ((4 * cg + j) << 2) | cg);
    }
}

template <int TP, typename TIN, bool ALIGNED>
__device__ __forceinline__ void wave_load(const TIN* __restrict__ mat, int T, int lane, float (&v)[WGeo<TP>::R][4],
                                          bool followed = false) {
    using W = WGeo<TP>;
    const int c4 = 4 * (lane % W::CG), s0 = W::R * (lane / W::CG);
    if (ALIGNED) {
#pragma unroll
        for (int k = 0; k < W::R; ++k) {
            const int s = s0 + k;
            const TIN* row = mat + (size_t)(s < T ? s : T - 1) * T;
            Elem<TIN>::get4(row + (c4 < T ? c4 : T - 4), v[k]);
        }
    } else if (followed && T > 1) {  // (the same for the whole wave: one scalar branch)
#pragma unroll
        for (int k = 0; k < W::R; ++k) load_row4_anywhere<TIN, true>(mat, T, s0 + k, c4, v[k]);
    } else {
#pragma unroll
        for (int k = 0; k < W::R; ++k) load_row4_anywhere<TIN, false>(mat, T, s0 + k, c4, v[k]);
    }
}
// What has to follow wave_load where the tile is consumed (nothing if the tag count is a multiple of four).
template <int TP, bool ALIGNED>
__device__ __forceinline__ void wave_settle(float (&v)[WGeo<TP>::R][4], int T, int lane) {
    if constexpr (!ALIGNED) {
        const int c4 = 4 * (lane % WGeo<TP>::CG);
#pragma unroll
        for (int k = 0; k < WGeo<TP>::R; ++k) settle_row4(v[k], T, c4);
    }
}

// The same lane's share of an emission row (row 0 of the slot) for structured potentials.
template <int TP, bool ALIGNED>
__device__ __forceinline__ void wave_load_emit(const float* __restrict__ emit_row, int T, int lane, float (&v)[WGeo<TP>::R][4],
                                               bool followed = false) {
    load_emit4<ALIGNED>(emit_row, T, 4 * (lane % WGeo<TP>::CG), v[0], followed);
}
// What has to come between wave_load_emit and add_trans (nothing if the tag count is a multiple of four).
template <int TP, bool ALIGNED>
__device__ __forceinline__ void wave_settle_emit(float (&v)[WGeo<TP>::R][4], int T, int lane) {
    settle_emit4<ALIGNED>(v[0], T, 4 * (lane % WGeo<TP>::CG));
}

__device__ __forceinline__ float max4(const float (&x)[4]) { return fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])); }

// One forward position: r(t) = log2 sum_s 2^(ua(s) + phi2(s,t)), ua in row form, r in column form.
// With WITH_MU it also writes mu(s,t) = 2^(ua(s) + phi2(s,t) + ubK(t)) and returns their sum.
// The speculative form shifts everything by c; it stands only if every sum it made is in range.
// With WITH_H it also advances the conditional entropy of the path behind the current tag (base 2):
//     h_new(t) = sum_s q(s|t) [h(s) - log2 q(s|t)],  q(s|t) = 2^(ua(s) + phi2(s,t)) / sum_s' (same),
// computed as U(t) / S(t) + log2 S(t) with U(t) = sum_s e(s,t) [h(s) - log2 e(s,t)] for the same
// shifted exponentials e the step already forms (hin in row form, hout in column form).

// With ENT = 1 (and WITH_MU) the marginals mu_i(s,t) are not stored: the step adds the conditional entropy
// of the edge, H(y_i | y_{i-1}) = sum_s m(s) log2 m(s) - sum_{s,t} mu log2 mu with m(s) = sum_t mu_i(s,t)
// (base 2, every term in the lane that holds it; the caller sums hacc over the wave at the end).
// ENT = 2: neither are they stored; the step adds sum_{s,t} mu_i(s,t) wt(s,t) for the weights wt handed in
// (natural units: the expectation of a second chain's potentials under this chain).
template <int TP, bool WITH_MU, bool ALIGNED, bool WITH_H = false, int ENT = 0>
__device__ __forceinline__ void wave_fwd_step(float (&v)[WGeo<TP>::R][4], const float (&ua)[WGeo<TP>::R], float c,
                                              const float (&ubK)[4], float* __restrict__ mu_out, int T, int lane,
                                              bool exact_only, float (&r)[4], float& tot,
                                              const float (&hin)[WGeo<TP>::R], float (&hout)[4], float& hacc,
                                              const float (*wt)[4] = nullptr) {
    using W = WGeo<TP>;
    constexpr int R = W::R;
    const int c4 = 4 * (lane % W::CG), s0 = R * (lane / W::CG);
    bool accepted = false;
    if (!exact_only) {
        float ls[4] = {0.f, 0.f, 0.f, 0.f}, gm[4] = {0.f, 0.f, 0.f, 0.f}, lu[4] = {0.f, 0.f, 0.f, 0.f};
        float lgm[4] = {0.f, 0.f, 0.f, 0.f}, hstep = 0.f;
        if (WITH_MU) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                lgm[j] = c + ubK[j];
                gm[j] = ex2(lgm[j]);
            }
        }
#pragma unroll
        for (int k = 0; k < R; ++k) {
            const float uac = ua[k] - c;
            float e[4], rowl = 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float arg = __builtin_fmaf(v[k][j], kLog2e, uac);
                e[j] = ex2(arg);
                ls[j] += e[j];
                if (WITH_H) lu[j] = __builtin_fmaf(e[j], hin[k] - log2_term(arg), lu[j]);
                if (ENT == 1) {
                    const float w = e[j] * gm[j];
                    rowl += w;
                    hstep -= w > 0.f ? w * (arg + lgm[j]) : 0.f;
                }
                if (ENT == 2) {
                    const float w = e[j] * gm[j];
                    hstep += w > 0.f ? w * wt[k][j] : 0.f;
                }
            }
            if (ENT == 1) {
                const float m = xor_sum<1, W::CG>(rowl);
                hstep += (c4 == 0 && m > 0.f) ? m * lg2(m) : 0.f;
            } else if (ENT == 0 && WITH_MU) {
                store4<ALIGNED>(mu_out, T, s0 + k, c4, e[0] * gm[0], e[1] * gm[1], e[2] * gm[2], e[3] * gm[3]);
            }
        }
        const float part = (ls[0] * gm[0] + ls[1] * gm[1]) + (ls[2] * gm[2] + ls[3] * gm[3]);
        bool ok = true;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float S = xor_sum<W::CG, 64>(ls[j]);
            const bool inm = c4 + j < T;
            r[j] = inm ? c + lg2(S) : LCCRF_NEG_INF;
            ok = ok && (!inm || sum_in_range(S));
            if (WITH_H) hout[j] = inm ? entropy_of(xor_sum<W::CG, 64>(lu[j]), S) : 0.f;
        }
        accepted = __builtin_amdgcn_ballot_w64(!ok) == 0;
        if (WITH_MU && accepted) tot = xor_sum<1, 64>(part);
        if (ENT != 0 && accepted) hacc += hstep;
    }
    if (!accepted) {
        float lm[4] = {LCCRF_NEG_INF, LCCRF_NEG_INF, LCCRF_NEG_INF, LCCRF_NEG_INF};
#pragma unroll
        for (int k = 0; k < R; ++k)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                v[k][j] = __builtin_fmaf(v[k][j], kLog2e, ua[k]);
                lm[j] = fmaxf(lm[j], v[k][j]);
            }
        float M[4], g[4], ls[4] = {0.f, 0.f, 0.f, 0.f}, gm[4] = {0.f, 0.f, 0.f, 0.f}, lu[4] = {0.f, 0.f, 0.f, 0.f};
        float lgm[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            M[j] = xor_max<W::CG, 64>(lm[j]);
            g[j] = finite_or_zero(M[j]);
            if (WITH_MU) {
                lgm[j] = g[j] + ubK[j];
                gm[j] = ex2(lgm[j]);
            }
        }
#pragma unroll
        for (int k = 0; k < R; ++k) {
            float e[4], rowl = 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float arg = v[k][j] - g[j];
                e[j] = ex2(arg);
                ls[j] += e[j];
                if (WITH_H) lu[j] = __builtin_fmaf(e[j], hin[k] - log2_term(arg), lu[j]);
                if (ENT == 1) {
                    const float w = e[j] * gm[j];
                    rowl += w;
                    hacc -= w > 0.f ? w * (arg + lgm[j]) : 0.f;
                }
                if (ENT == 2) {
                    const float w = e[j] * gm[j];
                    hacc += w > 0.f ? w * wt[k][j] : 0.f;
                }
            }
            if (ENT == 1) {
                const float m = xor_sum<1, W::CG>(rowl);
                hacc += (c4 == 0 && m > 0.f) ? m * lg2(m) : 0.f;
            } else if (ENT == 0 && WITH_MU) {
                store4<ALIGNED>(mu_out, T, s0 + k, c4, e[0] * gm[0], e[1] * gm[1], e[2] * gm[2], e[3] * gm[3]);
            }
        }
        if (WITH_MU) tot = xor_sum<1, 64>((ls[0] * gm[0] + ls[1] * gm[1]) + (ls[2] * gm[2] + ls[3] * gm[3]));
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float S = xor_sum<W::CG, 64>(ls[j]);
            r[j] = (c4 + j < T) ? M[j] + lg2(S) : LCCRF_NEG_INF;  // M = -inf gives S = 0: -inf
            if (WITH_H) hout[j] = (c4 + j < T) ? entropy_of(xor_sum<W::CG, 64>(lu[j]), S) : 0.f;
        }
    }
}

// One backward position: r(s) = log2 sum_t 2^(phi2(s,t) + ub(t)), ub in column form, r in row form.
// WITH_H: the conditional entropy of the path ahead of the current tag (hin in column form, hout in row form).
// ENT as in wave_fwd_step; here m(s) = S(s) f(s) and the factor f(s) of row s drops out of log2 (mu / m).
template <int TP, bool WITH_MU, bool ALIGNED, bool WITH_H = false, int ENT = 0>
__device__ __forceinline__ void wave_bwd_step(float (&v)[WGeo<TP>::R][4], const float (&ub)[4], float c,
                                              const float (&uaK)[WGeo<TP>::R], float* __restrict__ mu_out, int T,
                                              int lane, bool exact_only, float (&r)[WGeo<TP>::R], float& tot,
                                              const float (&hin)[4], float (&hout)[WGeo<TP>::R], float& hacc,
                                              const float (*wt)[4] = nullptr) {
    using W = WGeo<TP>;
    constexpr int R = W::R;
    const int c4 = 4 * (lane % W::CG), s0 = R * (lane / W::CG);
    bool accepted = false;
    if (!exact_only) {
        const float ubc[4] = {ub[0] - c, ub[1] - c, ub[2] - c, ub[3] - c};
        float part = 0.f, hstep = 0.f;
        bool ok = true;
#pragma unroll
        for (int k = 0; k < R; ++k) {
            float e[4], Ul = 0.f, El = 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float arg = __builtin_fmaf(v[k][j], kLog2e, ubc[j]);
                e[j] = ex2(arg);
                if (WITH_H) Ul = __builtin_fmaf(e[j], hin[j] - log2_term(arg), Ul);
                if (ENT == 1) El += e[j] > 0.f ? e[j] * arg : 0.f;
                if (ENT == 2) El += e[j] > 0.f ? e[j] * wt[k][j] : 0.f;
            }
            const float Sl = (e[0] + e[1]) + (e[2] + e[3]);
            const float S = xor_sum<1, W::CG>(Sl);
            if (WITH_MU) {
                const float f = ex2(c + uaK[k]);
                if (ENT == 1) hstep += f > 0.f ? f * (((c4 == 0 && S > 0.f) ? S * lg2(S) : 0.f) - El) : 0.f;
                else if (ENT == 2) hstep += f > 0.f ? f * El : 0.f;
                else store4<ALIGNED>(mu_out, T, s0 + k, c4, e[0] * f, e[1] * f, e[2] * f, e[3] * f);
                part += Sl * f;
            }
            const bool inm = s0 + k < T;
            r[k] = inm ? c + lg2(S) : LCCRF_NEG_INF;
            ok = ok && (!inm || sum_in_range(S));
            if (WITH_H) hout[k] = inm ? entropy_of(xor_sum<1, W::CG>(Ul), S) : 0.f;
        }
        accepted = __builtin_amdgcn_ballot_w64(!ok) == 0;
        if (WITH_MU && accepted) tot = xor_sum<1, 64>(part);
        if (ENT != 0 && accepted) hacc += hstep;
    }
    if (!accepted) {
        float part = 0.f;
#pragma unroll
        for (int k = 0; k < R; ++k) {
#pragma unroll
            for (int j = 0; j < 4; ++j) v[k][j] = __builtin_fmaf(v[k][j], kLog2e, ub[j]);
            const float m = xor_max<1, W::CG>(max4(v[k]));
            const float g = finite_or_zero(m);
            float e[4], Ul = 0.f, El = 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float arg = v[k][j] - g;
                e[j] = ex2(arg);
                if (WITH_H) Ul = __builtin_fmaf(e[j], hin[j] - log2_term(arg), Ul);
                if (ENT == 1) El += e[j] > 0.f ? e[j] * arg : 0.f;
                if (ENT == 2) El += e[j] > 0.f ? e[j] * wt[k][j] : 0.f;
            }
            const float Sl = (e[0] + e[1]) + (e[2] + e[3]);
            const float S = xor_sum<1, W::CG>(Sl);
            if (WITH_MU) {
                const float f = ex2(g + uaK[k]);
                if (ENT == 1) hacc += f > 0.f ? f * (((c4 == 0 && S > 0.f) ? S * lg2(S) : 0.f) - El) : 0.f;
                else if (ENT == 2) hacc += f > 0.f ? f * El : 0.f;
                else store4<ALIGNED>(mu_out, T, s0 + k, c4, e[0] * f, e[1] * f, e[2] * f, e[3] * f);
                part += Sl * f;
            }
            r[k] = (s0 + k < T) ? m + lg2(S) : LCCRF_NEG_INF;
            if (WITH_H) hout[k] = (s0 + k < T) ? entropy_of(xor_sum<1, W::CG>(Ul), S) : 0.f;
        }
        if (WITH_MU) tot = xor_sum<1, 64>(part);
    }
}

// -log2 of the sum of the marginals the last step wrote (0 if nothing usable was written).
__device__ __forceinline__ float drift_of(float tot) { return (tot > 0.5f && tot < 2.0f) ? -lg2(tot) : 0.f; }

// Tiles in flight per wave: more in the first pass, whose slots are smaller (no stored vector rides along).
constexpr int wave_ring_depth(int TP, bool second_pass) { return second_pass ? (TP == 16 ? 2 : 2) : (TP == 16 ? 8 : 6); }

// ---------------------------------------------------------------------------------------
// Pass 1: both half chains, vectors stored.
// STRUCT: potentials are trans + emit (a compile-time choice: a branch around the loads would cost the
// exact wait counts that keep the ring of tiles in flight).
// Where the two passes keep the vectors of a chain: position `pos` of the sequence at index
// pos - origin (device memory: the sequence's rows of the workspace arrays, origin 0; LDS: the
// positions of one chunk, origin = its first position).
struct VecStore {
    float* ua;
    float* ub;
    double* Oa;
    double* Ob;
    int origin;
};

__device__ __forceinline__ VecStore device_vectors(const ChainArgs& a, int b) {
    const size_t vb = (size_t)b * a.N;
    return VecStore{a.ua + vb * a.T, a.ub + vb * a.T, a.Oa + vb, a.Ob + vb, 0};
}

// MEET_ONLY: only the vectors of the meeting position are stored (all a log-partition needs).
template <int TP, typename TIN, bool ALIGNED, bool WITH_H, bool STRUCT, int PF = wave_ring_depth(TP, false), bool MEET_ONLY = false>
__device__ __forceinline__ void wave_half_body(const ChainArgs& a, const Span& sp, int dir, int lane, const VecStore& vs) {
    using W = WGeo<TP>;
    constexpr int R = W::R;
    const int cg = lane % W::CG, rg = lane / W::CG, c4 = 4 * cg, s0 = R * rg;
    if (sp.empty) return;
    const int b = sp.b, N = a.N, T = a.T;
    const int p0 = sp.p0, e = sp.e;
    const int h = forward_end(a, p0, e);
    if (a.full_forward && dir == 1) return;
    const size_t TT = (size_t)T * T;
    const TIN* phib = static_cast<const TIN*>(a.phi) + (size_t)b * N * TT;
    const bool exact_only = a.exact_only != 0;
    float ring[PF][R][4];
    constexpr bool structured = STRUCT;
    const float* emb = structured ? a.emit + (size_t)b * N * T : nullptr;
    float tr[R][4];
    if constexpr (structured) {
        wave_load<TP, float, ALIGNED>(a.trans, T, lane, tr);
        wave_settle<TP, ALIGNED>(tr, T, lane);
    }
    auto load = [&](int i, int slot) {
        if constexpr (structured) wave_load_emit<TP, ALIGNED>(emb + (size_t)i * T, T, lane, ring[slot], b != a.B - 1 || i != N - 1);
        else wave_load<TP, TIN, ALIGNED>(phib + (size_t)i * TT, T, lane, ring[slot], b != a.B - 1 || i != N - 1);
    };
    const float none4[4] = {0.f, 0.f, 0.f, 0.f};
    float noneR[R];
#pragma unroll
    for (int k = 0; k < R; ++k) noneR[k] = 0.f;
    float tot = 0.f;
    double O = 0.0;

    if (dir == 0) {
        float vc[4];  // alpha, column form
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int t = c4 + j;
            vc[j] = LCCRF_NEG_INF;
            if (t < T)
                vc[j] = !sp.first ? a.Fv[((size_t)b * a.C + sp.c - 1) * T + t]
                        : (structured ? a.trans[t] + emb[t] : Elem<TIN>::get(phib + t)) * kLog2e;
        }
        if (!sp.first) O = a.OF[(size_t)b * a.C + sp.c - 1];
        auto settle = [&](int pos) {  // normalise the vector of position `pos` and store it
            const float d = finite_or_zero(xor_max<1, W::CG>(max4(vc)));
            O += (double)d;
#pragma unroll
            for (int j = 0; j < 4; ++j) vc[j] -= d;
            if ((WITH_H || MEET_ONLY) && pos != h) return d;  // an entropy query needs the vectors of the meeting position only
            if (rg == 0) {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (c4 + j < T) vs.ua[(pos - vs.origin) * T + c4 + j] = vc[j];
            }
            if (lane == 0) vs.Oa[pos - vs.origin] = O;
            return d;
        };
        float hc[4] = {0.f, 0.f, 0.f, 0.f};  // entropy of the path behind each tag, column form
        walk<PF>(p0 + 1, h, +1, load, [&](int i, int slot) {
            if constexpr (structured) {
                wave_settle_emit<TP, ALIGNED>(ring[slot], T, lane);
                add_trans<R>(ring[slot], tr);
            }
            else wave_settle<TP, ALIGNED>(ring[slot], T, lane);
            const float d = settle(i - 1);
            float ua[R], hrow[R];
            col_to_row<TP>(vc, ua, lane);
            if (WITH_H) col_to_row<TP>(hc, hrow, lane);
            wave_fwd_step<TP, false, ALIGNED, WITH_H>(ring[slot], ua, d, none4, nullptr, T, lane, exact_only, vc, tot, hrow, hc, tot);
        });
        settle(h);
        if (WITH_H && rg == 0) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (c4 + j < T) a.ha[(size_t)b * T + c4 + j] = hc[j];
        }
    } else {
        float vr[R];  // beta, row form
#pragma unroll
        for (int k = 0; k < R; ++k) {
            const int s = s0 + k;
            vr[k] = LCCRF_NEG_INF;
            if (s < T) vr[k] = sp.last ? 0.f : a.Gv[((size_t)b * a.C + sp.c) * T + s];
        }
        if (!sp.last) O = a.OG[(size_t)b * a.C + sp.c];
        auto settle = [&](int pos) {
            float m = vr[0];
#pragma unroll
            for (int k = 1; k < R; ++k) m = fmaxf(m, vr[k]);
            const float d = finite_or_zero(xor_max<W::CG, 64>(m));
            O += (double)d;
#pragma unroll
            for (int k = 0; k < R; ++k) vr[k] -= d;
            if ((WITH_H || MEET_ONLY) && pos != h) return d;
            if (cg == 0) {
#pragma unroll
                for (int k = 0; k < R; ++k)
                    if (s0 + k < T) vs.ub[(pos - vs.origin) * T + s0 + k] = vr[k];
            }
            if (lane == 0) vs.Ob[pos - vs.origin] = O;
            return d;
        };
        float hr[R];  // entropy of the path ahead of each tag, row form
#pragma unroll
        for (int k = 0; k < R; ++k) hr[k] = 0.f;
        walk<PF>(e, h + 1, -1, load, [&](int i, int slot) {
            if constexpr (structured) {
                wave_settle_emit<TP, ALIGNED>(ring[slot], T, lane);
                add_trans<R>(ring[slot], tr);
            }
            else wave_settle<TP, ALIGNED>(ring[slot], T, lane);
            const float d = settle(i);
            float ub[4], hcol[4];
            row_to_col<TP>(vr, ub, lane);
            if (WITH_H) row_to_col<TP>(hr, hcol, lane);
            wave_bwd_step<TP, false, ALIGNED, WITH_H>(ring[slot], ub, d, noneR, nullptr, T, lane, exact_only, vr, tot, hcol, hr, tot);
        });
        settle(h);
        if (WITH_H && cg == 0) {
#pragma unroll
            for (int k = 0; k < R; ++k)
                if (s0 + k < T) a.hb[(size_t)b * T + s0 + k] = hr[k];
        }
    }
}

template <int TP, typename TIN, bool ALIGNED, bool WITH_H, bool STRUCT>
__global__ __launch_bounds__(64) void wave_half_kernel(ChainArgs a) {
    const Span sp = make_span(a, blockIdx.x >> 1);
    wave_half_body<TP, TIN, ALIGNED, WITH_H, STRUCT>(a, sp, blockIdx.x & 1, threadIdx.x, device_vectors(a, sp.b));
}

// ---------------------------------------------------------------------------------------
// Pass 2: both chains continue past the meeting point and write the marginals.
// ENT: no marginal is written; every wave adds up the conditional entropies H(y_i | y_{i-1}) of its
// edges (the wave of position 0 also H(y_0)) and leaves the sum, base 2, in a.ent[2 (b C + c) + dir]:
// by the chain rule their total is the entropy of the sequence.
// ENT = 2: the same with the expectation of a second chain's potentials a.psi under this chain's
// marginals, sum_e mu(e) psi(e) (a.ent_kind = 2), or of psi - phi (a.ent_kind = 3), in natural units.
template <int TP, typename TIN, bool ALIGNED, bool STRUCT, int ENT = 0>
__device__ __forceinline__ void wave_marginal_body(const ChainArgs& a, const Span& sp, int dir, int lane, const VecStore& vs) {
    using W = WGeo<TP>;
    constexpr int R = W::R, PF = wave_ring_depth(TP, true);
    const int cg = lane % W::CG, rg = lane / W::CG, c4 = 4 * cg, s0 = R * rg;
    const int b = sp.b, N = a.N, T = a.T, L = sp.L;
    const size_t TT = (size_t)T * T;
    const int og = vs.origin;
    float* mub = ENT != 0 ? nullptr : a.mu + (size_t)b * N * TT;
    const bool exact_only = a.exact_only != 0;
    float hacc = 0.f;

    if (ENT == 0 && dir == 0) {
        // positions past the end carry no edge: their marginals are zero (a chunk clears its own range)
        const int zfrom = a.chunk > 0 ? (sp.c * a.chunk > L ? sp.c * a.chunk : L) : L;
        const int zto = a.chunk > 0 ? ((sp.c + 1) * a.chunk < N ? (sp.c + 1) * a.chunk : N) : N;
        const size_t z0 = (size_t)zfrom * TT, z1 = (size_t)(zto > zfrom ? zto : zfrom) * TT;
        if (ALIGNED) {
            float4* p = reinterpret_cast<float4*>(mub);
            for (size_t k = z0 / 4 + lane; k < z1 / 4; k += 64) p[k] = make_float4(0.f, 0.f, 0.f, 0.f);
        } else {
            for (size_t k = z0 + lane; k < z1; k += 64) mub[k] = 0.f;
        }
    }
    if (L == 0) {
        if (dir == 0 && sp.c == 0 && lane == 0 && a.logZ) a.logZ[b] = 0.f;
        return;
    }
    if (sp.empty) return;
    const int p0 = sp.p0, e = sp.e;
    const int h = meeting_point(p0, e);
    const TIN* phib = static_cast<const TIN*>(a.phi) + (size_t)b * N * TT;

    // log2 Z from the two vectors stored for the meeting position
    double lz2;
    {
        float z[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int t = c4 + j;
            z[j] = (t < T) ? vs.ua[(h - og) * T + t] + vs.ub[(h - og) * T + t] : LCCRF_NEG_INF;
        }
        const float M = xor_max<1, W::CG>(max4(z));
        const float g = finite_or_zero(M);
        const float S = xor_sum<1, W::CG>((ex2(z[0] - g) + ex2(z[1] - g)) + (ex2(z[2] - g) + ex2(z[3] - g)));
        lz2 = (double)(M + lg2(S)) + vs.Oa[h - og] + vs.Ob[h - og];
    }
    const bool feasible = lz2 > -1.0e300;  // false: no path has a finite score, marginals are 0
    if (dir == 0 && sp.c == 0 && lane == 0 && a.logZ) a.logZ[b] = (float)(lz2 * kLn2);

    float ring[PF][R][4];
    constexpr bool structured = STRUCT;
    static_assert(!(STRUCT && ENT == 2), "no expectations over structured potentials");
    const float* emb = structured ? a.emit + (size_t)b * N * T : nullptr;
    float tr[R][4];
    if constexpr (structured) {
        wave_load<TP, float, ALIGNED>(a.trans, T, lane, tr);
        wave_settle<TP, ALIGNED>(tr, T, lane);
    }
    const TIN* psib = ENT == 2 ? static_cast<const TIN*>(a.psi) + (size_t)b * N * TT : nullptr;
    const bool difference = a.ent_kind == 3;
    float ringq[ENT == 2 ? PF : 1][R][4];
    auto load_phi = [&](int i, int slot) {
        if constexpr (structured) wave_load_emit<TP, ALIGNED>(emb + (size_t)i * T, T, lane, ring[slot], b != a.B - 1 || i != N - 1);
        else wave_load<TP, TIN, ALIGNED>(phib + (size_t)i * TT, T, lane, ring[slot], b != a.B - 1 || i != N - 1);
        if constexpr (ENT == 2) wave_load<TP, TIN, ALIGNED>(psib + (size_t)i * TT, T, lane, ringq[slot], b != a.B - 1 || i != N - 1);
    };
    // the weights of the expectation for the tile in `slot` (before the step rewrites the tile)
    float wt[R][4];
    auto weights = [&](int slot) {
        if constexpr (ENT == 2) {
#pragma unroll
            for (int k = 0; k < R; ++k)
#pragma unroll
                for (int j = 0; j < 4; ++j) wt[k][j] = difference ? ringq[slot][k][j] - ring[slot][k][j] : ringq[slot][k][j];
        }
    };
    float kappa = 0.f, tot = 0.f;
    float noh_c[4] = {0.f, 0.f, 0.f, 0.f}, noh_r[R];  // no entropy carried in this pass
#pragma unroll
    for (int k = 0; k < R; ++k) noh_r[k] = 0.f;

    if (dir == 0) {
        double O = vs.Oa[h - og];
        float vc[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) vc[j] = (c4 + j < T) ? vs.ua[(h - og) * T + c4 + j] : LCCRF_NEG_INF;
        float aux[PF][4];
        double ob[PF];
        auto load = [&](int i, int slot) {
            load_phi(i, slot);
#pragma unroll
            for (int j = 0; j < 4; ++j) aux[slot][j] = vs.ub[(i - og) * T + (c4 + j < T ? c4 + j : T - 1)];
            ob[slot] = vs.Ob[i - og];
        };
        walk<PF>(h + 1, e, +1, load, [&](int i, int slot) {
            if constexpr (structured) {
                wave_settle_emit<TP, ALIGNED>(ring[slot], T, lane);
                add_trans<R>(ring[slot], tr);
            }
            else wave_settle<TP, ALIGNED>(ring[slot], T, lane);
            if constexpr (ENT == 2) wave_settle<TP, ALIGNED>(ringq[slot], T, lane);
            const float d = finite_or_zero(xor_max<1, W::CG>(max4(vc)));
            kappa += drift_of(tot);
            O += (double)d;
#pragma unroll
            for (int j = 0; j < 4; ++j) vc[j] -= d;
            float ua[R];
            col_to_row<TP>(vc, ua, lane);
            const float K = feasible ? (float)(O + ob[slot] - lz2) + kappa : LCCRF_NEG_INF;
            float ubK[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) ubK[j] = (c4 + j < T) ? aux[slot][j] + K : LCCRF_NEG_INF;
            weights(slot);
            wave_fwd_step<TP, true, ALIGNED, false, ENT>(ring[slot], ua, d, ubK, ENT != 0 ? nullptr : mub + (size_t)i * TT, T, lane, exact_only, vc, tot, noh_r, noh_c, hacc, wt);
        });
    } else {
        double O = vs.Ob[h - og];
        float vr[R];
#pragma unroll
        for (int k = 0; k < R; ++k) vr[k] = (s0 + k < T) ? vs.ub[(h - og) * T + s0 + k] : LCCRF_NEG_INF;
        float aux[PF][R];
        double oa[PF];
        auto load = [&](int i, int slot) {
            load_phi(i, slot);
#pragma unroll
            for (int k = 0; k < R; ++k) aux[slot][k] = vs.ua[(i - 1 - og) * T + (s0 + k < T ? s0 + k : T - 1)];
            oa[slot] = vs.Oa[i - 1 - og];
        };
        walk<PF>(h, p0 + 1, -1, load, [&](int i, int slot) {
            if constexpr (structured) {
                wave_settle_emit<TP, ALIGNED>(ring[slot], T, lane);
                add_trans<R>(ring[slot], tr);
            }
            else wave_settle<TP, ALIGNED>(ring[slot], T, lane);
            if constexpr (ENT == 2) wave_settle<TP, ALIGNED>(ringq[slot], T, lane);
            float m = vr[0];
#pragma unroll
            for (int k = 1; k < R; ++k) m = fmaxf(m, vr[k]);
            const float d = finite_or_zero(xor_max<W::CG, 64>(m));
            kappa += drift_of(tot);
            O += (double)d;
#pragma unroll
            for (int k = 0; k < R; ++k) vr[k] -= d;
            float ub[4];
            row_to_col<TP>(vr, ub, lane);
            const float K = feasible ? (float)(oa[slot] + O - lz2) + kappa : LCCRF_NEG_INF;
            float uaK[R];
#pragma unroll
            for (int k = 0; k < R; ++k) uaK[k] = (s0 + k < T) ? aux[slot][k] + K : LCCRF_NEG_INF;
            weights(slot);
            wave_bwd_step<TP, true, ALIGNED, false, ENT>(ring[slot], ub, d, uaK, ENT != 0 ? nullptr : mub + (size_t)i * TT, T, lane, exact_only, vr, tot, noh_c, noh_r, hacc, wt);
        });
        // position 0: p(y_0 = t) = softmax_t(alpha_0(t) + beta_0(t)) in row 0, zeros elsewhere
        if (!sp.first) {
            if (ENT != 0) {
                hacc = xor_sum<1, 64>(hacc);
                if (lane == 0) a.ent[2 * ((size_t)b * a.C + sp.c) + 1] = hacc;
            }
            return;
        }
        if (ENT == 0)
            for (int k = T + lane; k < (int)TT; k += 64) mub[k] = 0.f;
        float z[R], m = LCCRF_NEG_INF;
#pragma unroll
        for (int k = 0; k < R; ++k) {
            z[k] = (s0 + k < T) ? vs.ua[(0 - og) * T + s0 + k] + vr[k] : LCCRF_NEG_INF;
            m = fmaxf(m, z[k]);
        }
        m = finite_or_zero(xor_max<W::CG, 64>(m));
        float S = 0.f;
#pragma unroll
        for (int k = 0; k < R; ++k) S += ex2(z[k] - m);
        S = xor_sum<W::CG, 64>(S);
        const float cnorm = (feasible && S > 0.f) ? 1.0f / S : 0.f;
        if (cg == 0) {
#pragma unroll
            for (int k = 0; k < R; ++k) {
                if (s0 + k >= T) continue;
                const float p = cnorm * ex2(z[k] - m);
                if (ENT == 1) {
                    hacc -= p > 0.f ? p * (z[k] - m - lg2(S)) : 0.f;  // H(y_0)
                } else if (ENT == 2) {  // the first row of the first matrix
                    const float q0 = Elem<TIN>::get(psib + s0 + k);
                    hacc += p > 0.f ? p * (difference ? q0 - Elem<TIN>::get(phib + s0 + k) : q0) : 0.f;
                } else {
                    mub[s0 + k] = p;
                }
            }
        }
    }
    if (ENT != 0) {
        hacc = xor_sum<1, 64>(hacc);
        if (lane == 0) a.ent[2 * ((size_t)b * a.C + sp.c) + dir] = hacc;
    }
}

template <int TP, typename TIN, bool ALIGNED, bool STRUCT, int ENT = 0>
__global__ __launch_bounds__(64) void wave_marginal_kernel(ChainArgs a) {
    const Span sp = make_span(a, blockIdx.x >> 1);
    wave_marginal_body<TP, TIN, ALIGNED, STRUCT, ENT>(a, sp, blockIdx.x & 1, threadIdx.x, device_vectors(a, sp.b));
}

// Both passes of one chunk in one workgroup of two waves (the forward and the backward chain), the
// vectors of the chunk's positions in LDS instead of the workspace: one launch and no trip through
// device memory between the passes.  Chunks of at most kFusedChunk positions.
constexpr int kFusedChunk = 64;
constexpr int kFusedFirstDepth = 3;  // tiles in flight in its first half (registers are what bounds its waves a SIMD)

template <int TP, typename TIN, bool ALIGNED, int ENT>
__global__ __launch_bounds__(128) void wave_chunk_kernel(ChainArgs a) {
    __shared__ float sua[(kFusedChunk + 1) * TP], sub[(kFusedChunk + 1) * TP];
    __shared__ double sOa[kFusedChunk + 1], sOb[kFusedChunk + 1];
    const int lane = threadIdx.x & 63, dir = threadIdx.x >> 6;
    const Span sp = make_span(a, blockIdx.x);
    const VecStore vs{sua, sub, sOa, sOb, sp.p0};
    wave_half_body<TP, TIN, ALIGNED, false, false, kFusedFirstDepth>(a, sp, dir, lane, vs);
    __syncthreads();
    wave_marginal_body<TP, TIN, ALIGNED, false, ENT>(a, sp, dir, lane, vs);
}

// The log-partition of whole sequences in one launch: the two half chains of a sequence as the two
// waves of a workgroup, their vectors at the meeting position in LDS, combined by the first wave.
template <int TP, typename TIN, bool ALIGNED>
__global__ __launch_bounds__(128) void wave_logz_kernel(ChainArgs a) {
    __shared__ float sua[TP], sub[TP];
    __shared__ double sO[2];
    const int lane = threadIdx.x & 63, dir = threadIdx.x >> 6;
    const Span sp = make_span(a, blockIdx.x);
    const int b = sp.b, T = a.T, L = sp.L;
    if (L == 0) {
        if (threadIdx.x == 0 && a.logZ) a.logZ[b] = 0.f;
        if (threadIdx.x == 0 && a.logZ64) a.logZ64[b] = 0.0;
        return;
    }
    const VecStore vs{sua, sub, &sO[0], &sO[1], meeting_point(sp.p0, sp.e)};
    wave_half_body<TP, TIN, ALIGNED, false, false, wave_ring_depth(TP, false), true>(a, sp, dir, lane, vs);
    __syncthreads();
    if (dir == 0) {
        const float z = lane < T ? sua[lane] + sub[lane] : LCCRF_NEG_INF;
        const float m = xor_max<1, 64>(z);
        const float S = xor_sum<1, 64>(ex2(z - finite_or_zero(m)));
        const double lz = ((double)(m + lg2(S)) + sO[0] + sO[1]) * kLn2;
        if (lane == 0 && a.logZ) a.logZ[b] = (float)lz;
        if (lane == 0 && a.logZ64) a.logZ64[b] = lz;
    }
}

// ---------------------------------------------------------------------------------------
bool wave_supported(int T) { return T >= 1 && T <= 32; }

template <int TP>
static hipError_t launch_wave_logz_tp(int dtype, const ChainArgs& a, hipStream_t st) {
    const dim3 grid(a.B), block(128);
    const bool aligned = (a.T % 4) == 0;
    if (dtype == 0) {
        if (aligned) hipLaunchKernelGGL((wave_logz_kernel<TP, float, true>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((wave_logz_kernel<TP, float, false>), grid, block, 0, st, a);
    } else {
        if (aligned) hipLaunchKernelGGL((wave_logz_kernel<TP, uint16_t, true>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((wave_logz_kernel<TP, uint16_t, false>), grid, block, 0, st, a);
    }
    return hipGetLastError();
}

// logZ (a.logZ and/or a.logZ64) of whole sequences, plain potentials, T <= 32.
hipError_t launch_wave_logz(int dtype, const ChainArgs& a, hipStream_t st) {
    return a.T <= 16 ? launch_wave_logz_tp<16>(dtype, a, st) : launch_wave_logz_tp<32>(dtype, a, st);
}
bool wave_chunks_fused(int chunk) { return chunk >= 1 && chunk <= kFusedChunk; }

template <int TP, typename TIN, bool ALIGNED>
static hipError_t launch_wave_chunks_tp(const ChainArgs& a, hipStream_t st) {
    const dim3 grid(a.B * a.C), block(128);
    if (a.ent && a.ent_kind >= 2) hipLaunchKernelGGL((wave_chunk_kernel<TP, TIN, ALIGNED, 2>), grid, block, 0, st, a);
    else if (a.ent) hipLaunchKernelGGL((wave_chunk_kernel<TP, TIN, ALIGNED, 1>), grid, block, 0, st, a);
    else hipLaunchKernelGGL((wave_chunk_kernel<TP, TIN, ALIGNED, 0>), grid, block, 0, st, a);
    return hipGetLastError();
}

// Both passes over every chunk of `a` in one launch (a.chunk > 0, wave_chunks_fused(a.chunk), plain potentials).
hipError_t launch_wave_chunks(int dtype, const ChainArgs& a, hipStream_t st) {
    const bool aligned = (a.T % 4) == 0;
    if (a.T <= 16) {
        if (dtype == 0) return aligned ? launch_wave_chunks_tp<16, float, true>(a, st) : launch_wave_chunks_tp<16, float, false>(a, st);
        return aligned ? launch_wave_chunks_tp<16, uint16_t, true>(a, st) : launch_wave_chunks_tp<16, uint16_t, false>(a, st);
    }
    if (dtype == 0) return aligned ? launch_wave_chunks_tp<32, float, true>(a, st) : launch_wave_chunks_tp<32, float, false>(a, st);
    return aligned ? launch_wave_chunks_tp<32, uint16_t, true>(a, st) : launch_wave_chunks_tp<32, uint16_t, false>(a, st);
}

template <int TP, typename TIN, bool ALIGNED>
static hipError_t launch_wave_tp(bool second_pass, const ChainArgs& a, hipStream_t st) {
    const dim3 grid(2 * a.B * a.C);
    if constexpr (std::is_same<TIN, float>::value) {
        if (a.emit) {  // structured potentials: float only, no entropy mode
            if (second_pass)
                hipLaunchKernelGGL((wave_marginal_kernel<TP, float, ALIGNED, true>), grid, dim3(64), 0, st, a);
            else
                hipLaunchKernelGGL((wave_half_kernel<TP, float, ALIGNED, false, true>), grid, dim3(64), 0, st, a);
            return hipGetLastError();
        }
    }
    if (second_pass && a.ent && a.ent_kind >= 2)
        hipLaunchKernelGGL((wave_marginal_kernel<TP, TIN, ALIGNED, false, 2>), grid, dim3(64), 0, st, a);
    else if (second_pass && a.ent)
        hipLaunchKernelGGL((wave_marginal_kernel<TP, TIN, ALIGNED, false, 1>), grid, dim3(64), 0, st, a);
    else if (second_pass)
        hipLaunchKernelGGL((wave_marginal_kernel<TP, TIN, ALIGNED, false>), grid, dim3(64), 0, st, a);
    else if (a.ha)
        hipLaunchKernelGGL((wave_half_kernel<TP, TIN, ALIGNED, true, false>), grid, dim3(64), 0, st, a);
    else
        hipLaunchKernelGGL((wave_half_kernel<TP, TIN, ALIGNED, false, false>), grid, dim3(64), 0, st, a);
    return hipGetLastError();
}

// One pass over all chains of `a` (a.C = 1 for whole sequences): the first stores the vectors of
// both half chains, the second writes the marginals.
hipError_t launch_wave_pass(bool second_pass, int dtype, const ChainArgs& a, hipStream_t st) {
    const bool aligned = (a.T % 4) == 0;
    if (a.T <= 16) {
        if (dtype == 0)
            return aligned ? launch_wave_tp<16, float, true>(second_pass, a, st) : launch_wave_tp<16, float, false>(second_pass, a, st);
        return aligned ? launch_wave_tp<16, uint16_t, true>(second_pass, a, st)
                       : launch_wave_tp<16, uint16_t, false>(second_pass, a, st);
    }
    if (dtype == 0)
        return aligned ? launch_wave_tp<32, float, true>(second_pass, a, st) : launch_wave_tp<32, float, false>(second_pass, a, st);
    return aligned ? launch_wave_tp<32, uint16_t, true>(second_pass, a, st)
                   : launch_wave_tp<32, uint16_t, false>(second_pass, a, st);
}

}  // namespace lccrf
