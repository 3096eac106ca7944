// Sum-product chains for 8 .. 64 tags with the recursion taken off the streaming work: one wave of a
// workgroup runs the chain, the others stream the potentials.
//
// The sequential forward recursion (section "Sequence Tagging": O(m^2 n) work, n dependent steps) is
// what bounds batches that do not fill the chip: a step of the kernels in lccrf_wave.hip / lccrf_chain.hip
// costs 1400 to 2000 cycles, most of them the exponentials, the logarithm and the lane reductions of a
// log-sum-exp that all sit on the chain of dependent instructions.  Here a step of the chain is a plain
// vector-matrix product in the linear domain,
//     V'(u) = sum_v V(v) E(u, v),      E = 2^(phi log2 e - m),  m = ceil(max of the matrix),
// by ONE wave with lane u holding V(u): sixteen fused multiply-adds per block of sixteen source tags,
// the source values arriving by DPP row rotation (v_fmac_f32_dpp row_ror:n), the blocks by the gfx950
// permlane swaps; no exponential, no logarithm and no reduction tree on the dependent path.  The matrix
// entries a lane needs, in the order its rotations consume them, wait in LDS: the other waves of the
// workgroup ("producers") load the potentials (coalesced 16-byte loads, the next matrix of a wave in flight
// while it works on the current one), exponentiate them and scatter them into a ring of LDS slots in that
// rotated order.  A producer then waits for the chain to accept the step its matrix belongs to and does the
// step's stores: in the first pass the resulting vector (base-2 logarithms plus a double offset, the format of
// the other sum-product kernels, so either pass may be combined with theirs), in the second pass the marginals
// mu = V(s) E(s,t) G(t) of that position from the matrix it still holds in registers (coalesced 16-byte
// stores).  The waves meet only through words in LDS (ready / done / stop), never at a barrier.
//
// Vectors are kept as V 2^O with O = O0 + an integer: every matrix is shifted by an integer m, and after every
// step the vector is rescaled by the power of two that brings tag 0's entry into [1/2, 1) (any accepted entry
// serves as the reference; lane 0's comes without a reduction).  A step is accepted only if every sum lies in
// [2^-60, 2^60] (kSumLo, kSumHi): then whatever underflowed in it is below 2^-66 of the sum it belongs to, for
// every entry separately, so the loss does not compound from step to step.  A step that is not accepted (a
// hard zero from a potential of -inf, entries of one matrix hundreds of bits apart) is taken by the chain wave
// itself in the log domain, straight from memory, every log-sum-exp shifted by its own maximum, stores and
// marginals included; the fast path resumes as soon as the vector is one that scaled single precision holds
// faithfully again.  Eight such steps in a row, or a producer that does not deliver within the poll limit,
// send the chain wave into the log-domain tail for the rest of its half chain; the producers see `stop` and
// leave.
#include "lccrf_chain_args.h"
#include "lccrf_device.h"
#include "lccrf_launch.h"
#include "lccrf_lds_flags.h"

#include <type_traits>

namespace lccrf {

// Waves of a workgroup: wave 0 runs the chain (at raised priority), the others are producers.  Up to 32 tags a
// producer needs few registers and eleven of them keep the second pass fed (B=128 N=256 T=32: second pass
// 51.8 -> 47.9 us against seven); above, seven is what the register file holds at two waves a SIMD.
constexpr int lane_waves(int nblk) { return nblk <= 2 ? 12 : 8; }
constexpr int kLaneMaxProducers = 11;
constexpr int kLaneVecRing = 16;        // published vectors kept (the chain leads a producer by fewer than that)

template <int NBLK>
struct LaneShape {
    static_assert(NBLK >= 1 && NBLK <= 4, "one to four blocks of sixteen tags");
    static constexpr int U = 16 * NBLK;  // padded tag count
    static constexpr int RS = U + 4;     // floats per LDS row: 16-byte reads of consecutive rows hit distinct banks
    static constexpr int RING = 8;       // LDS slots for matrices (a power of two: slot = step & 7)
    static constexpr int NG = NBLK * NBLK;  // groups of four entries a producer lane holds of one matrix
    static constexpr int PF = 2;  // matrices per producer wave: one in hand, one in flight
};

template <int NBLK>
struct LaneShared {
    using S = LaneShape<NBLK>;
    float E[S::RING][S::U + 1][S::RS];  // E[slot][u][16 b + n] = the entry lane u multiplies with rotation n of block b
                                        // (row U stays zero: read by the lanes of the chain wave that hold no tag)
    float V[kLaneVecRing][64];      // V_q, the vector that enters step q, at [q % kLaneVecRing]
    int VOi[kLaneVecRing];          // twice its offset less O0 (the shifts and rescales so far: an integer), plus 1
                                    // if the step that produced it was taken in the log domain by the chain wave
    double O0;                      // offset of V_0
    float G[kLaneMaxProducers][64]; // per producer wave: the factors of the stored vector of the other chain
    unsigned long long ready[S::RING];  // once the matrix of step q sits in slot q % RING: q + 1 in the high word,
                                        // the matrix's shift (an integer) in the low word: one read brings both
    int done;                       // steps the chain has accepted
    int stop;                       // first step of the log-domain tail (INT_MAX: none)
};

// acc[0] + .. + acc[3] += sum over n of (a of the lane n places to the left in its row of sixteen) * e[n]
// (four accumulators: a lone wave sees the full latency of every dependent instruction).
#define LCCRF_FM(N, ACC, E) "v_fmac_f32_dpp %" #ACC ", %4, %" #E " row_ror:" #N " row_mask:0xf bank_mask:0xf\n\t"
__device__ __forceinline__ void fmac_rotations(float (&acc)[4], float a, const float (&e)[16]) {
    asm volatile("s_nop 1\n\t"  // a vector result needs two wait states before a DPP read
        "v_fmac_f32_e32 %0, %4, %5\n\t"
        LCCRF_FM(1, 1, 6) LCCRF_FM(2, 2, 7) LCCRF_FM(3, 3, 8) LCCRF_FM(4, 0, 9) LCCRF_FM(5, 1, 10) LCCRF_FM(6, 2, 11)
        LCCRF_FM(7, 3, 12) LCCRF_FM(8, 0, 13) LCCRF_FM(9, 1, 14) LCCRF_FM(10, 2, 15) LCCRF_FM(11, 3, 16)
        LCCRF_FM(12, 0, 17) LCCRF_FM(13, 1, 18) LCCRF_FM(14, 2, 19) LCCRF_FM(15, 3, 20)
        : "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3])
        : "v"(a), "v"(e[0]), "v"(e[1]), "v"(e[2]), "v"(e[3]), "v"(e[4]), "v"(e[5]), "v"(e[6]), "v"(e[7]), "v"(e[8]),
          "v"(e[9]), "v"(e[10]), "v"(e[11]), "v"(e[12]), "v"(e[13]), "v"(e[14]), "v"(e[15]));
}
#undef LCCRF_FM

__device__ __forceinline__ float lane_value(float x, int src) {  // src uniform over the wave
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), src));
}

// What a chain is working on (uniform over the workgroup).
struct LaneJob {
    int b, dir, L, h;
    int first, sdir, count;  // step q consumes the matrix of position first + q sdir
};

// Where the potentials of sequence b come from: a dense tensor of TIN, or (StructF) trans[s][t] + emit[b][i][t],
// the single-precision sum the materialised tensor would hold.  at(): one potential; piece(): the four of row s,
// columns t0 .. t0 + 3 (flat offset off = s T + t0), `fixed` being what fixed_part() returned for that piece.
// AL: the tag count is a multiple of four and every piece lies on a 16-byte boundary.  Otherwise the rows start at any
// multiple of the element size: the last piece of a row is moved back to end where the row ends (it overlaps the
// piece before it; the entries both hold are the same numbers, written to the same places), and a piece is loaded and
// stored through types that promise the compiler no more than the element's alignment.
struct StructF {};
template <bool AL, typename E>
__device__ __forceinline__ void lane_load4(const E* p, float (&o)[4]) {
    if constexpr (AL) Elem<E>::get4(p, o);
    else Elem<E>::get4_anywhere(p, o);
}
template <bool AL>
__device__ __forceinline__ void lane_store4(float* p, float a, float b, float c, float d) {
    if constexpr (AL) {
        *reinterpret_cast<float4*>(p) = make_float4(a, b, c, d);
    } else {
        store4_anywhere(p, a, b, c, d);
    }
}
template <typename TIN, bool AL>
struct LaneSource {
    static constexpr bool kStruct = false;
    const TIN* phib;
    size_t TT;
    int T;
    __device__ __forceinline__ LaneSource(const ChainArgs& a, int b)
        : phib(static_cast<const TIN*>(a.phi) + (size_t)b * a.N * a.T * a.T), TT((size_t)a.T * a.T), T(a.T) {}
    __device__ __forceinline__ float at(int i, int s, int t) const { return Elem<TIN>::get(phib + (size_t)i * TT + (size_t)s * T + t); }
    __device__ __forceinline__ void fixed_part(int, int, float (&f)[4]) const { f[0] = f[1] = f[2] = f[3] = 0.f; }
    __device__ __forceinline__ void piece(int i, int off, int, const float (&)[4], float (&o)[4]) const {
        lane_load4<AL>(phib + (size_t)i * TT + off, o);
    }
};
template <bool AL>
struct LaneSource<StructF, AL> {
    static constexpr bool kStruct = true;
    const float* emb;
    const float* trans;
    int T;
    __device__ __forceinline__ LaneSource(const ChainArgs& a, int b) : emb(a.emit + (size_t)b * a.N * a.T), trans(a.trans), T(a.T) {}
    __device__ __forceinline__ float at(int i, int s, int t) const { return trans[(size_t)s * T + t] + emb[(size_t)i * T + t]; }
    __device__ __forceinline__ void fixed_part(int off, int, float (&f)[4]) const { lane_load4<AL>(trans + off, f); }
    __device__ __forceinline__ void piece(int i, int, int t0, const float (&f)[4], float (&o)[4]) const {
        float e[4];
        lane_load4<AL>(emb + (size_t)i * T + t0, e);
#pragma unroll
        for (int k = 0; k < 4; ++k) o[k] = f[k] + e[k];
    }
};

// One position in the log domain by the chain wave alone, straight from memory: every log-sum-exp shifted by
// its own maximum.  lv: the vector that enters step q, base-2 logarithms, lane = tag (-inf from T on), O its
// offset; on return lv is the result less the integer shift that is returned (its maximum then lies in (-1, 0]).
// Writes what the step owes to memory: the marginals of its position (second pass), the stored vector (first).
template <typename TIN, bool AL, bool PASS2>
__device__ __forceinline__ int lane_log_step(const ChainArgs& a, const LaneJob& jb, int q, float& lv, double O,
                                             double lz2, int meet_only) {
    const int lane = threadIdx.x & 63, T = a.T, N = a.N, b = jb.b;
    const size_t TT = (size_t)T * T;
    const LaneSource<TIN, AL> src(a, b);
    const size_t vb = (size_t)b * N;
    const int i = jb.first + q * jb.sdir;
    const bool on = lane < T;
    const int me = on ? lane : 0;
    float other = LCCRF_NEG_INF, K = 0.f;
    float* mu_i = nullptr;
    if (PASS2) {
        // forward: beta_i(t) and its offset; backward: alpha_{i-1}(s) and its offset
        const size_t vp = jb.dir == 0 ? vb + i : vb + i - 1;
        other = on ? (jb.dir == 0 ? a.ub : a.ua)[vp * T + me] : LCCRF_NEG_INF;
        K = (float)(O + (jb.dir == 0 ? a.Ob : a.Oa)[vp] - lz2);
        mu_i = a.mu + (vb + i) * TT;
    }
    float mx = LCCRF_NEG_INF;
    for (int v = 0; v < T; ++v) {
        const float x = lane_value(lv, v) + (jb.dir == 0 ? src.at(i, v, me) : src.at(i, me, v)) * kLog2e;
        mx = fmaxf(mx, x);
    }
    const float g = finite_or_zero(mx);
    float sum = 0.f;
    for (int v = 0; v < T; ++v) {
        const float x = lane_value(lv, v) + (jb.dir == 0 ? src.at(i, v, me) : src.at(i, me, v)) * kLog2e;
        sum += ex2(x - g);
        if (PASS2 && on) {
            const float m = ex2(x + other + K);
            if (jb.dir == 0) mu_i[(size_t)v * T + lane] = m;
            else mu_i[(size_t)lane * T + v] = m;
        }
    }
    const float r = on ? mx + lg2(sum) : LCCRF_NEG_INF;
    // an integer shift, clamped far inside the range of an int: the offsets stay O0 plus an integer
    const float d = fminf(fmaxf(ceilf(finite_or_zero(xor_max<1, 64>(r))), -0x1p30f), 0x1p30f);
    lv = r - d;
    if (!PASS2) {
        const int pos = jb.dir == 0 ? i : i - 1;
        if (!meet_only || pos == jb.h) {
            if (on) (jb.dir == 0 ? a.ua : a.ub)[(vb + pos) * T + lane] = lv;
            if (lane == 0) (jb.dir == 0 ? a.Oa : a.Ob)[vb + pos] = O + (double)d;
        }
    }
    return __builtin_amdgcn_readfirstlane((int)d);  // (the same in every lane; said so, it stays in a scalar register)
}

// The log-domain tail: steps q0 .. count - 1 of the job.  Returns with lv / O the last vector.
template <typename TIN, bool AL, bool PASS2>
__device__ __forceinline__ void lane_log_tail(const ChainArgs& a, const LaneJob& jb, int q0, float& lv, double& O,
                                              double lz2, int meet_only) {
    for (int q = q0; q < jb.count; ++q) O += (double)lane_log_step<TIN, AL, PASS2>(a, jb, q, lv, O, lz2, meet_only);
}

// The chain wave.
template <int NBLK, typename TIN, bool AL, bool PASS2>
__device__ __forceinline__ void lane_chain_wave(const ChainArgs& a, const LaneJob& jb, LaneShared<NBLK>& sh, double lz2,
                                                bool feasible, int meet_only, int poll_limit) {
    using S = LaneShape<NBLK>;
    const int lane = threadIdx.x & 63, T = a.T, N = a.N, b = jb.b;
    const size_t TT = (size_t)T * T;
    const size_t vb = (size_t)b * N;
    // Up to 32 tags the 64 lanes hold the vector twice and each copy sums over one block of sixteen source
    // tags (half the products a step; the halves meet through one permlane swap); above, lane = tag.
    constexpr bool kSplit = NBLK == 2;
    const int u = kSplit ? (lane & 31) : lane;  // the tag of this lane
    const int copy = kSplit ? (lane >> 5) : 0;
    bool on = u < T;
    const int me = on ? u : 0;
    const int urow = u < S::U ? (u < T ? u : S::U) : S::U;  // its row of the matrices in LDS (row U: zeros)
    // the vector that enters step 0
    float lv;  // base-2 logarithm, used for the stores of the first pass and by the tail
    double O = 0.0;
    if (!PASS2) {
        if (jb.dir == 0) {
            const float x = on ? LaneSource<TIN, AL>(a, b).at(0, 0, me) * kLog2e : LCCRF_NEG_INF;  // row 0 of the first matrix
            const float d = ceilf(finite_or_zero(xor_max<1, 64>(x)));
            lv = x - d;
            O = (double)d;
        } else {
            lv = on ? 0.f : LCCRF_NEG_INF;
        }
        const int pos = jb.dir == 0 ? 0 : jb.L - 1;
        if (!meet_only || pos == jb.h) {
            if (on && copy == 0) (jb.dir == 0 ? a.ua : a.ub)[(vb + pos) * T + u] = lv;
            if (lane == 0) (jb.dir == 0 ? a.Oa : a.Ob)[vb + pos] = O;
        }
    } else {
        lv = on ? (jb.dir == 0 ? a.ua : a.ub)[(vb + jb.h) * T + me] : LCCRF_NEG_INF;
        O = (jb.dir == 0 ? a.Oa : a.Ob)[vb + jb.h];
    }
    float V = ex2(lv);  // 0 for lanes past T
    const double O0 = O;
    int Oi = 0;  // O = O0 + Oi: the shifts of the matrices and the rescales so far
    if (copy == 0) sh.V[0][u] = V;
    if (lane == 0) {
        sh.VOi[0] = 0;
        sh.O0 = O0;
    }
    const unsigned long long onmask = __builtin_amdgcn_ballot_w64(on);
    unsigned q = 0;
    const unsigned count = (unsigned)jb.count;
    bool tail = false, carried = false;
    float lv_carry = LCCRF_NEG_INF;  // the vector in logarithms, where the log-domain steps leave it to the tail
    // The matrix of a step: the entries of this lane in the order its rotations consume them, and the shift.
    constexpr int NB = kSplit ? 1 : NBLK;  // blocks of sixteen source tags a lane sums over
    struct Tile {
        float e[NB][16];
        int m;
    };
    const auto read_entries = [&](unsigned step, Tile& t) {
        const unsigned slot = step % S::RING;
#pragma unroll
        for (int bk = 0; bk < NB; ++bk)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const float4 v = *reinterpret_cast<const float4*>(&sh.E[slot][urow][16 * (kSplit ? copy : bk) + 4 * g]);
                t.e[bk][4 * g] = v.x; t.e[bk][4 * g + 1] = v.y; t.e[bk][4 * g + 2] = v.z; t.e[bk][4 * g + 3] = v.w;
            }
    };
    const auto read_tile = [&](unsigned step, Tile& t, unsigned long long word) {
        t.m = __builtin_amdgcn_readfirstlane((int)(unsigned)word);
        read_entries(step, t);
    };
    // waits for the matrix of `step` (bounded) and reads it; false: it did not come
    const auto fetch = [&](unsigned step, Tile& t) -> bool {
        int spins = 0;
        unsigned long long word;
        while ((unsigned)__builtin_amdgcn_readfirstlane((int)((word = lds_load_acquire(&sh.ready[step % S::RING])) >> 32)) < step + 1)
            if (++spins > poll_limit) return false;
        read_tile(step, t, word);
        return true;
    };
    // Steps that the fast path does not accept (a sum out of range: entries of one matrix hundreds of bits
    // apart, or a hard zero) are taken in the log domain by this wave itself, one position at a time, until the
    // vector is again one that scaled single precision holds faithfully (every entry an exact zero or within
    // 2^-60 of the largest): then the fast path resumes with the next matrix.  The producers are told through
    // the low bit of the published offset to leave those positions alone.  After eight such steps in a row
    // (hard constraints throughout) the chain gives the producers up for good.
    // 0: go on (the matrix of step q is in `nxt`), 2: it did not come, 3: that was the last step, 4: give up.
    const auto slow_steps = [&](Tile& nxt) -> int {
        float lvs = lane < T ? lg2(V) : LCCRF_NEG_INF;
        for (int n = 0;; ++n) {
            const int d = lane_log_step<TIN, AL, PASS2>(a, jb, (int)q, lvs, O0 + (double)Oi, lz2, meet_only);
            Oi += d;
            float lall = lvs;  // every copy of the vector gets its tag's value
            if constexpr (kSplit) {
                const auto h = __builtin_amdgcn_permlane32_swap(__float_as_int(lvs), __float_as_int(lvs), false, false);
                lall = __int_as_float(h[0]);
            }
            V = on ? ex2(lall) : 0.f;
            ++q;
            sh.V[q % kLaneVecRing][u] = V;
            sh.VOi[q % kLaneVecRing] = (Oi << 1) | 1;
            lds_store_release(&sh.done, (int)q);
            if (q == count) return 3;
            const bool faithful = !(lane < T) || lvs == LCCRF_NEG_INF || lvs >= -60.f;
            const bool inside = (unsigned)(Oi + (1 << 28)) < (1u << 29);
            if (__builtin_amdgcn_ballot_w64(!faithful) == 0 && inside) break;
            if (n >= 7 || !inside) {
                lv_carry = lvs;
                carried = true;
                return 4;
            }
        }
        return fetch(q, nxt) ? 0 : 2;
    };
    // One step from the matrix in `cur`; meanwhile the matrix of the next step is read into `nxt`, whether it is
    // there or not, so that it comes back under the products: its flag is looked at before (LDS executes a wave's
    // instructions in order: a flag that was up when it was read means that the reads behind it found the matrix);
    // if it was not up, the matrix is waited for at the end of the step and read again.  Everything the step leaves behind for the other waves is the vector, one
    // integer and the step count in LDS: the stores to memory are theirs.
    // 0: go on, 1: the step was not accepted (q and the vector are unchanged), 2: the next matrix did not come,
    // 3: that was the last step.
    // (Flags and offsets are written by every lane, the same value to the same address: cheaper for a lone
    // wave than masking the write down to one lane.)
    const auto step = [&](const Tile& cur, Tile& nxt) __attribute__((always_inline)) -> int {
        unsigned long long word_next = lds_load_acquire(&sh.ready[(q + 1) % S::RING]);
        read_entries(q + 1, nxt);
        __builtin_amdgcn_sched_barrier(0);
        float Ab[4];
        if constexpr (NBLK == 1) {
            Ab[0] = V;
        } else {
            const auto p = __builtin_amdgcn_permlane16_swap(__float_as_int(V), __float_as_int(V), false, false);
            if constexpr (NBLK == 2) {
                Ab[0] = copy == 0 ? __int_as_float(p[0]) : __int_as_float(p[1]);  // block `copy` in both rows of the copy
            } else {
                const auto x = __builtin_amdgcn_permlane32_swap(p[0], p[0], false, false);
                const auto w = __builtin_amdgcn_permlane32_swap(p[1], p[1], false, false);
                Ab[0] = __int_as_float(x[0]); Ab[2] = __int_as_float(x[1]);
                Ab[1] = __int_as_float(w[0]); Ab[3] = __int_as_float(w[1]);
            }
        }
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int bk = 0; bk < NB; ++bk) fmac_rotations(acc, Ab[bk], cur.e[bk]);
        // (the flag is looked at only here, behind the products: its read has had their time to come back)
        asm volatile("" : "+v"(word_next));
        float Ssum = (acc[0] + acc[1]) + (acc[2] + acc[3]);
        if constexpr (kSplit) {  // the two halves of the sum
            const auto h = __builtin_amdgcn_permlane32_swap(__float_as_int(Ssum), __float_as_int(Ssum), false, false);
            Ssum = __int_as_float(h[0]) + __int_as_float(h[1]);
        }
        const int Onew = Oi + cur.m;
        // accepted: every sum in range, and the integer offset far from overflow
        // (S in [kSumLo, kSumHi] as one unsigned comparison of its bits: positive floats order like their bit patterns,
        // negative ones and NaNs fall outside; the comparison leaves the lane mask in scalar registers directly)
        const unsigned long long inr = __builtin_amdgcn_uicmp(__float_as_uint(Ssum) - __float_as_uint(kSumLo),
                                                              __float_as_uint(kSumHi) - __float_as_uint(kSumLo), 37 /* unsigned <= */);
        if ((inr & onmask) != onmask || (unsigned)(Onew + (1 << 28)) >= (1u << 29)) return 1;
        // Rescale by the power of two that brings tag 0 into [1/2, 1): any accepted entry serves as the
        // reference (what bounds the vector is the range test above, not where its largest entry lies), and
        // lane 0's comes without a reduction over the lanes.  Lanes without a tag hold an exact zero.
        const int k = __builtin_amdgcn_readfirstlane(__builtin_amdgcn_frexp_expf(Ssum));
        V = __builtin_amdgcn_ldexpf(Ssum, -k);
        Oi = Onew + k;
        ++q;
        sh.V[q % kLaneVecRing][u] = V;
        sh.VOi[q % kLaneVecRing] = Oi << 1;
        lds_store_release(&sh.done, (int)q);
        if (q == count) return 3;
        if ((unsigned)__builtin_amdgcn_readfirstlane((int)(word_next >> 32)) >= q + 1) nxt.m = __builtin_amdgcn_readfirstlane((int)(unsigned)word_next);
        else if (!fetch(q, nxt)) return 2;
        return 0;
    };
    Tile tA, tB;
    if (count > 0) {
        int why = fetch(0, tA) ? 0 : 2;
        for (;;) {
            while (why == 0) {
                why = step(tA, tB);
                if (why != 0) break;
                why = step(tB, tA);
            }
            if (why != 1) break;
            why = slow_steps(tA);  // (outside the loop of the fast path, which stays as tight as it was)
        }
        tail = why != 3;
    }
    O = O0 + (double)Oi;
    on = lane < T;  // from here on lane = tag again (the first copy)
    lv = !on ? LCCRF_NEG_INF : carried ? lv_carry : lg2(V);
    if (tail) {
        if (lane == 0) lds_store_release(&sh.stop, (int)q);
        lane_log_tail<TIN, AL, PASS2>(a, jb, (int)q, lv, O, lz2, meet_only);
    } else if (!PASS2 && meet_only && count > 0) {
        // a log-partition call keeps the vectors of the meeting position only: the last of this chain
        if (on) (jb.dir == 0 ? a.ua : a.ub)[(vb + jb.h) * T + lane] = lv;
        if (lane == 0) (jb.dir == 0 ? a.Oa : a.Ob)[vb + jb.h] = O;
    }
    if (PASS2 && jb.dir == 1) {
        // position 0: p(y_0 = t) = 2^(alpha_0(t) + beta_0(t) - log2 Z) in row 0 (the other rows were cleared at the start)
        const float z = on ? a.ua[vb * T + me] + lv + (float)(a.Oa[vb] + O - lz2) : LCCRF_NEG_INF;
        if (on) a.mu[vb * TT + lane] = feasible ? ex2(z) : 0.f;
    }
}

// A producer wave.
template <int NBLK, typename TIN, bool AL, bool PASS2>
__device__ __forceinline__ void lane_producer_wave(const ChainArgs& a, const LaneJob& jb, LaneShared<NBLK>& sh, int w,
                                                   double lz2, int meet_only, int poll_limit) {
    using S = LaneShape<NBLK>;
    constexpr int NG = S::NG, PF = S::PF, W = lane_waves(NBLK) - 1;
    const int lane = threadIdx.x & 63, T = a.T, N = a.N, b = jb.b;
    const size_t TT = (size_t)T * T;
    const size_t vb = (size_t)b * N;
    const LaneSource<TIN, AL> src(a, b);
    const int nj = w < jb.count ? (jb.count - w + W - 1) / W : 0;  // matrices of this wave: steps w, w + W, ...
    if (nj == 0) return;
    // group m of this lane: piece g = lane + 64 m of the matrix, row s = g / Q, columns t0 .. t0 + 3, Q pieces a row:
    // t0 = 4 (g % Q), but the last piece of a row ends with the row (T - 4: only a tag count that is no multiple of
    // four moves it)
    int goff[NG], grow[NG], gcol[NG], laddr[NG][4];
    unsigned valid = 0;
    const int Q = (T + 3) >> 2;
#pragma unroll
    for (int m = 0; m < NG; ++m) {
        const int g = lane + 64 * m;
        const bool ok = g < T * Q;
        valid |= ok ? (1u << m) : 0u;
        const int s = ok ? g / Q : 0, t0 = ok ? min(4 * (g % Q), T - 4) : 0;
        goff[m] = s * T + t0;
        grow[m] = s;
        gcol[m] = t0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int t = t0 + k;
            const int u = jb.dir == 0 ? t : s, v = jb.dir == 0 ? s : t;
            laddr[m][k] = u * S::RS + 16 * (v >> 4) + ((u - v) & 15);
        }
    }
    float x[PF][NG][4], aux[PF];
    double oo[PF];
    float fixed[LaneSource<TIN, AL>::kStruct ? NG : 1][4];  // structured potentials: this lane's entries of the transition matrix
    if constexpr (LaneSource<TIN, AL>::kStruct) {
#pragma unroll
        for (int m = 0; m < NG; ++m) src.fixed_part(goff[m], gcol[m], fixed[m]);
    }
    const auto load = [&](int j, int p) {
        const int q = w + (j < nj ? j : nj - 1) * W;
        const int i = jb.first + q * jb.sdir;
#pragma unroll
        for (int m = 0; m < NG; ++m) src.piece(i, goff[m], gcol[m], fixed[LaneSource<TIN, AL>::kStruct ? m : 0], x[p][m]);
        if (PASS2) {
            const size_t vp = jb.dir == 0 ? vb + i : vb + i - 1;
            aux[p] = (jb.dir == 0 ? a.ub : a.ua)[vp * T + (lane < T ? lane : 0)];
            oo[p] = (jb.dir == 0 ? a.Ob : a.Oa)[vp];
        }
    };
    // Waits until the flag reaches `target` (true) or the chain has stopped at or before step `q` (false).
    // The chain wave always does one or the other: each of its own waits is bounded by the poll limit of the call.
    // The limit here, a thousand times the default, is a last resort that only keeps a wave from spinning for ever.
    const auto wait_for = [&](const int* flag, int target, int q) -> bool {
        long long spins = 0;
        while (lds_load_acquire(flag) < target) {
            if (lds_load_acquire(&sh.stop) <= q || ++spins > 1000ll * (poll_limit + 65536)) return false;
            __builtin_amdgcn_s_sleep(1);
        }
        return true;
    };
    // One matrix (number j of this wave, in buffer p): exponentiate, hand to the chain, write its marginals.
    // false: the chain has stopped before this matrix, nothing more to do.
    const auto process = [&](int j, auto pc) -> bool {
        constexpr int p = decltype(pc)::value;
        const int q = w + j * W;
        const int i = jb.first + q * jb.sdir;
        const int slot = q % S::RING;
        // the shift of this matrix: the smallest integer at or above its largest entry (base 2)
        float mxr = LCCRF_NEG_INF;
#pragma unroll
        for (int m = 0; m < NG; ++m) {
            const float gm = max3_raw(fmaxf(x[p][m][0], x[p][m][1]), x[p][m][2], x[p][m][3]);
            mxr = fmaxf(mxr, (valid >> m) & 1 ? gm : LCCRF_NEG_INF);
        }
        // (clamped far inside the range of an int: beyond, the chain's offset check sends the step to the tail)
        const float sh_m = fminf(fmaxf(ceilf(finite_or_zero(xor_max<1, 64>(mxr)) * kLog2e), -0x1p30f), 0x1p30f);
#pragma unroll
        for (int m = 0; m < NG; ++m)
#pragma unroll
            for (int k = 0; k < 4; ++k) x[p][m][k] = ex2(__builtin_fmaf(x[p][m][k], kLog2e, -sh_m));
        // the slot is free once the chain has accepted step q - RING
        if (!wait_for(&sh.done, q - S::RING + 1, q)) return false;
        float* Es = &sh.E[slot][0][0];
#pragma unroll
        for (int m = 0; m < NG; ++m)
            if ((valid >> m) & 1) {
#pragma unroll
                for (int k = 0; k < 4; ++k) Es[laddr[m][k]] = x[p][m][k];
            }
        if (lane == 0)
            lds_store_release(&sh.ready[slot], ((unsigned long long)(unsigned)(q + 1) << 32) | (unsigned)(int)sh_m);
        if (PASS2) {
            // the chain has accepted step q: V_q and this matrix make the marginals of position i
            if (!wait_for(&sh.done, q + 1, q)) return false;
            if (sh.VOi[(q + 1) % kLaneVecRing] & 1) return true;  // (the chain wave took this step itself)
            const double Oq = sh.O0 + (double)(sh.VOi[q % kLaneVecRing] >> 1);
            const float c = (float)(Oq + (double)sh_m + oo[p] - lz2);
            sh.G[w][lane] = lane < T ? ex2(aux[p] + c) : 0.f;
            const float* rowf = jb.dir == 0 ? sh.V[q % kLaneVecRing] : sh.G[w];
            const float* colf = jb.dir == 0 ? sh.G[w] : sh.V[q % kLaneVecRing];
            float* mu_i = a.mu + (vb + i) * TT;
#pragma unroll
            for (int m = 0; m < NG; ++m)
                if ((valid >> m) & 1) {
                    const float rf = rowf[grow[m]];
                    float cf[4];
                    lane_load4<AL>(colf + gcol[m], cf);
                    lane_store4<AL>(mu_i + goff[m], x[p][m][0] * rf * cf[0], x[p][m][1] * rf * cf[1], x[p][m][2] * rf * cf[2],
                                    x[p][m][3] * rf * cf[3]);
                }
        }
        if (!PASS2 && !meet_only) {
            // the chain has accepted step q: its result is the vector of position i (forward) or i - 1 (backward)
            if (!wait_for(&sh.done, q + 1, q)) return false;
            const int pos = jb.dir == 0 ? i : i - 1;
            const int word = sh.VOi[(q + 1) % kLaneVecRing];
            if (word & 1) return true;  // (the chain wave took this step itself, stores included)
            const float v = sh.V[(q + 1) % kLaneVecRing][lane];
            if (lane < T) (jb.dir == 0 ? a.ua : a.ub)[(vb + pos) * T + lane] = lg2(v);
            if (lane == 0) (jb.dir == 0 ? a.Oa : a.Ob)[vb + pos] = sh.O0 + (double)(word >> 1);
        }
        return true;
    };
    // Two buffers: the next matrix is requested just before the current one is worked on, so the only loads in
    // flight during a matrix are those of its successor (whatever the compiler then waits for at the top of the
    // loop, it is data the wave needs at once).
    using Buf0 = std::integral_constant<int, 0>;
    using Buf1 = std::integral_constant<int, 1>;
    load(0, 0);
    for (int j = 0; j < nj; j += 2) {
        load(j + 1, 1);
        __builtin_amdgcn_sched_barrier(0);
        if (!process(j, Buf0{})) break;
        load(j + 2, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (j + 1 < nj && !process(j + 1, Buf1{})) break;
    }
}

template <int NBLK, typename TIN, bool AL, bool PASS2>
__global__ __launch_bounds__(64 * lane_waves(NBLK)) void lane_chain_kernel(ChainArgs a, int meet_only, int poll_limit) {
    using S = LaneShape<NBLK>;
    constexpr int kLaneWaves = lane_waves(NBLK);
    extern __shared__ __attribute__((aligned(16))) unsigned char lane_smem[];
    LaneShared<NBLK>& sh = *reinterpret_cast<LaneShared<NBLK>*>(lane_smem);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform: loops over a wave's work stay scalar
    const int T = a.T, N = a.N;
    LaneJob jb;
    jb.b = blockIdx.x >> 1;
    jb.dir = blockIdx.x & 1;
    jb.L = clamp_length(a.lengths, jb.b, N);
    const int b = jb.b, L = jb.L;
    const size_t TT = (size_t)T * T;
    const size_t vb = (size_t)b * N;
    // Marginals that carry no edge are zero: the positions past the end (forward workgroup) and rows
    // 1 .. T - 1 of position 0 (backward workgroup).  Cleared by the wave that has no other work
    // (by everyone for an empty sequence).
    const auto zero_floats = [&](float* d, size_t n, int first, int threads) {  // n floats from d on, by threads first, first + 1, ...
        for (size_t k = first; k < n / 4; k += threads) lane_store4<AL>(d + 4 * k, 0.f, 0.f, 0.f, 0.f);
        if (!AL && first < (int)(n % 4)) d[n - 1 - first] = 0.f;
    };
    const auto clear_edgeless = [&](int first_thread, int threads) {
        if (jb.dir == 0) zero_floats(a.mu + (vb + L) * TT, (size_t)(N - L) * TT, tid - first_thread, threads);
        else if (L > 0) zero_floats(a.mu + vb * TT + T, TT - T, tid - first_thread, threads);
    };
    if (L == 0) {
        if (PASS2) clear_edgeless(0, 64 * kLaneWaves);
        if (PASS2 && jb.dir == 0 && tid == 0 && a.logZ) a.logZ[b] = 0.f;
        return;
    }
    const int e = L - 1;
    jb.h = meeting_point(0, e);
    if (!PASS2) {
        if (jb.dir == 0) { jb.first = 1; jb.sdir = +1; jb.count = jb.h; }
        else { jb.first = e; jb.sdir = -1; jb.count = e - jb.h; }
    } else {
        if (jb.dir == 0) { jb.first = jb.h + 1; jb.sdir = +1; jb.count = e - jb.h; }
        else { jb.first = jb.h; jb.sdir = -1; jb.count = jb.h; }
    }
    // log2 Z from the two vectors stored for the meeting position
    double lz2 = 0.0;
    bool feasible = true;
    if (PASS2) {
        const float z = lane < T ? a.ua[(vb + jb.h) * T + lane] + a.ub[(vb + jb.h) * T + lane] : LCCRF_NEG_INF;
        const float M = xor_max<1, 64>(z);
        const float Ssum = xor_sum<1, 64>(ex2(z - finite_or_zero(M)));
        lz2 = (double)(M + lg2(Ssum)) + a.Oa[vb + jb.h] + a.Ob[vb + jb.h];
        feasible = lz2 > -1.0e300;
        if (jb.dir == 0 && tid == 0 && a.logZ) a.logZ[b] = (float)(lz2 * kLn2);
        if (!feasible) {  // no path has a finite score: every marginal is zero
            for (int q = 0; q < jb.count; ++q) {
                zero_floats(a.mu + (vb + jb.first + q * jb.sdir) * TT, TT, tid, 64 * kLaneWaves);
            }
            if (jb.dir == 1 && tid < T) a.mu[vb * TT + tid] = 0.f;
            clear_edgeless(0, 64 * kLaneWaves);
            return;
        }
    }
    // flags, and zeros where no producer ever writes (source tags past T)
    if (tid < S::RING) sh.ready[tid] = 0ull;
    if (tid == 0) { sh.done = 0; sh.stop = 0x7fffffff; }
    if (T != S::U) {
        float* Ez = &sh.E[0][0][0];
        for (int k = tid; k < S::RING * (S::U + 1) * S::RS; k += 64 * kLaneWaves) Ez[k] = 0.f;
    } else {
        for (int k = tid; k < S::RING * S::RS; k += 64 * kLaneWaves) sh.E[k / S::RS][S::U][k % S::RS] = 0.f;
    }
    __syncthreads();
    if (wv == 0) {
        __builtin_amdgcn_s_setprio(3);
        lane_chain_wave<NBLK, TIN, AL, PASS2>(a, jb, sh, lz2, feasible, meet_only, poll_limit);
    } else {
        if (PASS2 && wv == 4) clear_edgeless(4 * 64, 64);  // (the producer that shares the chain's SIMD)
        lane_producer_wave<NBLK, TIN, AL, PASS2>(a, jb, sh, wv - 1, lz2, meet_only, poll_limit);
    }
}

// ---------------------------------------------------------------------------------------
// Dense or structured potentials, whole sequences, 8 .. 64 tags: multiples of four (16-byte pieces of a row) at every
// size, other counts (element loads) up to 48.
bool lane_supported(int T) { return T >= 8 && T <= 64 && (T % 4 == 0 || T <= 48); }

template <int NBLK, typename TIN, bool AL, bool PASS2>
static hipError_t launch_lane_kernel(const ChainArgs& a, int meet_only, int poll_limit, hipStream_t st) {
    const size_t bytes = sizeof(LaneShared<NBLK>);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&lane_chain_kernel<NBLK, TIN, AL, PASS2>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((lane_chain_kernel<NBLK, TIN, AL, PASS2>), dim3(2 * a.B), dim3(64 * lane_waves(NBLK)), bytes, st, a, meet_only, poll_limit);
    return hipGetLastError();
}
template <int NBLK, bool AL>
static hipError_t launch_lane_al(bool second_pass, int dtype, const ChainArgs& a, int meet_only, int poll_limit, hipStream_t st) {
    if (a.emit)
        return second_pass ? launch_lane_kernel<NBLK, StructF, AL, true>(a, meet_only, poll_limit, st)
                           : launch_lane_kernel<NBLK, StructF, AL, false>(a, meet_only, poll_limit, st);
    if (dtype == 0)
        return second_pass ? launch_lane_kernel<NBLK, float, AL, true>(a, meet_only, poll_limit, st)
                           : launch_lane_kernel<NBLK, float, AL, false>(a, meet_only, poll_limit, st);
    return second_pass ? launch_lane_kernel<NBLK, uint16_t, AL, true>(a, meet_only, poll_limit, st)
                       : launch_lane_kernel<NBLK, uint16_t, AL, false>(a, meet_only, poll_limit, st);
}
template <int NBLK>
static hipError_t launch_lane_nblk(bool second_pass, int dtype, const ChainArgs& a, int meet_only, int poll_limit, hipStream_t st) {
    if (a.T % 4 == 0) return launch_lane_al<NBLK, true>(second_pass, dtype, a, meet_only, poll_limit, st);
    if constexpr (NBLK <= 3) return launch_lane_al<NBLK, false>(second_pass, dtype, a, meet_only, poll_limit, st);
    return hipErrorInvalidValue;
}

hipError_t launch_lane_pass(bool second_pass, int dtype, const ChainArgs& a, bool meet_only, int poll_limit, hipStream_t st) {
    if (!lane_supported(a.T) || a.chunk > 0 || (a.emit && (dtype != 0 || !a.trans))) return hipErrorInvalidValue;
    const int mo = meet_only ? 1 : 0;
    if (a.T <= 16) return launch_lane_nblk<1>(second_pass, dtype, a, mo, poll_limit, st);
    if (a.T <= 32) return launch_lane_nblk<2>(second_pass, dtype, a, mo, poll_limit, st);
    if (a.T <= 48) return launch_lane_nblk<3>(second_pass, dtype, a, mo, poll_limit, st);
    return launch_lane_nblk<4>(second_pass, dtype, a, mo, poll_limit, st);
}

}  // namespace lccrf
