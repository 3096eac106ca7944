// Max-plus (Viterbi) chains for up to 64 tags with the recursion taken off everything else: one wave of a
// workgroup runs the chain of scores, the others stream the potentials and find the pointers.
//
// The recursion of section "Computing Most Probable Structure" (the forward algorithm with max in place of
// log-sum-exp), delta_i(t) = max_s delta_{i-1}(s) + phi_i(s, t), is a chain of n dependent steps, and in
// the one-wave and four-wave kernels of lccrf_viterbi.hip a step carries everything: the loads' conversion
// to double precision, the additions, and a tournament in which every comparison moves a score AND the tag
// it came from (a compare and three selects where a plain maximum is one instruction).  Only the scores are
// on the chain of dependencies: the pointer of position i needs delta_{i-1}, nothing needs the pointer
// before the trace.  So, as in the sum-product kernels of lccrf_lane.hip:
//
//   chain wave (wave 0):  out(x) = max_y in(y) + M(y, x) in double precision, v_add_f64 and v_max_f64 only,
//       M read from LDS as doubles in the order its lanes consume them (up to 32 tags: the next matrix is read
//       into registers behind the additions of the current step and comes back under its maxima), the vector
//       published in LDS;
//   helper waves (1 .. 7): each takes every seventh position: loads the matrix as it lies in memory (coalesced
//       16-byte pieces, or single elements if the tag count is no multiple of four; the next matrix in flight
//       while it works on the current one), converts it and scatters
//       it into a ring of LDS slots in the chain wave's order, then, as soon as the vector that enters the
//       position is published, finds the pointers (smallest best source tag, the tie rule of the other kernels)
//       from the matrix as it sits in the slot and keeps them for a store one matrix later.  A slot is written
//       again only after the chain wave has finished its step and its helper has read it back (`kept`).
//
// Forward and backward chains differ only in where a helper scatters an entry: M(y, x) = phi_i(y, x) for the
// forward chain (delta), phi_i(x, y) for the backward one (eps), y the tag the vector comes in on.  Lane
// part * TP + x of a wave works on column x and the RPL source tags from part * RPL on.
//
// Scores are sums in double precision of the same operands as in the other kernels and the oracle, a maximum
// is exact, and the pointer is the smallest tag that attains it: results are bit-identical whichever kernel
// ran.  The waves meet through words in LDS (ready / kept / done / stop), never at a barrier; every wait is
// bounded: a chain wave whose matrix does not come within the poll limit goes on alone (loads, scores and
// pointers, a position at a time), tells the helpers through `stop`, and they leave.
//
// What bounds a step (32 tags, cycles of a lone wave): sixteen additions and nineteen maxima at 4.75 to 8 each,
// the vector's way through LDS (a write, then eight 16-byte reads: about 190) and the LDS pipe it shares with the
// helpers (8 KB a matrix written, 8 KB read back for the pointers, 8 KB read by the chain): about 560 a step
// against 1700 in the one-wave kernel.
#include "lccrf_chain_args.h"
#include "lccrf_device.h"
#include "lccrf_launch.h"
#include "lccrf_lds_flags.h"
#include "lccrf_viterbi_args.h"

#include <type_traits>

namespace lccrf {

constexpr int kMaxWaves = 8;      // wave 0 runs the chain, the others are helpers
constexpr int kMaxHelpers = kMaxWaves - 1;
constexpr int kMaxVecRing = 16;   // published vectors kept (the chain leads a helper by fewer than that)

// TP: padded tag count (lanes per copy of the columns), ROWS: source tags covered (TP, or 48 of 64).
template <int TP, int ROWS>
struct MaxShape {
    static_assert(TP == 16 || TP == 32 || TP == 64, "16, 32 or 64 columns");
    static_assert(ROWS % 16 == 0 && ROWS <= TP && (ROWS == TP || TP == 64), "rows in blocks of sixteen");
    static constexpr int P = 64 / TP;       // lanes that share a column
    static constexpr int RPL = ROWS / P;    // source tags a lane works on: 4, 16, 48 or 64
    static constexpr int CH = RPL < 16 ? RPL : 16;  // ... in pieces of this many
    static constexpr int RING = TP < 64 ? 8 : ROWS == 48 ? 6 : 4;  // LDS slots for matrices
    static constexpr int NG = RPL / 4;      // 16-byte pieces of a matrix a helper lane loads
    static constexpr bool PRELOAD = TP <= 32;  // the chain wave holds the next matrix in registers
    static_assert(kMaxHelpers + 1 < kMaxVecRing, "a helper reads its vector before the chain can overwrite it");
};

template <int TP, int ROWS>
struct MaxShared {
    using S = MaxShape<TP, ROWS>;
    double M[S::RING][S::RPL / 2][65][2];  // M[slot][k / 2][lane][k % 2]: entry k of that lane (16-byte reads, lane after lane;
                                           // 65: the helpers' scattered writes of one instruction spread over the banks)
    double V[kMaxVecRing][TP];             // V_q, the vector that enters step q, at [q % kMaxVecRing]
    double own[2][TP];                     // the vectors of a chain wave that goes on alone
    float emis[kMaxHelpers][64];           // structured potentials: the emission scores of the position a helper works on
    int ready[S::RING];                    // q + 1 once the matrix of step q sits in slot q % RING
    int kept[S::RING];                     // q + 1 once the helper of step q has read the matrix back for its pointers
    int done;                              // steps the chain wave has finished (V_done is published)
    int stop;                              // first step the chain wave takes alone (INT_MAX: none)
};

struct MaxJob {
    int dir;
    int first, sdir, count;  // step q consumes the matrix of position first + q sdir
};

// Where the potentials of sequence b come from: a dense tensor of TIN, or (MaxStructF) trans[s][t] + emit[b][i][t],
// the single-precision sum the materialised tensor would hold.  AL: T is a multiple of four (16-byte loads).
//   first(t): the score of tag t at position 0;
//   fixed_part(s, t0, f) / piece(i, s, t0, f, o, followed): the four potentials of row s, columns t0 .. t0 + 3 of
//       position i (what lies past the end of the row if T is no multiple of four is for the caller to mask), f being
//       what fixed_part returned for that piece; followed: see Anywhere below, the other sources ignore it;
//   entries(i, dir, y0, x, v): v[k] = M(y0 + k, x), the entries one lane of the chain wave works on (addresses
//       clamped into the matrix; what lies outside is masked when it is used, max_entry).
struct MaxStructF {};
template <typename E, bool AL>
__device__ __forceinline__ void max_load4(const E* row, int T, int t0, float (&o)[4]) {  // row[t0 .. t0 + 3]
    if constexpr (AL) {
        Elem<E>::get4(row + t0, o);
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) o[k] = Elem<E>::get(row + (t0 + k < T ? t0 + k : T - 1));
    }
}
template <typename TIN, bool AL>
struct MaxSource {
    static constexpr bool kStruct = false;
    static constexpr bool kQuad = false;
    const TIN* phib;
    size_t TT;
    int T;
    __device__ __forceinline__ MaxSource(const VitArgs& a, int b)
        : phib(static_cast<const TIN*>(a.phi) + (size_t)b * a.N * a.T * a.T), TT((size_t)a.T * a.T), T(a.T) {}
    __device__ __forceinline__ float first(int t) const { return Elem<TIN>::get(phib + t); }
    __device__ __forceinline__ void fixed_part(int, int, float (&f)[4]) const { f[0] = f[1] = f[2] = f[3] = 0.f; }
    __device__ __forceinline__ void piece(int i, int s, int t0, const float (&)[4], float (&o)[4], bool) const {
        max_load4<TIN, AL>(phib + (size_t)i * TT + (size_t)s * T, T, t0, o);
    }
    template <int RPL>
    __device__ __forceinline__ void entries(int i, int dir, int y0, int x, float (&v)[RPL]) const {
        const TIN* mat = phib + (size_t)i * TT;
        const int xc = x < T ? x : T - 1;
        if (dir == 0) {
#pragma unroll
            for (int k = 0; k < RPL; ++k) v[k] = Elem<TIN>::get(mat + (size_t)(y0 + k < T ? y0 + k : T - 1) * T + xc);
        } else {
            const TIN* row = mat + (size_t)xc * T;
#pragma unroll
            for (int k = 0; k < RPL; k += 4) {
                float q[4];
                max_load4<TIN, AL>(row, T, AL ? (y0 + k < T ? y0 + k : T - 4) : y0 + k, q);
                v[k] = q[0]; v[k + 1] = q[1]; v[k + 2] = q[2]; v[k + 3] = q[3];
            }
        }
    }
};
// A dense tensor of E whose tag count is no multiple of four (and at least five), every piece of a matrix as one
// load from wherever it starts: a piece that ends a row brings the first entries of the next row with it (the caller
// masks them), and the piece that ends a matrix the first of the next matrix.  `followed` (the same for the whole
// wave) says that there is a next matrix; if there is none, the piece that ends the matrix is loaded from four
// entries earlier, where the matrix ends, and settle_last() moves its entries to their places when the piece is used.
template <typename E>
struct Anywhere {};
template <typename E, bool AL>
struct MaxSource<Anywhere<E>, AL> : MaxSource<E, false> {
    static_assert(!AL, "for tag counts that are no multiple of four");
    static constexpr bool kQuad = true;
    using Base = MaxSource<E, false>;
    __device__ __forceinline__ MaxSource(const VitArgs& a, int b) : Base(a, b) {}
    __device__ __forceinline__ void piece(int i, int s, int t0, const float (&)[4], float (&o)[4], bool followed) const {
        const int off = s * Base::T + t0, last = (int)Base::TT - 4;
        Elem<E>::get4_anywhere(Base::phib + (size_t)i * Base::TT + (followed || off < last ? off : last), o);
    }
    // The piece that ends a matrix, loaded from the matrix's last four entries: its T % 4 entries inside the matrix sit
    // at the end of what was loaded and belong at its front (`mine`: this lane holds that piece).
    __device__ __forceinline__ void settle_last(bool mine, float& o0, float& o1, float& o2, float o3) const {
        const int r = 4 - (Base::T & 3);  // 1 .. 3, the same in every lane
        const float n0 = r == 1 ? o1 : r == 2 ? o2 : o3, n1 = r == 1 ? o2 : o3;
        o0 = mine ? n0 : o0;
        o1 = mine ? n1 : o1;
        o2 = mine ? o3 : o2;
    }
};
template <bool AL>
struct MaxSource<MaxStructF, AL> {
    static constexpr bool kStruct = true;
    static constexpr bool kQuad = false;
    const float* emb;
    const float* trans;
    int T;
    __device__ __forceinline__ MaxSource(const VitArgs& a, int b) : emb(a.emit + (size_t)b * a.N * a.T), trans(a.trans), T(a.T) {}
    __device__ __forceinline__ float first(int t) const { return trans[t] + emb[t]; }
    __device__ __forceinline__ void fixed_part(int s, int t0, float (&f)[4]) const { max_load4<float, AL>(trans + (size_t)s * T, T, t0, f); }
    __device__ __forceinline__ void piece(int i, int, int t0, const float (&f)[4], float (&o)[4], bool) const {
        float e[4];
        max_load4<float, AL>(emb + (size_t)i * T, T, t0, e);
#pragma unroll
        for (int k = 0; k < 4; ++k) o[k] = f[k] + e[k];
    }
    __device__ __forceinline__ float emission(int i, int t) const { return emb[(size_t)i * T + (t < T ? t : T - 1)]; }
    template <int RPL>
    __device__ __forceinline__ void entries(int i, int dir, int y0, int x, float (&v)[RPL]) const {
        const int xc = x < T ? x : T - 1;
        const float* er = emb + (size_t)i * T;
#pragma unroll
        for (int k = 0; k < RPL; ++k) {
            const int y = y0 + k < T ? y0 + k : T - 1;
            v[k] = dir == 0 ? trans[(size_t)y * T + xc] + er[xc] : trans[(size_t)xc * T + y] + er[y];
        }
    }
};
__device__ __forceinline__ double max_entry(float v, bool inside) { return (double)(inside ? v : LCCRF_NEG_INF); }

// Best source tag per column: the winner of in(y) + M(y, x) over the lane's RPL source tags and then over the
// lanes that share the column; ties to the smaller tag, kNoArg if nothing is finite.
// A piece of CH source tags from tag ya on: vin: the vector in LDS from that tag on; entry(k): M(ya + k, x) and
// M(ya + k + 1, x) as doubles, -inf outside the matrix.  The maximum by plain maxima (one instruction a
// candidate), then the first candidate equal to it.
template <int CH, typename Entry>
__device__ __forceinline__ Best max_pointer_piece(const double* vin, int ya, Entry entry) {
    double val[CH];
#pragma unroll
    for (int k2 = 0; k2 < CH / 2; ++k2) {
        const double2 in = *reinterpret_cast<const double2*>(vin + 2 * k2);
        const double2 m = entry(2 * k2);
        val[2 * k2] = in.x + m.x;
        val[2 * k2 + 1] = in.y + m.y;
    }
    double m[CH];
#pragma unroll
    for (int k = 0; k < CH; ++k) m[k] = val[k];
#pragma unroll
    for (int w = 1; w < CH; w <<= 1)
#pragma unroll
        for (int k = 0; k + w < CH; k += 2 * w) m[k] = __builtin_fmax(m[k], m[k + w]);
    int arg = kNoArg;
#pragma unroll
    for (int k = CH - 1; k >= 0; --k) arg = val[k] == m[0] ? ya + k : arg;
    return Best{m[0], m[0] == -__builtin_huge_val() ? kNoArg : arg};
}
template <int P>
__device__ __forceinline__ Best max_pointer_parts(Best best) {
    if (P >= 4) best = swap_best<16>(best);
    if (P >= 2) best = swap_best<32>(best);
    return best;
}
template <int TP, int ROWS, typename Entry>
__device__ __forceinline__ Best max_pointer(const double* vin, int y0, Entry entry) {
    using S = MaxShape<TP, ROWS>;
    Best best{-__builtin_huge_val(), kNoArg};
#pragma unroll 1
    for (int c = 0; c < S::RPL; c += S::CH) {  // (a piece at a time: the pieces unrolled side by side would not fit the registers)
        const Best wc = max_pointer_piece<S::CH>(vin + y0 + c, y0 + c, [&](int k) { return entry(c + k); });
        if (wc.v > best.v) best = wc;  // ascending pieces: the first maximum stays
    }
    return max_pointer_parts<S::P>(best);
}

// max over the lanes that share a column (every one of them gets it)
__device__ __forceinline__ double max_raw(double a, double b) {  // (operands that are never signalling NaNs: no quieting first)
    double r;
    asm("v_max_f64 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
template <int P>
__device__ __forceinline__ double max_over_parts(double r) {
    if (P >= 4) {
        const long long b = __double_as_longlong(r);
        const int lo = (int)(b & 0xffffffffll), hi = (int)(b >> 32);
        const auto rl = __builtin_amdgcn_permlane16_swap(lo, lo, false, false);
        const auto rh = __builtin_amdgcn_permlane16_swap(hi, hi, false, false);
        r = max_raw(__longlong_as_double(((long long)(int)rh[0] << 32) | (unsigned int)rl[0]),
                    __longlong_as_double(((long long)(int)rh[1] << 32) | (unsigned int)rl[1]));
    }
    if (P >= 2) {
        const long long b = __double_as_longlong(r);
        const int lo = (int)(b & 0xffffffffll), hi = (int)(b >> 32);
        const auto rl = __builtin_amdgcn_permlane32_swap(lo, lo, false, false);
        const auto rh = __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
        r = max_raw(__longlong_as_double(((long long)(int)rh[0] << 32) | (unsigned int)rl[0]),
                    __longlong_as_double(((long long)(int)rh[1] << 32) | (unsigned int)rl[1]));
    }
    return r;
}

// The chain wave.
template <int TP, int ROWS, typename TIN, bool AL>
__device__ __forceinline__ void max_chain_wave(const VitArgs& a, const VitSpan& sp, const MaxJob& jb, MaxShared<TP, ROWS>& sh,
                                               double* mid, int poll_limit) {
    using S = MaxShape<TP, ROWS>;
    constexpr int RPL = S::RPL;
    const int lane = threadIdx.x & 63, T = a.T;
    const int part = lane / TP, x = lane % TP, y0 = part * RPL;
    const unsigned count = (unsigned)jb.count;
    unsigned q = 0;
    struct Tile {
        double m[S::PRELOAD ? RPL : 2];
    };
    const auto read_tile = [&](unsigned step, Tile& t) {
        if constexpr (S::PRELOAD) {
            const unsigned slot = step % S::RING;
#pragma unroll
            for (int k2 = 0; k2 < RPL / 2; ++k2) {
                const double2 d = *reinterpret_cast<const double2*>(&sh.M[slot][k2][lane][0]);
                t.m[2 * k2] = d.x;
                t.m[2 * k2 + 1] = d.y;
            }
        }
    };
    // waits for the matrix of `step` (bounded) and reads it; false: it did not come
    const auto fetch = [&](unsigned step, Tile& t) -> bool {
        int spins = 0;
        while ((unsigned)__builtin_amdgcn_readfirstlane(lds_load_acquire(&sh.ready[step % S::RING])) < step + 1)
            if (++spins > poll_limit) return false;
        read_tile(step, t);
        return true;
    };
    // One step from the matrix in `cur` (read from LDS inside the step at 64 columns).  The matrix of the next step
    // is read into `nxt` behind the additions, whether it is there or not, so that it comes back under the maxima;
    // the flag that says whether it was there is looked at before, at the start of the step (LDS executes a wave's
    // instructions in order: a flag that was up when it was read means that the reads behind it found the matrix).
    // If it was not, the matrix is waited for at the end of the step and read again.
    // 0: go on, 2: the next matrix did not come, 3: that was the last step.
    const auto step = [&](const Tile& cur, Tile& nxt) __attribute__((always_inline)) -> int {
        const double* vin = &sh.V[q % kMaxVecRing][y0];
        const unsigned slot = q % S::RING;
        double2 in[S::CH / 2];
        if constexpr (S::PRELOAD) {
#pragma unroll
            for (int k2 = 0; k2 < S::CH / 2; ++k2) in[k2] = *reinterpret_cast<const double2*>(vin + 2 * k2);
        }
        const int flag_next = lds_load_acquire(&sh.ready[(q + 1) % S::RING]);
        double r = 0.0;
#pragma unroll
        for (int c = 0; c < RPL; c += S::CH) {
            double val[S::CH];
#pragma unroll
            for (int k2 = 0; k2 < S::CH / 2; ++k2) {
                double m0, m1;
                if constexpr (S::PRELOAD) {
                    m0 = cur.m[c + 2 * k2];
                    m1 = cur.m[c + 2 * k2 + 1];
                } else {
                    in[k2] = *reinterpret_cast<const double2*>(vin + c + 2 * k2);
                    const double2 d = *reinterpret_cast<const double2*>(&sh.M[slot][c / 2 + k2][lane][0]);
                    m0 = d.x;
                    m1 = d.y;
                }
                val[2 * k2] = in[k2].x + m0;
                val[2 * k2 + 1] = in[k2].y + m1;
            }
            if constexpr (S::PRELOAD) {
                __builtin_amdgcn_sched_barrier(0);
                read_tile(q + 1, nxt);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int w = 1; w < S::CH; w <<= 1)
#pragma unroll
                for (int k = 0; k + w < S::CH; k += 2 * w) val[k] = __builtin_fmax(val[k], val[k + w]);
            r = c == 0 ? val[0] : __builtin_fmax(r, val[0]);
            if constexpr (!S::PRELOAD) __builtin_amdgcn_sched_barrier(0);  // (a piece at a time in the registers)
        }
        r = max_over_parts<S::P>(r);
        ++q;
        sh.V[q % kMaxVecRing][x] = r;  // (the lanes that share a column write the same value)
        lds_store_release(&sh.done, (int)q);
        if (q == count) return 3;
        if ((unsigned)__builtin_amdgcn_readfirstlane(flag_next) < q + 1 && !fetch(q, nxt)) return 2;
        return 0;
    };
    bool alone = false;
    if (count > 0) {
        Tile tA, tB;
        int why = fetch(0, tA) ? 0 : 2;
        while (why == 0) {
            why = step(tA, tB);
            if (why != 0) break;
            why = step(tB, tA);
        }
        alone = why != 3;
    }
    const double* last = sh.V[q % kMaxVecRing];
    if (alone) {
        // The rest of the chain by this wave alone: loads, scores and pointers, a position at a time.  The
        // published vectors stay as they are for the helpers that still work on earlier positions.
        lds_store_release(&sh.stop, (int)q);
        const MaxSource<TIN, AL> src(a, sp.b);
        uint8_t* bpb = a.bp + (size_t)sp.b * a.N * T;
        int buf = 0;
        sh.own[0][x] = last[x];
        for (; q < count; ++q) {
            const int i = jb.first + (int)q * jb.sdir;
            Best w{-__builtin_huge_val(), kNoArg};
#pragma unroll 1
            for (int c = 0; c < RPL; c += S::CH) {  // (a piece of the source tags at a time: few registers)
                float v[S::CH];
                src.template entries<S::CH>(i, jb.dir, y0 + c, x, v);
                const Best wc = max_pointer_piece<S::CH>(sh.own[buf] + y0 + c, y0 + c, [&](int k) {
                    double2 d;
                    d.x = max_entry(v[k], y0 + c + k < T && x < T);
                    d.y = max_entry(v[k + 1], y0 + c + k + 1 < T && x < T);
                    return d;
                });
                if (wc.v > w.v) w = wc;  // ascending pieces: the first maximum stays
            }
            w = max_pointer_parts<S::P>(w);
            sh.own[buf ^ 1][x] = w.v;
            if (part == 0 && x < T) bpb[(size_t)i * T + x] = (uint8_t)(w.a == kNoArg ? 0 : w.a);
            buf ^= 1;
        }
        last = sh.own[buf];
    }
    if (lane < T) mid[lane] = last[lane];
}

// A helper wave.
template <int TP, int ROWS, typename TIN, bool AL>
__device__ __forceinline__ void max_helper_wave(const VitArgs& a, const VitSpan& sp, const MaxJob& jb, MaxShared<TP, ROWS>& sh,
                                                int w, int poll_limit) {
    using S = MaxShape<TP, ROWS>;
    constexpr int RPL = S::RPL, NG = S::NG, W = kMaxHelpers;
    const int lane = threadIdx.x & 63, T = a.T;
    const int part = lane / TP, x = lane % TP, y0 = part * RPL;
    const int nj = w < jb.count ? (jb.count - w + W - 1) / W : 0;  // matrices of this wave: steps w, w + W, ...
    if (nj == 0) return;
    const MaxSource<TIN, AL> src(a, sp.b);
    uint8_t* bpb = a.bp + (size_t)sp.b * a.N * T;
    // The matrix is loaded as it lies in memory, piece lane + 64 m of 16 bytes (row s, columns t0 .. t0 + 3), and
    // scattered into the slot in the chain wave's order: entry (y, x) = (s, t) of a forward chain, (t, s) of a
    // backward one, sits at M[slot][k / 2][part TP + x][k % 2] with y = part RPL + k.
    int lidx[NG];  // index (in doubles) of the first entry of piece m in a slot
    int grow[NG], gcol[NG];  // row and first column of piece m
    unsigned valid = 0;
    const int Q = (T + 3) / 4;  // pieces a row (the last one of a row is cut off at T if T is no multiple of four)
#pragma unroll
    for (int m = 0; m < NG; ++m) {
        const int g = lane + 64 * m;
        const bool ok = g < T * Q;
        valid |= ok ? (1u << m) : 0u;
        const int s_ = (ok ? g : 0) / Q, t0 = 4 * ((ok ? g : 0) % Q);
        const int yy = jb.dir == 0 ? s_ : t0, xx = jb.dir == 0 ? t0 : s_;
        const int k = yy % RPL;
        lidx[m] = (((k >> 1) * 65 + (yy / RPL) * TP + xx) << 1) + (k & 1);
        grow[m] = s_;
        gcol[m] = t0;
    }
    // Dense potentials: the lane's pieces of two matrices, one in hand, one in flight.  Structured potentials: the
    // lane's entries of the transition matrix once, and of a position only the emission score of tag `lane` (one
    // load a matrix): the helper spreads the scores of a position over its lanes through LDS when it works on it.
    constexpr bool kStruct = MaxSource<TIN, AL>::kStruct;
    float raw[kStruct ? 1 : 2][kStruct ? 1 : NG][4];
    float fixed[kStruct ? NG : 1][4];
    float emis[2] = {0.f, 0.f};
    if constexpr (kStruct) {
#pragma unroll
        for (int m = 0; m < NG; ++m) src.fixed_part(grow[m], gcol[m], fixed[m]);
    }
    const auto load = [&](int j, int p) {
        const int q = w + (j < nj ? j : nj - 1) * W;
        const int i = jb.first + q * jb.sdir;
        if constexpr (kStruct) {
            emis[p] = src.emission(i, lane);
        } else {
            const bool followed = sp.b != a.B - 1 || i != a.N - 1;  // another matrix of the tensor lies behind this one
#pragma unroll
            for (int m = 0; m < NG; ++m) src.piece(i, grow[m], gcol[m], fixed[0], raw[p][m], followed);
        }
    };
    // Waits until the flag reaches `target` (true) or the chain wave has gone on alone at or before step `q`
    // (false).  The chain wave always does one or the other: each of its own waits is bounded by the poll limit
    // of the call.  The limit here is a last resort that only keeps a wave from spinning for ever.
    const auto wait_for = [&](const int* flag, int target, int q) -> bool {
        long long spins = 0;
        while (lds_load_acquire(flag) < target) {
            if (lds_load_acquire(&sh.stop) <= q || ++spins > 1000ll * (poll_limit + 65536)) return false;
            __builtin_amdgcn_s_sleep(1);
        }
        return true;
    };
    // The pointers of a position are stored a matrix later, ahead of a wait that is long anyway: the counter that
    // tells when loaded data has arrived counts stores as well, in order, so a store issued just before the next
    // matrix is needed would make the wave wait for the store's acknowledgement (more than a thousand cycles).
    uint8_t held = 0;
    uint8_t* held_at = nullptr;
    const auto flush = [&]() {
        if (held_at && part == 0 && x < T) *held_at = held;
        held_at = nullptr;
    };
    // One matrix (number j of this wave, in buffer p).  false: the chain wave has taken over, nothing more to do.
    const auto process = [&](int j, auto pc) -> bool {
        constexpr int p = decltype(pc)::value;
        const int q = w + j * W;
        const int i = jb.first + q * jb.sdir;
        const int slot = q % S::RING;
        // the slot is free once the chain wave has finished step q - RING and that step's helper has its pointers
        if (!wait_for(&sh.done, q - S::RING + 1, q) || !wait_for(&sh.kept[slot], q - S::RING + 1, q)) return false;
        double* Ms = &sh.M[slot][0][0][0];
        if constexpr (MaxSource<TIN, AL>::kQuad) {
            if (sp.b == a.B - 1 && i == a.N - 1) {  // the last matrix of the tensor: its last piece was loaded from further up
                const int glast = T * Q - 1;
#pragma unroll
                for (int m = 0; m < NG; ++m)
                    src.settle_last(m == (glast >> 6) && lane == (glast & 63), raw[p][m][0], raw[p][m][1], raw[p][m][2], raw[p][m][3]);
            }
        }
        if constexpr (kStruct) sh.emis[w][lane] = emis[p];  // (read back below by this wave only: its LDS instructions run in order)
#pragma unroll
        for (int m = 0; m < NG; ++m)
            if ((valid >> m) & 1) {
                double d[4];
                if constexpr (kStruct) {
                    const float4 e = *reinterpret_cast<const float4*>(&sh.emis[w][gcol[m]]);
                    d[0] = max_entry(fixed[m][0] + e.x, true);
                    d[1] = max_entry(fixed[m][1] + e.y, AL || gcol[m] + 1 < T);
                    d[2] = max_entry(fixed[m][2] + e.z, AL || gcol[m] + 2 < T);
                    d[3] = max_entry(fixed[m][3] + e.w, AL || gcol[m] + 3 < T);
                } else {
#pragma unroll
                    for (int k = 0; k < 4; ++k) d[k] = max_entry(raw[p][m][k], AL || gcol[m] + k < T);  // (-inf past the last column)
                }
                if (jb.dir == 0) {  // four columns of one source tag: 16 bytes apart
#pragma unroll
                    for (int k = 0; k < 4; ++k) Ms[lidx[m] + 2 * k] = d[k];
                } else {            // four source tags of one column: two pairs
                    double2 d0, d1;
                    d0.x = d[0]; d0.y = d[1];
                    d1.x = d[2]; d1.y = d[3];
                    *reinterpret_cast<double2*>(Ms + lidx[m]) = d0;
                    *reinterpret_cast<double2*>(Ms + lidx[m] + 130) = d1;
                }
            }
        if (lane == 0) lds_store_release(&sh.ready[slot], q + 1);
        flush();
        // the pointers of position i once the vector that enters it is published, from the matrix as it sits in the slot
        if (!wait_for(&sh.done, q, q)) return false;
        const Best b = max_pointer<TP, ROWS>(sh.V[q % kMaxVecRing], y0, [&](int k) {
            return *reinterpret_cast<const double2*>(&sh.M[slot][k >> 1][lane][0]);
        });
        if (lane == 0) lds_store_release(&sh.kept[slot], q + 1);
        held = (uint8_t)(b.a == kNoArg ? 0 : b.a);
        held_at = bpb + (size_t)i * T + x;
        return true;
    };
    // Two buffers: the next matrix is requested just before the current one is worked on.
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
    flush();
}

// (At 17 .. 32 tags two workgroups share a compute unit, four waves a SIMD: 128 vector registers a lane.  The aligned
// dense kernels need fewer anyway; the others spill a few values of their chain wave's lone path for it and gain a
// fifth on batches of more than one sequence for every two compute units: B=256 N=128 T=30 56 -> 48 us.)
template <int TP, int ROWS, typename TIN, bool AL>
__global__ __launch_bounds__(64 * kMaxWaves, (TP == 32 ? 4 : 1)) void viterbi_lane_kernel(VitArgs a, int poll_limit) {
    using S = MaxShape<TP, ROWS>;
    extern __shared__ __attribute__((aligned(16))) unsigned char max_smem[];
    MaxShared<TP, ROWS>& sh = *reinterpret_cast<MaxShared<TP, ROWS>*>(max_smem);
    const int tid = threadIdx.x;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform: loops over a wave's work stay scalar
    const int dir = blockIdx.x & 1;
    const VitSpan sp = vit_span(a, blockIdx.x >> 1);
    if (sp.empty) return;
    const int b = sp.b, T = a.T;
    const int p0 = sp.p0, e = sp.e, h = meeting_point(p0, e);
    MaxJob jb;
    jb.dir = dir;
    if (dir == 0) { jb.first = p0 + 1; jb.sdir = +1; jb.count = h - p0; }
    else { jb.first = e; jb.sdir = -1; jb.count = e - h; }
    double* mid = a.mid + (((size_t)b * a.C + sp.c) * 2 + dir) * T;
    // the vector that enters step 0
    if (tid < TP) {
        const double ninf = -__builtin_huge_val();
        double v0 = ninf;
        if (tid < T) {
            if (dir == 0) {
                if (sp.t0 == 0) v0 = (double)MaxSource<TIN, AL>(a, b).first(tid);
                else v0 = (tid == a.pin[(size_t)b * a.C + sp.c - 1]) ? 0.0 : ninf;
            } else {
                // a whole sequence may end in any tag; a chunk must end in its pinned tag
                v0 = (a.chunk <= 0 || tid == a.pin[(size_t)b * a.C + sp.c]) ? 0.0 : ninf;
            }
        }
        sh.V[0][tid] = v0;
    }
    if (tid < S::RING) { sh.ready[tid] = 0; sh.kept[tid] = 0; }
    if (tid == 0) { sh.done = 0; sh.stop = 0x7fffffff; }
    if (T != TP) {  // entries past the tag set: the helpers never write them
        double* Mz = &sh.M[0][0][0][0];
        for (int k = tid; k < S::RING * S::RPL * 65; k += 64 * kMaxWaves) Mz[k] = -__builtin_huge_val();
    }
    __syncthreads();
    if (wv == 0) {
        __builtin_amdgcn_s_setprio(3);
        max_chain_wave<TP, ROWS, TIN, AL>(a, sp, jb, sh, mid, poll_limit);
    } else {
        max_helper_wave<TP, ROWS, TIN, AL>(a, sp, jb, sh, wv - 1, poll_limit);
    }
}

// ---------------------------------------------------------------------------------------
// Dense or structured potentials, whole sequences, up to 64 tags.
bool lane_max_supported(int T) { return T >= 1 && T <= 64; }

template <int TP, int ROWS, typename TIN, bool AL>
static hipError_t launch_max_kernel(const VitArgs& a, int poll_limit, hipStream_t st) {
    const size_t bytes = sizeof(MaxShared<TP, ROWS>);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&viterbi_lane_kernel<TP, ROWS, TIN, AL>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((viterbi_lane_kernel<TP, ROWS, TIN, AL>), dim3(2 * a.B * a.C), dim3(64 * kMaxWaves), bytes, st, a, poll_limit);
    return hipGetLastError();
}
template <typename TIN, bool AL>
static hipError_t launch_max_T(const VitArgs& a, int poll_limit, hipStream_t st) {
    if (a.T <= 16) return launch_max_kernel<16, 16, TIN, AL>(a, poll_limit, st);
    if (a.T <= 32) return launch_max_kernel<32, 32, TIN, AL>(a, poll_limit, st);
    if (a.T <= 48) return launch_max_kernel<64, 48, TIN, AL>(a, poll_limit, st);
    return launch_max_kernel<64, 64, TIN, AL>(a, poll_limit, st);
}
template <typename TIN>
static hipError_t launch_max_src(const VitArgs& a, int poll_limit, hipStream_t st) {
    if ((a.T % 4) == 0) return launch_max_T<TIN, true>(a, poll_limit, st);
    if constexpr (!std::is_same<TIN, MaxStructF>::value) {
        // (from five tags on: below, a matrix is too small for its last four entries to be a piece's)
        if (a.T >= 5) return launch_max_T<Anywhere<TIN>, false>(a, poll_limit, st);
        return launch_max_kernel<16, 16, TIN, false>(a, poll_limit, st);
    } else {
        return launch_max_T<TIN, false>(a, poll_limit, st);
    }
}

hipError_t launch_lane_max_chains(int dtype, const VitArgs& a, int poll_limit, hipStream_t st) {
    if (!lane_max_supported(a.T) || a.chunk > 0 || (a.emit && (dtype != 0 || !a.trans))) return hipErrorInvalidValue;
    if (a.emit) return launch_max_src<MaxStructF>(a, poll_limit, st);
    return dtype == 0 ? launch_max_src<float>(a, poll_limit, st) : launch_max_src<uint16_t>(a, poll_limit, st);
}

}  // namespace lccrf
