// Chunked log-semiring scan over the positions of long chains with a small tag set (T <= 64; the
// max-plus variant T <= 16).
//
// The paper (section "Sequence Tagging") notes that the forward algorithm can also be run as a
// parallel scan over products of T x T matrices, at T times the arithmetic of the sequential
// recursion, which pays when T is much smaller than the length.  Here the scan is a three-phase
// chunked one sized for one GPU:
//
//   phase A (chunk_product_kernel, one wave per chunk of `chunk` positions, all chunks at once):
//       P_c = phi_first (x) ... (x) phi_last, the log-semiring product of the chunk's matrices,
//       P_c[r][s] = log sum over paths that enter the chunk from tag r and leave it in tag s;
//   phase B (chunk_boundary_kernel, two waves per sequence, serial over the chunks only):
//       alpha at the last position of every chunk (F_c = F_{c-1} (x) P_c) and beta at the last
//       position of every chunk (G_{c-1} = P_c (x) G_c), and logZ from the last F.  With many
//       chunks this is itself run as a scan: group_product_kernel multiplies the products of
//       every group of chunks (all groups at once, the very code of phase A with chunk products in
//       the place of potentials), phase B runs over the groups, and then over the chunks of
//       every group at once from the group's boundary vectors;
//   phase C (the chain kernels of lccrf_chain.hip, one pair of workgroups per chunk):
//       the ordinary two-chain forward-backward inside every chunk, started from F and G.
//
// Phase A keeps each product in the linear domain, in double precision, scaled per entry tag by
// an exact power of two after every position, so that one position costs T^2 exponentials and
// four v_mfma_f64_16x16x4_f64 instead of T^3 exponentials.  A product is accepted only if no
// entry ever fell below 2^-900 of its scale unless no path leads to it at all (the zero pattern
// is carried along as a product of 0/1 matrices): then no term that matters was flushed to zero.
// Otherwise the wave recomputes its chunk with the exact log-domain
// product, every log-sum-exp shifted by its own maximum.  Both forms write the same format:
// log2 of the scaled product, one integer log2 scale per entry tag and one common offset.
#include "lccrf_device.h"
#include "lccrf_launch.h"

#include <type_traits>

namespace lccrf {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef double f64x4 __attribute__((ext_vector_type(4)));

constexpr int kScanPF = 8;

// Value of lane `src_lane` (any lane, computed per lane).
__device__ __forceinline__ float lane_bperm(float x, int src_lane) {
    return __int_as_float(__builtin_amdgcn_ds_bpermute(src_lane << 2, __float_as_int(x)));
}

struct ScanArgs {
    const void* phi;
    const int32_t* lengths;
    int B, N, T;
    int chunk, C;
    // log2 P_c[r][s] = Pl[b][c][s][r] + rel[b][c][r] + base[b][c]   (r: entry tag, s: exit tag;
    // tags >= T are padded with -inf up to TP = 16 or 32, the padded tag count of the launch)
    float* Pl;     // [B][C][TP][TP]
    float* rel;    // [B][C][TP]  integer valued, <= 0
    double* base;  // [B][C]
    float* Fv;     // [B][C][T]   alpha at the last position of chunk c, maximum 0 ...
    double* OF;    // [B][C]      ... plus this offset (base-2 logarithms)
    float* Gv;     // [B][C][T]   beta at the last position of chunk c
    double* OG;    // [B][C]
    float* logZ;   // [B] or null
    int with_beta;
    double* logZ64;  // [B] or null: the same in double precision
    // Grouped runs (GS > 0): a unit of work covers GS consecutive chunks, G = ceil(C / GS) groups a
    // sequence.  group_product_kernel writes the product of every group to (Pl2, rel2, base2), laid
    // out like (Pl, rel, base) with G in the place of C; chunk_boundary_kernel starts every group
    // from the boundary vectors of the groups (Fin .. OGin, [B][G] like Fv .. OG) instead of walking
    // the whole sequence.
    int GS, G;
    float* Pl2;
    float* rel2;
    double* base2;
    const float* Fin;
    const double* OFin;
    const float* Gin;
    const double* OGin;
    // Structured potentials (emit non-null; phi is then not read): phi[b][i][s][t] = trans[s][t] + emit[b][i][t].
    const float* emit;   // [B][N][T]
    const float* trans;  // [T][T]
};

// First and last position whose matrix belongs to chunk c (first > last: none).
__device__ __forceinline__ void chunk_range(int c, int chunk, int L, int& first, int& last) {
    const int t0 = c * chunk, t1 = t0 + chunk;
    first = c == 0 ? 1 : t0;
    last = (t1 < L ? t1 : L) - 1;
}

// ---------------------------------------------------------------------------------------
// Phase A.
//
// TP is the padded tag count (16, 32, 48 or 64); matrices are handled as NB x NB blocks of 16 x 16,
// NB = TP / 16.  Lane (g = lane / 16, j = lane % 16) handles, of block (sb, tb), four entries of
// the column at position j of block tb (row: tag before, column: tag after), entry number
// e = (sb NB + tb) 4 + v: the rows an accumulator register v of that lane holds after a 16x16x4 MFMA,
// which sit at positions g + 4v of block sb for the f64 instruction (F64) and 4g + v for the f32 one.  Sources hand out matrices in base-2
// logarithms, -inf outside T x T; every matrix may carry a common offset besides.
//
// Up to 32 tags one wave holds the whole running product D.  Above, a workgroup of NB waves serves a
// chunk and wave w holds block column w of D (the entry tags 16 w .. 16 w + 15): a block column of
// D_new = E^T D needs all of E but only its own columns of D, so every wave reads the whole matrix of
// a position (and exponentiates it: the same T^2 exponentials a wave, on four SIMDs at once), issues
// a quarter of the matrix instructions and keeps a quarter of the product in registers, and the waves
// exchange nothing until the product is complete.
template <int TP, bool F64 = true>
struct ScanShape {
    static_assert(TP == 16 || TP == 32 || TP == 48 || TP == 64, "padded tag count");
    static constexpr int NB = TP / 16, NE = 4 * NB * NB;
    static constexpr int NW = TP <= 32 ? 1 : NB;  // waves per product
    static constexpr int RB = NB / NW;            // block columns of D a wave holds
    static constexpr int LPRow = TP <= 32 ? 64 / TP : 1;  // lanes sharing a row in phase B (one wave per vector)
    static constexpr int CPL = TP / LPRow;                // columns per lane there
    static constexpr int XL = 64 * NW / TP;  // threads sharing a row in the exact product (all waves of the workgroup)
    static constexpr int XC = TP / XL;       // columns per thread there
    // Tag held by position w (0 .. 15) of block b: blocks are interleaved, tag = NB w + b, so that the NB
    // columns a lane holds of one row (position j of every block) are neighbours in memory: one vector load
    // per row instead of NB scalar ones, and the sixteen lanes of a row read one contiguous stretch.
    static __device__ __forceinline__ int tag(int b, int w) { return NB * w + b; }
    static __device__ __forceinline__ int row(int lane, int e) {
        return tag(e / (4 * NB), F64 ? (lane >> 4) + 4 * (e & 3) : 4 * (lane >> 4) + (e & 3));
    }
    static __device__ __forceinline__ int col(int lane, int e) { return tag((e / 4) % NB, lane & 15); }
};
// One bit per entry a lane holds of a matrix.
template <int NE>
using ScanMask = std::conditional_t<(NE > 32), unsigned long long, unsigned>;
template <typename M>
__device__ __forceinline__ M shfl_mask(M m, int src) {
    if constexpr (sizeof(M) == 8) {
        const unsigned lo = (unsigned)__shfl((int)(unsigned)(m & 0xffffffffull), src, 64);
        const unsigned hi = (unsigned)__shfl((int)(unsigned)(m >> 32), src, 64);
        return ((unsigned long long)hi << 32) | lo;
    } else {
        return (M)__shfl((int)m, src, 64);
    }
}
// What the waves of one product tell each other when it is complete (one slot per precision tried).
struct ProductShared {
    float emax[2][4];
    int rejected[2][4];
};

// NB consecutive elements starting at p (NB = 2, 3 or 4; p aligned to NB elements for 2 and 4, to one for 3).
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x3 __attribute__((ext_vector_type(3)));
template <int NB>
__device__ __forceinline__ void load_row(const float* p, float (&v)[NB]) {
    if constexpr (NB == 2) {
        const f32x2 q = *reinterpret_cast<const f32x2*>(p);
        v[0] = q[0]; v[1] = q[1];
    } else if constexpr (NB == 3) {
        struct __attribute__((packed, aligned(4))) Three { float a, b, c; };
        const Three q = *reinterpret_cast<const Three*>(p);
        v[0] = q.a; v[1] = q.b; v[2] = q.c;
    } else {
        const f32x4 q = *reinterpret_cast<const f32x4*>(p);
        v[0] = q[0]; v[1] = q[1]; v[2] = q[2]; v[3] = q[3];
    }
}
template <int NB>
__device__ __forceinline__ void load_row(const uint16_t* p, float (&v)[NB]) {
    if constexpr (NB == 2) {
        const unsigned q = *reinterpret_cast<const unsigned*>(p);
        v[0] = __uint_as_float(q << 16); v[1] = __uint_as_float(q & 0xffff0000u);
    } else if constexpr (NB == 3) {
#pragma unroll
        for (int k = 0; k < 3; ++k) v[k] = bf16_to_f32(p[k]);
    } else {
        const uint2 q = *reinterpret_cast<const uint2*>(p);
        v[0] = __uint_as_float(q.x << 16); v[1] = __uint_as_float(q.x & 0xffff0000u);
        v[2] = __uint_as_float(q.y << 16); v[3] = __uint_as_float(q.y & 0xffff0000u);
    }
}

// VEC: T is a multiple of NB (and, for four-wide loads, of 4): a lane's NB columns of a row are loaded
// with one instruction.  Otherwise one scalar load per entry.
template <typename TIN, int TP, bool F64, bool VEC>
struct PotentialMatrices {  // the potentials phi_i of one sequence
    using S = ScanShape<TP, F64>;
    static constexpr int NB = S::NB;
    // tiles in flight: the counter of outstanding loads a wave can wait on ends at 63, so a ring of scalar
    // loads (NE a tile) must stay below that or every step waits for all of them
    static constexpr int PF = TP == 16 ? kScanPF : TP == 32 ? 3 : VEC ? (TP == 48 ? 3 : 2) : 1;
    struct Slot { float x[S::NE]; };
    // entries outside T x T are loaded from the nearest entry inside: whatever a slot holds is a potential
    static constexpr bool kPaddingIsFinite = true;
    const TIN* phib;
    int T;
    size_t TT;
    // entry e = (sb NB + tb) 4 + v sits at row offset roff[4 sb + v] plus column coff[tb] (both clamped into the matrix)
    int roff[4 * NB], coff[NB];
    ScanMask<S::NE> in;  // bit e: entry e lies inside T x T
    __device__ PotentialMatrices(const TIN* p, int T_, int lane) : phib(p), T(T_), TT((size_t)T_ * T_), in(0) {
#pragma unroll
        for (int e = 0; e < S::NE; ++e) {
            const int s = S::row(lane, e), t = S::col(lane, e);
            in |= (s < T && t < T) ? (ScanMask<S::NE>(1) << e) : ScanMask<S::NE>(0);
        }
#pragma unroll
        for (int k = 0; k < 4 * NB; ++k) {
            const int s = S::row(lane, (k / 4) * 4 * NB + (k & 3));
            roff[k] = (s < T ? s : T - 1) * T;
        }
#pragma unroll
        for (int tb = 0; tb < NB; ++tb) {
            const int t = S::col(lane, 4 * tb);
            coff[tb] = t < T ? t : T - 1;
        }
        // vector loads: the lane's columns NB j .. NB j + NB - 1 (T a multiple of NB: all inside or all outside)
        if (VEC) coff[0] = coff[0] + NB <= T ? coff[0] : T - NB;
    }
    __device__ __forceinline__ void load(int i, Slot& sl) const {
        const TIN* m = phib + (size_t)i * TT;
        if constexpr (VEC && NB > 1) {
#pragma unroll
            for (int k = 0; k < 4 * NB; ++k) {
                float v[NB];
                load_row<NB>(m + roff[k] + coff[0], v);
#pragma unroll
                for (int tb = 0; tb < NB; ++tb) sl.x[((k / 4) * NB + tb) * 4 + (k & 3)] = v[tb];
            }
        } else {
#pragma unroll
            for (int e = 0; e < S::NE; ++e) sl.x[e] = Elem<TIN>::get(m + roff[(e / (4 * NB)) * 4 + (e & 3)] + coff[(e / 4) % NB]);
        }
    }
    __device__ __forceinline__ double entries(const Slot& sl, float (&x)[S::NE]) const {
#pragma unroll
        for (int e = 0; e < S::NE; ++e) x[e] = (in >> e) & 1 ? sl.x[e] * kLog2e : LCCRF_NEG_INF;
        return 0.0;
    }
    __device__ __forceinline__ float smallest_loaded(const Slot& sl) const {
        float lo = sl.x[0];
#pragma unroll
        for (int e = 1; e < S::NE; ++e) lo = fminf(lo, sl.x[e]);
        return lo;
    }
    __device__ __forceinline__ float entry(int i, int r, int t) const {  // one entry, straight from memory
        return (r < T && t < T) ? Elem<TIN>::get(phib + (size_t)i * TT + r * T + t) * kLog2e : LCCRF_NEG_INF;
    }
    __device__ __forceinline__ double offset(int) const { return 0.0; }
};

// The same matrices from structured potentials, phi_i[s][t] = trans[s][t] + emit_i[t]: the transition entries of a
// lane stay in registers (in base-2 logarithms, -inf outside T x T) and a position brings the emissions of the lane's
// NB columns.
template <int TP, bool F64>
struct StructuredMatrices {
    using S = ScanShape<TP, F64>;
    static constexpr int NB = S::NB;
    static constexpr int PF = 4;
    struct Slot { float em[NB]; };
    static constexpr bool kPaddingIsFinite = false;  // entries outside T x T are handed out as -inf
    const float* emb;
    const float* trans;
    int T;
    float tr[S::NE];
    int coff[NB];
    __device__ StructuredMatrices(const float* emit_b, const float* trans_, int T_, int lane) : emb(emit_b), trans(trans_), T(T_) {
#pragma unroll
        for (int e = 0; e < S::NE; ++e) {
            const int s = S::row(lane, e), t = S::col(lane, e);
            tr[e] = (s < T && t < T) ? trans[s * T + t] * kLog2e : LCCRF_NEG_INF;
        }
#pragma unroll
        for (int tb = 0; tb < NB; ++tb) {
            const int t = S::col(lane, 4 * tb);
            coff[tb] = t < T ? t : T - 1;
        }
    }
    __device__ __forceinline__ void load(int i, Slot& sl) const {
        const float* m = emb + (size_t)i * T;
#pragma unroll
        for (int tb = 0; tb < NB; ++tb) sl.em[tb] = m[coff[tb]];
    }
    __device__ __forceinline__ double entries(const Slot& sl, float (&x)[S::NE]) const {
#pragma unroll
        for (int e = 0; e < S::NE; ++e) x[e] = tr[e] + sl.em[(e / 4) % NB] * kLog2e;
        return 0.0;
    }
    __device__ __forceinline__ float entry(int i, int r, int t) const {
        return (r < T && t < T) ? (trans[r * T + t] + emb[(size_t)i * T + t]) * kLog2e : LCCRF_NEG_INF;
    }
    __device__ __forceinline__ double offset(int) const { return 0.0; }
};

template <int TP, bool F64>
struct ChunkMatrices {  // the chunk products of one sequence, as phase A has written them
    using S = ScanShape<TP, F64>;
    static constexpr int PF = TP == 16 ? 4 : 2;
    struct Slot { float p[S::NE], r[4 * S::NB]; double b; };  // r: the scale of row 16 sb + (row of register v), at [4 sb + v]
    static constexpr bool kPaddingIsFinite = false;  // stored products are -inf outside T x T
    const float* Pl;
    const float* rel;
    const double* base;
    int T, lane;
    __device__ ChunkMatrices(const float* Pl_, const float* rel_, const double* base_, int T_, int lane_)
        : Pl(Pl_), rel(rel_), base(base_), T(T_), lane(lane_) {}
    __device__ __forceinline__ void load(int c, Slot& sl) const {
#pragma unroll
        for (int e = 0; e < S::NE; ++e) sl.p[e] = Pl[(size_t)c * TP * TP + S::col(lane, e) * TP + S::row(lane, e)];
#pragma unroll
        for (int k = 0; k < 4 * S::NB; ++k) sl.r[k] = rel[(size_t)c * TP + S::row(lane, (k / 4) * 4 * S::NB + (k & 3))];
        sl.b = base[c];
    }
    __device__ __forceinline__ double entries(const Slot& sl, float (&x)[S::NE]) const {
#pragma unroll
        for (int e = 0; e < S::NE; ++e)
            x[e] = (S::row(lane, e) < T && S::col(lane, e) < T) ? sl.p[e] + sl.r[(e / (4 * S::NB)) * 4 + (e & 3)] : LCCRF_NEG_INF;
        return sl.b;
    }
    __device__ __forceinline__ float entry(int c, int r, int t) const {
        return (r < T && t < T) ? Pl[(size_t)c * TP * TP + t * TP + r] + rel[(size_t)c * TP + r] : LCCRF_NEG_INF;
    }
    __device__ __forceinline__ double offset(int c) const { return base[c]; }
};

// The arithmetic of the linear-domain product in the two precisions it is tried in.
template <bool F64>
struct Linear;
template <>
struct Linear<true> {
    using scalar = double;
    using vec = f64x4;
    // 2^d in double: the fraction through the float exponential, the integer part through the exponent field
    static __device__ __forceinline__ double pow2(float d) {
        const float di = floorf(d);
        return d > -1000.f ? ldexp((double)ex2(d - di), (int)di) : 0.0;
    }
    static __device__ __forceinline__ vec mfma(double a, double b, vec c) { return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0); }
    // exponent field of a non-negative number; entries below 2^-900 are not accepted
    static constexpr unsigned kBias = 1023, kMinField = 1023 - 900, kNoField = 0x7ff;
    static __device__ __forceinline__ unsigned field(double x) { return __builtin_amdgcn_ubfe((unsigned)__double2hiint(x), 20, 11); }
    static __device__ __forceinline__ double scaled(double x, int e) { return ldexp(x, -e); }
    static __device__ __forceinline__ float log2_of(double x) { return (float)log2(x); }
};
template <>
struct Linear<false> {
    using scalar = float;
    using vec = f32x4;
    static __device__ __forceinline__ float pow2(float d) { return ex2(d); }
    static __device__ __forceinline__ vec mfma(float a, float b, vec c) { return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0); }
    // entries below 2^-90 are not accepted: with them a term that underflowed could matter
    static constexpr unsigned kBias = 127, kMinField = 127 - 90, kNoField = 0xff;
    static __device__ __forceinline__ unsigned field(float x) { return __builtin_amdgcn_ubfe((unsigned)__float_as_int(x), 23, 8); }
    static __device__ __forceinline__ float scaled(float x, int e) { return ldexpf(x, -e); }
    static __device__ __forceinline__ float log2_of(float x) { return lg2(x); }
};

// Product of matrices first .. last of `src` (none: the identity) in the linear domain on the matrix
// cores, by one wave; written, if accepted (the return value), as
// log2 P[r][s] = Pout[s * TP + r] + rel_out[r] + *base_out.
// Block (sb, rb) of D (exit tag s, entry tag r) sits in the accumulator layout of the 16x16x4
// MFMA of its precision: lane (g, j) holds D[row(v)][16 rb + j], v = 0..3.  The same lane loads
// phi_i[row(v)][16 tb + j]; as the A operand of an MFMA that is E^T[j][k = g] for the inner
// indices s = row(v), and register v of D's block (sb, rb) is the matching B operand, so block
// (tb, rb) of
//     D_new[t][r] = sum_s E[s][t] D[s][r]
// is the sum over sb and v of those MFMAs, and nothing moves between lanes from one position
// to the next.  F64 = false is the product in single precision (half the matrix time and no
// double-precision conversions); its narrower exponent range makes it give up on peaked
// potentials, which take the double-precision product from the start.
//
// Which products try single precision first.  Measured on independent normal potentials: with 17 to
// 32 tags it takes a quarter off the scan's log-partition (all kernels) up to a standard deviation
// of 7, costs nothing at 8 to 9 and adds a tenth to a fifth from 10 on, where some wave of the
// launch gives up late in its chunk; with up to 16 tags the matrix cores are a small part of the
// time, the gain is half as large and the same loss would fall on long chains of peaked
// potentials, so those stay in double precision.
template <int TP>
constexpr bool kSingleFirst = TP >= 32;

template <int TP, bool F64, typename Src>
__device__ __forceinline__ bool linear_product(const Src& src, int first, int last, int T, float* __restrict__ Pout,
                                               float* __restrict__ rel_out, double* __restrict__ base_out,
                                               ProductShared& shared) {
    using S = ScanShape<TP, F64>;
    using L = Linear<F64>;
    using scalar = typename L::scalar;
    using vec = typename L::vec;
    using Mask = ScanMask<S::NE>;
    constexpr int NB = S::NB, NE = S::NE, RB = S::RB;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int rb0 = wv * RB;  // this wave holds block columns rb0 .. rb0 + RB - 1 of D
    const int g = lane >> 4, j = lane & 15;
    Mask in = 0;
#pragma unroll
    for (int e = 0; e < NE; ++e) in |= (S::row(lane, e) < T && S::col(lane, e) < T) ? (Mask(1) << e) : Mask(0);
    // entry (tb, rb, v) of D lies inside T x T (the numbering of the entries of a matrix, rb in the place of tb)
    const auto inside = [&](int tb, int rl, int v) { return ((in >> ((tb * NB + rb0 + rl) * 4 + v)) & 1) != 0; };
    // The zero pattern of D (1 where some path exists) is carried along by a product of 0/1
    // matrices on the f32 MFMA, from the first matrix with a -inf entry on (until then D is
    // the identity or has no zero).  That instruction numbers its output rows 4g + v; beside the
    // f64 product it therefore runs on rows renamed by pi(4g + v) = g + 4v: its A operand is the
    // flag of column pi(j).
    const int pj = F64 ? ((lane & 48) | (4 * (j & 3) + (j >> 2))) : lane;
    scalar D[NB][RB][4];
    float Z[NB][RB][4];
    double Msum = 0.0;
    int esum[RB];
    bool bad = false, tracking = false, started = false, rejected = false;
#pragma unroll
    for (int sb = 0; sb < NB; ++sb)
#pragma unroll
        for (int rl = 0; rl < RB; ++rl)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const bool diag = sb == rb0 + rl && (F64 ? g + 4 * v : 4 * g + v) == j;
                D[sb][rl][v] = diag ? (scalar)1 : (scalar)0;
                Z[sb][rl][v] = diag ? 1.f : 0.f;
            }
#pragma unroll
    for (int rl = 0; rl < RB; ++rl) esum[rl] = 0;
    typename Src::Slot ring[Src::PF];
    auto load = [&](int i, int slot) { src.load(i, ring[slot]); };
    // The single-precision product looks at every position whether it still holds, and ends at
    // once if not; the double-precision one hardly ever fails and is judged at the end.
    const auto step = [&](int, int slot) -> bool {
        float x[NE];
        const double common = src.entries(ring[slot], x);
        float mloc = x[0];
#pragma unroll
        for (int e = 1; e < NE; ++e) mloc = fmaxf(mloc, x[e]);
        const float m = finite_or_zero(xor_max<1, 64>(mloc));
        Msum += (double)m + common;
        vec acc[NB][RB];
#pragma unroll
        for (int tb = 0; tb < NB; ++tb)
#pragma unroll
            for (int rl = 0; rl < RB; ++rl) acc[tb][rl] = vec{0, 0, 0, 0};
#pragma unroll
        for (int sb = 0; sb < NB; ++sb)
#pragma unroll
            for (int tb = 0; tb < NB; ++tb)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const scalar E = L::pow2(x[(sb * NB + tb) * 4 + v] - m);
#pragma unroll
                    for (int rl = 0; rl < RB; ++rl) acc[tb][rl] = L::mfma(E, D[sb][rl][v], acc[tb][rl]);
                }
        // bit e of nz: entry e of this matrix is not a structural zero
        const auto nonzero_mask = [&]() {
            Mask nz = 0;
#pragma unroll
            for (int e = 0; e < NE; ++e) nz |= (x[e] > LCCRF_NEG_INF) ? (Mask(1) << e) : Mask(0);
            return nz;
        };
        Mask nz = 0;
        bool hole;
        if constexpr (Src::kPaddingIsFinite) {
            hole = src.smallest_loaded(ring[slot]) == LCCRF_NEG_INF;
        } else {
            nz = nonzero_mask();
            hole = (in & ~nz) != 0;
        }
        if (!tracking && __builtin_amdgcn_ballot_w64(hole) != 0) {
            tracking = true;
            if (started) {
#pragma unroll
                for (int sb = 0; sb < NB; ++sb)
#pragma unroll
                    for (int rl = 0; rl < RB; ++rl)
#pragma unroll
                        for (int v = 0; v < 4; ++v) Z[sb][rl][v] = inside(sb, rl, v) ? 1.f : 0.f;
            }
        }
        started = true;
        // Exponent fields of the new entries: their largest gives each column's rescale, the
        // smallest among the entries that some path reaches says whether the product still holds.
        unsigned fld[NB][RB][4], fmin = L::kNoField;
#pragma unroll
        for (int tb = 0; tb < NB; ++tb)
#pragma unroll
            for (int rl = 0; rl < RB; ++rl)
#pragma unroll
                for (int v = 0; v < 4; ++v) fld[tb][rl][v] = L::field(acc[tb][rl][v]);
        if (tracking) {
            if constexpr (Src::kPaddingIsFinite) nz = nonzero_mask();
            const Mask nzp = shfl_mask(nz, pj);
            f32x4 pat[NB][RB];
#pragma unroll
            for (int tb = 0; tb < NB; ++tb)
#pragma unroll
                for (int rl = 0; rl < RB; ++rl) pat[tb][rl] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int sb = 0; sb < NB; ++sb)
#pragma unroll
                for (int tb = 0; tb < NB; ++tb)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const float flag = (nzp >> ((sb * NB + tb) * 4 + v)) & 1 ? 1.f : 0.f;
#pragma unroll
                        for (int rl = 0; rl < RB; ++rl)
                            pat[tb][rl] = __builtin_amdgcn_mfma_f32_16x16x4f32(flag, Z[sb][rl][v], pat[tb][rl], 0, 0, 0);
                    }
#pragma unroll
            for (int tb = 0; tb < NB; ++tb)
#pragma unroll
                for (int rl = 0; rl < RB; ++rl)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const bool reached = pat[tb][rl][v] > 0.f;
                        Z[tb][rl][v] = reached ? 1.f : 0.f;
                        fmin = min(fmin, reached ? fld[tb][rl][v] : L::kNoField);
                    }
        } else {
#pragma unroll
            for (int tb = 0; tb < NB; ++tb)
#pragma unroll
                for (int rl = 0; rl < RB; ++rl)
#pragma unroll
                    for (int v = 0; v < 4; ++v) fmin = min(fmin, inside(tb, rl, v) ? fld[tb][rl][v] : L::kNoField);
        }
        bad |= fmin < L::kMinField;  // also zero and subnormal entries (field 0)
        if (!F64 && __builtin_amdgcn_ballot_w64(bad) != 0) {
            rejected = true;
            return false;
        }
        // With the column maxima of D in [1, 2) and E at most 1, a term lost to underflow is
        // below the smallest normal number: it cannot matter to a sum of the accepted size.
        // Power-of-two rescale of each entry tag's column (exact): the largest exponent.
#pragma unroll
        for (int rl = 0; rl < RB; ++rl) {
            unsigned ef = 0;
#pragma unroll
            for (int tb = 0; tb < NB; ++tb)
#pragma unroll
                for (int v = 0; v < 4; ++v) ef = max(ef, fld[tb][rl][v]);
            const auto r16 = __builtin_amdgcn_permlane16_swap(ef, ef, false, false);
            ef = max(r16[0], r16[1]);
            const auto r32 = __builtin_amdgcn_permlane32_swap(ef, ef, false, false);
            ef = max(r32[0], r32[1]);
            const int ex = ef > 0 ? (int)ef - (int)L::kBias : 0;  // a column without any path keeps its zeros
            esum[rl] += ex;
#pragma unroll
            for (int tb = 0; tb < NB; ++tb)
#pragma unroll
                for (int v = 0; v < 4; ++v) D[tb][rl][v] = L::scaled(acc[tb][rl][v], ex);
        }
        return true;
    };
    if constexpr (F64) walk<Src::PF>(first, last, +1, load, step);
    else walk_while<Src::PF>(first, last, +1, load, step);
    rejected |= __builtin_amdgcn_ballot_w64(bad) != 0;
    float ef[RB], emax = LCCRF_NEG_INF;
#pragma unroll
    for (int rl = 0; rl < RB; ++rl) {
        ef[rl] = S::tag(rb0 + rl, j) < T ? (float)esum[rl] : LCCRF_NEG_INF;
        emax = fmaxf(emax, xor_max<1, 16>(ef[rl]));
    }
    if constexpr (S::NW > 1) {
        // the waves of the workgroup agree on the verdict and on the largest column scale (a wave that gave up
        // early waits here for the others)
        if (lane == 0) {
            shared.emax[F64][wv] = emax;
            shared.rejected[F64][wv] = rejected ? 1 : 0;
        }
        __syncthreads();
#pragma unroll
        for (int w = 0; w < S::NW; ++w) {
            emax = fmaxf(emax, shared.emax[F64][w]);
            rejected |= shared.rejected[F64][w] != 0;
        }
    }
    if (!rejected) {
        emax = finite_or_zero(emax);
#pragma unroll
        for (int tb = 0; tb < NB; ++tb)
#pragma unroll
            for (int rl = 0; rl < RB; ++rl)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    Pout[S::row(lane, (tb * NB + rb0 + rl) * 4 + v) * TP + S::tag(rb0 + rl, j)] =
                        (inside(tb, rl, v) && D[tb][rl][v] > 0) ? L::log2_of(D[tb][rl][v]) : LCCRF_NEG_INF;
        if (g == 0) {
#pragma unroll
            for (int rl = 0; rl < RB; ++rl) rel_out[S::tag(rb0 + rl, j)] = ef[rl] - emax;
        }
        if (threadIdx.x == 0) *base_out = Msum + (double)emax;
        return true;
    }
    return false;
}

// The same product in the log domain, every log-sum-exp shifted by its own maximum (rare: taken when
// both linear products gave up), by all threads of the workgroup.  Thread (r = tid / XL, q = tid % XL)
// owns P[r][XC q .. XC q + XC - 1]; P and the current matrix are exchanged through LDS.
template <int TP, typename Src>
__device__ __forceinline__ void exact_product(const Src& src, int first, int last, int T, float* __restrict__ Pout,
                                              float* __restrict__ rel_out, double* __restrict__ base_out,
                                              float (*Pc)[TP + 1], float (*Ph)[TP + 1]) {
    using S = ScanShape<TP, true>;
    const int tid = threadIdx.x;
    constexpr int XL = S::XL, XC = S::XC;
    const int r = tid / XL, q = tid % XL;
    float out[XC];
#pragma unroll
    for (int jj = 0; jj < XC; ++jj) out[jj] = (r == XC * q + jj) ? 0.f : LCCRF_NEG_INF;
    float sg = 0.f;  // integer valued
    double osum = 0.0;
    for (int i = first; i <= last; ++i) {
        osum += src.offset(i);
        __syncthreads();
#pragma unroll
        for (int jj = 0; jj < XC; ++jj) {
            const int t = XC * q + jj;
            Pc[r][t] = out[jj];
            Ph[r][t] = src.entry(i, r, t);
        }
        __syncthreads();
        float mx[XC], sm[XC];
#pragma unroll
        for (int jj = 0; jj < XC; ++jj) {
            mx[jj] = LCCRF_NEG_INF;
            sm[jj] = 0.f;
        }
        for (int s = 0; s < TP; ++s) {
            const float p = Pc[r][s];
#pragma unroll
            for (int jj = 0; jj < XC; ++jj) mx[jj] = fmaxf(mx[jj], p + Ph[s][XC * q + jj]);
        }
        for (int s = 0; s < TP; ++s) {
            const float p = Pc[r][s];
#pragma unroll
            for (int jj = 0; jj < XC; ++jj) sm[jj] += ex2(p + Ph[s][XC * q + jj] - finite_or_zero(mx[jj]));
        }
        float rm = LCCRF_NEG_INF;
#pragma unroll
        for (int jj = 0; jj < XC; ++jj) {
            out[jj] = mx[jj] + lg2(sm[jj]);
            rm = fmaxf(rm, out[jj]);
        }
        // shift the row by the integer part of its maximum: scales stay integers, hence exact
        rm = xor_max<1, XL>(rm);
        const float sh = floorf(finite_or_zero(rm));
        sg += sh;
#pragma unroll
        for (int jj = 0; jj < XC; ++jj) out[jj] -= sh;
    }
    const float ef = r < T ? sg : LCCRF_NEG_INF;
    // the largest row scale, over all rows of the workgroup: through LDS
    __syncthreads();
    if (q == 0) Pc[0][r] = ef;
    __syncthreads();
    float emax = LCCRF_NEG_INF;
    for (int k = 0; k < TP; ++k) emax = fmaxf(emax, Pc[0][k]);
    emax = finite_or_zero(emax);
#pragma unroll
    for (int jj = 0; jj < XC; ++jj) {
        const int t = XC * q + jj;
        Pout[t * TP + r] = (r < T && t < T) ? out[jj] : LCCRF_NEG_INF;
    }
    if (q == 0) rel_out[r] = ef - emax;
    if (tid == 0) *base_out = osum + (double)emax;
}

// One wave (up to 32 tags) or NB waves per chunk: the product of the chunk's potentials.
template <typename TIN, int TP, bool VEC, bool STRUCT = false>
__global__ __launch_bounds__(64 * ScanShape<TP>::NW) void chunk_product_kernel(ScanArgs a) {
    __shared__ float Pc[TP][TP + 1];
    __shared__ float Ph[TP][TP + 1];
    __shared__ ProductShared shared;
    const int b = blockIdx.x / a.C, c = blockIdx.x % a.C;
    const int T = a.T, N = a.N;
    const int L = clamp_length(a.lengths, b, N);
    if (c * a.chunk >= L) return;
    int first, last;
    chunk_range(c, a.chunk, L, first, last);
    const size_t bc = (size_t)b * a.C + c;
    float* Pout = a.Pl + bc * TP * TP;
    float* rel_out = a.rel + bc * TP;
    const int lane = threadIdx.x & 63;
    if constexpr (STRUCT) {
        const float* emb = a.emit + (size_t)b * N * T;
        if constexpr (kSingleFirst<TP>) {
            const StructuredMatrices<TP, false> src(emb, a.trans, T, lane);
            if (linear_product<TP, false>(src, first, last, T, Pout, rel_out, a.base + bc, shared)) return;
        }
        const StructuredMatrices<TP, true> src(emb, a.trans, T, lane);
        if (linear_product<TP, true>(src, first, last, T, Pout, rel_out, a.base + bc, shared)) return;
        exact_product<TP>(src, first, last, T, Pout, rel_out, a.base + bc, Pc, Ph);
        return;
    }
    const TIN* phib = static_cast<const TIN*>(a.phi) + (size_t)b * N * T * T;
    if constexpr (kSingleFirst<TP>) {
        const PotentialMatrices<TIN, TP, false, VEC> src(phib, T, lane);
        if (linear_product<TP, false>(src, first, last, T, Pout, rel_out, a.base + bc, shared)) return;
    }
    const PotentialMatrices<TIN, TP, true, VEC> src(phib, T, lane);
    if (linear_product<TP, true>(src, first, last, T, Pout, rel_out, a.base + bc, shared)) return;
    exact_product<TP>(src, first, last, T, Pout, rel_out, a.base + bc, Pc, Ph);
}

// One wave (or NB waves) per group of GS chunks: the product of the group's chunk products.
template <int TP>
__global__ __launch_bounds__(64 * ScanShape<TP>::NW) void group_product_kernel(ScanArgs a) {
    __shared__ float Pc[TP][TP + 1];
    __shared__ float Ph[TP][TP + 1];
    __shared__ ProductShared shared;
    const int b = blockIdx.x / a.G, g = blockIdx.x % a.G;
    const int L = clamp_length(a.lengths, b, a.N);
    const int Cb = (L + a.chunk - 1) / a.chunk;  // chunks of this sequence
    const int c0 = g * a.GS;
    if (c0 >= Cb) return;
    const int c1 = (c0 + a.GS < Cb ? c0 + a.GS : Cb) - 1;
    const size_t cb = (size_t)b * a.C, bg = (size_t)b * a.G + g;
    float* Pout = a.Pl2 + bg * TP * TP;
    float* rel_out = a.rel2 + bg * TP;
    const int lane = threadIdx.x & 63;
    if constexpr (kSingleFirst<TP>) {
        const ChunkMatrices<TP, false> src(a.Pl + cb * TP * TP, a.rel + cb * TP, a.base + cb, a.T, lane);
        if (linear_product<TP, false>(src, c0, c1, a.T, Pout, rel_out, a.base2 + bg, shared)) return;
    }
    const ChunkMatrices<TP, true> src(a.Pl + cb * TP * TP, a.rel + cb * TP, a.base + cb, a.T, lane);
    if (linear_product<TP, true>(src, c0, c1, a.T, Pout, rel_out, a.base2 + bg, shared)) return;
    exact_product<TP>(src, c0, c1, a.T, Pout, rel_out, a.base2 + bg, Pc, Ph);
}

// ---------------------------------------------------------------------------------------
// Phase B.  One wave runs the forward vector through a run of chunk products, another the
// backward vector: the whole sequence (GS = 0: waves 2b and 2b + 1), or the chunks of one group
// (GS > 0: waves 2 (b G + g) and 2 (b G + g) + 1), started from the boundary vectors of the
// groups.  Lane (o = lane / LPRow, q = lane % LPRow) produces output entry o from the CPL input
// entries CPL q .. CPL q + CPL - 1; the vector travels from step to step in registers: entry t of
// the new vector sits in lanes LPRow t .. LPRow t + LPRow - 1, a lane fetches its input entries
// with lane reads.  It is normalised by the maximum of the PREVIOUS vector (one step stale:
// consecutive maxima differ little), so the wave-wide maximum is off the chain of dependent
// instructions.
template <typename TIN, int TP>
__global__ __launch_bounds__(64) void chunk_boundary_kernel(ScanArgs a) {
    using S = ScanShape<TP, true>;
    constexpr int LPRow = S::LPRow, CPL = S::CPL, PF = TP == 16 ? kScanPF : TP == 32 ? 4 : 2;
    const int lane = threadIdx.x, o = lane / LPRow, q = lane % LPRow;
    const int oc = o < TP ? o : TP - 1;  // (48 tags: the last 16 lanes have no entry; they load what lane 47 loads)
    const int dir = blockIdx.x & 1;
    const int unit = blockIdx.x >> 1;
    const bool grouped = a.GS > 0;
    const int b = grouped ? unit / a.G : unit, g = grouped ? unit % a.G : 0;
    const int T = a.T, N = a.N;
    const int L = clamp_length(a.lengths, b, N);
    if (L == 0) {
        if (!grouped && dir == 0 && lane == 0 && a.logZ) a.logZ[b] = 0.f;
        if (!grouped && dir == 0 && lane == 0 && a.logZ64) a.logZ64[b] = 0.0;
        return;
    }
    if (dir == 1 && !a.with_beta) return;
    const int Cb = (L + a.chunk - 1) / a.chunk;
    const int c0 = grouped ? g * a.GS : 0;  // chunks c0 .. c1 are this wave's
    if (c0 >= Cb) return;
    const int c1 = (grouped && c0 + a.GS < Cb ? c0 + a.GS : Cb) - 1;
    const size_t cb = (size_t)b * a.C, bg = (size_t)b * a.G;
    double O = 0.0;
    // one step: x[jj] holds (input entry) + (matrix entry); returns log2 of the sum of their powers
    auto lse = [&](const float (&x)[CPL]) {
        float mx = x[0];
#pragma unroll
        for (int jj = 1; jj < CPL; ++jj) mx = fmaxf(mx, x[jj]);
        mx = xor_max<1, LPRow>(mx);
        const float mf = finite_or_zero(mx);
        float s = 0.f;
#pragma unroll
        for (int jj = 0; jj < CPL; ++jj) s += ex2(x[jj] - mf);
        return mx + lg2(xor_sum<1, LPRow>(s));
    };

    if (dir == 0) {
        float nv;  // alpha before chunk c0, entry o in lanes LPRow o ..
        if (c0 == 0) {
            const TIN* phib = static_cast<const TIN*>(a.phi) + (size_t)b * N * T * T;
            const float v = lane >= T ? LCCRF_NEG_INF  // alpha_0
                            : (a.emit ? a.trans[lane] + a.emit[(size_t)b * N * T + lane] : Elem<TIN>::get(phib + lane)) * kLog2e;
            const float d = finite_or_zero(xor_max<1, 64>(v));
            O = (double)d;
            nv = (o < T) ? __shfl(v, o, 64) - d : LCCRF_NEG_INF;
        } else {
            nv = (o < T) ? a.Fin[(bg + g - 1) * T + o] : LCCRF_NEG_INF;
            O = a.OFin[bg + g - 1];
        }
        float pm[PF][CPL], rl[PF][CPL];
        double bs[PF];
        auto load = [&](int c, int slot) {
            const float* P = a.Pl + (cb + c) * TP * TP + oc * TP + CPL * q;
            const float* E = a.rel + (cb + c) * TP + CPL * q;
#pragma unroll
            for (int k = 0; k < CPL; k += 4) {
                const float4 p = *reinterpret_cast<const float4*>(P + k);
                const float4 e = *reinterpret_cast<const float4*>(E + k);
                pm[slot][k] = p.x; pm[slot][k + 1] = p.y; pm[slot][k + 2] = p.z; pm[slot][k + 3] = p.w;
                rl[slot][k] = e.x; rl[slot][k + 1] = e.y; rl[slot][k + 2] = e.z; rl[slot][k + 3] = e.w;
            }
            bs[slot] = a.base[cb + c];
        };
        float dprev = 0.f;
        walk<PF>(c0, c1, +1, load, [&](int c, int slot) {
            float x[CPL];
#pragma unroll
            for (int jj = 0; jj < CPL; ++jj) x[jj] = lane_bperm(nv, LPRow * (CPL * q + jj)) + (pm[slot][jj] + rl[slot][jj]);
            const float r = lse(x);
            O += bs[slot] + (double)dprev;
            nv = o < TP ? r - dprev : LCCRF_NEG_INF;  // (lanes past the padded tag count hold no entry)
            dprev = finite_or_zero(xor_max<LPRow, 64>(nv));  // used by the next step
            if (q == 0 && o < T) a.Fv[(cb + c) * T + o] = nv;
            if (lane == 0) a.OF[cb + c] = O;
        });
        if (!grouped && (a.logZ || a.logZ64)) {
            // entry t sits in LPRow lanes: count it once
            const float Ssum = xor_sum<1, 64>(q == 0 ? ex2(nv - dprev) : 0.f);
            const double lz = (O + (double)dprev + (double)lg2(Ssum)) * kLn2;
            if (lane == 0 && a.logZ) a.logZ[b] = (float)lz;
            if (lane == 0 && a.logZ64) a.logZ64[b] = lz;
        }
    } else {
        float nv;  // beta at the last position of chunk c1, entry o in lanes LPRow o ..
        if (c1 == Cb - 1) {
            nv = (o < T) ? 0.f : LCCRF_NEG_INF;
        } else {
            nv = (o < T) ? a.Gin[(bg + g) * T + o] : LCCRF_NEG_INF;
            O = a.OGin[bg + g];
        }
        float dprev = 0.f;
        float pm[PF][CPL], rl[PF];
        double bs[PF];
        auto load = [&](int c, int slot) {
            const float* P = a.Pl + (cb + c) * TP * TP;
#pragma unroll
            for (int jj = 0; jj < CPL; ++jj) pm[slot][jj] = P[(CPL * q + jj) * TP + oc];
            rl[slot] = a.rel[(cb + c) * TP + oc];
            bs[slot] = a.base[cb + c];
        };
        // chunk c takes beta at its last position to beta at the last position of chunk c - 1
        walk<PF>(c1, c0 > 1 ? c0 : 1, -1, load, [&](int c, int slot) {
            float x[CPL];
#pragma unroll
            for (int jj = 0; jj < CPL; ++jj) x[jj] = pm[slot][jj] + lane_bperm(nv, LPRow * (CPL * q + jj));
            const float r = lse(x) + rl[slot];
            O += bs[slot] + (double)dprev;
            nv = o < TP ? r - dprev : LCCRF_NEG_INF;  // (lanes past the padded tag count hold no entry)
            dprev = finite_or_zero(xor_max<LPRow, 64>(nv));
            if (q == 0 && o < T) a.Gv[(cb + c - 1) * T + o] = nv;
            if (lane == 0) a.OG[cb + c - 1] = O;
        });
    }
}


// ---------------------------------------------------------------------------------------
// Max-plus analogue (section "Computing Most Probable Structure": the same recursion with max in
// place of log-sum-exp).  Scores stay unscaled in double precision like the sequential Viterbi
// kernel's, so the scan compares the same sums up to the rounding of their last bit.
//
//   phase A: M_c[r][s] = best score of a path through chunk c from tag r (one position before
//       the chunk) to tag s (its last position);
//   phase B: delta at the last position of every chunk with the best entry tag per exit tag,
//       then the back-trace over chunks: the tag at the last position of every chunk (pin);
//   phase C (viterbi_kernel of lccrf_viterbi.hip, one workgroup per chunk): the best path
//       inside every chunk between its two pinned tags, so the stitched path is one valid path.
struct MaxScanArgs {
    const void* phi;
    const int32_t* lengths;
    int B, N, T;
    int chunk, C;
    double* Mx;     // [B][C][TP][TP]  M_c[r][s], -inf padded (TP = 16 up to 16 tags, 32 above)
    uint8_t* K;     // [B][C][TP]      best entry tag for each exit tag
    int32_t* pin;   // [B][C]
    float* best_score;
    // Grouped runs (GS > 0; G = ceil(C / GS) groups a sequence): group_maxplus_kernel writes the
    // max-plus product of every group's chunk matrices to Mx2 ([B][G][TP][TP]); the boundary
    // kernel then handles one group per wave, between the tags pin_in ([B][G]) already fixed at
    // the last position of every group.
    int GS, G;
    double* Mx2;
    const int32_t* pin_in;
    // Structured potentials (emit non-null; phi is then not read), as in ScanArgs.
    const float* emit;
    const float* trans;
};

// Lanes and entries of the max-plus scan's matrices: a TP x TP matrix (TP = 16 or 32) over the 64 lanes of a wave,
// QL lanes a row, EPL consecutive entries of the row a lane.
template <int TP>
struct MaxScanShape {
    static_assert(TP == 16 || TP == 32, "padded tag counts of the max-plus scan");
    static constexpr int QL = 64 / TP;    // 4 or 2
    static constexpr int EPL = TP / QL;   // 4 or 16
    static constexpr int SB = TP == 16 ? 16 : 2;  // rows of a matrix read from LDS at a time (16 tags)
};

// A double of lane `K` of every aligned group of QL lanes (four: a quad; two: lanes 2n and 2n + 1).
template <int QL, int K>
__device__ __forceinline__ double group_read(double x) {
    constexpr int CTRL = QL == 4 ? K * 0x55 : (K == 0 ? 0xA0 : 0xF5);  // quad_perm [K,K,K,K] / [0,0,2,2], [1,1,3,3]
    const long long bits = __double_as_longlong(x);
    const int lo = dpp_i<CTRL>((int)(bits & 0xffffffffll)), hi = dpp_i<CTRL>((int)(bits >> 32));
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}

// Max-plus product of matrices first .. last (none: the identity) by one wave.  Lane
// (r = lane / QL, q = lane % QL) owns M[r][EPL q .. EPL q + EPL - 1]; row r of M is spread over the QL lanes of a
// group and is read from their registers, the entries X_i[s][EPL q ..] of every matrix, which all the
// lanes of column group q need, go through LDS in the type XT (16 tags: potentials as floats would halve the LDS
// bytes, doubles save every reader the conversion; 32 tags: doubles, the conversions would cost half as much again
// as the additions and maxima).  get(slot, jj) returns this lane's entry jj of a matrix.  One wave per workgroup:
// the barrier is only the wait for the LDS writes, and the two tile buffers keep the next matrix's writes off the
// tile that is being read.
template <int TP, int PF, typename Slot, typename XT, typename Load, typename Get>
__device__ __forceinline__ void maxplus_product(int first, int last, int T, double* __restrict__ out, Load load_slot,
                                                Get get, XT (*Xs)[TP][TP]) {
    using S = MaxScanShape<TP>;
    constexpr int QL = S::QL, EPL = S::EPL, SB = S::SB;
    const int lane = threadIdx.x, r = lane / QL, q = lane % QL;
    const double ninf = -__builtin_huge_val();
    double M[EPL];
#pragma unroll
    for (int jj = 0; jj < EPL; ++jj) M[jj] = (r == EPL * q + jj) ? 0.0 : ninf;
    Slot ring[PF];
    auto load = [&](int i, int slot) { load_slot(i, ring[slot]); };
    int buf = 0;
    walk<PF>(first, last, +1, load, [&](int, int slot) {
        buf ^= 1;
        XT(*X)[TP] = Xs[buf];
#pragma unroll
        for (int jj = 0; jj < EPL; ++jj) X[r][EPL * q + jj] = get(ring[slot], jj);
        __syncthreads();
        double best[EPL];
#pragma unroll
        for (int jj = 0; jj < EPL; ++jj) best[jj] = ninf;
        // SB rows of this lane's columns at a time, all their reads first (left to itself the compiler waits for
        // every LDS read before it issues the next), then the arithmetic; row s of M's row r is entry s % EPL of
        // lane s / EPL of the group
#pragma unroll
        for (int s0 = 0; s0 < TP; s0 += SB) {
            XT xr[SB][EPL];
#pragma unroll
            for (int s = 0; s < SB; ++s)
#pragma unroll
                for (int jj = 0; jj < EPL; ++jj) xr[s][jj] = X[s0 + s][EPL * q + jj];
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int s = 0; s < SB; ++s) {
                constexpr int kNone = 0;
                (void)kNone;
                const int sg = s0 + s;
                double m;
                if constexpr (QL == 4) {
                    const int k = sg / EPL;
                    m = k == 0 ? group_read<4, 0>(M[sg % EPL]) : k == 1 ? group_read<4, 1>(M[sg % EPL])
                        : k == 2 ? group_read<4, 2>(M[sg % EPL]) : group_read<4, 3>(M[sg % EPL]);
                } else {
                    m = sg / EPL == 0 ? group_read<2, 0>(M[sg % EPL]) : group_read<2, 1>(M[sg % EPL]);
                }
#pragma unroll
                for (int jj = 0; jj < EPL; ++jj) best[jj] = fmax(best[jj], m + (double)xr[s][jj]);
            }
        }
#pragma unroll
        for (int jj = 0; jj < EPL; ++jj) M[jj] = best[jj];
    });
#pragma unroll
    for (int jj = 0; jj < EPL; ++jj) out[r * TP + EPL * q + jj] = (r < T && EPL * q + jj < T) ? M[jj] : ninf;
}

// The plain instruction: the running maxima are loop-carried, and fmax() quiets them once an iteration (a ninth of
// the product's instructions) although no operand here is ever a NaN (sums of finite values and -inf).
__device__ __forceinline__ double scan_max_raw(double a, double b) {
    double r;
    asm("v_max_f64 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

// The same product for 17 .. 32 tags (32 x 32 matrices, 1024 candidates a position and lane pair).  Lane (a = lane / 8,
// b = lane % 8) owns the 4 x 4 block M[4a .. 4a+3][4b .. 4b+3]: for a source tag s it needs four entries of column s
// of M and four of row s of X, 48 or 64 bytes of LDS for sixteen candidates (a lane that owned part of a row, as
// above, would read 136 bytes for thirty-two, and the product was bound by LDS bandwidth at five times the cost of
// its arithmetic).  M goes through LDS transposed (Mt[s][r]), X (X[s][t]) in the type XT it is given in (potentials as floats,
// chunk products as doubles); the loop over source tags stays a loop (unrolled, a position kept a thousand values
// in flight and spilled), with the reads of the next source tag issued before the arithmetic of the current one.
// get(slot, i, j): entry (4a + i, 4b + j) of a matrix.
template <int PF, typename Slot, typename XT, typename Load, typename Get>
__device__ __forceinline__ void maxplus_product32(int first, int last, int T, double* __restrict__ out, Load load_slot,
                                                  Get get, XT (*Xs)[32][32], double (*Mt)[32]) {
    const int lane = threadIdx.x, a4 = 4 * (lane >> 3), b4 = 4 * (lane & 7);
    const double ninf = -__builtin_huge_val();
    double M[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) M[i][j] = (a4 + i == b4 + j) ? 0.0 : ninf;
    Slot ring[PF];
    auto load = [&](int i, int slot) { load_slot(i, ring[slot]); };
    int buf = 0;
    walk<PF>(first, last, +1, load, [&](int, int slot) {
        buf ^= 1;
        XT(*X)[32] = Xs[buf];  // (two tiles: the writes of a position need not wait behind the reads of the one before)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) X[a4 + i][b4 + j] = get(ring[slot], i, j);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            double2 lo, hi;
            lo.x = M[0][j]; lo.y = M[1][j]; hi.x = M[2][j]; hi.y = M[3][j];
            *reinterpret_cast<double2*>(&Mt[b4 + j][a4]) = lo;
            *reinterpret_cast<double2*>(&Mt[b4 + j][a4 + 2]) = hi;
        }
        __syncthreads();
        double best[4][4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) best[i][j] = ninf;
        const auto read = [&](int sg, double (&m)[4], XT (&x)[4]) {
            const double2 lo = *reinterpret_cast<const double2*>(&Mt[sg][a4]);
            const double2 hi = *reinterpret_cast<const double2*>(&Mt[sg][a4 + 2]);
            m[0] = lo.x; m[1] = lo.y; m[2] = hi.x; m[3] = hi.y;
#pragma unroll
            for (int j = 0; j < 4; ++j) x[j] = X[sg][b4 + j];
        };
        const auto fold = [&](const double (&m)[4], const XT (&x)[4]) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const double xj = (double)x[j];
#pragma unroll
                for (int i = 0; i < 4; ++i) best[i][j] = scan_max_raw(best[i][j], m[i] + xj);
            }
        };
        double ma[4], mb[4];
        XT xa[4], xb[4];
        read(0, ma, xa);
#pragma unroll 2
        for (int sg = 0; sg < 32; sg += 2) {
            read(sg + 1, mb, xb);
            fold(ma, xa);
            read(sg + 2 < 32 ? sg + 2 : 31, ma, xa);
            fold(mb, xb);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) M[i][j] = best[i][j];
    });
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) out[(a4 + i) * 32 + b4 + j] = (a4 + i < T && b4 + j < T) ? M[i][j] : ninf;
}

struct MaxBlockF { float x[4][4]; };
struct MaxBlockD { double x[4][4]; };
struct MaxBlockE { float e[4]; };

// Phase A at 17 .. 32 tags.
template <typename TIN, bool STRUCT = false>
__global__ __launch_bounds__(64) void chunk_maxplus32_kernel(MaxScanArgs a) {
    __shared__ __attribute__((aligned(16))) float Xs[2][32][32];
    __shared__ __attribute__((aligned(16))) double Mt[32][32];
    const int lane = threadIdx.x, a4 = 4 * (lane >> 3), b4 = 4 * (lane & 7);
    const int b = blockIdx.x / a.C, c = blockIdx.x % a.C;
    const int T = a.T, N = a.N;
    const int L = clamp_length(a.lengths, b, N);
    if (c * a.chunk >= L) return;
    int first, last;
    chunk_range(c, a.chunk, L, first, last);
    const size_t TT = (size_t)T * T;
    int off[4][4];
    unsigned in = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int r = a4 + i, t = b4 + j;
            in |= (r < T && t < T) ? (1u << (4 * i + j)) : 0u;
            off[i][j] = (r < T ? r : T - 1) * T + (t < T ? t : T - 1);
        }
    double* out = a.Mx + ((size_t)b * a.C + c) * 1024;
    if constexpr (STRUCT) {
        // the candidates are the single-precision sums trans + emit, as the materialised tensor would hold them
        const float* emb = a.emit + (size_t)b * N * T;
        float tr[4][4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) tr[i][j] = a.trans[off[i][j]];
        maxplus_product32<3, MaxBlockE, float>(
            first, last, T, out,
            [&](int i, MaxBlockE& sl) {
                const float* m = emb + (size_t)i * T;
#pragma unroll
                for (int j = 0; j < 4; ++j) sl.e[j] = m[b4 + j < T ? b4 + j : T - 1];
            },
            [&](const MaxBlockE& sl, int i, int j) { return (in >> (4 * i + j)) & 1 ? tr[i][j] + sl.e[j] : LCCRF_NEG_INF; }, Xs, Mt);
        return;
    }
    const TIN* phib = static_cast<const TIN*>(a.phi) + (size_t)b * N * TT;
    maxplus_product32<3, MaxBlockF, float>(
        first, last, T, out,
        [&](int i, MaxBlockF& sl) {
            const TIN* m = phib + (size_t)i * TT;
#pragma unroll
            for (int ii = 0; ii < 4; ++ii)
#pragma unroll
                for (int j = 0; j < 4; ++j) sl.x[ii][j] = Elem<TIN>::get(m + off[ii][j]);
        },
        [&](const MaxBlockF& sl, int i, int j) { return (in >> (4 * i + j)) & 1 ? sl.x[i][j] : LCCRF_NEG_INF; }, Xs, Mt);
}

// One wave per group of GS chunks at 17 .. 32 tags.
__global__ __launch_bounds__(64) void group_maxplus32_kernel(MaxScanArgs a) {
    __shared__ __attribute__((aligned(16))) double Xs[2][32][32];
    __shared__ __attribute__((aligned(16))) double Mt[32][32];
    const int lane = threadIdx.x, a4 = 4 * (lane >> 3), b4 = 4 * (lane & 7);
    const int b = blockIdx.x / a.G, g = blockIdx.x % a.G;
    const int L = clamp_length(a.lengths, b, a.N);
    const int Cb = (L + a.chunk - 1) / a.chunk;
    const int c0 = g * a.GS;
    if (c0 >= Cb) return;
    const int c1 = (c0 + a.GS < Cb ? c0 + a.GS : Cb) - 1;
    const double* Mb = a.Mx + (size_t)b * a.C * 1024 + a4 * 32 + b4;
    maxplus_product32<2, MaxBlockD, double>(
        c0, c1, a.T, a.Mx2 + ((size_t)b * a.G + g) * 1024,
        [&](int c, MaxBlockD& sl) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) sl.x[i][j] = Mb[(size_t)c * 1024 + i * 32 + j];
        },
        [&](const MaxBlockD& sl, int i, int j) { return sl.x[i][j]; }, Xs, Mt);
}

template <int EPL> struct MaxSlotF { float x[EPL]; };
template <int EPL> struct MaxSlotD { double x[EPL]; };

template <int TP, typename TIN, bool STRUCT = false>
__global__ __launch_bounds__(64) void chunk_maxplus_kernel(MaxScanArgs a) {
    using S = MaxScanShape<TP>;
    constexpr int QL = S::QL, EPL = S::EPL, PF = TP == 16 ? kScanPF : 3;
    __shared__ __attribute__((aligned(16))) double Xs[2][TP][TP];
    const int lane = threadIdx.x, r = lane / QL, q = lane % QL;
    const int b = blockIdx.x / a.C, c = blockIdx.x % a.C;
    const int T = a.T, N = a.N;
    const int L = clamp_length(a.lengths, b, N);
    if (c * a.chunk >= L) return;
    int first, last;
    chunk_range(c, a.chunk, L, first, last);
    const size_t TT = (size_t)T * T;
    int off[EPL];
    unsigned in = 0;
#pragma unroll
    for (int jj = 0; jj < EPL; ++jj) {
        const int t = EPL * q + jj;
        in |= (r < T && t < T) ? (1u << jj) : 0u;
        off[jj] = (r < T ? r : T - 1) * T + (t < T ? t : T - 1);
    }
    if constexpr (STRUCT) {
        // the candidates are the single-precision sums trans + emit, as the materialised tensor would hold them
        const float* emb = a.emit + (size_t)b * N * T;
        float tr[EPL];
#pragma unroll
        for (int jj = 0; jj < EPL; ++jj) tr[jj] = a.trans[off[jj]];
        const int col0 = EPL * q;
        maxplus_product<TP, PF, MaxSlotF<EPL>, double>(
            first, last, T, a.Mx + ((size_t)b * a.C + c) * (TP * TP),
            [&](int i, MaxSlotF<EPL>& sl) {
                const float* m = emb + (size_t)i * T;
#pragma unroll
                for (int jj = 0; jj < EPL; ++jj) sl.x[jj] = m[col0 + jj < T ? col0 + jj : T - 1];
            },
            [&](const MaxSlotF<EPL>& sl, int jj) { return (double)((in >> jj) & 1 ? tr[jj] + sl.x[jj] : LCCRF_NEG_INF); }, Xs);
        return;
    }
    const TIN* phib = static_cast<const TIN*>(a.phi) + (size_t)b * N * TT;
    maxplus_product<TP, PF, MaxSlotF<EPL>, double>(
        first, last, T, a.Mx + ((size_t)b * a.C + c) * (TP * TP),
        [&](int i, MaxSlotF<EPL>& sl) {
            const TIN* m = phib + (size_t)i * TT;
#pragma unroll
            for (int jj = 0; jj < EPL; ++jj) sl.x[jj] = Elem<TIN>::get(m + off[jj]);
        },
        [&](const MaxSlotF<EPL>& sl, int jj) { return (double)((in >> jj) & 1 ? sl.x[jj] : LCCRF_NEG_INF); }, Xs);
}

// One wave per group of GS chunks: the max-plus product of the group's chunk matrices.
template <int TP>
__global__ __launch_bounds__(64) void group_maxplus_kernel(MaxScanArgs a) {
    using S = MaxScanShape<TP>;
    constexpr int QL = S::QL, EPL = S::EPL;
    __shared__ __attribute__((aligned(16))) double Xs[2][TP][TP];
    const int lane = threadIdx.x, r = lane / QL, q = lane % QL;
    const int b = blockIdx.x / a.G, g = blockIdx.x % a.G;
    const int L = clamp_length(a.lengths, b, a.N);
    const int Cb = (L + a.chunk - 1) / a.chunk;
    const int c0 = g * a.GS;
    if (c0 >= Cb) return;
    const int c1 = (c0 + a.GS < Cb ? c0 + a.GS : Cb) - 1;
    const double* Mb = a.Mx + (size_t)b * a.C * (TP * TP) + r * TP + EPL * q;
    maxplus_product<TP, (TP == 16 ? 4 : 2), MaxSlotD<EPL>, double>(
        c0, c1, a.T, a.Mx2 + ((size_t)b * a.G + g) * (TP * TP),
        [&](int c, MaxSlotD<EPL>& sl) {
#pragma unroll
            for (int jj = 0; jj < EPL; ++jj) sl.x[jj] = Mb[(size_t)c * (TP * TP) + jj];
        },
        [&](const MaxSlotD<EPL>& sl, int jj) { return sl.x[jj]; }, Xs);
}

constexpr int kPinWindow = 1024;  // chunks of back-pointers held in LDS at a time by the back-trace

// Phase B of the max-plus scan.  One wave per sequence (GS = 0) or per group of chunks (GS > 0):
// delta through the chunk matrices with the best entry tag per exit tag (K), then the back-trace
// over those chunks, which fixes the tag at the last position of every chunk (pin).  A whole
// sequence starts from delta_0 and ends in its best final tag; a group starts from the tag
// already fixed at the end of the group before it (group 0: delta_0) and ends in the tag fixed at
// its own end, so what it finds is a best path between those two tags.
// (Exit tag t in lanes QL t .. QL t + QL - 1, lane q of them taking the entry tags EPL q .. EPL q + EPL - 1.)
template <int TP, typename TIN>
__global__ __launch_bounds__(64) void chunk_maxplus_boundary_kernel(MaxScanArgs a) {
    using S = MaxScanShape<TP>;
    constexpr int QL = S::QL, EPL = S::EPL, PF = TP == 16 ? kScanPF : 3;
    __shared__ uint8_t win[kPinWindow * TP];
    const int lane = threadIdx.x, t = lane / QL, q = lane % QL;
    const bool grouped = a.GS > 0;
    const int b = grouped ? blockIdx.x / a.G : blockIdx.x, g = grouped ? blockIdx.x % a.G : 0;
    const int T = a.T, N = a.N;
    const int L = clamp_length(a.lengths, b, N);
    if (L == 0) {
        if (!grouped && lane == 0 && a.best_score) a.best_score[b] = 0.f;
        return;
    }
    const int Cb = (L + a.chunk - 1) / a.chunk;
    const int c0 = grouped ? g * a.GS : 0;  // chunks c0 .. c1 are this wave's
    if (c0 >= Cb) return;
    const int c1 = (grouped && c0 + a.GS < Cb ? c0 + a.GS : Cb) - 1;
    const size_t cb = (size_t)b * a.C, bg = (size_t)b * a.G;
    const double ninf = -__builtin_huge_val();
    // delta of the last boundary, entry t in lanes 4t .. 4t+3: it travels from step to step in registers
    double dv;
    if (c0 == 0) {
        const TIN* phib = static_cast<const TIN*>(a.phi) + (size_t)b * N * T * T;
        dv = t >= T ? ninf  // delta_0
             : a.emit ? (double)(a.trans[t] + a.emit[(size_t)b * N * T + t]) : (double)Elem<TIN>::get(phib + t);
    } else {
        dv = (t == a.pin_in[bg + g - 1]) ? 0.0 : ninf;  // the tag fixed at the end of the group before
    }
    double mm[PF][EPL];
    auto load = [&](int c, int slot) {
        const double* M = a.Mx + (cb + c) * (TP * TP);
#pragma unroll
        for (int jj = 0; jj < EPL; ++jj) mm[slot][jj] = M[(EPL * q + jj) * TP + t];
    };
    walk<PF>(c0, c1, +1, load, [&](int c, int slot) {
        double bv = ninf;
        int ba = 0x7fffffff;
        double in[EPL];
#pragma unroll
        for (int jj = 0; jj < EPL; ++jj) in[jj] = __shfl(dv, QL * (EPL * q + jj), 64);
#pragma unroll
        for (int jj = 0; jj < EPL; ++jj) {  // ascending entry tags: the first maximum wins
            const double val = in[jj] + mm[slot][jj];
            if (val > bv) { bv = val; ba = EPL * q + jj; }
        }
#pragma unroll
        for (int off = 1; off < QL; off <<= 1) {
            const double pv = __shfl_xor(bv, off, 64);
            const int pa = __shfl_xor(ba, off, 64);
            if (pv > bv || (pv == bv && pa < ba)) { bv = pv; ba = pa; }
        }
        dv = bv;
        if (q == 0) a.K[(cb + c) * TP + t] = (uint8_t)(ba == 0x7fffffff ? 0 : ba);
    });
    int y;
    if (!grouped) {
        // best tag at the last position: first maximum (entry t sits in lanes QL t .. QL t + QL - 1)
        double bv = (q == 0 && t < T) ? dv : ninf;
        int ba = (q == 0 && t < T) ? t : 0x7fffffff;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const double pv = __shfl_xor(bv, off, 64);
            const int pa = __shfl_xor(ba, off, 64);
            if (pv > bv || (pv == bv && pa < ba)) { bv = pv; ba = pa; }
        }
        if (ba == 0x7fffffff) ba = 0;
        if (lane == 0 && a.best_score) a.best_score[b] = (float)bv;
        y = ba;
    } else {
        y = a.pin_in[bg + g];
        if (y < 0 || y >= T) y = 0;
    }
    __threadfence();  // K written above is read back below by other lanes
    __syncthreads();
    // back-trace over the chunks through an LDS window of K: chunk c maps the tag at its end to the
    // tag at the end of chunk c - 1
    int hi = c1 + 1;  // chunks (c0, hi) still to walk
    if (lane == 0) a.pin[cb + c1] = y;
    while (hi > c0 + 1) {
        const int lo = (hi - kPinWindow > c0 + 1) ? hi - kPinWindow : c0 + 1;
        const int nbytes = (hi - lo) * TP;
        const uint8_t* src = a.K + (cb + lo) * TP;
        for (int k = lane; k < nbytes; k += 64) win[k] = src[k];
        __syncthreads();
        if (lane == 0) {
            for (int c = hi - 1; c >= lo; --c) {
                y = win[(c - lo) * TP + y];
                a.pin[cb + c - 1] = y;
            }
        }
        __syncthreads();
        hi = lo;
    }
}

// ---------------------------------------------------------------------------------------
// Sum queries: tag sets up to 64 (matrices in 1, 4, 9 or 16 blocks of 16 x 16); the max-plus scan: up to 32.
bool scan_supported(int T) { return T >= 1 && T <= 64; }
bool scan_supported_max(int T) { return T >= 1 && T <= 32; }
int scan_padded_tags_max(int T) { return T <= 16 ? 16 : 32; }
int scan_padded_tags(int T) { return (T + 15) / 16 * 16; }

// Chunks per group when phase B is itself run as a scan; 0: one serial pass over all chunks.  The
// group products cost about 3.5 times a vector step each and two serial stages follow them
// (over groups, over the chunks of a group), which puts the best group near sqrt(C) / 2.
int scan_group_size(int C) {
    if (C < 64) return 0;
    int gs = 4;
    while (gs * gs * 4 < C) gs *= 2;
    return gs;
}

template <typename TIN, int TP>
static hipError_t launch_scan_boundaries_t(ScanArgs a, const ScanGroupBuffers& gb, hipStream_t st) {
    constexpr int kProductThreads = 64 * ScanShape<TP>::NW;
    // vector loads of a lane's NB neighbouring columns: T a multiple of NB, and the rows aligned for them
    constexpr int NB = ScanShape<TP>::NB;
    const bool vec = NB > 1 && a.T % NB == 0 && (NB == 3 ? sizeof(TIN) == 4 : true);
    if (a.emit)
        hipLaunchKernelGGL((chunk_product_kernel<float, TP, false, true>), dim3(a.B * a.C), dim3(kProductThreads), 0, st, a);
    else if (vec)
        hipLaunchKernelGGL((chunk_product_kernel<TIN, TP, true>), dim3(a.B * a.C), dim3(kProductThreads), 0, st, a);
    else
        hipLaunchKernelGGL((chunk_product_kernel<TIN, TP, false>), dim3(a.B * a.C), dim3(kProductThreads), 0, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int gs = scan_group_size(a.C);
    if (gs == 0) {
        hipLaunchKernelGGL((chunk_boundary_kernel<TIN, TP>), dim3(2 * a.B), dim3(64), 0, st, a);
        return hipGetLastError();
    }
    const int G = (a.C + gs - 1) / gs;
    // products of the groups
    ScanArgs p = a;
    p.GS = gs; p.G = G; p.Pl2 = gb.Pl2; p.rel2 = gb.rel2; p.base2 = gb.base2;
    hipLaunchKernelGGL(group_product_kernel<TP>, dim3(a.B * G), dim3(kProductThreads), 0, st, p);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    // phase B over the groups: the same kernel, a group in the place of a chunk (this launch writes logZ)
    ScanArgs u = a;
    u.chunk = a.chunk * gs; u.C = G;
    u.Pl = gb.Pl2; u.rel = gb.rel2; u.base = gb.base2; u.Fv = gb.Fv2; u.OF = gb.OF2; u.Gv = gb.Gv2; u.OG = gb.OG2;
    hipLaunchKernelGGL((chunk_boundary_kernel<TIN, TP>), dim3(2 * a.B), dim3(64), 0, st, u);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    // ... and over the chunks of every group at once
    ScanArgs l = a;
    l.GS = gs; l.G = G; l.logZ = nullptr; l.logZ64 = nullptr;
    l.Fin = gb.Fv2; l.OFin = gb.OF2; l.Gin = gb.Gv2; l.OGin = gb.OG2;
    hipLaunchKernelGGL((chunk_boundary_kernel<TIN, TP>), dim3(2 * a.B * G), dim3(64), 0, st, l);
    return hipGetLastError();
}

hipError_t launch_scan_boundaries(int dtype, const void* phi, const int32_t* lengths, int B, int N, int T, int chunk,
                                  float* Pl, float* rel, double* base, float* Fv, double* OF, float* Gv, double* OG,
                                  const ScanGroupBuffers& gb, float* logZ, bool with_beta, hipStream_t st,
                                  double* logZ64, const float* emit, const float* trans) {
    const int C = (N + chunk - 1) / chunk;
    ScanArgs a{phi, lengths, B, N, T, chunk, C, Pl, rel, base, Fv, OF, Gv, OG, logZ, with_beta ? 1 : 0, logZ64,
               0, 1, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, emit, trans};
    if (emit && (dtype != 0 || !trans)) return hipErrorInvalidValue;
    if (T <= 16)
        return dtype == 0 ? launch_scan_boundaries_t<float, 16>(a, gb, st) : launch_scan_boundaries_t<uint16_t, 16>(a, gb, st);
    if (T <= 32)
        return dtype == 0 ? launch_scan_boundaries_t<float, 32>(a, gb, st) : launch_scan_boundaries_t<uint16_t, 32>(a, gb, st);
    if (T <= 48)
        return dtype == 0 ? launch_scan_boundaries_t<float, 48>(a, gb, st) : launch_scan_boundaries_t<uint16_t, 48>(a, gb, st);
    if (T <= 64)
        return dtype == 0 ? launch_scan_boundaries_t<float, 64>(a, gb, st) : launch_scan_boundaries_t<uint16_t, 64>(a, gb, st);
    return hipErrorInvalidValue;
}


template <int TP, typename TIN>
static hipError_t launch_scan_pins_t(MaxScanArgs a, const MaxGroupBuffers& gb, hipStream_t st) {
    if constexpr (TP == 32) {
        if (a.emit) hipLaunchKernelGGL((chunk_maxplus32_kernel<float, true>), dim3(a.B * a.C), dim3(64), 0, st, a);
        else hipLaunchKernelGGL((chunk_maxplus32_kernel<TIN>), dim3(a.B * a.C), dim3(64), 0, st, a);
    } else {
        if (a.emit) hipLaunchKernelGGL((chunk_maxplus_kernel<TP, float, true>), dim3(a.B * a.C), dim3(64), 0, st, a);
        else hipLaunchKernelGGL((chunk_maxplus_kernel<TP, TIN>), dim3(a.B * a.C), dim3(64), 0, st, a);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int gs = scan_group_size(a.C);
    if (gs == 0) {
        hipLaunchKernelGGL((chunk_maxplus_boundary_kernel<TP, TIN>), dim3(a.B), dim3(64), 0, st, a);
        return hipGetLastError();
    }
    const int G = (a.C + gs - 1) / gs;
    MaxScanArgs p = a;
    p.GS = gs; p.G = G; p.Mx2 = gb.Mx2;
    if constexpr (TP == 32) hipLaunchKernelGGL(group_maxplus32_kernel, dim3(a.B * G), dim3(64), 0, st, p);
    else hipLaunchKernelGGL(group_maxplus_kernel<TP>, dim3(a.B * G), dim3(64), 0, st, p);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    // phase B over the groups: the same kernel, a group in the place of a chunk (best score, tags at group ends)
    MaxScanArgs u = a;
    u.chunk = a.chunk * gs; u.C = G; u.Mx = gb.Mx2; u.K = gb.K2; u.pin = gb.pin2;
    hipLaunchKernelGGL((chunk_maxplus_boundary_kernel<TP, TIN>), dim3(a.B), dim3(64), 0, st, u);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    // ... and inside every group at once, between the tags just fixed
    MaxScanArgs l = a;
    l.GS = gs; l.G = G; l.best_score = nullptr; l.pin_in = gb.pin2;
    hipLaunchKernelGGL((chunk_maxplus_boundary_kernel<TP, TIN>), dim3(a.B * G), dim3(64), 0, st, l);
    return hipGetLastError();
}

hipError_t launch_scan_pins(int dtype, const void* phi, const int32_t* lengths, int B, int N, int T, int chunk,
                            double* Mx, uint8_t* K, int32_t* pin, const MaxGroupBuffers& gb, float* best_score,
                            hipStream_t st, const float* emit, const float* trans) {
    const int C = (N + chunk - 1) / chunk;
    MaxScanArgs a{phi, lengths, B, N, T, chunk, C, Mx, K, pin, best_score, 0, 1, nullptr, nullptr, emit, trans};
    if (emit && (dtype != 0 || !trans)) return hipErrorInvalidValue;
    if (!scan_supported_max(T)) return hipErrorInvalidValue;
    if (T <= 16) return dtype == 0 ? launch_scan_pins_t<16, float>(a, gb, st) : launch_scan_pins_t<16, uint16_t>(a, gb, st);
    return dtype == 0 ? launch_scan_pins_t<32, float>(a, gb, st) : launch_scan_pins_t<32, uint16_t>(a, gb, st);
}

}  // namespace lccrf
