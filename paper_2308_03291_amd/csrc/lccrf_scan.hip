// Chunked log-semiring scan over the positions of long chains with a small tag set (T <= 32; the
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
// TP is the padded tag count (16 or 32); matrices are handled as NB x NB blocks of 16 x 16,
// NB = TP / 16.  Lane (g = lane / 16, j = lane % 16) handles, of block (sb, tb), four entries of
// column 16 tb + j (row: tag before, column: tag after), entry number e = (sb NB + tb) 4 + v: the rows
// an accumulator register v of that lane holds after a 16x16x4 MFMA, which are 16 sb + g + 4v for the
// f64 instruction (F64) and 16 sb + 4g + v for the f32 one.  Sources hand out matrices in base-2
// logarithms, -inf outside T x T; every matrix may carry a common offset besides.
template <int TP, bool F64 = true>
struct ScanShape {
    static constexpr int NB = TP / 16, NE = 4 * NB * NB;
    static constexpr int LPRow = 64 / TP;    // lanes sharing a row in the row-wise layouts (exact product, phase B)
    static constexpr int CPL = TP / LPRow;   // columns per lane there
    static_assert(TP == 16 || TP == 32, "padded tag count");
    static __device__ __forceinline__ int row(int lane, int e) {
        return 16 * (e / (4 * NB)) + (F64 ? (lane >> 4) + 4 * (e & 3) : 4 * (lane >> 4) + (e & 3));
    }
    static __device__ __forceinline__ int col(int lane, int e) { return 16 * ((e / 4) % NB) + (lane & 15); }
};

template <typename TIN, int TP, bool F64>
struct PotentialMatrices {  // the potentials phi_i of one sequence
    using S = ScanShape<TP, F64>;
    static constexpr int PF = TP == 16 ? kScanPF : 3;
    struct Slot { float x[S::NE]; };
    // entries outside T x T are loaded from the nearest entry inside: whatever a slot holds is a potential
    static constexpr bool kPaddingIsFinite = true;
    const TIN* phib;
    int T;
    size_t TT;
    int off[S::NE];
    unsigned in;  // bit e: entry e lies inside T x T
    __device__ PotentialMatrices(const TIN* p, int T_, int lane) : phib(p), T(T_), TT((size_t)T_ * T_), in(0) {
#pragma unroll
        for (int e = 0; e < S::NE; ++e) {
            const int s = S::row(lane, e), t = S::col(lane, e);
            in |= (s < T && t < T) ? (1u << e) : 0u;
            off[e] = (s < T ? s : T - 1) * T + (t < T ? t : T - 1);
        }
    }
    __device__ __forceinline__ void load(int i, Slot& sl) const {
        const TIN* m = phib + (size_t)i * TT;
#pragma unroll
        for (int e = 0; e < S::NE; ++e) sl.x[e] = Elem<TIN>::get(m + off[e]);
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

template <int TP, bool F64>
struct ChunkMatrices {  // the chunk products of one sequence, as phase A has written them
    using S = ScanShape<TP, F64>;
    static constexpr int PF = TP == 16 ? 4 : 2;
    struct Slot { float p[S::NE], r[S::NE]; double b; };
    static constexpr bool kPaddingIsFinite = false;  // stored products are -inf outside T x T
    const float* Pl;
    const float* rel;
    const double* base;
    int T, lane;
    __device__ ChunkMatrices(const float* Pl_, const float* rel_, const double* base_, int T_, int lane_)
        : Pl(Pl_), rel(rel_), base(base_), T(T_), lane(lane_) {}
    __device__ __forceinline__ void load(int c, Slot& sl) const {
#pragma unroll
        for (int e = 0; e < S::NE; ++e) {
            sl.p[e] = Pl[(size_t)c * TP * TP + S::col(lane, e) * TP + S::row(lane, e)];
            sl.r[e] = rel[(size_t)c * TP + S::row(lane, e)];
        }
        sl.b = base[c];
    }
    __device__ __forceinline__ double entries(const Slot& sl, float (&x)[S::NE]) const {
#pragma unroll
        for (int e = 0; e < S::NE; ++e)
            x[e] = (S::row(lane, e) < T && S::col(lane, e) < T) ? sl.p[e] + sl.r[e] : LCCRF_NEG_INF;
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
constexpr bool kSingleFirst = TP == 32;

template <int TP, bool F64, typename Src>
__device__ __forceinline__ bool linear_product(const Src& src, int first, int last, int T, float* __restrict__ Pout,
                                               float* __restrict__ rel_out, double* __restrict__ base_out) {
    using S = ScanShape<TP, F64>;
    using L = Linear<F64>;
    using scalar = typename L::scalar;
    using vec = typename L::vec;
    constexpr int NB = S::NB, NE = S::NE;
    const int lane = threadIdx.x;
    const int g = lane >> 4, j = lane & 15;
    unsigned in = 0;
#pragma unroll
    for (int e = 0; e < NE; ++e) in |= (S::row(lane, e) < T && S::col(lane, e) < T) ? (1u << e) : 0u;
    // The zero pattern of D (1 where some path exists) is carried along by a product of 0/1
    // matrices on the f32 MFMA, from the first matrix with a -inf entry on (until then D is
    // the identity or has no zero).  That instruction numbers its output rows 4g + v; beside the
    // f64 product it therefore runs on rows renamed by pi(4g + v) = g + 4v: its A operand is the
    // flag of column pi(j).
    const int pj = F64 ? ((lane & 48) | (4 * (j & 3) + (j >> 2))) : lane;
    scalar D[NB][NB][4];
    float Z[NB][NB][4];
    double Msum = 0.0;
    int esum[NB];
    bool bad = false, tracking = false, started = false, rejected = false;
#pragma unroll
    for (int sb = 0; sb < NB; ++sb)
#pragma unroll
        for (int rb = 0; rb < NB; ++rb)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const bool diag = sb == rb && (F64 ? g + 4 * v : 4 * g + v) == j;
                D[sb][rb][v] = diag ? (scalar)1 : (scalar)0;
                Z[sb][rb][v] = diag ? 1.f : 0.f;
            }
#pragma unroll
    for (int rb = 0; rb < NB; ++rb) esum[rb] = 0;
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
        vec acc[NB][NB];
#pragma unroll
        for (int tb = 0; tb < NB; ++tb)
#pragma unroll
            for (int rb = 0; rb < NB; ++rb) acc[tb][rb] = vec{0, 0, 0, 0};
#pragma unroll
        for (int sb = 0; sb < NB; ++sb)
#pragma unroll
            for (int tb = 0; tb < NB; ++tb)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const scalar E = L::pow2(x[(sb * NB + tb) * 4 + v] - m);
#pragma unroll
                    for (int rb = 0; rb < NB; ++rb) acc[tb][rb] = L::mfma(E, D[sb][rb][v], acc[tb][rb]);
                }
        // bit e of nz: entry e of this matrix is not a structural zero
        const auto nonzero_mask = [&]() {
            unsigned nz = 0;
#pragma unroll
            for (int e = 0; e < NE; ++e) nz |= (x[e] > LCCRF_NEG_INF) ? (1u << e) : 0u;
            return nz;
        };
        unsigned nz = 0;
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
                    for (int rb = 0; rb < NB; ++rb)
#pragma unroll
                        for (int v = 0; v < 4; ++v) Z[sb][rb][v] = (in >> ((sb * NB + rb) * 4 + v)) & 1 ? 1.f : 0.f;
            }
        }
        started = true;
        // Exponent fields of the new entries: their largest gives each column's rescale, the
        // smallest among the entries that some path reaches says whether the product still holds.
        unsigned fld[NB][NB][4], fmin = L::kNoField;
#pragma unroll
        for (int tb = 0; tb < NB; ++tb)
#pragma unroll
            for (int rb = 0; rb < NB; ++rb)
#pragma unroll
                for (int v = 0; v < 4; ++v) fld[tb][rb][v] = L::field(acc[tb][rb][v]);
        if (tracking) {
            if constexpr (Src::kPaddingIsFinite) nz = nonzero_mask();
            const unsigned nzp = (unsigned)__shfl((int)nz, pj, 64);
            f32x4 pat[NB][NB];
#pragma unroll
            for (int tb = 0; tb < NB; ++tb)
#pragma unroll
                for (int rb = 0; rb < NB; ++rb) pat[tb][rb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int sb = 0; sb < NB; ++sb)
#pragma unroll
                for (int tb = 0; tb < NB; ++tb)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const float flag = (nzp >> ((sb * NB + tb) * 4 + v)) & 1 ? 1.f : 0.f;
#pragma unroll
                        for (int rb = 0; rb < NB; ++rb)
                            pat[tb][rb] = __builtin_amdgcn_mfma_f32_16x16x4f32(flag, Z[sb][rb][v], pat[tb][rb], 0, 0, 0);
                    }
#pragma unroll
            for (int tb = 0; tb < NB; ++tb)
#pragma unroll
                for (int rb = 0; rb < NB; ++rb)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const bool reached = pat[tb][rb][v] > 0.f;
                        Z[tb][rb][v] = reached ? 1.f : 0.f;
                        fmin = min(fmin, reached ? fld[tb][rb][v] : L::kNoField);
                    }
        } else {
#pragma unroll
            for (int tb = 0; tb < NB; ++tb)
#pragma unroll
                for (int rb = 0; rb < NB; ++rb)
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        fmin = min(fmin, (in >> ((tb * NB + rb) * 4 + v)) & 1 ? fld[tb][rb][v] : L::kNoField);
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
        for (int rb = 0; rb < NB; ++rb) {
            unsigned ef = 0;
#pragma unroll
            for (int tb = 0; tb < NB; ++tb)
#pragma unroll
                for (int v = 0; v < 4; ++v) ef = max(ef, fld[tb][rb][v]);
            const auto r16 = __builtin_amdgcn_permlane16_swap(ef, ef, false, false);
            ef = max(r16[0], r16[1]);
            const auto r32 = __builtin_amdgcn_permlane32_swap(ef, ef, false, false);
            ef = max(r32[0], r32[1]);
            const int ex = ef > 0 ? (int)ef - (int)L::kBias : 0;  // a column without any path keeps its zeros
            esum[rb] += ex;
#pragma unroll
            for (int tb = 0; tb < NB; ++tb)
#pragma unroll
                for (int v = 0; v < 4; ++v) D[tb][rb][v] = L::scaled(acc[tb][rb][v], ex);
        }
        return true;
    };
    if constexpr (F64) walk<Src::PF>(first, last, +1, load, step);
    else walk_while<Src::PF>(first, last, +1, load, step);
    rejected |= __builtin_amdgcn_ballot_w64(bad) != 0;
    if (!rejected) {
        float ef[NB], emax = LCCRF_NEG_INF;
#pragma unroll
        for (int rb = 0; rb < NB; ++rb) {
            ef[rb] = 16 * rb + j < T ? (float)esum[rb] : LCCRF_NEG_INF;
            emax = fmaxf(emax, xor_max<1, 16>(ef[rb]));
        }
        emax = finite_or_zero(emax);
#pragma unroll
        for (int tb = 0; tb < NB; ++tb)
#pragma unroll
            for (int rb = 0; rb < NB; ++rb)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const bool inside = (in >> ((tb * NB + rb) * 4 + v)) & 1;
                    Pout[S::row(lane, (tb * NB + rb) * 4 + v) * TP + 16 * rb + j] =
                        (inside && D[tb][rb][v] > 0) ? L::log2_of(D[tb][rb][v]) : LCCRF_NEG_INF;
                }
        if (g == 0) {
#pragma unroll
            for (int rb = 0; rb < NB; ++rb) rel_out[16 * rb + j] = ef[rb] - emax;
        }
        if (lane == 0) *base_out = Msum + (double)emax;
        return true;
    }
    return false;
}

// The same product in the log domain, every log-sum-exp shifted by its own maximum (rare: taken when
// both linear products gave up).  Lane (r = lane / LPRow, q = lane % LPRow) owns
// P[r][CPL q .. CPL q + CPL - 1]; P and the current matrix are exchanged through LDS.
template <int TP, typename Src>
__device__ __forceinline__ void exact_product(const Src& src, int first, int last, int T, float* __restrict__ Pout,
                                              float* __restrict__ rel_out, double* __restrict__ base_out,
                                              float (*Pc)[TP + 1], float (*Ph)[TP + 1]) {
    using S = ScanShape<TP, true>;
    const int lane = threadIdx.x;
    constexpr int LPRow = S::LPRow, CPL = S::CPL;
    const int r = lane / LPRow, q = lane % LPRow;
    float out[CPL];
#pragma unroll
    for (int jj = 0; jj < CPL; ++jj) out[jj] = (r == CPL * q + jj) ? 0.f : LCCRF_NEG_INF;
    float sg = 0.f;  // integer valued
    double osum = 0.0;
    for (int i = first; i <= last; ++i) {
        osum += src.offset(i);
        __syncthreads();
#pragma unroll
        for (int jj = 0; jj < CPL; ++jj) {
            const int t = CPL * q + jj;
            Pc[r][t] = out[jj];
            Ph[r][t] = src.entry(i, r, t);
        }
        __syncthreads();
        float mx[CPL], sm[CPL];
#pragma unroll
        for (int jj = 0; jj < CPL; ++jj) {
            mx[jj] = LCCRF_NEG_INF;
            sm[jj] = 0.f;
        }
        for (int s = 0; s < TP; ++s) {
            const float p = Pc[r][s];
#pragma unroll
            for (int jj = 0; jj < CPL; ++jj) mx[jj] = fmaxf(mx[jj], p + Ph[s][CPL * q + jj]);
        }
        for (int s = 0; s < TP; ++s) {
            const float p = Pc[r][s];
#pragma unroll
            for (int jj = 0; jj < CPL; ++jj) sm[jj] += ex2(p + Ph[s][CPL * q + jj] - finite_or_zero(mx[jj]));
        }
        float rm = LCCRF_NEG_INF;
#pragma unroll
        for (int jj = 0; jj < CPL; ++jj) {
            out[jj] = mx[jj] + lg2(sm[jj]);
            rm = fmaxf(rm, out[jj]);
        }
        // shift the row by the integer part of its maximum: scales stay integers, hence exact
        rm = xor_max<1, LPRow>(rm);
        const float sh = floorf(finite_or_zero(rm));
        sg += sh;
#pragma unroll
        for (int jj = 0; jj < CPL; ++jj) out[jj] -= sh;
    }
    const float ef = r < T ? sg : LCCRF_NEG_INF;
    const float emax = finite_or_zero(xor_max<LPRow, 64>(ef));
#pragma unroll
    for (int jj = 0; jj < CPL; ++jj) {
        const int t = CPL * q + jj;
        Pout[t * TP + r] = (r < T && t < T) ? out[jj] : LCCRF_NEG_INF;
    }
    if (q == 0) rel_out[r] = ef - emax;
    if (lane == 0) *base_out = osum + (double)emax;
}

// One wave per chunk: the product of the chunk's potentials.
template <typename TIN, int TP>
__global__ __launch_bounds__(64) void chunk_product_kernel(ScanArgs a) {
    __shared__ float Pc[TP][TP + 1];
    __shared__ float Ph[TP][TP + 1];
    const int b = blockIdx.x / a.C, c = blockIdx.x % a.C;
    const int T = a.T, N = a.N;
    const int L = clamp_length(a.lengths, b, N);
    if (c * a.chunk >= L) return;
    int first, last;
    chunk_range(c, a.chunk, L, first, last);
    const TIN* phib = static_cast<const TIN*>(a.phi) + (size_t)b * N * T * T;
    const size_t bc = (size_t)b * a.C + c;
    float* Pout = a.Pl + bc * TP * TP;
    float* rel_out = a.rel + bc * TP;
    if constexpr (kSingleFirst<TP>) {
        const PotentialMatrices<TIN, TP, false> src(phib, T, threadIdx.x);
        if (linear_product<TP, false>(src, first, last, T, Pout, rel_out, a.base + bc)) return;
    }
    const PotentialMatrices<TIN, TP, true> src(phib, T, threadIdx.x);
    if (linear_product<TP, true>(src, first, last, T, Pout, rel_out, a.base + bc)) return;
    exact_product<TP>(src, first, last, T, Pout, rel_out, a.base + bc, Pc, Ph);
}

// One wave per group of GS chunks: the product of the group's chunk products.
template <int TP>
__global__ __launch_bounds__(64) void group_product_kernel(ScanArgs a) {
    __shared__ float Pc[TP][TP + 1];
    __shared__ float Ph[TP][TP + 1];
    const int b = blockIdx.x / a.G, g = blockIdx.x % a.G;
    const int L = clamp_length(a.lengths, b, a.N);
    const int Cb = (L + a.chunk - 1) / a.chunk;  // chunks of this sequence
    const int c0 = g * a.GS;
    if (c0 >= Cb) return;
    const int c1 = (c0 + a.GS < Cb ? c0 + a.GS : Cb) - 1;
    const size_t cb = (size_t)b * a.C, bg = (size_t)b * a.G + g;
    float* Pout = a.Pl2 + bg * TP * TP;
    float* rel_out = a.rel2 + bg * TP;
    if constexpr (kSingleFirst<TP>) {
        const ChunkMatrices<TP, false> src(a.Pl + cb * TP * TP, a.rel + cb * TP, a.base + cb, a.T, threadIdx.x);
        if (linear_product<TP, false>(src, c0, c1, a.T, Pout, rel_out, a.base2 + bg)) return;
    }
    const ChunkMatrices<TP, true> src(a.Pl + cb * TP * TP, a.rel + cb * TP, a.base + cb, a.T, threadIdx.x);
    if (linear_product<TP, true>(src, c0, c1, a.T, Pout, rel_out, a.base2 + bg)) return;
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
    constexpr int LPRow = S::LPRow, CPL = S::CPL, PF = TP == 16 ? kScanPF : 4;
    const int lane = threadIdx.x, o = lane / LPRow, q = lane % LPRow;
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
            const float v = (lane < T) ? Elem<TIN>::get(phib + lane) * kLog2e : LCCRF_NEG_INF;  // alpha_0
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
            const float* P = a.Pl + (cb + c) * TP * TP + o * TP + CPL * q;
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
            nv = r - dprev;
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
            for (int jj = 0; jj < CPL; ++jj) pm[slot][jj] = P[(CPL * q + jj) * TP + o];
            rl[slot] = a.rel[(cb + c) * TP + o];
            bs[slot] = a.base[cb + c];
        };
        // chunk c takes beta at its last position to beta at the last position of chunk c - 1
        walk<PF>(c1, c0 > 1 ? c0 : 1, -1, load, [&](int c, int slot) {
            float x[CPL];
#pragma unroll
            for (int jj = 0; jj < CPL; ++jj) x[jj] = pm[slot][jj] + lane_bperm(nv, LPRow * (CPL * q + jj));
            const float r = lse(x) + rl[slot];
            O += bs[slot] + (double)dprev;
            nv = r - dprev;
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
    double* Mx;     // [B][C][16][16]  M_c[r][s], -inf padded
    uint8_t* K;     // [B][C][16]      best entry tag for each exit tag
    int32_t* pin;   // [B][C]
    float* best_score;
    // Grouped runs (GS > 0; G = ceil(C / GS) groups a sequence): group_maxplus_kernel writes the
    // max-plus product of every group's chunk matrices to Mx2 ([B][G][16][16]); the boundary
    // kernel then handles one group per wave, between the tags pin_in ([B][G]) already fixed at
    // the last position of every group.
    int GS, G;
    double* Mx2;
    const int32_t* pin_in;
};

// A double of lane `K` of every aligned group of four lanes.
template <int K>
__device__ __forceinline__ double quad_read(double x) {
    const long long bits = __double_as_longlong(x);
    const int lo = dpp_i<K * 0x55>((int)(bits & 0xffffffffll)), hi = dpp_i<K * 0x55>((int)(bits >> 32));
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}

// Max-plus product of matrices first .. last (none: the identity) by one wave.  Lane
// (r = lane / 4, q = lane % 4) owns M[r][4q .. 4q+3]; row r of M is spread over the four lanes of a
// quad and is read from their registers, the entries X_i[s][4q .. 4q+3] of every matrix, which the
// sixteen lanes of column group q all need, go through LDS in the type XT they are stored in
// (potentials as floats: the conversion to double is repeated by every reader, half the LDS bytes
// are what eight such waves on a compute unit wait for).  get(slot, jj) returns this lane's four
// entries of a matrix.  One wave per workgroup: the barrier is only the wait for the LDS writes, and
// the two tile buffers keep the next matrix's writes off the tile that is being read.
template <int PF, typename Slot, typename XT, typename Load, typename Get>
__device__ __forceinline__ void maxplus_product(int first, int last, int T, double* __restrict__ out, Load load_slot,
                                                Get get, XT (*Xs)[16][16]) {
    const int lane = threadIdx.x, r = lane >> 2, q = lane & 3;
    const double ninf = -__builtin_huge_val();
    double M[4];
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) M[jj] = (r == 4 * q + jj) ? 0.0 : ninf;
    Slot ring[PF];
    auto load = [&](int i, int slot) { load_slot(i, ring[slot]); };
    int buf = 0;
    walk<PF>(first, last, +1, load, [&](int, int slot) {
        buf ^= 1;
        XT(*X)[16] = Xs[buf];
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) X[r][4 * q + jj] = get(ring[slot], jj);
        __syncthreads();
        double best[4] = {ninf, ninf, ninf, ninf};
        const auto row = [&](int s, double m) {
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) best[jj] = fmax(best[jj], m + (double)X[s][4 * q + jj]);
        };
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            row(jj, quad_read<0>(M[jj]));
            row(4 + jj, quad_read<1>(M[jj]));
            row(8 + jj, quad_read<2>(M[jj]));
            row(12 + jj, quad_read<3>(M[jj]));
        }
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) M[jj] = best[jj];
    });
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) out[r * 16 + 4 * q + jj] = (r < T && 4 * q + jj < T) ? M[jj] : ninf;
}

struct MaxSlotF { float x[4]; };
struct MaxSlotD { double x[4]; };

template <typename TIN>
__global__ __launch_bounds__(64) void chunk_maxplus_kernel(MaxScanArgs a) {
    __shared__ __attribute__((aligned(16))) float Xs[2][16][16];
    const int lane = threadIdx.x, r = lane >> 2, q = lane & 3;
    const int b = blockIdx.x / a.C, c = blockIdx.x % a.C;
    const int T = a.T, N = a.N;
    const int L = clamp_length(a.lengths, b, N);
    if (c * a.chunk >= L) return;
    int first, last;
    chunk_range(c, a.chunk, L, first, last);
    const size_t TT = (size_t)T * T;
    const TIN* phib = static_cast<const TIN*>(a.phi) + (size_t)b * N * TT;
    int off[4];
    bool in[4];
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
        const int t = 4 * q + jj;
        in[jj] = r < T && t < T;
        off[jj] = (r < T ? r : T - 1) * T + (t < T ? t : T - 1);
    }
    maxplus_product<kScanPF, MaxSlotF, float>(
        first, last, T, a.Mx + ((size_t)b * a.C + c) * 256,
        [&](int i, MaxSlotF& sl) {
            const TIN* m = phib + (size_t)i * TT;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) sl.x[jj] = Elem<TIN>::get(m + off[jj]);
        },
        [&](const MaxSlotF& sl, int jj) { return in[jj] ? sl.x[jj] : LCCRF_NEG_INF; }, Xs);
}

// One wave per group of GS chunks: the max-plus product of the group's chunk matrices.
__global__ __launch_bounds__(64) void group_maxplus_kernel(MaxScanArgs a) {
    __shared__ __attribute__((aligned(16))) double Xs[2][16][16];
    const int lane = threadIdx.x, r = lane >> 2, q = lane & 3;
    const int b = blockIdx.x / a.G, g = blockIdx.x % a.G;
    const int L = clamp_length(a.lengths, b, a.N);
    const int Cb = (L + a.chunk - 1) / a.chunk;
    const int c0 = g * a.GS;
    if (c0 >= Cb) return;
    const int c1 = (c0 + a.GS < Cb ? c0 + a.GS : Cb) - 1;
    const double* Mb = a.Mx + (size_t)b * a.C * 256 + r * 16 + 4 * q;
    maxplus_product<4, MaxSlotD, double>(
        c0, c1, a.T, a.Mx2 + ((size_t)b * a.G + g) * 256,
        [&](int c, MaxSlotD& sl) {
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) sl.x[jj] = Mb[(size_t)c * 256 + jj];
        },
        [&](const MaxSlotD& sl, int jj) { return sl.x[jj]; }, Xs);
}

constexpr int kPinWindow = 1024;  // chunks of back-pointers held in LDS at a time by the back-trace

// Phase B of the max-plus scan.  One wave per sequence (GS = 0) or per group of chunks (GS > 0):
// delta through the chunk matrices with the best entry tag per exit tag (K), then the back-trace
// over those chunks, which fixes the tag at the last position of every chunk (pin).  A whole
// sequence starts from delta_0 and ends in its best final tag; a group starts from the tag
// already fixed at the end of the group before it (group 0: delta_0) and ends in the tag fixed at
// its own end, so what it finds is a best path between those two tags.
template <typename TIN>
__global__ __launch_bounds__(64) void chunk_maxplus_boundary_kernel(MaxScanArgs a) {
    __shared__ uint8_t win[kPinWindow * 16];
    const int lane = threadIdx.x, t = lane >> 2, q = lane & 3;
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
        dv = (t < T) ? (double)Elem<TIN>::get(phib + t) : ninf;  // delta_0
    } else {
        dv = (t == a.pin_in[bg + g - 1]) ? 0.0 : ninf;  // the tag fixed at the end of the group before
    }
    double mm[kScanPF][4];
    auto load = [&](int c, int slot) {
        const double* M = a.Mx + (cb + c) * 256;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) mm[slot][jj] = M[(4 * q + jj) * 16 + t];
    };
    walk<kScanPF>(c0, c1, +1, load, [&](int c, int slot) {
        double bv = ninf;
        int ba = 0x7fffffff;
        double in[4];
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) in[jj] = __shfl(dv, 16 * q + 4 * jj, 64);
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {  // ascending entry tags: the first maximum wins
            const double val = in[jj] + mm[slot][jj];
            if (val > bv) { bv = val; ba = 4 * q + jj; }
        }
#pragma unroll
        for (int off = 1; off < 4; off <<= 1) {
            const double pv = __shfl_xor(bv, off, 64);
            const int pa = __shfl_xor(ba, off, 64);
            if (pv > bv || (pv == bv && pa < ba)) { bv = pv; ba = pa; }
        }
        dv = bv;
        if (q == 0) a.K[(cb + c) * 16 + t] = (uint8_t)(ba == 0x7fffffff ? 0 : ba);
    });
    int y;
    if (!grouped) {
        // best tag at the last position: first maximum (entry t sits in lanes 4t .. 4t+3)
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
        const int nbytes = (hi - lo) * 16;
        const uint8_t* src = a.K + (cb + lo) * 16;
        for (int k = lane; k < nbytes; k += 64) win[k] = src[k];
        __syncthreads();
        if (lane == 0) {
            for (int c = hi - 1; c >= lo; --c) {
                y = win[(c - lo) * 16 + y];
                a.pin[cb + c - 1] = y;
            }
        }
        __syncthreads();
        hi = lo;
    }
}

// ---------------------------------------------------------------------------------------
// Sum queries: tag sets up to 32 (matrices in one or four 16 x 16 blocks); the max-plus scan: up to 16.
bool scan_supported(int T) { return T >= 1 && T <= 32; }
bool scan_supported_max(int T) { return T >= 1 && T <= 16; }
int scan_padded_tags(int T) { return T <= 16 ? 16 : 32; }

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
    hipLaunchKernelGGL((chunk_product_kernel<TIN, TP>), dim3(a.B * a.C), dim3(64), 0, st, a);
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
    hipLaunchKernelGGL(group_product_kernel<TP>, dim3(a.B * G), dim3(64), 0, st, p);
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
                                  double* logZ64) {
    const int C = (N + chunk - 1) / chunk;
    ScanArgs a{phi, lengths, B, N, T, chunk, C, Pl, rel, base, Fv, OF, Gv, OG, logZ, with_beta ? 1 : 0, logZ64,
               0, 1, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
    if (T <= 16)
        return dtype == 0 ? launch_scan_boundaries_t<float, 16>(a, gb, st) : launch_scan_boundaries_t<uint16_t, 16>(a, gb, st);
    return dtype == 0 ? launch_scan_boundaries_t<float, 32>(a, gb, st) : launch_scan_boundaries_t<uint16_t, 32>(a, gb, st);
}


template <typename TIN>
static hipError_t launch_scan_pins_t(MaxScanArgs a, const MaxGroupBuffers& gb, hipStream_t st) {
    hipLaunchKernelGGL(chunk_maxplus_kernel<TIN>, dim3(a.B * a.C), dim3(64), 0, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int gs = scan_group_size(a.C);
    if (gs == 0) {
        hipLaunchKernelGGL(chunk_maxplus_boundary_kernel<TIN>, dim3(a.B), dim3(64), 0, st, a);
        return hipGetLastError();
    }
    const int G = (a.C + gs - 1) / gs;
    MaxScanArgs p = a;
    p.GS = gs; p.G = G; p.Mx2 = gb.Mx2;
    hipLaunchKernelGGL(group_maxplus_kernel, dim3(a.B * G), dim3(64), 0, st, p);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    // phase B over the groups: the same kernel, a group in the place of a chunk (best score, tags at group ends)
    MaxScanArgs u = a;
    u.chunk = a.chunk * gs; u.C = G; u.Mx = gb.Mx2; u.K = gb.K2; u.pin = gb.pin2;
    hipLaunchKernelGGL(chunk_maxplus_boundary_kernel<TIN>, dim3(a.B), dim3(64), 0, st, u);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    // ... and inside every group at once, between the tags just fixed
    MaxScanArgs l = a;
    l.GS = gs; l.G = G; l.best_score = nullptr; l.pin_in = gb.pin2;
    hipLaunchKernelGGL(chunk_maxplus_boundary_kernel<TIN>, dim3(a.B * G), dim3(64), 0, st, l);
    return hipGetLastError();
}

hipError_t launch_scan_pins(int dtype, const void* phi, const int32_t* lengths, int B, int N, int T, int chunk,
                            double* Mx, uint8_t* K, int32_t* pin, const MaxGroupBuffers& gb, float* best_score,
                            hipStream_t st) {
    const int C = (N + chunk - 1) / chunk;
    MaxScanArgs a{phi, lengths, B, N, T, chunk, C, Mx, K, pin, best_score, 0, 1, nullptr, nullptr};
    return dtype == 0 ? launch_scan_pins_t<float>(a, gb, st) : launch_scan_pins_t<uint16_t>(a, gb, st);
}

}  // namespace lccrf
