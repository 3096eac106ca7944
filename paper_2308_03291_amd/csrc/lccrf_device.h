// Device-side building blocks shared by the linear-chain CRF kernels (gfx950 only).
//
// Thread mapping used by every chain kernel.  One T x T matrix phi_i (row s = previous
// tag, column t = current tag, t contiguous in memory) is spread over a workgroup of
// W = 64 * WAVES threads as follows: LPR consecutive lanes cover one row, each lane owning
// four consecutive columns (t = 4c .. 4c+3, c = tid % LPR); the W / LPR row groups cover
// rows r0, r0 + RPP, r0 + 2 RPP, ... (r0 = tid / LPR, RPP = W / LPR), ITEMS rows per
// thread.  A wave therefore reads whole, contiguous rows: every global load is coalesced,
// and 16 bytes wide: aligned when T is a multiple of 4, from wherever the piece starts otherwise
// (load_row4_anywhere).
//
//   reduction over s (forward recursion): in-thread over ITEMS rows, then across the
//       64 / LPR row groups of a wave by lane exchange, then across waves through LDS;
//   reduction over t (backward recursion): in-thread over 4 columns, then across the LPR
//       lanes of the row by lane exchange; never leaves the wave.
//
// All recursions run in base-2 logarithms: x2 = x * log2(e), so that the hardware
// v_exp_f32 / v_log_f32 (base 2) are used directly and the multiply folds into one fma.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lccrf {

constexpr float kLog2e = 1.44269504088896340736f;
constexpr double kLn2 = 0.69314718055994530942;
#define LCCRF_NEG_INF (-__builtin_huge_valf())

__device__ __forceinline__ float ex2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float lg2(float x) { return __builtin_amdgcn_logf(x); }

__device__ __forceinline__ float bf16_to_f32(uint16_t h) {
    return __uint_as_float(static_cast<uint32_t>(h) << 16);
}

typedef float vec4f __attribute__((ext_vector_type(4)));
typedef unsigned int vec2u __attribute__((ext_vector_type(2)));
// The same vectors at an address that is aligned like a single element only (rows of a matrix whose tag count is no
// multiple of four): types that promise the compiler no more than that.  (Vector types, not structs of four members:
// a struct's load is taken apart into its members early, and does not always come together again.)
typedef vec4f vec4f_anywhere __attribute__((aligned(4)));
typedef vec2u vec2u_anywhere __attribute__((aligned(2)));
__device__ __forceinline__ void stream_store4(float* p, float a0, float a1, float a2, float a3) {
    __builtin_nontemporal_store(vec4f{a0, a1, a2, a3}, reinterpret_cast<vec4f*>(p));
}

__device__ __forceinline__ void store4_anywhere(float* p, float a0, float a1, float a2, float a3) {
    *reinterpret_cast<vec4f_anywhere*>(p) = vec4f{a0, a1, a2, a3};
}

template <typename TIN> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float get(const float* p) { return *p; }
    static __device__ __forceinline__ void get4_anywhere(const float* p, float (&o)[4]) {
        const vec4f v = *reinterpret_cast<const vec4f_anywhere*>(p);
        o[0] = v[0]; o[1] = v[1]; o[2] = v[2]; o[3] = v[3];
    }
    static __device__ __forceinline__ void get4(const float* p, float (&o)[4]) {
        const float4 v = *reinterpret_cast<const float4*>(p);
        o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
    }
    // The same with the non-temporal hint, for kernels whose batches do not fit the caches anyway
    // (T > 64): potentials are read once per pass and marginals written once.  Measured on config 4:
    // second pass 0.915 -> 0.867 ms, first pass 0.44 -> 0.43 ms; on cache-sized batches (T <= 64
    // shapes) it costs 5-10 %, so the small-T kernels keep ordinary loads and stores.
    static __device__ __forceinline__ void get4_stream(const float* p, float (&o)[4]) {
        const vec4f v = __builtin_nontemporal_load(reinterpret_cast<const vec4f*>(p));
        o[0] = v[0]; o[1] = v[1]; o[2] = v[2]; o[3] = v[3];
    }
};
template <> struct Elem<uint16_t> {
    static __device__ __forceinline__ float get(const uint16_t* p) { return bf16_to_f32(*p); }
    static __device__ __forceinline__ void get4_anywhere(const uint16_t* p, float (&o)[4]) {
        const vec2u v = *reinterpret_cast<const vec2u_anywhere*>(p);
        o[0] = __uint_as_float(v[0] << 16);
        o[1] = __uint_as_float(v[0] & 0xffff0000u);
        o[2] = __uint_as_float(v[1] << 16);
        o[3] = __uint_as_float(v[1] & 0xffff0000u);
    }
    static __device__ __forceinline__ void get4(const uint16_t* p, float (&o)[4]) {
        const uint2 v = *reinterpret_cast<const uint2*>(p);
        o[0] = __uint_as_float(v.x << 16);
        o[1] = __uint_as_float(v.x & 0xffff0000u);
        o[2] = __uint_as_float(v.y << 16);
        o[3] = __uint_as_float(v.y & 0xffff0000u);
    }
    static __device__ __forceinline__ void get4_stream(const uint16_t* p, float (&o)[4]) {
        const vec2u v = __builtin_nontemporal_load(reinterpret_cast<const vec2u*>(p));
        o[0] = __uint_as_float(v[0] << 16);
        o[1] = __uint_as_float(v[0] & 0xffff0000u);
        o[2] = __uint_as_float(v[1] << 16);
        o[3] = __uint_as_float(v[1] & 0xffff0000u);
    }
};

// Geometry of one instantiation.
template <int LPR_, int WAVES_, int ITEMS_>
struct Geo {
    static constexpr int LPR = LPR_;        // lanes per row (power of two, <= 64)
    static constexpr int WAVES = WAVES_;
    static constexpr int ITEMS = ITEMS_;    // rows per thread
    static constexpr int W = 64 * WAVES_;   // threads per workgroup
    static constexpr int RPP = W / LPR_;    // rows covered by one pass of the workgroup
    static constexpr int TCAP = 4 * LPR_;   // largest T this geometry covers
    static constexpr int RGW = 64 / LPR_;   // row groups per wave
    static constexpr int COLWAVES = (TCAP + 63) / 64;  // waves holding one thread per column
    static_assert(RPP * ITEMS_ >= TCAP || RPP * ITEMS_ >= 1, "rows not covered");
};

// Columns c4 .. c4 + 3 of row s of a T x T matrix whose rows lie anywhere an element may (T no multiple of four).
// A thread whose row or columns lie outside the matrix takes the last row, or the columns from 0 on, instead.  The
// four elements come as one load wherever four elements follow in the matrix: those past the end of the row are then
// the first of the next row.  Only the piece that ends the matrix (the last columns of the last row) is loaded element
// by element, and that only if nothing follows the matrix in memory (FOLLOWED says that something does: another
// matrix of the tensor, of two tags or more, so that the three elements a load may run over are there; then the
// load is the same instruction in every thread, with no branch around it).
// settle_row4() makes of what was loaded the piece every consumer may rely on; nothing here touches the loaded
// values, so the loads stay in flight.
template <typename TIN, bool FOLLOWED>
__device__ __forceinline__ void load_row4_anywhere(const TIN* __restrict__ mat, int T, int s, int c4, float (&o)[4]) {
    const int cc = c4 < T ? c4 : 0;
    const int off = (s < T ? s : T - 1) * T + cc;
    if (FOLLOWED || off + 4 <= T * T) {
        Elem<TIN>::get4_anywhere(mat + off, o);
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) o[j] = Elem<TIN>::get(mat + off + (cc + j < T ? j : 0));
    }
}
// The entries of such a piece that lie past the end of the row become copies of its first entry: data of the row
// itself, which the thread works on anyway.
__device__ __forceinline__ void settle_row4(float (&o)[4], int T, int c4) {
    const int cc = c4 < T ? c4 : 0;
#pragma unroll
    for (int j = 1; j < 4; ++j) o[j] = cc + j < T ? o[j] : o[0];
}

// Issue the loads of this thread's part of one matrix.  Addresses are clamped into the
// matrix, so every lane issues the same loads with no branch around them, and nothing here
// touches the loaded values: the loads stay in flight until the tile is consumed.  There settle_tile()
// comes first (it does nothing when the tag count is a multiple of four), then whatever the kernel does
// about the entries outside the matrix (mask_tile(), or weights that drop them).
template <typename G, typename TIN, bool ALIGNED>
__device__ __forceinline__ void load_tile(const TIN* __restrict__ mat, int T, int c4, int r0,
                                          float (&v)[G::ITEMS][4], bool followed = false) {
    if (ALIGNED) {
#pragma unroll
        for (int k = 0; k < G::ITEMS; ++k) {
            const int s = r0 + k * G::RPP;
            const TIN* row = mat + (size_t)(s < T ? s : T - 1) * T;
            if (G::TCAP > 64) Elem<TIN>::get4_stream(row + (c4 < T ? c4 : T - 4), v[k]);  // T % 4 == 0 here, so T >= 4
            else Elem<TIN>::get4(row + (c4 < T ? c4 : T - 4), v[k]);
        }
    } else if (followed && T > 1) {  // (the same for the whole workgroup: one scalar branch)
#pragma unroll
        for (int k = 0; k < G::ITEMS; ++k) load_row4_anywhere<TIN, true>(mat, T, r0 + k * G::RPP, c4, v[k]);
    } else {
#pragma unroll
        for (int k = 0; k < G::ITEMS; ++k) load_row4_anywhere<TIN, false>(mat, T, r0 + k * G::RPP, c4, v[k]);
    }
}
template <typename G, bool ALIGNED>
__device__ __forceinline__ void settle_tile(float (&v)[G::ITEMS][4], int T, int c4) {
    if constexpr (!ALIGNED) {
#pragma unroll
        for (int k = 0; k < G::ITEMS; ++k) settle_row4(v[k], T, c4);
    }
}

// Structured potentials phi[i][s][t] = trans[s][t] + emit[i][t] (the usual tagging parameterisation;
// the dense layout of the paper's linear-chain CRF with the per-position part factored out): the
// transition tile stays in registers (loaded once with load_tile / wave_load), a position brings
// only its T emission scores.  load_emit4 puts this thread's four columns into row 0 of the slot;
// add_trans then turns the slot into the tile of that position.
// (T no multiple of four: the columns a settled tile of the transition matrix holds, see load_row4_anywhere; as one
// load if another row of emission scores follows this one in memory (`followed`, the same for the whole workgroup),
// what it brings in from that row being replaced by settle_row4() before add_trans; element by element otherwise.)
template <bool ALIGNED>
__device__ __forceinline__ void load_emit4(const float* __restrict__ emit_row, int T, int c4, float (&o)[4], bool followed = false) {
    if (ALIGNED) {
        Elem<float>::get4(emit_row + (c4 < T ? c4 : T - 4), o);
    } else if (followed && T >= 4) {
        Elem<float>::get4_anywhere(emit_row + (c4 < T ? c4 : 0), o);
    } else {
        const int cc = c4 < T ? c4 : 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) o[j] = emit_row[cc + j < T ? cc + j : cc];
    }
}
template <bool ALIGNED>
__device__ __forceinline__ void settle_emit4(float (&o)[4], int T, int c4) {
    if constexpr (!ALIGNED) settle_row4(o, T, c4);
}
template <int ROWS>
__device__ __forceinline__ void add_trans(float (&v)[ROWS][4], const float (&tr)[ROWS][4]) {
    const float em[4] = {v[0][0], v[0][1], v[0][2], v[0][3]};
#pragma unroll
    for (int k = 0; k < ROWS; ++k)
#pragma unroll
        for (int j = 0; j < 4; ++j) v[k][j] = tr[k][j] + em[j];
}

// Replace the entries of a loaded tile that lie outside the T x T matrix by -inf, the
// neutral element of both max and log-sum-exp.
template <typename G>
__device__ __forceinline__ void mask_tile(float (&v)[G::ITEMS][4], int T, int c4, int r0) {
#pragma unroll
    for (int k = 0; k < G::ITEMS; ++k) {
        const bool row_ok = r0 + k * G::RPP < T;
#pragma unroll
        for (int j = 0; j < 4; ++j) v[k][j] = (row_ok && c4 + j < T) ? v[k][j] : LCCRF_NEG_INF;
    }
}

// Store this thread's part of one matrix of marginals.
template <typename G, bool ALIGNED>
__device__ __forceinline__ void store_tile(float* __restrict__ mat, int T, int c4, int r0,
                                           const float (&v)[G::ITEMS][4]) {
#pragma unroll
    for (int k = 0; k < G::ITEMS; ++k) {
        const int s = r0 + k * G::RPP;
        if (s < T && c4 < T) {
            float* p = mat + (size_t)s * T + c4;
            if (ALIGNED) {
                *reinterpret_cast<float4*>(p) = make_float4(v[k][0], v[k][1], v[k][2], v[k][3]);
            } else if (c4 + 4 <= T) {
                store4_anywhere(p, v[k][0], v[k][1], v[k][2], v[k][3]);
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (c4 + j < T) p[j] = v[k][j];
            }
        }
    }
}

// Cross-lane moves on the DPP path (no LDS).  Written with a zero `old` value and bound_ctrl set,
// the form the compiler can fold into the consuming add or max (v_add_f32_dpp) instead of a copy,
// a hazard nop and a separate move.
// A translation unit may define LCCRF_LANE_EXCHANGE_CLASSIC before including this header to get
// the plain forms instead (a move with its own register and the LDS swizzle at distance 4).
#ifdef LCCRF_LANE_EXCHANGE_CLASSIC
constexpr bool kNoMirror = true;
#else
constexpr bool kNoMirror = false;
#endif
constexpr int kDppQuadXor1 = 0xB1;     // quad_perm [1,0,3,2]
constexpr int kDppQuadXor2 = 0x4E;     // quad_perm [2,3,0,1]
constexpr int kDppRowRor4 = 0x124;     // rotate right by 4 within a row of 16 lanes
constexpr int kDppRowRor8 = 0x128;
constexpr int kDppHalfMirror = 0x141;  // lane i <-> 7 - i within each group of 8 lanes
template <int CTRL>
__device__ __forceinline__ float dpp(float x) {
#ifdef LCCRF_LANE_EXCHANGE_CLASSIC
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(x), __float_as_int(x), CTRL, 0xF, 0xF, false));
#else
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true));
#endif
}
template <int CTRL>
__device__ __forceinline__ int dpp_i(int x) { return __builtin_amdgcn_update_dpp(0, x, CTRL, 0xF, 0xF, true); }

// Value held by lane (id ^ OFF) of the same wave, without touching LDS memory where the
// hardware offers a cross-lane path: DPP quad permutes and row rotates inside a row of 16
// lanes, the LDS crossbar swizzle for a distance of 4, and the gfx950 permlane swaps
// between rows of 16 and between the two halves of the wave.
template <int OFF>
__device__ __forceinline__ int lane_xor_i(int x) {
    static_assert(OFF == 1 || OFF == 2 || OFF == 4 || OFF == 8 || OFF == 16 || OFF == 32, "power of two < 64");
    if (OFF == 1) return dpp_i<kDppQuadXor1>(x);
    if (OFF == 2) return dpp_i<kDppQuadXor2>(x);
    if (OFF == 4) return __builtin_amdgcn_ds_swizzle(x, 0x101F);                     // bit mode, xor 4
    if (OFF == 8) return dpp_i<kDppRowRor8>(x);
    const int lane = __lane_id();
    if (OFF == 16) {
        const auto r = __builtin_amdgcn_permlane16_swap(x, x, false, false);
        return (lane & 16) ? (int)r[0] : (int)r[1];
    }
    const auto r = __builtin_amdgcn_permlane32_swap(x, x, false, false);
    return (lane & 32) ? (int)r[0] : (int)r[1];
}
template <int OFF>
__device__ __forceinline__ float lane_xor(float x) { return __int_as_float(lane_xor_i<OFF>(__float_as_int(x))); }
template <int OFF>
__device__ __forceinline__ double lane_xor(double x) {
    const long long b = __double_as_longlong(x);
    const int lo = lane_xor_i<OFF>((int)(b & 0xffffffffll)), hi = lane_xor_i<OFF>((int)(b >> 32));
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}

// Maxima as the bare instructions.  In front of a max whose operand comes from memory or from another lane the
// compiler puts a canonicalising copy of that operand (it cannot rule out a signalling NaN), which also keeps the
// cross-lane move from folding into the max: three instructions where one does.  NaN operands are ignored in favour
// of the others, as by fmaxf.  The DPP form waits out the two states a vector result needs before a DPP read.
__device__ __forceinline__ float max3_raw(float a, float b, float c) {
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
template <int CTRL>
__device__ __forceinline__ float max_with_dpp(float x) {  // max(x, value of the lane CTRL names); all lanes active
    float r;
    static_assert(CTRL == kDppQuadXor1 || CTRL == kDppQuadXor2 || CTRL == kDppHalfMirror || CTRL == kDppRowRor4 ||
                      CTRL == kDppRowRor8, "one of the lane patterns above");
    if constexpr (CTRL == kDppQuadXor1)
        asm("s_nop 1\n\tv_max_f32_dpp %0, %1, %1 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf" : "=v"(r) : "v"(x));
    else if constexpr (CTRL == kDppQuadXor2)
        asm("s_nop 1\n\tv_max_f32_dpp %0, %1, %1 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf" : "=v"(r) : "v"(x));
    else if constexpr (CTRL == kDppHalfMirror)
        asm("s_nop 1\n\tv_max_f32_dpp %0, %1, %1 row_half_mirror row_mask:0xf bank_mask:0xf" : "=v"(r) : "v"(x));
    else if constexpr (CTRL == kDppRowRor4)
        asm("s_nop 1\n\tv_max_f32_dpp %0, %1, %1 row_ror:4 row_mask:0xf bank_mask:0xf" : "=v"(r) : "v"(x));
    else
        asm("s_nop 1\n\tv_max_f32_dpp %0, %1, %1 row_ror:8 row_mask:0xf bank_mask:0xf" : "=v"(r) : "v"(x));
    return r;
}

// All-reduce over the lanes of a wave whose ids differ only in the bits [LO, HI) (LO, HI
// powers of two, LO >= HI means a single lane: nothing to do).  Every lane of a group ends
// with the bit-identical result (both partners of an exchange add the same two numbers).
// Once the four lanes of every quad hold the same value (LO = 1), the partner at distance 4 is
// reached by mirroring the group of 8 lanes (lane i takes 7 - i, which sits in the other quad
// and holds that quad's value): a DPP move instead of a trip through the LDS crossbar.
template <int LO, int HI>
__device__ __forceinline__ float xor_max(float x) {
#ifdef LCCRF_LANE_EXCHANGE_CLASSIC
    if (LO <= 1 && 1 < HI) x = fmaxf(x, dpp<kDppQuadXor1>(x));
    if (LO <= 2 && 2 < HI) x = fmaxf(x, dpp<kDppQuadXor2>(x));
    if (LO <= 4 && 4 < HI) x = fmaxf(x, lane_xor<4>(x));
    if (LO <= 8 && 8 < HI) x = fmaxf(x, dpp<kDppRowRor8>(x));
#else
    if (LO <= 1 && 1 < HI) x = max_with_dpp<kDppQuadXor1>(x);
    if (LO <= 2 && 2 < HI) x = max_with_dpp<kDppQuadXor2>(x);
    if (LO <= 4 && 4 < HI) x = (LO <= 1) ? max_with_dpp<kDppHalfMirror>(x) : fmaxf(x, lane_xor<4>(x));
    if (LO <= 8 && 8 < HI) x = max_with_dpp<kDppRowRor8>(x);
#endif
    if (LO <= 16 && 16 < HI) {  // both halves of the swapped pair: no select needed for a symmetric op
        const auto r = __builtin_amdgcn_permlane16_swap(__float_as_int(x), __float_as_int(x), false, false);
        x = max3_raw(__int_as_float(r[0]), __int_as_float(r[1]), __int_as_float(r[1]));
    }
    if (LO <= 32 && 32 < HI) {
        const auto r = __builtin_amdgcn_permlane32_swap(__float_as_int(x), __float_as_int(x), false, false);
        x = max3_raw(__int_as_float(r[0]), __int_as_float(r[1]), __int_as_float(r[1]));
    }
    return x;
}
template <int LO, int HI>
__device__ __forceinline__ float xor_sum(float x) {
    if (LO <= 1 && 1 < HI) x += dpp<kDppQuadXor1>(x);
    if (LO <= 2 && 2 < HI) x += dpp<kDppQuadXor2>(x);
    if (LO <= 4 && 4 < HI) x += (LO <= 1 && !kNoMirror) ? dpp<kDppHalfMirror>(x) : lane_xor<4>(x);
    if (LO <= 8 && 8 < HI) x += dpp<kDppRowRor8>(x);
    if (LO <= 16 && 16 < HI) {
        const auto r = __builtin_amdgcn_permlane16_swap(__float_as_int(x), __float_as_int(x), false, false);
        x = __int_as_float(r[0]) + __int_as_float(r[1]);
    }
    if (LO <= 32 && 32 < HI) {
        const auto r = __builtin_amdgcn_permlane32_swap(__float_as_int(x), __float_as_int(x), false, false);
        x = __int_as_float(r[0]) + __int_as_float(r[1]);
    }
    return x;
}

// Sums of four values per lane (S0..S3, e.g. the partial sums of four matrix rows) over the LPR
// lanes of a group (LPR = 16, 32 or 64 consecutive lanes), at a third of the exchanges four
// separate all-reduces would take: the first two levels halve the number of values a lane
// carries instead of doubling the copies.  Every lane returns the complete sum of value number
// 2 * (lane & 1) + ((lane >> 1) & 1).  Lanes of one group that own the same value may differ in
// the last bit (they add in different orders); each caller lets one lane per value publish it.
template <int LPR>
__device__ __forceinline__ float reduce4_over_lanes(float S0, float S1, float S2, float S3, int lane) {
    static_assert(LPR == 16 || LPR == 32 || LPR == 64, "a row spans 16, 32 or 64 lanes");
    const bool b0 = (lane & 1) != 0, b1 = (lane & 2) != 0;
    const float keepA = (b0 ? S2 : S0) + dpp<kDppQuadXor1>(b0 ? S0 : S2);
    const float keepB = (b0 ? S3 : S1) + dpp<kDppQuadXor1>(b0 ? S1 : S3);
    float x = (b1 ? keepB : keepA) + dpp<kDppQuadXor2>(b1 ? keepA : keepB);
    x += dpp<kDppRowRor4>(x);
    x += dpp<kDppRowRor8>(x);
    if (LPR >= 32) {
        const auto r = __builtin_amdgcn_permlane16_swap(__float_as_int(x), __float_as_int(x), false, false);
        x = __int_as_float(r[0]) + __int_as_float(r[1]);
    }
    if (LPR >= 64) {
        const auto r = __builtin_amdgcn_permlane32_swap(__float_as_int(x), __float_as_int(x), false, false);
        x = __int_as_float(r[0]) + __int_as_float(r[1]);
    }
    return x;
}

// LDS layout of a tile that is written row by row and read back column-block by column-block
// (forward chains at 64 < T <= 128): two buffers of 128 rows.
constexpr int kTurnStride = 132;  // floats per LDS row: 128 + 4 keeps 16-byte accesses conflict free
constexpr int kTurnFloats = 2 * 128 * kTurnStride;

// A candidate of a max-plus step: its score and the tag it comes from.  Ties go to the smaller tag,
// which makes `better` commutative and associative: any reduction order gives the same winner.
struct Best {
    double v;
    int a;
};
__device__ __forceinline__ Best better(Best x, Best y) {
    const bool take_y = y.v > x.v || (y.v == x.v && y.a < x.a);
    return take_y ? y : x;
}
template <int CTRL>
__device__ __forceinline__ Best dpp_best(Best x) {
    const long long b = __double_as_longlong(x.v);
    const int lo = dpp_i<CTRL>((int)(b & 0xffffffffll)), hi = dpp_i<CTRL>((int)(b >> 32));
    return Best{__longlong_as_double(((long long)hi << 32) | (unsigned int)lo), dpp_i<CTRL>(x.a)};
}
// The better of this lane's candidate and that of the lane 16 (W = 16) or 32 (W = 32) away.
template <int W>
__device__ __forceinline__ Best swap_best(Best x) {
    const long long b = __double_as_longlong(x.v);
    const int lo = (int)(b & 0xffffffffll), hi = (int)(b >> 32);
    if (W == 16) {
        const auto rl = __builtin_amdgcn_permlane16_swap(lo, lo, false, false);
        const auto rh = __builtin_amdgcn_permlane16_swap(hi, hi, false, false);
        const auto ra = __builtin_amdgcn_permlane16_swap(x.a, x.a, false, false);
        return better(Best{__longlong_as_double(((long long)(int)rh[0] << 32) | (unsigned int)rl[0]), (int)ra[0]},
                      Best{__longlong_as_double(((long long)(int)rh[1] << 32) | (unsigned int)rl[1]), (int)ra[1]});
    }
    const auto rl = __builtin_amdgcn_permlane32_swap(lo, lo, false, false);
    const auto rh = __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
    const auto ra = __builtin_amdgcn_permlane32_swap(x.a, x.a, false, false);
    return better(Best{__longlong_as_double(((long long)(int)rh[0] << 32) | (unsigned int)rl[0]), (int)ra[0]},
                  Best{__longlong_as_double(((long long)(int)rh[1] << 32) | (unsigned int)rl[1]), (int)ra[1]});
}
// reduce4_over_lanes for candidates: the best of b0..b3 (four rows or columns per lane) over the
// LPR lanes of a group; every lane returns the winner of number 2 * (lane & 1) + ((lane >> 1) & 1).
template <int LPR>
__device__ __forceinline__ Best reduce4_best_over_lanes(Best b0, Best b1, Best b2, Best b3, int lane) {
    static_assert(LPR == 16 || LPR == 32 || LPR == 64, "a group spans 16, 32 or 64 lanes");
    const bool o0 = (lane & 1) != 0, o1 = (lane & 2) != 0;
    const Best keepA = better(o0 ? b2 : b0, dpp_best<kDppQuadXor1>(o0 ? b0 : b2));
    const Best keepB = better(o0 ? b3 : b1, dpp_best<kDppQuadXor1>(o0 ? b1 : b3));
    Best x = better(o1 ? keepB : keepA, dpp_best<kDppQuadXor2>(o1 ? keepA : keepB));
    x = better(x, dpp_best<kDppRowRor4>(x));
    x = better(x, dpp_best<kDppRowRor8>(x));
    if (LPR >= 32) x = swap_best<16>(x);
    if (LPR >= 64) x = swap_best<32>(x);
    return x;
}

// Walks positions first, first+dir, ..., last (dir = +1 or -1) with a ring of PF tiles:
// `load(i, slot)` issues the loads of position i into ring slot `slot`; `step(i, slot)`
// consumes the slot, which is refilled with the tile PF positions ahead right after.
//
// Every refill is issued unconditionally (past the end of the walk the last position is
// simply loaded again and never used).  That costs PF redundant tile loads per chain and buys
// a loop in which the number of loads issued after any tile is the same on every path, which
// is what lets the compiler wait for exactly the oldest tile (s_waitcnt vmcnt(n) with n > 0)
// and keep the PF - 1 younger ones in flight.
template <int PF, typename Load, typename Step>
__device__ __forceinline__ void walk(int first, int last, int dir, Load load, Step step) {
    const int n = (last - first) * dir + 1;  // number of positions (<= 0: nothing to do)
    if (n <= 0) return;
#pragma unroll
    for (int p = 0; p < PF; ++p) load(first + (p < n ? p : n - 1) * dir, p);
    int done = 0;
    while (true) {
#pragma unroll
        for (int p = 0; p < PF; ++p) {
            const int i = first + done * dir;
            step(i, p);
            const int ahead = done + PF;
            load(first + (ahead < n ? ahead : n - 1) * dir, p);
            if (++done >= n) return;
        }
    }
}

// The same walk for a step that may give up: it returns false to end the walk at once (loads
// already issued for later positions land in ring slots nobody reads any more).
template <int PF, typename Load, typename Step>
__device__ __forceinline__ void walk_while(int first, int last, int dir, Load load, Step step) {
    const int n = (last - first) * dir + 1;
    if (n <= 0) return;
#pragma unroll
    for (int p = 0; p < PF; ++p) load(first + (p < n ? p : n - 1) * dir, p);
    int done = 0;
    while (true) {
#pragma unroll
        for (int p = 0; p < PF; ++p) {
            if (!step(first + done * dir, p)) return;
            const int ahead = done + PF;
            load(first + (ahead < n ? ahead : n - 1) * dir, p);
            if (++done >= n) return;
        }
    }
}

constexpr float kSumLo = 0x1p-60f, kSumHi = 0x1p60f;  // accepted range of a speculative sum
__device__ __forceinline__ bool sum_in_range(float S) { return S >= kSumLo && S <= kSumHi; }  // false for NaN

// Store 4 consecutive marginals of row s (columns c4 .. c4+3), only those inside the matrix.
// STREAM: with the non-temporal hint (see Elem::get4_stream).
template <bool ALIGNED, bool STREAM = false>
__device__ __forceinline__ void store4(float* __restrict__ mu_out, int T, int s, int c4,
                                       float a0, float a1, float a2, float a3) {
    if (s < T && c4 < T) {
        float* p = mu_out + (size_t)s * T + c4;
        if (ALIGNED) {
            if (STREAM) stream_store4(p, a0, a1, a2, a3);
            else *reinterpret_cast<float4*>(p) = make_float4(a0, a1, a2, a3);
        } else if (c4 + 4 <= T) {
            store4_anywhere(p, a0, a1, a2, a3);
        } else {  // the piece that ends the row holds T % 4 columns: the same count in every thread that gets here
            const int nv = T & 3;
            p[0] = a0;
            if (nv > 1) p[1] = a1;
            if (nv > 2) p[2] = a2;
        }
    }
}

// Pieces of the conditional-entropy recursion: with e = 2^arg the shifted exponentials of a step,
// S = sum e and U = sum e (h - arg), the new entropy is U / S + log2 S (0 for an unreachable tag).
__device__ __forceinline__ float log2_term(float arg) { return fmaxf(arg, -200.f); }  // 2^arg is 0 below: keeps 0 * inf away
__device__ __forceinline__ float entropy_of(float U, float S) { return S > 0.f ? U * __builtin_amdgcn_rcpf(S) + __builtin_amdgcn_logf(S) : 0.f; }

__device__ __forceinline__ float finite_or_zero(float m) { return (m == LCCRF_NEG_INF) ? 0.0f : m; }

__device__ __forceinline__ int clamp_length(const int32_t* __restrict__ lengths, int b, int N) {
    int L = lengths ? lengths[b] : N;
    L = L < 0 ? 0 : L;
    return L > N ? N : L;
}

}  // namespace lccrf
