// Max-plus (Viterbi) chains for the linear-chain CRF: the recursion of the forward
// algorithm with (max, +) in place of (logsumexp, +), as the paper's section "Computing
// Most Probable Structure" prescribes, followed by the trace that reads off the path.
//
// Like the sum-product chains, every sequence (or every chunk of the scan) is served by two
// chains that meet in the middle, at half the serial depth:
//
//   forward  workgroup: delta_i(t) = max_s delta_{i-1}(s) + phi_i(s,t) for i <= h, with the
//       back-pointer bp_i(t) = the best s;
//   backward workgroup: eps_{i-1}(s) = max_t phi_i(s,t) + eps_i(t) for i > h, with the
//       forward pointer fp_i(s) = the best t (stored in the same table, rows i > h);
//   trace (viterbi_trace_kernel): y_h = argmax_t delta_h(t) + eps_h(t), then y_{i-1} = bp_i(y_i)
//       down to the first position and y_i = fp_i(y_{i-1}) up to the last, by two threads.
//
// Scores are carried in double precision and never rescaled: max-plus needs only additions and
// comparisons, both at the full vector rate in fp64 on this chip, and every candidate is then one
// correctly rounded fp64 addition of exactly representable inputs, whichever thread forms it.
// Ties go to the smaller tag.
#include "lccrf_chain_args.h"
#include "lccrf_device.h"
#include "lccrf_launch.h"
#include "lccrf_viterbi_args.h"

namespace lccrf {

constexpr int kTraceBytes = 8192;  // LDS window of pointers walked by each direction of a trace

// Forward chains at 64 < T <= 128 turn their tiles through LDS like the sum-product
// first pass does (lccrf_chain.hip): a wave then owns 8 complete columns and the maximum over
// rows never leaves it, so the per-wave candidates below are not needed.
template <typename G, bool ALIGNED>
constexpr bool vit_turns() { return G::LPR == 32 && G::WAVES == 16 && G::ITEMS == 4; }

template <typename G, bool TURNED>
struct VitSmem {
    double pv[G::WAVES][G::TCAP];  // per-wave best candidate per column (forward merge)
    int pi[G::WAVES][G::TCAP];     // and its previous tag
    double dvec[2][G::TCAP];
};
template <typename G>
struct VitSmem<G, true> {
    double dvec[2][G::TCAP];
};

// STRUCT: potentials are trans + emit (float, T <= 128; a compile-time choice so that the dense path
// keeps its loads free of branches).
template <typename G, typename TIN, bool ALIGNED, bool STRUCT = false>
__global__ __launch_bounds__(G::W) void viterbi_half_kernel(VitArgs a) {
    constexpr bool TURNED = vit_turns<G, ALIGNED>() && !STRUCT;  // structured tiles are formed in registers: nothing to turn
    __shared__ VitSmem<G, TURNED> sm;
    constexpr int ITEMS = G::ITEMS;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int dir = blockIdx.x & 1;
    const VitSpan sp = vit_span(a, blockIdx.x >> 1);
    if (sp.empty) return;
    const int b = sp.b, N = a.N, T = a.T;
    const int p0 = sp.p0, e = sp.e, h = meeting_point(p0, e);
    const int c4 = 4 * (tid % G::LPR), r0 = tid / G::LPR;
    const size_t TT = (size_t)T * T;
    const TIN* phib = static_cast<const TIN*>(a.phi) + (size_t)b * N * TT;
    uint8_t* bpb = a.bp + (size_t)b * N * T;
    double* mid = a.mid + (((size_t)b * a.C + sp.c) * 2 + dir) * T;
    const double ninf = -__builtin_huge_val();

    for (int k = tid; k < 2 * G::TCAP; k += G::W) (&sm.dvec[0][0])[k] = ninf;
    __syncthreads();
    constexpr bool CAN_STRUCT = STRUCT;
    constexpr bool structured = STRUCT;
    const float* emb = structured ? a.emit + (size_t)b * N * T : nullptr;
    float tr[CAN_STRUCT ? ITEMS : 1][4];
    if constexpr (CAN_STRUCT) {
        load_tile<G, float, ALIGNED>(a.trans, T, c4, r0, tr);
    }
    if (tid < T) {
        if (dir == 0) {
            if (sp.t0 == 0) sm.dvec[0][tid] = structured ? (double)(a.trans[tid] + emb[tid]) : (double)Elem<TIN>::get(phib + tid);
            else sm.dvec[0][tid] = (tid == a.pin[(size_t)b * a.C + sp.c - 1]) ? 0.0 : ninf;
        } else {
            // a whole sequence may end in any tag; a chunk must end in its pinned tag
            sm.dvec[0][tid] = (a.chunk <= 0 || tid == a.pin[(size_t)b * a.C + sp.c]) ? 0.0 : ninf;
        }
    }
    __syncthreads();

    int buf = 0;
    float A[ITEMS][4], Bq[ITEMS][4];
    // forward: column maxima over rows, merged across waves through LDS
    auto fetch = [&](int i, float (&v)[ITEMS][4]) {
        if constexpr (CAN_STRUCT) {
            load_emit4<ALIGNED>(emb + (size_t)i * T, T, c4, v[0], b != a.B - 1 || i != N - 1);
            return;
        }
        load_tile<G, TIN, ALIGNED>(phib + (size_t)i * TT, T, c4, r0, v, b != a.B - 1 || i != N - 1);
    };
    auto tile_ready = [&](float (&v)[ITEMS][4]) {
        if constexpr (CAN_STRUCT) {
            settle_emit4<ALIGNED>(v[0], T, c4);
            add_trans<ITEMS>(v, tr);
        }
    };
    auto fwd_step = [&](int i, float (&v)[ITEMS][4]) {
      if constexpr (!TURNED) {
        tile_ready(v);
        mask_tile<G>(v, T, c4, r0);
        double best[4] = {ninf, ninf, ninf, ninf};
        int arg[4] = {kNoArg, kNoArg, kNoArg, kNoArg};
#pragma unroll
        for (int k = 0; k < ITEMS; ++k) {
            const int s = r0 + k * G::RPP;
            const double dk = sm.dvec[buf][s];  // s < TCAP; tags >= T hold -inf: no branch around the read
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const double val = dk + (double)v[k][j];
                if (val > best[j]) { best[j] = val; arg[j] = s; }
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {  // over the row groups of the wave: lanes LPR, 2 LPR, ... apart
            Best x{best[j], arg[j]};
            if (G::LPR <= 16) x = swap_best<16>(x);
            if (G::LPR <= 32) x = swap_best<32>(x);
            best[j] = x.v;
            arg[j] = x.a;
        }
        if (lane < G::LPR) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                sm.pv[wave][c4 + j] = best[j];
                sm.pi[wave][c4 + j] = arg[j];
            }
        }
        __syncthreads();
        if (tid < G::TCAP) {
            double bv = ninf;
            int ba = kNoArg;
#pragma unroll
            for (int w = 0; w < G::WAVES; ++w) take_better(bv, ba, sm.pv[w][tid], sm.pi[w][tid]);
            sm.dvec[buf ^ 1][tid] = bv;
            if (tid < T) bpb[(size_t)i * T + tid] = (uint8_t)(ba == kNoArg ? 0 : ba);
        }
        __syncthreads();
        buf ^= 1;
      }
    };
    // backward: row maxima over columns, inside the wave
    auto bwd_step = [&](int i, float (&v)[ITEMS][4]) {
        tile_ready(v);
        mask_tile<G>(v, T, c4, r0);
        double ek[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) ek[j] = sm.dvec[buf][c4 + j];  // -inf for tags >= T
        if constexpr (ITEMS % 4 == 0 && G::LPR >= 16) {
            // four rows at a time: each lane ends up with the winner of one of them
            const int kk = 2 * (lane & 1) + ((lane >> 1) & 1);
#pragma unroll
            for (int k0 = 0; k0 < ITEMS; k0 += 4) {
                Best c[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    c[q] = Best{ninf, kNoArg};
#pragma unroll
                    for (int j = 0; j < 4; ++j) {  // ascending columns: the first maximum wins
                        const double val = (double)v[k0 + q][j] + ek[j];
                        if (val > c[q].v) c[q] = Best{val, c4 + j};
                    }
                }
                const Best w = reduce4_best_over_lanes<G::LPR>(c[0], c[1], c[2], c[3], lane);
                const int s = r0 + (k0 + kk) * G::RPP;
                if ((tid % G::LPR) < 4 && s < T) {
                    sm.dvec[buf ^ 1][s] = w.v;
                    bpb[(size_t)i * T + s] = (uint8_t)(w.a == kNoArg ? 0 : w.a);
                }
            }
        } else
#pragma unroll
        for (int k = 0; k < ITEMS; ++k) {
            double bv = ninf;
            int ba = kNoArg;
#pragma unroll
            for (int j = 0; j < 4; ++j) {  // ascending columns: the first maximum wins
                const double val = (double)v[k][j] + ek[j];
                if (val > bv) { bv = val; ba = c4 + j; }
            }
#pragma unroll
            for (int off = 1; off < G::LPR; off <<= 1) {
                const double pv = __shfl_xor(bv, off, 64);
                const int pa = __shfl_xor(ba, off, 64);
                take_better(bv, ba, pv, pa);
            }
            const int s = r0 + k * G::RPP;
            if (c4 == 0 && s < T) {
                sm.dvec[buf ^ 1][s] = bv;
                bpb[(size_t)i * T + s] = (uint8_t)(ba == kNoArg ? 0 : ba);
            }
        }
        __syncthreads();
        buf ^= 1;
    };
    auto run = [&](int first, int last, int step_dir, auto step) {  // two-deep software pipeline over the tiles
        int i = first;
        const int n = (last - first) * step_dir + 1;
        if (n <= 0) return;
        int left = n;
        if constexpr (ITEMS >= 16) {
            // 64 potentials a thread and tile: a second tile in flight would not fit the registers
            for (; left > 0; --left, i += step_dir) {
                fetch(i, A);
                step(i, A);
            }
            return;
        }
        fetch(i, A);
        while (left > 0) {
            if (left > 1) fetch(i + step_dir, Bq);
            step(i, A);
            i += step_dir;
            if (--left == 0) break;
            if (left > 1) fetch(i + step_dir, A);
            step(i, Bq);
            i += step_dir;
            --left;
        }
    };
    if constexpr (TURNED) {
        if (dir == 0) {
            extern __shared__ __attribute__((aligned(16))) float turn_tiles[];
            float* tiles = turn_tiles;
            constexpr int PF = 4;
            const int rowl = lane & 31, colw = 8 * wave + 4 * (lane >> 5);
            const int kk = 2 * (lane & 1) + ((lane >> 1) & 1);
            const int first = p0 + 1, n = h - p0;
            if (n > 0) {
                float ring[PF][4][4];
                // (entries outside the matrix hold other entries of it: rows >= T meet -inf, columns >= T are dropped)
                auto load = [&](int i, int slot) { load_tile<G, TIN, ALIGNED>(phib + (size_t)i * TT, T, c4, r0, ring[slot], b != a.B - 1 || i != N - 1); };
                auto to_lds = [&](int slot, int wb) {
#pragma unroll
                    for (int k = 0; k < 4; ++k)
                        *reinterpret_cast<float4*>(&tiles[(wb * 128 + r0 + 32 * k) * kTurnStride + c4]) =
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
                        const int nslot = (p + 1) % PF;
                        const float* mine = &tiles[((p & 1) * 128 + rowl) * kTurnStride + colw];
                        Best c[4] = {Best{ninf, kNoArg}, Best{ninf, kNoArg}, Best{ninf, kNoArg}, Best{ninf, kNoArg}};
#pragma unroll
                        for (int k = 0; k < 4; ++k) {  // ascending rows: the first maximum wins
                            const int s = rowl + 32 * k;
                            const double dk = sm.dvec[buf][s];  // -inf for rows >= T
                            const float4 q = *reinterpret_cast<const float4*>(mine + 32 * k * kTurnStride);
                            const double v0 = dk + (double)q.x, v1 = dk + (double)q.y, v2 = dk + (double)q.z, v3 = dk + (double)q.w;
                            if (v0 > c[0].v) c[0] = Best{v0, s};
                            if (v1 > c[1].v) c[1] = Best{v1, s};
                            if (v2 > c[2].v) c[2] = Best{v2, s};
                            if (v3 > c[3].v) c[3] = Best{v3, s};
                        }
                        to_lds(nslot, nslot & 1);
                        {
                            const int ahead = done + 1 + PF;
                            load(first + (ahead < n ? ahead : n - 1), nslot);
                        }
                        const Best w = reduce4_best_over_lanes<32>(c[0], c[1], c[2], c[3], lane);
                        const int col = colw + kk;
                        if (rowl < 4 && col < T) {
                            sm.dvec[buf ^ 1][col] = w.v;
                            bpb[(size_t)i * T + col] = (uint8_t)(w.a == kNoArg ? 0 : w.a);
                        }
                        __syncthreads();
                        buf ^= 1;
                        if (++done >= n) { running = false; break; }
                    }
                }
            }
        } else {
            run(e, h + 1, -1, bwd_step);
        }
    } else {
        if (dir == 0) run(p0 + 1, h, +1, fwd_step);
        else run(e, h + 1, -1, bwd_step);
    }
    if (tid < T) mid[tid] = sm.dvec[buf][tid];
}

// 129 .. 256 tags: the matrix of a position streams through registers in batches of 64 rows, as in the
// sum-product kernels for these tag sets (lccrf_stream.hip): lane l of wave w holds, of batch q, rows
// 64 q + 4 w + k (k < 4), columns 4 l .. 4 l + 3, and a ring of batch slots is refilled across position
// boundaries.  Held as one tile of 64 potentials a thread beside the double-precision candidates, the
// matrix spilled registers and allowed no load in flight during a step.
//   forward:  a thread keeps the best candidate of each of its four columns over its rows of all batches
//             (ascending rows: the first maximum wins), the 16 waves' candidates meet through LDS;
//   backward: a row is complete inside its wave and batch: four rows at a time by the packed reduction.
constexpr int kVitBatchRows = 64;
constexpr int kVitRing = 3;
using VSG = Geo<64, 16, 16>;

template <typename TIN, bool ALIGNED>
__global__ __launch_bounds__(1024) void viterbi_stream_kernel(VitArgs a) {
    __shared__ VitSmem<VSG, false> sm;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int dir = blockIdx.x & 1;
    const VitSpan sp = vit_span(a, blockIdx.x >> 1);
    if (sp.empty) return;
    const int b = sp.b, N = a.N, T = a.T;
    const int p0 = sp.p0, e = sp.e, h = meeting_point(p0, e);
    const int c4 = 4 * lane;
    const size_t TT = (size_t)T * T;
    const TIN* phib = static_cast<const TIN*>(a.phi) + (size_t)b * N * TT;
    uint8_t* bpb = a.bp + (size_t)b * N * T;
    double* mid = a.mid + (((size_t)b * a.C + sp.c) * 2 + dir) * T;
    const double ninf = -__builtin_huge_val();
    const int NBq = (T + kVitBatchRows - 1) / kVitBatchRows;  // 3 or 4

    for (int k = tid; k < 2 * VSG::TCAP; k += 1024) (&sm.dvec[0][0])[k] = ninf;
    __syncthreads();
    if (tid < T) {
        if (dir == 0) {
            if (sp.t0 == 0) sm.dvec[0][tid] = (double)Elem<TIN>::get(phib + tid);
            else sm.dvec[0][tid] = (tid == a.pin[(size_t)b * a.C + sp.c - 1]) ? 0.0 : ninf;
        } else {
            sm.dvec[0][tid] = (a.chunk <= 0 || tid == a.pin[(size_t)b * a.C + sp.c]) ? 0.0 : ninf;
        }
    }
    __syncthreads();

    int buf = 0;
    float ring[kVitRing][4][4];
    const int first = dir == 0 ? p0 + 1 : e;
    const int n = dir == 0 ? h - p0 : e - h;
    const int sdir = dir == 0 ? +1 : -1;
    // unit u = batch u % NBq of the matrix of position first + sdir (u / NBq); addresses clamped into the matrix
    auto load = [&](int u, int slot) {
        const TIN* mat = phib + (size_t)(first + sdir * (u / NBq)) * TT;
        const bool mat_followed = b != a.B - 1 || first + sdir * (u / NBq) != N - 1;
        const int row0 = kVitBatchRows * (u % NBq) + 4 * wave;
        if (ALIGNED) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int s = row0 + k;
                const TIN* row = mat + (size_t)(s < T ? s : T - 1) * T;
                Elem<TIN>::get4_stream(row + (c4 < T ? c4 : T - 4), ring[slot][k]);
            }
        } else if (mat_followed) {  // (entries outside the matrix hold other entries of it: they meet -inf, or are dropped)
#pragma unroll
            for (int k = 0; k < 4; ++k) load_row4_anywhere<TIN, true>(mat, T, row0 + k, c4, ring[slot][k]);
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k) load_row4_anywhere<TIN, false>(mat, T, row0 + k, c4, ring[slot][k]);
        }
    };
    if (dir == 0) {
        double best[4] = {ninf, ninf, ninf, ninf};
        int arg[4] = {kNoArg, kNoArg, kNoArg, kNoArg};
        walk<kVitRing>(0, n * NBq - 1, +1, load, [&](int u, int slot) {
            const int i = first + u / NBq, q = u % NBq;
            const int row0 = kVitBatchRows * q + 4 * wave;
            if (q == 0) {
#pragma unroll
                for (int j = 0; j < 4; ++j) { best[j] = ninf; arg[j] = kNoArg; }
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {  // ascending rows: the first maximum wins
                const int s = row0 + k;
                const double dk = sm.dvec[buf][s];  // -inf for rows >= T (s < 256 always)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const double val = dk + (double)ring[slot][k][j];
                    if (val > best[j]) { best[j] = val; arg[j] = s; }
                }
            }
            if (q == NBq - 1) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    sm.pv[wave][c4 + j] = best[j];
                    sm.pi[wave][c4 + j] = arg[j];
                }
                __syncthreads();
                if (tid < VSG::TCAP) {
                    double bv = ninf;
                    int ba = kNoArg;
                    if (tid < T) {
#pragma unroll
                        for (int w = 0; w < 16; ++w) take_better(bv, ba, sm.pv[w][tid], sm.pi[w][tid]);
                        bpb[(size_t)i * T + tid] = (uint8_t)(ba == kNoArg ? 0 : ba);
                    }
                    sm.dvec[buf ^ 1][tid] = bv;
                }
                __syncthreads();
                buf ^= 1;
            }
        });
    } else {
        double ek[4] = {ninf, ninf, ninf, ninf};
        walk<kVitRing>(0, n * NBq - 1, +1, load, [&](int u, int slot) {
            const int i = first - u / NBq, q = u % NBq;
            const int row0 = kVitBatchRows * q + 4 * wave;
            if (q == 0) {
#pragma unroll
                for (int j = 0; j < 4; ++j) ek[j] = sm.dvec[buf][c4 + j];  // -inf for tags >= T
            }
            Best c[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                c[k] = Best{ninf, kNoArg};
#pragma unroll
                for (int j = 0; j < 4; ++j) {  // ascending columns: the first maximum wins
                    const double val = (double)ring[slot][k][j] + ek[j];
                    if (val > c[k].v) c[k] = Best{val, c4 + j};
                }
            }
            // four rows at a time: each lane ends up with the winner of one of them
            const int kk = 2 * (lane & 1) + ((lane >> 1) & 1);
            const Best w = reduce4_best_over_lanes<64>(c[0], c[1], c[2], c[3], lane);
            const int s = row0 + kk;
            if (lane < 4 && s < T) {
                sm.dvec[buf ^ 1][s] = w.v;
                bpb[(size_t)i * T + s] = (uint8_t)(w.a == kNoArg ? 0 : w.a);
            }
            if (q == NBq - 1) {
                __syncthreads();
                buf ^= 1;
            }
        });
    }
    if (tid < T) mid[tid] = sm.dvec[buf][tid];
}

// One wave per chain for T <= 32 (TP = 16 or 32 padded tags): the whole matrix of a position is spread
// over the 64 lanes, the vector of the previous position sits in LDS, and nothing but that vector
// crosses lanes, so a step needs no barrier between waves and no merge through LDS.
//   forward:  LPC = 64 / TP lanes share a column t (lane = part TP + t), each takes the rows
//             part RPL .. part RPL + RPL - 1 in ascending order and the LPC partial winners are
//             merged with lane exchanges (for a fixed row the lanes read consecutive addresses);
//   backward: LPC lanes share a row s (lane = s LPC + part), each takes RPL consecutive columns
//             (vector loads), merged in the same way.
// Same outputs as viterbi_half_kernel: pointers in bp, the two vectors of the meeting point in mid.
// ALONE: the wave is the whole workgroup (its barrier is a wait for its own LDS writes).  Otherwise it shares a
// workgroup with waves that make a different number of steps, and must not meet them at a barrier: LDS executes a
// wave's instructions in order, so the wave's own writes are there for its later reads, and the compiler only has
// to keep the order.
template <bool ALONE>
__device__ __forceinline__ void wave_step_end() {
    if constexpr (ALONE) __syncthreads();
    else __atomic_signal_fence(__ATOMIC_SEQ_CST);
}
template <int TP, typename TIN, bool ALIGNED, bool STRUCT, bool ALONE>
__device__ __forceinline__ void viterbi_wave_chain(const VitArgs& a, const VitSpan& sp, int dir, int lane, double (*dvec)[TP]) {
    constexpr int LPC = 64 / TP, RPL = TP / LPC, PF = 3;
    const int b = sp.b, N = a.N, T = a.T;
    const int p0 = sp.p0, e = sp.e, h = meeting_point(p0, e);
    const size_t TT = (size_t)T * T;
    const TIN* phib = STRUCT ? nullptr : static_cast<const TIN*>(a.phi) + (size_t)b * N * TT;
    const float* emb = STRUCT ? a.emit + (size_t)b * N * T : nullptr;
    uint8_t* bpb = a.bp + (size_t)b * N * T;
    double* mid = a.mid + (((size_t)b * a.C + sp.c) * 2 + dir) * T;
    const double ninf = -__builtin_huge_val();

    if (lane < TP) {
        double v0 = ninf;
        if (lane < T) {
            if (dir == 0) {
                if (sp.t0 == 0) v0 = STRUCT ? (double)(a.trans[lane] + emb[lane]) : (double)Elem<TIN>::get(phib + lane);
                else v0 = (lane == a.pin[(size_t)b * a.C + sp.c - 1]) ? 0.0 : ninf;
            } else {
                // a whole sequence may end in any tag; a chunk must end in its pinned tag
                v0 = (a.chunk <= 0 || lane == a.pin[(size_t)b * a.C + sp.c]) ? 0.0 : ninf;
            }
        }
        dvec[0][lane] = v0;
    }
    wave_step_end<ALONE>();
    int buf = 0;
    float ring[PF][RPL];

    if (dir == 0) {
        const int part = lane / TP, t = lane % TP, s0 = part * RPL;
        const int tc = t < T ? t : T - 1;
        float tr[STRUCT ? RPL : 1];
        if constexpr (STRUCT) {
#pragma unroll
            for (int k = 0; k < RPL; ++k) tr[k] = a.trans[(size_t)(s0 + k < T ? s0 + k : T - 1) * T + tc];
        }
        auto load = [&](int i, int slot) {
            if constexpr (STRUCT) {
                ring[slot][0] = emb[(size_t)i * T + tc];
            } else {
                const TIN* m = phib + (size_t)i * TT + tc;
#pragma unroll
                for (int k = 0; k < RPL; ++k) ring[slot][k] = Elem<TIN>::get(m + (size_t)(s0 + k < T ? s0 + k : T - 1) * T);
            }
        };
        walk<PF>(p0 + 1, h, +1, load, [&](int i, int slot) {
            double val[RPL];
            int arg[RPL];
#pragma unroll
            for (int k = 0; k < RPL; ++k) {
                const int s = s0 + k;
                const float x = STRUCT ? tr[k] + ring[slot][0] : ring[slot][k];
                // the vector is read whatever the entry is (tags >= T hold -inf there): no branch around the LDS read
                val[k] = dvec[buf][s] + (double)((s < T && t < T) ? x : LCCRF_NEG_INF);
                arg[k] = s;
            }
            first_max_tree<RPL>(val, arg);
            double bv = val[0];
            int ba = bv == ninf ? kNoArg : arg[0];
#pragma unroll
            for (int off = TP; off < 64; off <<= 1) {
                const double pv = __shfl_xor(bv, off, 64);
                const int pa = __shfl_xor(ba, off, 64);
                take_better(bv, ba, pv, pa);
            }
            if (part == 0) {
                dvec[buf ^ 1][t] = bv;
                if (t < T) bpb[(size_t)i * T + t] = (uint8_t)(ba == kNoArg ? 0 : ba);
            }
            wave_step_end<ALONE>();
            buf ^= 1;
        });
    } else {
        const int s = lane / LPC, part = lane % LPC, c0 = part * RPL;
        const int sc = s < T ? s : T - 1;
        float tr[STRUCT ? RPL : 1];
        if constexpr (STRUCT) {
#pragma unroll
            for (int k = 0; k < RPL; ++k) tr[k] = a.trans[(size_t)sc * T + (c0 + k < T ? c0 + k : T - 1)];
        }
        auto load = [&](int i, int slot) {
            const float* erow = STRUCT ? emb + (size_t)i * T : nullptr;
            const TIN* row = STRUCT ? nullptr : phib + (size_t)i * TT + (size_t)sc * T;
            if constexpr (ALIGNED) {
#pragma unroll
                for (int k = 0; k < RPL; k += 4) {
                    float q[4];
                    const int c = c0 + k < T ? c0 + k : T - 4;  // T % 4 == 0 here
                    if constexpr (STRUCT) Elem<float>::get4(erow + c, q);
                    else Elem<TIN>::get4(row + c, q);
                    ring[slot][k] = q[0]; ring[slot][k + 1] = q[1]; ring[slot][k + 2] = q[2]; ring[slot][k + 3] = q[3];
                }
            } else if constexpr (STRUCT) {
#pragma unroll
                for (int k = 0; k < RPL; ++k) ring[slot][k] = erow[c0 + k < T ? c0 + k : T - 1];
            } else {  // (entries past the end of the row hold other entries of the matrix: they are masked below)
                const TIN* mat = phib + (size_t)i * TT;
                if ((sp.b != a.B - 1 || i != a.N - 1) && T > 1) {  // (the same for the whole wave: one scalar branch)
#pragma unroll
                    for (int k = 0; k < RPL; k += 4)
                        load_row4_anywhere<TIN, true>(mat, T, sc, c0 + k, *reinterpret_cast<float(*)[4]>(&ring[slot][k]));
                } else {
#pragma unroll
                    for (int k = 0; k < RPL; k += 4)
                        load_row4_anywhere<TIN, false>(mat, T, sc, c0 + k, *reinterpret_cast<float(*)[4]>(&ring[slot][k]));
                }
            }
        };
        walk<PF>(e, h + 1, -1, load, [&](int i, int slot) {
            double val[RPL];
            int arg[RPL];
#pragma unroll
            for (int k = 0; k < RPL; ++k) {
                const int t = c0 + k;
                const float x = STRUCT ? tr[k] + ring[slot][k] : ring[slot][k];
                val[k] = (double)((s < T && t < T) ? x : LCCRF_NEG_INF) + dvec[buf][t];
                arg[k] = t;
            }
            first_max_tree<RPL>(val, arg);
            double bv = val[0];
            int ba = bv == ninf ? kNoArg : arg[0];
#pragma unroll
            for (int off = 1; off < LPC; off <<= 1) {
                const double pv = __shfl_xor(bv, off, 64);
                const int pa = __shfl_xor(ba, off, 64);
                take_better(bv, ba, pv, pa);
            }
            if (part == 0) {
                dvec[buf ^ 1][s] = bv;
                if (s < T) bpb[(size_t)i * T + s] = (uint8_t)(ba == kNoArg ? 0 : ba);
            }
            wave_step_end<ALONE>();
            buf ^= 1;
        });
    }
    if (lane < T) mid[lane] = dvec[buf][lane];
}

template <int TP, typename TIN, bool ALIGNED, bool STRUCT>
__global__ __launch_bounds__(64) void viterbi_wave_kernel(VitArgs a) {
    __shared__ double dvec[2][TP];
    const VitSpan sp = vit_span(a, blockIdx.x >> 1);
    if (sp.empty) return;
    viterbi_wave_chain<TP, TIN, ALIGNED, STRUCT, true>(a, sp, blockIdx.x & 1, threadIdx.x, dvec);
}

// Joins the two chains at the meeting point and reads off the path.
//
// Following the pointers is a chain of dependent LDS reads, one per position (about a hundred cycles each).  It is
// cut by walking stretches of the path before their entry tag is known: a half of the workgroup serves a
// direction, its threads (stretch g, tag t) follow the pointers of stretch g from EVERY entry tag t and record
// the tags they pass; one thread then links the stretches (the tag a stretch is left on, given the tag it was
// entered on, enters the next), and all threads copy the recorded tags of the stretches' true entry tags out.
// The dependent chain is R / G + G lookups instead of R for R positions in G = threads / T stretches.
constexpr int kTraceThreads = 512;             // half of them per direction
template <int THREADS, int BYTES>
struct TraceShared {
    static constexpr int HALF = THREADS / 2;
    __attribute__((aligned(16))) uint8_t window[2][BYTES];  // pointers of the rows being walked
    uint8_t passed[2][BYTES + HALF];  // [step][stretch][entry tag]: the tag reached after that step
    uint8_t left_on[2][HALF];         // [stretch][entry tag]: the tag the stretch is left on
    int entered[2][HALF + 1];         // the tag every stretch is entered on
    int start;
};
// By all THREADS threads of a workgroup (every one of them must call it: it holds barriers).
template <int THREADS, int BYTES>
__device__ __forceinline__ void trace_span(const VitArgs& a, const VitSpan& sp, TraceShared<THREADS, BYTES>& sm) {
    constexpr int kHalf = THREADS / 2;
    const int tid = threadIdx.x, lane = tid & 63;
    const int dir = tid / kHalf, me = tid % kHalf;  // dir 0 walks down, 1 up
    const int b = sp.b, N = a.N, T = a.T, L = sp.L;
    int32_t* tags = a.tags + (size_t)b * N;
    for (int i = (L > sp.t0 ? L : sp.t0) + tid; i < sp.t1; i += THREADS) tags[i] = -1;
    if (L == 0) {
        if (a.chunk <= 0 && tid == 0 && a.best_score) a.best_score[b] = 0.f;
        return;
    }
    if (sp.empty) return;
    const int p0 = sp.p0, e = sp.e, h = meeting_point(p0, e);
    const uint8_t* bpb = a.bp + (size_t)b * N * T;
    const double* mid = a.mid + ((size_t)b * a.C + sp.c) * 2 * T;
    const double ninf = -__builtin_huge_val();

    if (tid < 64) {  // best tag at the meeting point: first maximum of delta_h + eps_h
        double bv = ninf;
        int ba = kNoArg;
        for (int t = lane; t < T; t += 64) {
            const double val = mid[t] + mid[T + t];
            if (val > bv) { bv = val; ba = t; }
        }
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const double pv = __shfl_xor(bv, off, 64);
            const int pa = __shfl_xor(ba, off, 64);
            take_better(bv, ba, pv, pa);
        }
        if (lane == 0) {
            sm.start = (ba == kNoArg) ? 0 : ba;
            if (a.chunk <= 0 && a.best_score) a.best_score[b] = (float)bv;
        }
    }
    __syncthreads();
    const int rows_per_window = BYTES / T;
    const int G = kHalf / T > 0 ? kHalf / T : 1;   // stretches walked at once
    const int g = me / T, t = me % T;
    int y = sm.start;               // the tag the next window is entered on (the same in every thread of a direction)
    if (tid == 0) tags[h] = y;
    // downwards row r yields the tag of position r - 1 (a chunk leaves the tag of its entry position p0 to the
    // chunk that ends there); upwards row r yields the tag of position r
    const int stop = sp.t0 == 0 ? 1 : sp.t0 + 1;
    int hi = h + 1;   // rows [stop, hi) still to walk down
    int lo = h + 1;   // rows [lo, e] still to walk up
    while (hi > stop || lo <= e) {  // both directions make the same number of trips: barriers stay matched
        const int dlo = (hi - rows_per_window > stop) ? hi - rows_per_window : stop;
        const int uhi = (lo + rows_per_window - 1 < e) ? lo + rows_per_window - 1 : e;
        // rows of this trip: the first of them in memory and their number
        const int first = dir == 0 ? dlo : lo;
        const int R = dir == 0 ? (hi > stop ? hi - dlo : 0) : (lo <= e ? uhi - lo + 1 : 0);
        {
            const int nbytes = R * T;
            const uint8_t* src = bpb + (size_t)first * T;
            int k0 = 0;
            if ((reinterpret_cast<uintptr_t>(src) & 15) == 0) {
                const int n16 = nbytes / 16;
                const uint4* s16 = reinterpret_cast<const uint4*>(src);
                uint4* d16 = reinterpret_cast<uint4*>(sm.window[dir]);
                for (int k = me; k < n16; k += kHalf) d16[k] = s16[k];
                k0 = n16 * 16;
            }
            for (int k = k0 + me; k < nbytes; k += kHalf) sm.window[dir][k] = src[k];
        }
        __syncthreads();
        const int S = (R + G - 1) / G;  // rows a stretch
        if (g < G && t < T && R > 0) {
            int yy = t;
            for (int j = 0; j < S; ++j) {
                const int k = g * S + j;  // the k-th row walked on this trip
                if (k >= R) break;
                yy = sm.window[dir][(dir == 0 ? R - 1 - k : k) * T + yy];
                sm.passed[dir][(j * G + g) * T + t] = (uint8_t)yy;
            }
            sm.left_on[dir][g * T + t] = (uint8_t)yy;
        }
        __syncthreads();
        if (me == 0 && R > 0) {
            int yy = y;
            for (int q = 0; q < G; ++q) {
                sm.entered[dir][q] = yy;
                yy = sm.left_on[dir][q * T + yy];
            }
            sm.entered[dir][G] = yy;
        }
        __syncthreads();
        if (R > 0) {
            for (int k = me; k < R; k += kHalf) {
                const int q = k / S, j = k % S;
                const int tag = sm.passed[dir][(j * G + q) * T + sm.entered[dir][q]];
                if (dir == 0) tags[first + R - 1 - k - 1] = tag;
                else tags[first + k] = tag;
            }
            y = sm.entered[dir][G];
        }
        __syncthreads();
        if (hi > stop) hi = dlo;
        if (lo <= e) lo = uhi + 1;
    }
}
__global__ __launch_bounds__(kTraceThreads) void viterbi_trace_kernel(VitArgs a) {
    __shared__ TraceShared<kTraceThreads, kTraceBytes> sm;
    trace_span<kTraceThreads, kTraceBytes>(a, vit_span(a, blockIdx.x), sm);
}

// A chunk of the scan (up to 32 tags) by one workgroup of two waves: its forward and its backward chain side by
// side, then, behind one barrier, its trace: the pointers and the two vectors of the meeting point come back
// from memory the same workgroup has just written (one launch and one trip through the launch queue less).
constexpr int kFusedTraceBytes = 2048;
template <int TP, typename TIN, bool ALIGNED, bool STRUCT>
__global__ __launch_bounds__(128) void viterbi_chunk_kernel(VitArgs a) {
    __shared__ double dvec[2][2][TP];
    __shared__ TraceShared<128, kFusedTraceBytes> sm;
    const VitSpan sp = vit_span(a, blockIdx.x);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (!sp.empty) viterbi_wave_chain<TP, TIN, ALIGNED, STRUCT, false>(a, sp, wave, threadIdx.x & 63, dvec[wave]);
    // The barrier orders what the two waves stored before what the trace loads at workgroup scope, which is all it
    // takes: the waves of a workgroup share their compute unit's vector cache, and stores go through it.  (A fence of
    // wider scope here would write the whole L2 back once per workgroup: 14 us became 160.)
    __syncthreads();
    trace_span<128, kFusedTraceBytes>(a, sp, sm);
}

template <typename G, typename TIN, bool ALIGNED>
static hipError_t launch_geo(const VitArgs& a, hipStream_t st) {
    hipError_t e = hipSuccess;
    size_t turn_bytes = 0;
    if constexpr (vit_turns<G, ALIGNED>()) {
        turn_bytes = kTurnFloats * sizeof(float);
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&viterbi_half_kernel<G, TIN, ALIGNED>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)turn_bytes);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((viterbi_half_kernel<G, TIN, ALIGNED>), dim3(2 * a.B * a.C), dim3(G::W), turn_bytes, st, a);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(viterbi_trace_kernel, dim3(a.B * a.C), dim3(kTraceThreads), 0, st, a);
    return hipGetLastError();
}

template <int TP, typename TIN, bool ALIGNED, bool STRUCT>
static hipError_t launch_wave_vit(const VitArgs& a, hipStream_t st) {
    if (a.chunk > 0) {
        hipLaunchKernelGGL((viterbi_chunk_kernel<TP, TIN, ALIGNED, STRUCT>), dim3(a.B * a.C), dim3(128), 0, st, a);
        return hipGetLastError();
    }
    hipLaunchKernelGGL((viterbi_wave_kernel<TP, TIN, ALIGNED, STRUCT>), dim3(2 * a.B * a.C), dim3(64), 0, st, a);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(viterbi_trace_kernel, dim3(a.B * a.C), dim3(kTraceThreads), 0, st, a);
    return hipGetLastError();
}

template <typename TIN, bool ALIGNED>
static hipError_t launch_T(const VitArgs& a, hipStream_t st) {
    const int T = a.T;
    if (T <= 16) return launch_wave_vit<16, TIN, ALIGNED, false>(a, st);
    if (T <= 32) return launch_wave_vit<32, TIN, ALIGNED, false>(a, st);
    if (T <= 64) return launch_geo<Geo<16, 4, 4>, TIN, ALIGNED>(a, st);
    if (T <= 128) return launch_geo<Geo<32, 16, 4>, TIN, ALIGNED>(a, st);
    hipLaunchKernelGGL((viterbi_stream_kernel<TIN, ALIGNED>), dim3(2 * a.B * a.C), dim3(1024), 0, st, a);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(viterbi_trace_kernel, dim3(a.B * a.C), dim3(kTraceThreads), 0, st, a);
    return hipGetLastError();
}

static hipError_t launch_any(int dtype, const VitArgs& a, hipStream_t st, bool lanes = false, int lane_poll_limit = 0) {
    if (lanes) {
        const hipError_t e = launch_lane_max_chains(dtype, a, lane_poll_limit, st);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(viterbi_trace_kernel, dim3(a.B * a.C), dim3(kTraceThreads), 0, st, a);
        return hipGetLastError();
    }
    const bool aligned = (a.T % 4) == 0;
    if (dtype == 0) return aligned ? launch_T<float, true>(a, st) : launch_T<float, false>(a, st);
    return aligned ? launch_T<uint16_t, true>(a, st) : launch_T<uint16_t, false>(a, st);
}

size_t viterbi_mid_doubles(int B, int C, int T) { return (size_t)B * C * 2 * T; }

hipError_t launch_sequential_max(int dtype, const void* phi, const int32_t* lengths, int B, int N, int T,
                                 uint8_t* bp, double* mid, float* best_score, int32_t* tags, hipStream_t st, bool lanes,
                                 int lane_poll_limit) {
    if (lanes && !lane_max_supported(T)) return hipErrorInvalidValue;
    return launch_any(dtype, VitArgs{phi, lengths, B, N, T, bp, mid, best_score, tags, 0, 1, nullptr, nullptr, nullptr}, st,
                      lanes, lane_poll_limit);
}

template <typename G, bool ALIGNED>
static hipError_t launch_structured_geo(const VitArgs& a, hipStream_t st) {
    hipLaunchKernelGGL((viterbi_half_kernel<G, float, ALIGNED, true>), dim3(2 * a.B * a.C), dim3(G::W), 0, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(viterbi_trace_kernel, dim3(a.B * a.C), dim3(kTraceThreads), 0, st, a);
    return hipGetLastError();
}
template <bool ALIGNED>
static hipError_t launch_structured_T(const VitArgs& a, hipStream_t st) {
    if (a.T <= 16) return launch_wave_vit<16, float, ALIGNED, true>(a, st);
    if (a.T <= 32) return launch_wave_vit<32, float, ALIGNED, true>(a, st);
    if (a.T <= 64) return launch_structured_geo<Geo<16, 4, 4>, ALIGNED>(a, st);
    return launch_structured_geo<Geo<32, 16, 4>, ALIGNED>(a, st);
}

// The same from structured potentials (float emit [B][N][T] + trans [T][T]; T <= 128).
hipError_t launch_structured_max(const float* emit, const float* trans, const int32_t* lengths, int B, int N, int T,
                                 uint8_t* bp, double* mid, float* best_score, int32_t* tags, hipStream_t st, bool lanes,
                                 int lane_poll_limit) {
    if (T > 128 || (lanes && !lane_max_supported(T))) return hipErrorInvalidValue;
    const VitArgs a{nullptr, lengths, B, N, T, bp, mid, best_score, tags, 0, 1, nullptr, emit, trans};
    if (lanes) return launch_any(0, a, st, true, lane_poll_limit);
    return (T % 4) == 0 ? launch_structured_T<true>(a, st) : launch_structured_T<false>(a, st);
}

// Best path inside every chunk between the tags the max-plus scan has pinned at the chunk ends.
hipError_t launch_chunked_max(int dtype, const void* phi, const int32_t* lengths, int B, int N, int T, uint8_t* bp,
                              double* mid, int32_t* tags, int chunk, const int32_t* pin, hipStream_t st,
                              const float* emit, const float* trans) {
    if (emit) {
        if (dtype != 0 || !trans || T > 128) return hipErrorInvalidValue;
        const VitArgs a{nullptr, lengths, B, N, T, bp, mid, nullptr, tags, chunk, (N + chunk - 1) / chunk, pin, emit, trans};
        return (T % 4) == 0 ? launch_structured_T<true>(a, st) : launch_structured_T<false>(a, st);
    }
    return launch_any(dtype, VitArgs{phi, lengths, B, N, T, bp, mid, nullptr, tags, chunk, (N + chunk - 1) / chunk, pin, nullptr, nullptr}, st);
}

}  // namespace lccrf
