// Second pass of the marginals for large tag sets and few sequences: TWO workgroups per chain.
//
// With B sequences there are only 2B chains (a forward and a backward one per sequence, see
// lccrf_chain.hip).  When 2B is well below the number of compute units, one workgroup per
// chain leaves most of the chip idle and the pass is held back by what a single CU can stream
// (about 50 GB/s) and issue.  Here every chain is served by a PAIR of workgroups on different
// CUs that split each T x T matrix in two:
//
//   forward chain  (alpha_i(t) = sum over s): partner p owns the columns [p T/2, (p+1) T/2),
//   backward chain (beta_{i-1}(s) = sum over t): partner p owns the rows  [p T/2, (p+1) T/2),
//
// so each partner produces half of the next vector from half of the matrix and needs the
// other half from its partner once per step.  The halves travel through a small mailbox in
// device memory: every float is packed with the step number into one 8-byte word, written
// with a single store and polled by the receiver, so no separate flag or fence is needed
// (about 0.8 us per exchange when both workgroups sit on the same XCD; the block index of the
// partner differs by 8, which is how consecutive workgroups are dealt to the 8 XCDs).
//
// Steps are speculative only (uniform shift, see lccrf_chain.hip): a pair whose sums leave the
// accepted range, whose sequence has no finite path, or whose partner does not answer within
// a bounded number of polls marks the sequence as failed and stops; the one-workgroup exact
// kernel then recomputes the failed sequences.  Correctness therefore never depends on both
// partners being resident at the same time, only the speed does (and the low-order bits: the exact
// kernel rounds differently from the pair, so a hand-over that depends on timing makes two runs
// differ within the tolerance).  A receiver that finds its sequence flagged stops at its next poll,
// so one expired wait ends all four workgroups of the sequence within a poll's time.
// Measured on this kernel: the folded DPP forms and the mirror step make the second pass 1-2 % slower
// (0.925 against 0.908 ms on config 4), although they are fewer instructions; the plain forms stay here.
#define LCCRF_LANE_EXCHANGE_CLASSIC
#include "lccrf_chain_args.h"
#include "lccrf_device.h"
#include "lccrf_launch.h"

namespace lccrf {


constexpr int kPairW = 512;        // threads that load and compute (8 waves)
constexpr int kPairWaves = 8;
constexpr int kPairThreads = kPairW + 64;  // plus one wave that only receives the partner's half
constexpr int kPairPF = 4;         // tiles in the register ring
constexpr int kPairMailWords = 128;  // words per mailbox slot (one per entry of a half vector, T <= 256)

// One mailbox word: [tag:16][extra:16][value:32], written and read as one 8-byte access, so a
// word whose tag matches carries this step's value; no flag, no fence.
__device__ __forceinline__ unsigned long long pack_word(float v, unsigned tag, unsigned extra) {
    return ((unsigned long long)(((tag & 0xffffu) << 16) | (extra & 0xffffu)) << 32) | (unsigned long long)__float_as_uint(v);
}

struct PairArgs {
    const void* phi;
    const int32_t* lengths;
    int B, N;
    const float* ua;   // stored by the first pass
    const float* ub;
    const double* Oa;
    const double* Ob;
    float* logZ;
    float* mu;
    unsigned long long* mail;  // [2B chains][2 partners][2 slots][kPairMailWords]
    int* failed;               // [B]
    int poll_limit;            // polls a receiver waits for its partner's words before it gives the sequence up
};

template <int T>
struct PairSmem {
    static constexpr int H = T / 2;
    alignas(16) float vec[2][T];                  // un-normalised vector V_j of step j in vec[j & 1]
    alignas(16) float psum[2][kPairWaves][H];     // forward: per-wave partial column sums of step j in psum[j & 1]
    alignas(16) float wtot[2][kPairWaves];        // per-wave sums of the marginals written by step j
    float red[2][4];    // scratch of the mid-point log-sum-exp
    float dmax[2];      // normaliser of V_j: maximum over partner 0's half
    float tot_own[2];   // marginal sum of step j: this workgroup's part ...
    float tot_oth[2];   // ... and the partner's part
    int stop_req;       // set (by anyone, at any time) when this pair must give up
    int stop_go[2];     // what the i/o wave has decided; written by it alone, read by all after the next barrier
};

// Sender side, executed by the i/o wave once this workgroup's half of the next vector is complete
// (lane t holds entry t + 64 q of this partner's half): one store per entry.  The marginal sum
// of the step rides in the extra bits of lanes 0 and 1, the "give up" vote in lane 2's.
template <int T>
__device__ __forceinline__ void send_half(unsigned long long* mine, unsigned tag, int lane,
                                          const float (&r)[T / 128 ? T / 128 : 1], float tot, bool bad) {
    unsigned long long* out = mine + (tag & 1) * kPairMailWords;
    const unsigned tb = __float_as_uint(tot);
    const unsigned extra = lane == 0 ? (tb >> 16) : (lane == 1 ? (tb & 0xffffu) : (lane == 2 ? (bad ? 1u : 0u) : 0u));
#pragma unroll
    for (int q = 0; q < (T / 128 ? T / 128 : 1); ++q)
        __hip_atomic_store(&out[lane + 64 * q], pack_word(r[q], tag, q == 0 ? extra : 0u), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
}

// Receiver side, executed by the i/o wave: polls the partner's words with this tag, puts the partner's half
// into vec[nbuf] and its scalars into shared memory (the partner's marginal sum belongs to the step
// before: slot nbuf ^ 1).  Returns false if the partner gave up, if the sequence has been flagged as
// failed, or if nothing arrives within poll_limit looks (0: gives up without looking).
template <int T>
__device__ __forceinline__ bool receive_half(PairSmem<T>& sm, const unsigned long long* theirs, const int* failed_flag,
                                             unsigned tag, int lane, int nbuf, int p, int poll_limit) {
    constexpr int H = T / 2;
    constexpr int NQ = H / 64;
    const unsigned long long* in = theirs + (tag & 1) * kPairMailWords;
    unsigned long long w[NQ];
    bool ok = false;
    // at most poll_limit looks (the limit is a kernel argument, the same in every lane): the wait always ends
    for (int looks = 0; looks < poll_limit; ++looks) {
        ok = true;
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            w[q] = __hip_atomic_load(&in[lane + 64 * q], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            ok = ok && (unsigned)(w[q] >> 48) == (tag & 0xffffu);
        }
        ok = __all(ok);
        if (ok || __hip_atomic_load(failed_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) break;
    }
    if (!ok) return false;
    float m = LCCRF_NEG_INF;
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        const float v = __uint_as_float((unsigned)w[q]);
        sm.vec[nbuf][(1 - p) * H + lane + 64 * q] = v;
        m = fmaxf(m, v);
    }
    const unsigned extra = (unsigned)(w[0] >> 32) & 0xffffu;
    const unsigned hi = __builtin_amdgcn_readlane(extra, 0), lo = __builtin_amdgcn_readlane(extra, 1);
    const unsigned badbit = __builtin_amdgcn_readlane(extra, 2);
    if (p == 1) {  // the normaliser is the maximum over partner 0's half, which is what arrived here
        m = xor_max<1, 64>(m);
        if (lane == 0) sm.dmax[nbuf] = finite_or_zero(m);
    }
    if (lane == 0) sm.tot_oth[nbuf ^ 1] = __uint_as_float((hi << 16) | lo);
    return badbit == 0;
}

// Step j of a pair takes the vector V_j of the position before (un-normalised, relative to the running
// offset O) to V_{j+1}.  A workgroup needs its partner's half of V_j for half of the step's terms only (a
// forward workgroup: the rows of the partner's half; a backward one: the columns), so it computes the
// other half of the terms first, while the partner's words are still on their way, and the exchange
// (about 0.8 us) is hidden behind them.  For that, nothing the first half uses may depend on the
// partner's newest data: the shift of a step is the normaliser of the vector ONE STEP BACK (consecutive
// normalisers differ by a few units; the accepted range of a speculative sum is 2^+-60), seeded from the
// last step of the first pass, and the drift feedback uses the marginal sum of two steps back with half
// the gain.  Per step every wave passes two barriers: B (the partner's half has arrived) and A (the
// workers' partial results are in shared memory).  The ninth wave does all the talking: after A it
// completes this workgroup's half of V_{j+1}, sends it, and polls for the partner's.  It alone decides
// on giving up (stop_go), which every wave reads right after B, so all nine leave together.
template <int T, typename TIN>
__global__ __launch_bounds__(kPairThreads) void pair_marginal_kernel(PairArgs a) {
    constexpr int H = T / 2;
    constexpr int NQ = H / 64;
    static_assert(T == 128, "tag-set size this kernel is laid out for");
    __shared__ PairSmem<T> sm;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const bool worker = wave < kPairWaves;
    // block index -> (chain, partner): partners are 8 blocks apart so that they share an XCD
    const int grp = blockIdx.x >> 4, low = blockIdx.x & 15;
    const int p = low >> 3;
    const int chain = grp * 8 + (low & 7);
    if (chain >= 2 * a.B) return;
    const int b = chain >> 1, dir = chain & 1;
    const int N = a.N;
    const int L = clamp_length(a.lengths, b, N);
    constexpr size_t TT = (size_t)T * T;
    const size_t vb = (size_t)b * N;
    float* mub = a.mu + (size_t)b * N * TT;
    int* failed = a.failed + b;

    if (dir == 0 && worker) {  // positions past the end carry no edge; the two partners split the zero fill
        float4* z = reinterpret_cast<float4*>(mub);
        const size_t z0 = (size_t)L * TT / 4, z1 = (size_t)N * TT / 4;
        for (size_t k = z0 + (size_t)p * kPairW + tid; k < z1; k += 2 * kPairW) z[k] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    if (L < 2) {  // degenerate chains go to the exact kernel
        if (tid == 0) *failed = 1;
        return;
    }
    const int h = meeting_point(0, L - 1);
    const TIN* phib = static_cast<const TIN*>(a.phi) + (size_t)b * N * TT;
    unsigned long long* mine = a.mail + ((size_t)chain * 2 + p) * 2 * kPairMailWords;
    const unsigned long long* theirs = a.mail + ((size_t)chain * 2 + (1 - p)) * 2 * kPairMailWords;

    // log2 Z at the meeting position, identical in all four workgroups of the sequence
    if (tid == 0) { sm.stop_req = 0; sm.stop_go[0] = 0; sm.stop_go[1] = 0; }
    float z = LCCRF_NEG_INF;
    if (tid < T) z = a.ua[(vb + h) * T + tid] + a.ub[(vb + h) * T + tid];
    if (wave < (T + 63) / 64) {
        const float wm = xor_max<1, 64>(z);
        if (lane == 0) sm.red[0][wave] = wm;
    }
    __syncthreads();
    float M = LCCRF_NEG_INF;
#pragma unroll
    for (int w = 0; w < (T + 63) / 64; ++w) M = fmaxf(M, sm.red[0][w]);
    if (wave < (T + 63) / 64) {
        const float ws = xor_sum<1, 64>(ex2(z - finite_or_zero(M)));
        if (lane == 0) sm.red[1][wave] = ws;
    }
    __syncthreads();
    float Sz = 0.f;
#pragma unroll
    for (int w = 0; w < (T + 63) / 64; ++w) Sz += sm.red[1][w];
    const double lz2 = (double)(M + lg2(Sz)) + a.Oa[vb + h] + a.Ob[vb + h];
    if (!(lz2 > -1.0e300)) {  // no finite path: the exact kernel writes the zeros
        if (tid == 0) *failed = 1;
        return;
    }
    if (dir == 0 && p == 0 && tid == 0 && a.logZ) a.logZ[b] = (float)(lz2 * kLn2);

    // V_0: the vector both chains start from (normalised in the first pass: maximum 0) plus the growth of
    // the first pass's last step, which seeds both the normaliser and the shift of step 0.
    const int n = (dir == 0) ? L - 1 - h : h;  // number of positions this pair walks
    float seed = 0.f;
    if (dir == 0) seed = (float)(a.Oa[vb + h] - a.Oa[vb + h - 1]);  // h >= 1 as L >= 2
    else if (h + 1 < L) seed = (float)(a.Ob[vb + h] - a.Ob[vb + h + 1]);
    if (!(seed > -1.0e30f && seed < 1.0e30f)) seed = 0.f;
    const float* start = (dir == 0 ? a.ua : a.ub) + (vb + h) * T;
    if (tid < T) sm.vec[0][tid] = start[tid] + seed;
    if (wave == 0) {  // normaliser of V_0: maximum over partner 0's half
        float m = LCCRF_NEG_INF;
#pragma unroll
        for (int q = 0; q < NQ; ++q) m = fmaxf(m, start[lane + 64 * q] + seed);
        m = xor_max<1, 64>(m);
        if (lane == 0) {
            sm.dmax[0] = finite_or_zero(m);
            sm.dmax[1] = 0.f;
            sm.tot_own[0] = sm.tot_own[1] = sm.tot_oth[0] = sm.tot_oth[1] = 0.f;
        }
    }
    __syncthreads();
    const double O0 = (dir == 0 ? a.Oa[vb + h] : a.Ob[vb + h]) - (double)seed;

    if (!worker) {
        // ---------------- the i/o wave ----------------
        float dst = seed;
        for (int j = 0; j < n; ++j) {
            if (j > 0) {
                if (!receive_half<T>(sm, theirs, failed, (unsigned)j, lane, j & 1, p, a.poll_limit) && lane == 0)
                    sm.stop_go[(j - 1) & 1] = 1;
            }
            __syncthreads();  // B_j
            if (j > 0 && sm.stop_go[(j - 1) & 1] != 0) return;
            const float dnext = sm.dmax[j & 1];
            __syncthreads();  // A_j
            float r[NQ];
            bool bad = false;
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                if (dir == 0) {
                    float S = 0.f;
#pragma unroll
                    for (int w = 0; w < kPairWaves; ++w) S += sm.psum[j & 1][w][lane + 64 * q];
                    r[q] = dst + lg2(S);
                    bad = bad || !(S >= 0x1p-60f && S <= 0x1p60f);
                } else {
                    r[q] = sm.vec[(j + 1) & 1][p * H + lane + 64 * q];  // written by the owners of the rows
                }
            }
            bad = !__all(!bad) || sm.stop_req != 0;
            float tp = lane < kPairWaves ? sm.wtot[j & 1][lane] : 0.f;
            tp = xor_sum<1, 8>(tp);
            tp = __builtin_amdgcn_readfirstlane(tp);
            send_half<T>(mine, (unsigned)(j + 1), lane, r, tp, bad);
            float rm = LCCRF_NEG_INF;
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                if (dir == 0) sm.vec[(j + 1) & 1][p * H + lane + 64 * q] = r[q];
                rm = fmaxf(rm, r[q]);
            }
            if (p == 0) rm = xor_max<1, 64>(rm);
            if (lane == 0) {
                if (p == 0) sm.dmax[(j + 1) & 1] = finite_or_zero(rm);
                sm.tot_own[j & 1] = tp;
                sm.stop_go[j & 1] = bad ? 1 : 0;
            }
            dst = dnext;
        }
        // the backward chain's last vector is beta_0, of which position 0 needs both halves
        if (dir == 1 && n > 0 && sm.stop_go[(n - 1) & 1] == 0) {
            if (!receive_half<T>(sm, theirs, failed, (unsigned)n, lane, n & 1, p, a.poll_limit) && lane == 0)
                sm.stop_go[(n - 1) & 1] = 1;
        }
        __syncthreads();  // F
        return;
    }

    // ---------------- the eight working waves ----------------
    // Every thread holds, of each matrix, 2 x 4 potentials that meet this workgroup's own half of the vector
    // (ring index 0, 1) and 2 x 4 that meet the partner's half (index 2, 3).
    const int cg = tid % 16, rg = tid / 16;  // 16 lanes of four columns, 32 row groups
    float ring[kPairPF][4][4];
    float aux[kPairPF][4];
    double off[kPairPF];
    double O = O0;
    float kappa = 0.f;
    float dst = seed;

    if (dir == 0) {
        // forward chain: this workgroup owns the columns [p H, p H + H) and takes all rows; rows
        // p H + rg + 32 kk meet its own half of alpha, rows (1 - p) H + rg + 32 kk the partner's
        const int c4 = p * H + 4 * cg;
        int rowi[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) rowi[k] = ((k < 2) ? p : 1 - p) * H + rg + 32 * (k & 1);
        auto load = [&](int i, int slot) {
#pragma unroll
            for (int k = 0; k < 4; ++k)
                Elem<TIN>::get4_stream(phib + (size_t)i * TT + (size_t)rowi[k] * T + c4, ring[slot][k]);
            const float4 q = *reinterpret_cast<const float4*>(a.ub + (vb + i) * T + c4);
            aux[slot][0] = q.x; aux[slot][1] = q.y; aux[slot][2] = q.z; aux[slot][3] = q.w;
            off[slot] = a.Ob[vb + i];
        };
        const int first = h + 1;
#pragma unroll
        for (int s = 0; s < kPairPF; ++s) load(first + (s < n ? s : (n > 0 ? n - 1 : -1)), s);  // n = 0: position h, unused
        float vown[2] = {sm.vec[0][rowi[0]], sm.vec[0][rowi[1]]};
        int done = 0;
        bool running = n > 0;
        while (running) {
#pragma unroll
            for (int slot = 0; slot < kPairPF; ++slot) {
                const int i = first + done, cur = done & 1;
                O += (double)dst;
                const float K = (float)(O + off[slot] - lz2) + kappa;
                float gm[4], ls[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) gm[jj] = ex2(dst + aux[slot][jj] + K);
                float* mrow = mub + (size_t)i * TT + c4;
                const auto half_step = [&](int k0, const float (&v)[2]) {
#pragma unroll
                    for (int kk = 0; kk < 2; ++kk) {
                        const float uac = v[kk] - dst - dst;
                        float e[4];
#pragma unroll
                        for (int jj = 0; jj < 4; ++jj) {
                            e[jj] = ex2(__builtin_fmaf(ring[slot][k0 + kk][jj], kLog2e, uac));
                            ls[jj] += e[jj];
                        }
                        stream_store4(mrow + (size_t)rowi[k0 + kk] * T, e[0] * gm[0], e[1] * gm[1], e[2] * gm[2], e[3] * gm[3]);
                    }
                };
                half_step(0, vown);  // the rows of this workgroup's own half: nothing of the partner's needed
                __syncthreads();     // B: the partner's half of V_j is in shared memory
                if (done > 0 && sm.stop_go[cur ^ 1] != 0) {
                    if (tid == 0) __hip_atomic_store(failed, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    return;
                }
                const float voth[2] = {sm.vec[cur][rowi[2]], sm.vec[cur][rowi[3]]};
                half_step(2, voth);
                {   // refill this slot with the tile kPairPF positions ahead (clamped: always issued)
                    const int ahead = done + kPairPF;
                    load(first + (ahead < n ? ahead : n - 1), slot);
                }
                const float dnext = sm.dmax[cur];
                if (done > 0) {  // drift feedback from the step before the last (both parts known by now), half gain
                    const float tprev = (p == 0) ? sm.tot_own[cur ^ 1] + sm.tot_oth[cur ^ 1] : sm.tot_oth[cur ^ 1] + sm.tot_own[cur ^ 1];
                    kappa += (tprev > 0.5f && tprev < 2.0f) ? -0.5f * lg2(tprev) : 0.f;
                }
                float tl = (ls[0] * gm[0] + ls[1] * gm[1]) + (ls[2] * gm[2] + ls[3] * gm[3]);
                tl = xor_sum<1, 64>(tl);
                if (lane == 0) sm.wtot[cur][wave] = tl;
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) ls[jj] = xor_sum<16, 64>(ls[jj]);
                if (lane < 16) *reinterpret_cast<float4*>(&sm.psum[cur][wave][4 * cg]) = make_float4(ls[0], ls[1], ls[2], ls[3]);
                __syncthreads();  // A: every wave's partial sums are in shared memory
                // this workgroup's half of V_{j+1}, for the rows this thread needs first in the next step
#pragma unroll
                for (int kk = 0; kk < 2; ++kk) {
                    float S = 0.f;
#pragma unroll
                    for (int w = 0; w < kPairWaves; ++w) S += sm.psum[cur][w][rg + 32 * kk];
                    vown[kk] = dst + lg2(S);
                }
                dst = dnext;
                if (++done >= n) { running = false; break; }
            }
        }
        __syncthreads();  // F
        if (n > 0 && sm.stop_go[(n - 1) & 1] != 0 && tid == 0) __hip_atomic_store(failed, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {
        // backward chain: this workgroup owns the rows [p H, p H + H): rows p H + rg + 32 kk; their columns
        // p H + 4 cg .. meet its own half of beta (ring index 0, 1), columns (1 - p) H + 4 cg .. the partner's
        const int co = p * H + 4 * cg, cx = (1 - p) * H + 4 * cg;
        const int row0 = p * H + rg;
        auto load = [&](int i, int slot) {
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                const TIN* rowp = phib + (size_t)i * TT + (size_t)(row0 + 32 * kk) * T;
                Elem<TIN>::get4_stream(rowp + co, ring[slot][kk]);
                Elem<TIN>::get4_stream(rowp + cx, ring[slot][2 + kk]);
                aux[slot][kk] = a.ua[(vb + i - 1) * T + row0 + 32 * kk];
            }
            off[slot] = a.Oa[vb + i - 1];
        };
        const int first = h;  // positions h, h-1, ..., 1
#pragma unroll
        for (int s = 0; s < kPairPF; ++s) load(first - (s < n ? s : n - 1), s);
        int done = 0;
        bool running = true;
        while (running) {
#pragma unroll
            for (int slot = 0; slot < kPairPF; ++slot) {
                const int i = first - done, cur = done & 1;
                O += (double)dst;
                const float K = (float)(off[slot] + O - lz2) + kappa;
                float f[2], S[2] = {0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < 2; ++kk) f[kk] = ex2(dst + aux[slot][kk] + K);
                float tl = 0.f;
                float* mpos = mub + (size_t)i * TT;
                const auto half_step = [&](int k0, int c0) {
                    const float4 q4 = *reinterpret_cast<const float4*>(&sm.vec[cur][c0]);
                    const float ubc[4] = {q4.x - dst - dst, q4.y - dst - dst, q4.z - dst - dst, q4.w - dst - dst};
#pragma unroll
                    for (int kk = 0; kk < 2; ++kk) {
                        float e[4];
#pragma unroll
                        for (int jj = 0; jj < 4; ++jj) e[jj] = ex2(__builtin_fmaf(ring[slot][k0 + kk][jj], kLog2e, ubc[jj]));
                        const float Se = (e[0] + e[1]) + (e[2] + e[3]);
                        S[kk] += Se;
                        stream_store4(mpos + (size_t)(row0 + 32 * kk) * T + c0, e[0] * f[kk], e[1] * f[kk], e[2] * f[kk], e[3] * f[kk]);
                        tl += Se * f[kk];
                    }
                };
                half_step(0, co);  // the columns of this workgroup's own half of beta
                __syncthreads();   // B: the partner's half of V_j is in shared memory
                if (done > 0 && sm.stop_go[cur ^ 1] != 0) {
                    if (tid == 0) __hip_atomic_store(failed, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    return;
                }
                half_step(2, cx);
                {
                    const int ahead = done + kPairPF;
                    load(first - (ahead < n ? ahead : n - 1), slot);
                }
                const float dnext = sm.dmax[cur];
                if (done > 0) {
                    const float tprev = (p == 0) ? sm.tot_own[cur ^ 1] + sm.tot_oth[cur ^ 1] : sm.tot_oth[cur ^ 1] + sm.tot_own[cur ^ 1];
                    kappa += (tprev > 0.5f && tprev < 2.0f) ? -0.5f * lg2(tprev) : 0.f;
                }
                bool bad = false;
#pragma unroll
                for (int kk = 0; kk < 2; ++kk) {
                    const float Sk = xor_sum<1, 16>(S[kk]);
                    bad = bad || !(Sk >= 0x1p-60f && Sk <= 0x1p60f);
                    if (cg == 0) sm.vec[cur ^ 1][row0 + 32 * kk] = dst + lg2(Sk);
                }
                tl = xor_sum<1, 64>(tl);
                if (lane == 0) sm.wtot[cur][wave] = tl;
                if (!__all(!bad) && lane == 0) sm.stop_req = 1;
                __syncthreads();  // A: this workgroup's half of V_{j+1} is in shared memory
                dst = dnext;
                if (++done >= n) { running = false; break; }
            }
        }
        __syncthreads();  // F: the partner's half of beta_0 has arrived (or the pair has given up)
        if (sm.stop_go[(n - 1) & 1] != 0) {
            if (tid == 0) __hip_atomic_store(failed, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return;
        }
        // position 0: p(y_0 = t) = softmax_t(alpha_0(t) + beta_0(t)) in row 0, zeros elsewhere
        const int buf = n & 1;
        for (int k = T + p * kPairW + tid; k < (int)TT; k += 2 * kPairW) mub[k] = 0.f;
        if (p == 0 && wave == 0) {
            float m = LCCRF_NEG_INF;
            for (int t = lane; t < T; t += 64) m = fmaxf(m, a.ua[vb * T + t] + sm.vec[buf][t]);
            m = xor_max<1, 64>(m);
            float S = 0.f;
            for (int t = lane; t < T; t += 64) S += ex2(a.ua[vb * T + t] + sm.vec[buf][t] - finite_or_zero(m));
            S = xor_sum<1, 64>(S);
            const float cinv = S > 0.f ? 1.0f / S : 0.f;
            for (int t = lane; t < T; t += 64) mub[t] = cinv * ex2(a.ua[vb * T + t] + sm.vec[buf][t] - finite_or_zero(m));
        }
    }
}

size_t pair_mail_words(int B) { return (size_t)2 * B * 2 * 2 * kPairMailWords; }

bool pair_supported(int T) { return T == 128; }

hipError_t launch_pair_marginals(int dtype, const void* phi, const int32_t* lengths, int B, int N, int T,
                                 const float* ua, const float* ub, const double* Oa, const double* Ob,
                                 float* logZ, float* mu, unsigned long long* mail, int* failed, int poll_limit,
                                 hipStream_t st) {
    PairArgs a{phi, lengths, B, N, ua, ub, Oa, Ob, logZ, mu, mail, failed, poll_limit};
    const int chains = 2 * B;
    const int grid = ((chains + 7) / 8) * 16;
    if (T == 128) {
        if (dtype == 0)
            hipLaunchKernelGGL((pair_marginal_kernel<128, float>), dim3(grid), dim3(kPairThreads), 0, st, a);
        else
            hipLaunchKernelGGL((pair_marginal_kernel<128, uint16_t>), dim3(grid), dim3(kPairThreads), 0, st, a);
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace lccrf
