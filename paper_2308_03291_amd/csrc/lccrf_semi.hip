// Semi-Markov CRF, log-partition (paper, section "Segmentation with Semi-Markov CRF": the linear
// chain's transition-matrix parametrisation, except that a transition may jump over several
// positions; forward algorithm in O(K T^2 L) for segments of at most K positions).
//
// phi[b][i][k][s][t]: log-potential of a segment tagged t that ends at position i and covers
// k + 1 positions, after a segment tagged s (row 0 for the first segment).  The forward step
//     alpha_i(t) = logsumexp over k = 0 .. min(K-1, i) and s of  alpha_{i-k-1}(s) + phi[i][k][s][t]
// is a vector-matrix product in the log semiring whose matrix is the (K T) x T block phi[b][i]
// (contiguous in memory) and whose vector is the last K alphas laid end to end.  One workgroup per
// sequence keeps those K vectors in LDS (a ring, each with a double-precision offset of its own)
// and streams the block through registers in batches of rows (every batch within one or a few of
// the K matrices, so which earlier vector it meets is the same for all threads), prefetched across
// step boundaries: the loads of a step do not depend on the step before it.  Per column a thread keeps a running
// maximum and a sum rescaled to it (exact log-sum-exp in one read), the partial results meet in
// LDS, and the new vector replaces the oldest one.
#include "lccrf_device.h"
#include "lccrf_launch.h"

namespace lccrf {

struct SemiArgs {
    const void* phi;
    const int32_t* lengths;
    int B, N, K, T;
    float* logZ;
};

constexpr int kSemiItems = 4;  // rows of a batch held by one thread
constexpr int kSemiPF = 3;     // batches in flight

// LDS: base[K] doubles (padded to an even count), ring[K][T] floats (padded to a multiple of 4), pmax and
// psum [WAVES][4 LPR]: every part starts on a 16-byte boundary.
static size_t semi_lds_bytes(int K, int T, int lpr, int waves) {
    const size_t ring = ((size_t)K * T + 3) / 4 * 4;
    return (size_t)((K + 1) / 2 * 2) * sizeof(double) + ring * sizeof(float) + (size_t)2 * waves * 4 * lpr * sizeof(float) + 16;
}

template <int LPR, int WAVES, typename TIN, bool ALIGNED>
__global__ __launch_bounds__(64 * WAVES) void semi_forward_kernel(SemiArgs a) {
    constexpr int W = 64 * WAVES, RPP = W / LPR, CAP = 4 * LPR, ITEMS = kSemiItems, PF = kSemiPF;
    // One pass of the workgroup covers RPP rows (thread: row r0, columns c4 .. c4+3): a part of one
    // T x T matrix, PPT passes covering it (RPP <= CAP), or TPP whole matrices of consecutive segment
    // lengths (RPP > CAP).  A batch is ITEMS passes.  Which row of its matrix a thread holds in
    // pass p, and which segment length that matrix belongs to, follow from p alone.
    constexpr int PPT = CAP / RPP > 0 ? CAP / RPP : 1, TPP = RPP / CAP > 0 ? RPP / CAP : 1;
    static_assert((PPT * RPP == CAP || TPP * CAP == RPP) && (PPT == 1 || PPT == 4 || PPT == 16) && ITEMS == 4, "geometry");
    extern __shared__ __attribute__((aligned(16))) unsigned char semi_smem[];
    const int K = a.K, T = a.T, N = a.N;
    const int KT = K * T;
    double* base = reinterpret_cast<double*>(semi_smem);
    float* ring = reinterpret_cast<float*>(base + (K + 1) / 2 * 2);
    float* pmax = ring + (KT + 3) / 4 * 4;
    float* psum = pmax + WAVES * CAP;
    float* dlast = psum + WAVES * CAP;  // maximum of the newest vector (T <= 64)

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b = blockIdx.x;
    const int L = clamp_length(a.lengths, b, N);
    if (L == 0) {
        if (tid == 0) a.logZ[b] = 0.f;
        return;
    }
    const int c4 = 4 * (tid % LPR), r0 = (tid / LPR) % CAP, k0 = (tid / LPR) / CAP;  // k0 = 0 unless TPP > 1
    const size_t TT = (size_t)T * T;
    const TIN* phib = static_cast<const TIN*>(a.phi) + (size_t)b * N * K * TT;
    const int nb = ((K + TPP - 1) / TPP * PPT + ITEMS - 1) / ITEMS;  // batches per position
    const int total = L * nb;

    // The empty prefix sits in the slot "position -1": potential 1 for row 0, nothing else.
    for (int k = tid; k < KT; k += W) ring[k] = LCCRF_NEG_INF;
    for (int k = tid; k < K; k += W) base[k] = 0.0;
    __syncthreads();
    if (tid == 0) {
        ring[(K - 1) * T] = 0.f;
        *dlast = 0.f;
    }
    __syncthreads();

    float tile[PF][ITEMS][4];
    int li = 0, lbt = 0;  // position and batch of the next load
    auto load = [&](int q, int slot) {
        const TIN* mat = phib + (size_t)li * K * TT;
#pragma unroll
        for (int m = 0; m < ITEMS; ++m) {
            const int p = ITEMS * lbt + m;
            const int k = (p / PPT) * TPP + k0, s = r0 + (p % PPT) * RPP;
            const TIN* matk = mat + (size_t)(k < K ? k : K - 1) * TT;
            if (ALIGNED) {
                const TIN* row = matk + (size_t)(s < T ? s : T - 1) * T;
                Elem<TIN>::get4(row + (c4 < T ? c4 : T - 4), tile[slot][m]);
            } else if ((b != a.B - 1 || li != N - 1) && T > 1) {  // (matrices of a later position lie behind these)
                load_row4_anywhere<TIN, true>(matk, T, s, c4, tile[slot][m]);
            } else {
                load_row4_anywhere<TIN, false>(matk, T, s, c4, tile[slot][m]);
            }
        }
        if (q < total - 1 && ++lbt == nb) {
            lbt = 0;
            ++li;
        }
    };

    int i = 0, bt = 0;  // position and batch being consumed
    int cur = K - 1;    // ring slot of position i - 1
    double R = 0.0;     // offset the new vector is relative to
    float mx[4], sm[4];
    walk<PF>(0, total - 1, +1, load, [&](int, int slot) {
        if (bt == 0) {
            // The newest vector is stored as it came out of its step; its maximum (found by the threads
            // that formed it, or here by every thread when they span several waves) moves into the
            // offset of the vector being formed.
            float d;
            if constexpr (CAP <= 64) {
                d = *dlast;
            } else {
                d = LCCRF_NEG_INF;
                for (int t = lane; t < T; t += 64) d = fmaxf(d, ring[cur * T + t]);
                d = finite_or_zero(xor_max<1, 64>(d));
            }
            R += (double)d;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                mx[j] = LCCRF_NEG_INF;
                sm[j] = 0.f;
            }
        }
        float x[ITEMS][4];
        float bm[4] = {LCCRF_NEG_INF, LCCRF_NEG_INF, LCCRF_NEG_INF, LCCRF_NEG_INF};
#pragma unroll
        for (int m = 0; m < ITEMS; ++m) {
            const int p = ITEMS * bt + m;
            const int k = (p / PPT) * TPP + k0, s = r0 + (p % PPT) * RPP;
            // a segment of k + 1 positions ending at i starts at i - k >= 0; the first segment reads row 0 only
            const bool row_ok = k < K && s < T && (k < i || (k == i && s == 0));
            int sl = cur - (k < K ? k : K - 1);  // ring slot of position i - 1 - k
            if (sl < 0) sl += K;
            // read whatever the row is (the address is inside the ring either way) and decide
            // afterwards: the reads of all rows of the batch are then in flight together
            float rv = ring[sl * T + (s < T ? s : T - 1)];
            asm volatile("" : "+v"(rv));
            const float v = rv + (float)(base[sl] - R);
            if constexpr (!ALIGNED) settle_row4(tile[slot][m], T, c4);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                x[m][j] = row_ok ? __builtin_fmaf(tile[slot][m][j], kLog2e, v) : LCCRF_NEG_INF;
                bm[j] = fmaxf(bm[j], x[m][j]);
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float mn = fmaxf(mx[j], bm[j]);
            const float mf = finite_or_zero(mn);
            float acc = sm[j] * ex2(mx[j] - mf);
#pragma unroll
            for (int m = 0; m < ITEMS; ++m) acc += ex2(x[m][j] - mf);
            sm[j] = acc;
            mx[j] = mn;
        }
        if (++bt == nb) {
            float M[4], S[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                M[j] = xor_max<LPR, 64>(mx[j]);
                S[j] = xor_sum<LPR, 64>(sm[j] * ex2(mx[j] - finite_or_zero(M[j])));
            }
            if (lane < LPR) {
                *reinterpret_cast<float4*>(&pmax[wave * CAP + c4]) = make_float4(M[0], M[1], M[2], M[3]);
                *reinterpret_cast<float4*>(&psum[wave * CAP + c4]) = make_float4(S[0], S[1], S[2], S[3]);
            }
            __syncthreads();  // every thread has read the ring for this position
            const int nxt = cur + 1 == K ? 0 : cur + 1;
            float rnew = LCCRF_NEG_INF;
            if (tid < T) {
                float Mt = LCCRF_NEG_INF;
#pragma unroll
                for (int w = 0; w < WAVES; ++w) Mt = fmaxf(Mt, pmax[w * CAP + tid]);
                const float mf = finite_or_zero(Mt);
                float St = 0.f;
#pragma unroll
                for (int w = 0; w < WAVES; ++w) St += psum[w * CAP + tid] * ex2(pmax[w * CAP + tid] - mf);
                rnew = Mt + lg2(St);  // no term at all: -inf
                ring[nxt * T + tid] = rnew;
            }
            if (CAP <= 64 && wave == 0) {  // T <= 64: all of the new vector is in wave 0
                const float d = xor_max<1, 64>(rnew);
                if (lane == 0) *dlast = finite_or_zero(d);
            }
            if (tid == 0) base[nxt] = R;
            __syncthreads();
            cur = nxt;
            bt = 0;
            ++i;
        }
    });

    // logZ = logsumexp of the vector of the last position
    if (wave == 0) {
        float d = LCCRF_NEG_INF;
        for (int t = lane; t < T; t += 64) d = fmaxf(d, ring[cur * T + t]);
        d = xor_max<1, 64>(d);
        float S = 0.f;
        for (int t = lane; t < T; t += 64) S += ex2(ring[cur * T + t] - finite_or_zero(d));
        S = xor_sum<1, 64>(S);
        if (lane == 0) a.logZ[b] = (d == LCCRF_NEG_INF) ? LCCRF_NEG_INF : (float)((base[cur] + (double)d + (double)lg2(S)) * kLn2);
    }
}

template <int LPR, int WAVES>
static hipError_t launch_semi_geo(int dtype, const SemiArgs& a, hipStream_t st) {
    const size_t lds = semi_lds_bytes(a.K, a.T, LPR, WAVES);
    const bool aligned = (a.T % 4) == 0;
    const dim3 grid(a.B), block(64 * WAVES);
    if (dtype == 0) {
        if (aligned) hipLaunchKernelGGL((semi_forward_kernel<LPR, WAVES, float, true>), grid, block, lds, st, a);
        else hipLaunchKernelGGL((semi_forward_kernel<LPR, WAVES, float, false>), grid, block, lds, st, a);
    } else {
        if (aligned) hipLaunchKernelGGL((semi_forward_kernel<LPR, WAVES, uint16_t, true>), grid, block, lds, st, a);
        else hipLaunchKernelGGL((semi_forward_kernel<LPR, WAVES, uint16_t, false>), grid, block, lds, st, a);
    }
    return hipGetLastError();
}

// Geometry by tag count: 4 LPR >= T columns; four waves up to T = 64 (one when T <= 16 and the K
// matrices have no more rows than one wave covers in a batch), sixteen above.
static void semi_geometry(int K, int T, int& lpr, int& waves) {
    lpr = T <= 16 ? 4 : T <= 32 ? 8 : T <= 64 ? 16 : T <= 128 ? 32 : 64;
    waves = T <= 16 ? (K <= 4 ? 1 : 4) : T <= 64 ? 4 : 16;
}

// The K vectors must fit the 64 KB of LDS a workgroup may take without opting in to more.
bool semi_markov_supported(int K, int T) {
    if (K < 1 || T < 1 || T > 256) return false;
    int lpr, waves;
    semi_geometry(K, T, lpr, waves);
    return semi_lds_bytes(K, T, lpr, waves) <= 64 * 1024 && K <= (1 << 24);
}

hipError_t launch_semi_markov_forward(int dtype, const void* phi, const int32_t* lengths, int B, int N, int K, int T,
                                      float* logZ, hipStream_t st) {
    const SemiArgs a{phi, lengths, B, N, K, T, logZ};
    if (T <= 16) return K <= 4 ? launch_semi_geo<4, 1>(dtype, a, st) : launch_semi_geo<4, 4>(dtype, a, st);
    if (T <= 32) return launch_semi_geo<8, 4>(dtype, a, st);
    if (T <= 64) return launch_semi_geo<16, 4>(dtype, a, st);
    if (T <= 128) return launch_semi_geo<32, 16>(dtype, a, st);
    return launch_semi_geo<64, 16>(dtype, a, st);
}

}  // namespace lccrf
