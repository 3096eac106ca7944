// Max-plus (Viterbi) chain for the linear-chain CRF: the recursion of the forward
// algorithm with (max, +) in place of (logsumexp, +), as the paper's section "Computing
// Most Probable Structure" prescribes, followed by the back-trace that reads off the path.
//
// delta is carried in double precision and never rescaled: max-plus needs only additions and
// comparisons, both run at the full vector rate in fp64 on this chip, and every candidate
// delta_{i-1}(s) + phi_i(s,t) is then one correctly rounded fp64 addition of exactly
// representable inputs, whichever thread forms it.  Ties go to the smaller previous tag.
#include "lccrf_device.h"
#include "lccrf_launch.h"

namespace lccrf {

constexpr int kNoArg = 0x7fffffff;
constexpr int kTraceBytes = 16384;  // LDS window of back-pointers walked by the back-trace

template <typename G>
struct VitSmem {
    union {
        struct {
            double pv[G::WAVES][G::TCAP];  // per-wave best candidate per column
            int pi[G::WAVES][G::TCAP];     // and its previous tag
        } f;
        uint8_t window[kTraceBytes];
    } u;
    double dvec[2][G::TCAP];
    double best;
    int last;
};

__device__ __forceinline__ void take_better(double& v, int& a, double pv, int pa) {
    if (pv > v || (pv == v && pa < a)) { v = pv; a = pa; }
}

struct VitArgs {
    const void* phi;
    const int32_t* lengths;
    int B, N, T;
    uint8_t* bp;  // [B][N][T]
    float* best_score;
    int32_t* tags;
    // Chunked schedule (chunk > 0): workgroup v serves chunk c = v % C of sequence v / C, the tag
    // positions [c chunk, (c+1) chunk), as a chain of its own that starts one position earlier in
    // the tag pin[b][c-1] and must end in the tag pin[b][c] (both chosen by the max-plus scan,
    // lccrf_scan.hip); the best score is the scan's and is not written here.
    int chunk, C;
    const int32_t* pin;  // [B][C] tag at the last position of each chunk
};

template <typename G, typename TIN, bool ALIGNED>
__global__ __launch_bounds__(G::W) void viterbi_kernel(VitArgs a) {
    __shared__ VitSmem<G> sm;
    constexpr int ITEMS = G::ITEMS;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const bool chunked = a.chunk > 0;
    const int b = chunked ? blockIdx.x / a.C : blockIdx.x;
    const int c = chunked ? blockIdx.x % a.C : 0;
    const int N = a.N, T = a.T;
    const int L = clamp_length(a.lengths, b, N);
    int32_t* tags = a.tags + (size_t)b * N;
    // this workgroup's stretch of tag positions [t0, t1), cut at the length: first position p0
    // (carries the start vector) and last position e of its chain
    const int t0 = chunked ? c * a.chunk : 0;
    const int t1 = chunked ? (t0 + a.chunk < N ? t0 + a.chunk : N) : N;
    for (int i = (L > t0 ? L : t0) + tid; i < t1; i += G::W) tags[i] = -1;
    if (L == 0) {
        if (!chunked && tid == 0 && a.best_score) a.best_score[b] = 0.f;
        return;
    }
    if (t0 >= L) return;
    const int p0 = t0 > 0 ? t0 - 1 : 0;
    const int e = (t1 < L ? t1 : L) - 1;
    const int c4 = 4 * (tid % G::LPR), r0 = tid / G::LPR;
    const size_t TT = (size_t)T * T;
    const TIN* phib = static_cast<const TIN*>(a.phi) + (size_t)b * N * TT;
    uint8_t* bpb = a.bp + (size_t)b * N * T;
    const double ninf = -__builtin_huge_val();

    for (int k = tid; k < 2 * G::TCAP; k += G::W) (&sm.dvec[0][0])[k] = ninf;
    __syncthreads();
    if (tid < T) {
        if (t0 == 0) sm.dvec[0][tid] = (double)Elem<TIN>::get(phib + tid);
        else sm.dvec[0][tid] = (tid == a.pin[(size_t)b * a.C + c - 1]) ? 0.0 : ninf;
    }
    __syncthreads();

    int buf = 0;
    float A[ITEMS][4], Bq[ITEMS][4];
    auto step = [&](int i, float (&v)[ITEMS][4]) {
        mask_tile<G>(v, T, c4, r0);
        double best[4] = {ninf, ninf, ninf, ninf};
        int arg[4] = {kNoArg, kNoArg, kNoArg, kNoArg};
#pragma unroll
        for (int k = 0; k < ITEMS; ++k) {
            const int s = r0 + k * G::RPP;
            const double dk = (s < T) ? sm.dvec[buf][s] : ninf;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const double val = dk + (double)v[k][j];
                if (val > best[j]) { best[j] = val; arg[j] = s; }
            }
        }
#pragma unroll
        for (int off = G::LPR; off < 64; off <<= 1) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const double pv = __shfl_xor(best[j], off, 64);
                const int pa = __shfl_xor(arg[j], off, 64);
                take_better(best[j], arg[j], pv, pa);
            }
        }
        if (lane < G::LPR) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                sm.u.f.pv[wave][c4 + j] = best[j];
                sm.u.f.pi[wave][c4 + j] = arg[j];
            }
        }
        __syncthreads();
        if (tid < G::TCAP) {
            double bv = ninf;
            int ba = kNoArg;
#pragma unroll
            for (int w = 0; w < G::WAVES; ++w) take_better(bv, ba, sm.u.f.pv[w][tid], sm.u.f.pi[w][tid]);
            sm.dvec[buf ^ 1][tid] = bv;
            if (tid < T) bpb[(size_t)i * T + tid] = (uint8_t)(ba == kNoArg ? 0 : ba);
        }
        __syncthreads();
        buf ^= 1;
    };
    int i = p0 + 1;
    if (i <= e) load_tile<G, TIN, ALIGNED>(phib + (size_t)i * TT, T, c4, r0, A);
    while (i <= e) {
        if (i + 1 <= e) load_tile<G, TIN, ALIGNED>(phib + (size_t)(i + 1) * TT, T, c4, r0, Bq);
        step(i, A);
        if (++i > e) break;
        if (i + 1 <= e) load_tile<G, TIN, ALIGNED>(phib + (size_t)(i + 1) * TT, T, c4, r0, A);
        step(i, Bq);
        ++i;
    }

    if (chunked) {
        if (tid == 0) sm.last = a.pin[(size_t)b * a.C + c];
    } else if (wave == 0) {
        // best final tag: first maximum of delta_{L-1}
        double bv = ninf;
        int ba = kNoArg;
        for (int t = lane; t < T; t += 64) {
            const double val = sm.dvec[buf][t];
            if (val > bv) { bv = val; ba = t; }
        }
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const double pv = __shfl_xor(bv, off, 64);
            const int pa = __shfl_xor(ba, off, 64);
            take_better(bv, ba, pv, pa);
        }
        if (lane == 0) {
            sm.best = bv;
            sm.last = (ba == kNoArg) ? 0 : ba;
            if (a.best_score) a.best_score[b] = (float)bv;
        }
    }
    __threadfence();  // back-pointers written above are read back below by other threads
    __syncthreads();

    // back-trace: y_{i-1} = bp_i(y_i), walked through an LDS window of back-pointers
    // (a chunk leaves the tag of its entry position p0 to the chunk that ends there)
    const int rows_per_window = kTraceBytes / T;
    int y = sm.last;
    if (tid == 0) tags[e] = y;
    const int stop = t0 == 0 ? 1 : t0 + 1;  // rows [stop, hi) still to walk; row r yields tag r - 1
    int hi = e + 1;
    while (hi > stop) {
        const int lo = (hi - rows_per_window > stop) ? hi - rows_per_window : stop;
        const int nbytes = (hi - lo) * T;
        const uint8_t* src = bpb + (size_t)lo * T;
        for (int k = tid; k < nbytes; k += G::W) sm.u.window[k] = src[k];
        __syncthreads();
        if (tid == 0) {
            for (int r = hi - 1; r >= lo; --r) {
                y = sm.u.window[(r - lo) * T + y];
                tags[r - 1] = y;
            }
        }
        __syncthreads();
        hi = lo;
    }
}

template <typename G, typename TIN, bool ALIGNED>
static hipError_t launch_geo(const VitArgs& a, hipStream_t st) {
    hipLaunchKernelGGL((viterbi_kernel<G, TIN, ALIGNED>), dim3(a.B * a.C), dim3(G::W), 0, st, a);
    return hipGetLastError();
}

template <typename TIN, bool ALIGNED>
static hipError_t launch_T(const VitArgs& a, hipStream_t st) {
    const int T = a.T;
    if (T <= 4) return launch_geo<Geo<1, 1, 1>, TIN, ALIGNED>(a, st);
    if (T <= 8) return launch_geo<Geo<2, 1, 1>, TIN, ALIGNED>(a, st);
    if (T <= 16) return launch_geo<Geo<4, 1, 1>, TIN, ALIGNED>(a, st);
    if (T <= 32) return launch_geo<Geo<8, 4, 1>, TIN, ALIGNED>(a, st);
    if (T <= 64) return launch_geo<Geo<16, 4, 4>, TIN, ALIGNED>(a, st);
    if (T <= 128) return launch_geo<Geo<32, 16, 4>, TIN, ALIGNED>(a, st);
    return launch_geo<Geo<64, 16, 16>, TIN, ALIGNED>(a, st);
}

hipError_t launch_sequential_max(int dtype, const void* phi, const int32_t* lengths, int B, int N, int T,
                                 uint8_t* bp, float* best_score, int32_t* tags, hipStream_t st) {
    VitArgs a{phi, lengths, B, N, T, bp, best_score, tags, 0, 1, nullptr};
    const bool aligned = (T % 4) == 0;
    if (dtype == 0) return aligned ? launch_T<float, true>(a, st) : launch_T<float, false>(a, st);
    return aligned ? launch_T<uint16_t, true>(a, st) : launch_T<uint16_t, false>(a, st);
}

// Best path inside every chunk between the tags the max-plus scan has pinned at the chunk ends.
hipError_t launch_chunked_max(int dtype, const void* phi, const int32_t* lengths, int B, int N, int T, uint8_t* bp,
                              int32_t* tags, int chunk, const int32_t* pin, hipStream_t st) {
    VitArgs a{phi, lengths, B, N, T, bp, nullptr, tags, chunk, (N + chunk - 1) / chunk, pin};
    const bool aligned = (T % 4) == 0;
    if (dtype == 0) return aligned ? launch_T<float, true>(a, st) : launch_T<float, false>(a, st);
    return aligned ? launch_T<uint16_t, true>(a, st) : launch_T<uint16_t, false>(a, st);
}

}  // namespace lccrf
