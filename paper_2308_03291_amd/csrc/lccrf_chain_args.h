// Arguments of the sum-product chain kernels and the stretch of positions one chain covers
// (shared by lccrf_chain.hip and lccrf_wave.hip).
#pragma once

#include "lccrf_device.h"

namespace lccrf {

struct ChainArgs {
    const void* phi;
    const int32_t* lengths;
    int B, N, T;
    float* ua;   // [B][N][T] normalised forward vectors (base-2 logs)
    float* ub;   // [B][N][T] normalised backward vectors
    double* Oa;  // [B][N] forward offsets:  alpha_i = (ua_i + Oa_i) * ln 2
    double* Ob;  // [B][N] backward offsets
    float* logZ;
    float* mu;
    int exact_only;  // 1: never take the speculative step (tests)
    const int* only_failed;  // second pass: if set, recompute only the sequences flagged here
    // Chunked schedule (chunk > 0): workgroup pair v serves chunk c = v % C of sequence v / C, the
    // tag positions [c chunk, (c+1) chunk), as a chain of its own that starts one position earlier
    // from the boundary vectors the scan has produced (lccrf_scan.hip).
    int chunk, C;
    const float* Fv;   // [B][C][T] alpha at the last position of each chunk, normalised
    const double* OF;  // [B][C] its offset
    const float* Gv;   // [B][C][T] beta at the last position of each chunk, normalised
    const double* OG;  // [B][C]
    // Scratch of the paired second pass, cleared by the first pass when it is going to be used
    // (null otherwise): pair_words 8-byte mailbox words and one failure flag per sequence.
    unsigned long long* pair_mail;
    int* pair_failed;
    int pair_words;
    double* logZ64;  // [B] or null: logZ in double precision (natural logarithm), for log-probabilities
    // Entropy mode (ha non-null, first pass only): the chains also carry the conditional entropy of
    // the path behind them given the current tag, and leave it here for the meeting position.
    float* ha;  // [B][T] H(y_0 .. y_{h-1} | y_h = t), base-2
    float* hb;  // [B][T] H(y_{h+1} .. y_{L-1} | y_h = t), base-2
    // Cross-entropy and KL divergence (psi non-null): ha and hb carry the conditional expectation of
    // the score under psi (of the score difference) instead, natural units, each less a common offset.
    const void* psi;  // potentials of the second chain, same layout and type as phi
    double* hoff;     // [B][2] the offsets of ha and hb
    // Entropy by edges (ent non-null, second pass of the one-wave kernels): no marginals are written, every
    // wave leaves the summed conditional entropies of its edges (base 2) in ent[2 (b C + c) + dir].
    float* ent;
    // What ent receives: 0 or 1 the entropy; 2 the expectation of the potentials psi under this chain's
    // marginals, sum_e mu(e) psi(e), in natural units; 3 that of psi - phi.
    int ent_kind;
    // Structured potentials (emit non-null; float only, T <= 64, whole sequences): phi is not read,
    // phi[b][i][s][t] = trans[s][t] + emit[b][i][t].
    const float* emit;   // [B][N][T]
    const float* trans;  // [T][T]
    // 1: the forward chain runs over the whole span and stores every alpha; no backward chain
    // (first pass of sampling, whose backward sweep needs alpha everywhere).
    int full_forward;
};

// The stretch of positions one pair of workgroups handles: all of a sequence, or one chunk.
struct Span {
    int b, c;
    int L;       // clamped length of the sequence
    int p0, e;   // first and last position of the chain (p0 carries the start vector)
    bool first;  // p0 is position 0: start from the first row of the first matrix
    bool last;   // e is the last position of the sequence: beta = 0 there
    bool empty;  // nothing to do
};

__device__ __forceinline__ Span make_span(const ChainArgs& a, int v) {
    Span s;
    if (a.chunk <= 0) {
        s.b = v; s.c = 0;
        s.L = clamp_length(a.lengths, s.b, a.N);
        s.p0 = 0; s.e = s.L - 1; s.first = true; s.last = true; s.empty = s.L == 0;
    } else {
        s.b = v / a.C; s.c = v % a.C;
        s.L = clamp_length(a.lengths, s.b, a.N);
        const int t0 = s.c * a.chunk;
        s.empty = t0 >= s.L;
        s.first = s.c == 0;
        s.p0 = s.first ? 0 : t0 - 1;
        const int t1 = t0 + a.chunk;
        s.e = (t1 < s.L ? t1 : s.L) - 1;
        s.last = s.e == s.L - 1;
    }
    return s;
}

// Where the forward and the backward chain of positions p0 .. e meet: the forward chain covers
// p0 .. h, the backward chain h .. e.  Every kernel of both passes derives it from here.
// (The middle: uneven splits were measured and lose more in the second pass than they gain in the first.)
__host__ __device__ __forceinline__ int meeting_point(int p0, int e) { return p0 + (e - p0 + 1) / 2; }
// Last position of the forward chain in a first pass: the meeting point, or the end of the span.
__device__ __forceinline__ int forward_end(const ChainArgs& a, int p0, int e) { return a.full_forward ? e : meeting_point(p0, e); }

// One-wave-per-chain kernels for T <= 32 (lccrf_wave.hip): one pass over all chains of `a`
// (a.C = 1 for whole sequences).  The first pass stores the vectors of both half chains, the
// second writes the marginals.  dtype 0: float, 1: bfloat16.
bool wave_supported(int T);
hipError_t launch_wave_pass(bool second_pass, int dtype, const ChainArgs& a, hipStream_t st);
// Chunked schedule with chunks short enough (wave_chunks_fused): both passes of every chunk in one
// launch, one workgroup of two waves per chunk, the chunk's vectors in LDS (ua, ub, Oa, Ob unused).
hipError_t launch_wave_logz(int dtype, const ChainArgs& a, hipStream_t st);  // whole sequences, logZ only, one launch
bool wave_chunks_fused(int chunk);
// Row-batch kernels for 128 < T <= 256 (lccrf_stream.hip): one pass over whole sequences, vectors and
// marginals exactly as launch_wave_pass.
bool stream_supported(int T);
hipError_t launch_stream_pass(bool second_pass, int dtype, const ChainArgs& a, hipStream_t st);
// The first pass in an expectation mode at those tag counts (0: entropy, a.ha / a.hb; 1: cross-entropy,
// 2: KL divergence, with a.psi and a.hoff), leaving what entropy_half_kernel leaves (lccrf_extras.hip).
hipError_t launch_stream_expect(int mode, int dtype, const ChainArgs& a, hipStream_t st);
hipError_t launch_wave_chunks(int dtype, const ChainArgs& a, hipStream_t st);
// One chain wave and six producer waves per half chain (lccrf_lane.hip): plain potentials, whole
// sequences, 8 <= T <= 64 in multiples of four.  One pass over all sequences of `a`, vectors and marginals
// exactly as launch_wave_pass; meet_only: a first pass that stores the vectors of the meeting position only;
// poll_limit: how many times the chain wave looks for a matrix that is late before it goes on alone.
bool lane_supported(int T);
hipError_t launch_lane_pass(bool second_pass, int dtype, const ChainArgs& a, bool meet_only, int poll_limit, hipStream_t st);

}  // namespace lccrf
