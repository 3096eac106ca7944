// Host-side launch entry points of the kernel translation units (internal to the library).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace lccrf {

// Sum-product chains, position by position.  op 0: logZ only; op 1: marginals (+ logZ if
// non-null).  dtype 0: float, 1: bfloat16.  ua/ub: [B][N][T] floats, Oa/Ob: [B][N] doubles of
// scratch.  Enqueues on `st`; returns the launch status.
// `between`, if non-null, is recorded on `st` after the first pass.  exact_only: skip the
// speculative uniform-shift step and run the exact step at every position.
// mail / failed: scratch of the paired second pass (pair_mail_words(B) 8-byte words and B ints),
// or null to always use one workgroup per chain; pair_poll_limit: how many polls a paired workgroup
// waits for its partner before the sequence goes to the one-workgroup kernel; cus: compute units of
// the device the stream belongs to (pairs are used when they fit the chip all at once).
hipError_t launch_sequential_sum(int op, int dtype, const void* phi, const int32_t* lengths, int B, int N, int T,
                                 float* ua, float* ub, double* Oa, double* Ob, float* logZ, float* mu,
                                 hipStream_t st, hipEvent_t between = nullptr, bool exact_only = false,
                                 unsigned long long* mail = nullptr, int* failed = nullptr, double* logZ64 = nullptr,
                                 const float* emit = nullptr, const float* trans = nullptr, int pair_poll_limit = 0,
                                 int cus = 0, bool lanes = false, int lane_poll_limit = 1 << 16);
// lanes: the chain-wave / producer-wave kernels of lccrf_lane.hip (lane_chains_supported(T); dense or structured potentials);
// lane_poll_limit: polls their chain wave spends on a late matrix before it continues in the log domain.
bool lane_chains_supported(int T);
// Sampling (lccrf_chain.hip, lccrf_extras.hip): forward chains over whole sequences with every alpha
// stored, then the backward sweep that draws the tags from the given uniforms [B][N].
hipError_t launch_full_forward(int dtype, const void* phi, const int32_t* lengths, int B, int N, int T, float* ua,
                               float* ub, double* Oa, double* Ob, hipStream_t st);
size_t sample_winmap_bytes(int B, int N, int T);
// uniforms null: drawn by the counter-based generator under `seed` instead (lccrf_extras.hip, Uniforms).
hipError_t launch_backward_sample(int dtype, const void* phi, const int32_t* lengths, const float* ua, const double* Oa,
                                  const float* uniforms, unsigned long long seed, int B, int N, int T, uint8_t* F,
                                  uint8_t* winmap, int32_t* tags, hipStream_t st);
// The forward pass of sampling under the chunked scan: every chunk's forward chain over its whole span from
// the boundary vectors Fv / OF, every alpha stored (T <= 32).
hipError_t launch_chunked_full_forward(int dtype, const void* phi, const int32_t* lengths, int B, int N, int T,
                                       float* ua, float* ub, double* Oa, double* Ob, int chunk, const float* Fv,
                                       const double* OF, hipStream_t st);
// Structured potentials (emit [B][N][T] + trans [T][T], float, phi unused) are served for these T.
bool structured_supported(int T);

// Paired second pass (two workgroups per chain; lccrf_pair.hip).
size_t pair_mail_words(int B);
bool pair_supported(int T);
hipError_t launch_pair_marginals(int dtype, const void* phi, const int32_t* lengths, int B, int N, int T,
                                 const float* ua, const float* ub, const double* Oa, const double* Ob,
                                 float* logZ, float* mu, unsigned long long* mail, int* failed, int poll_limit,
                                 hipStream_t st);

// Chunked scan over positions (lccrf_scan.hip), tag sets of at most 32 (TP = 16 or 32 padded tags).  Writes, per chunk of `chunk`
// positions (C = ceil(N / chunk) chunks per sequence), the chunk's transfer matrix (Pl: TP^2 floats, rel: TP
// floats, base: 1 double) and alpha / beta at the chunk's last position (Fv, Gv: T floats; OF, OG: 1
// double), and logZ if non-null.  with_beta false: forward vectors and logZ only.
// With many chunks the serial pass over chunks is itself split into groups of scan_group_size(C) chunks
// (0: not split); the group-level copies of the arrays above ([B][G], G = ceil(C / group size)) live in gb.
bool scan_supported(int T);      // sum queries (T <= 32)
bool scan_supported_max(int T);
int scan_padded_tags_max(int T);  // 16 or 32: the side of the max-plus scan's chunk matrices  // lccrf_argmax (T <= 16)
int scan_padded_tags(int T);     // 16 or 32: side of the stored chunk matrices
int scan_group_size(int C);
struct ScanGroupBuffers {
    float* Pl2;
    float* rel2;
    double* base2;
    float* Fv2;
    double* OF2;
    float* Gv2;
    double* OG2;
};
hipError_t launch_scan_boundaries(int dtype, const void* phi, const int32_t* lengths, int B, int N, int T, int chunk,
                                  float* Pl, float* rel, double* base, float* Fv, double* OF, float* Gv, double* OG,
                                  const ScanGroupBuffers& gb, float* logZ, bool with_beta, hipStream_t st,
                                  double* logZ64 = nullptr, const float* emit = nullptr, const float* trans = nullptr);
// emit non-null: structured potentials trans + emit (dtype 0; phi is not read), here and in the launchers below.

// log p(y) = score(y) - logZ for one tag path per sequence (lccrf_extras.hip); logZ64: [B] doubles
// already computed on the same stream.
hipError_t launch_path_log_prob(int dtype, const void* phi, const int32_t* lengths, const int32_t* tags, int B, int N,
                                int T, const double* logZ64, float* out, hipStream_t st);
// Two-pass forward-backward inside every chunk from those boundary vectors (lccrf_chain.hip); chunk >= 4.
hipError_t launch_chunked_marginals(int dtype, const void* phi, const int32_t* lengths, int B, int N, int T,
                                    float* ua, float* ub, double* Oa, double* Ob, float* mu, int chunk,
                                    const float* Fv, const double* OF, const float* Gv, const double* OG,
                                    hipStream_t st, hipEvent_t between, bool exact_only, float* ent = nullptr,
                                    const void* psi = nullptr, bool difference = false, const float* emit = nullptr,
                                    const float* trans = nullptr);
// ent non-null (T <= 32): the second pass writes no marginals (mu may be null) but the summed conditional
// entropies of every chunk's edges, [B][C][2] floats (base 2); launch_entropy_reduce adds them up to H [B].
// logZ: [B] floats from the boundary pass of the same run (-inf: no finite path, H is NaN).
hipError_t launch_entropy_reduce(const float* ent, const int32_t* lengths, const float* logZ, int B, int N, int chunk,
                                 float* H, hipStream_t st);
// ent and psi non-null: ent receives the expectation of the potentials psi (same layout and type as phi) under
// the chain of phi instead, sum_e mu(e) psi(e) over every chunk's edges in natural units, or that of psi - phi
// (difference).  launch_cross_reduce turns the sums into the cross-entropy logZq - E (logZp = the chain's own
// log-partition, only looked at for -inf: no finite path, NaN) or, with kl, into the Kullback-Leibler
// divergence logZq - logZp - E of the difference; both log-partitions [B] doubles, natural logarithm.
hipError_t launch_cross_reduce(bool kl, const float* ent, const int32_t* lengths, const double* logZq, const double* logZp,
                               int B, int N, int chunk, float* out, hipStream_t st);

// Max-plus chains (two per sequence, meeting in the middle) and the trace.  bp: [B][N][T] bytes,
// mid: viterbi_mid_doubles(B, 1, T) doubles of scratch.
size_t viterbi_mid_doubles(int B, int C, int T);
// lanes: the chains by a chain wave and helper waves (lccrf_lane_max.hip; lane_max_supported(T)), whose bounded
// waits take lane_poll_limit looks.
bool lane_max_supported(int T);
hipError_t launch_sequential_max(int dtype, const void* phi, const int32_t* lengths, int B, int N, int T,
                                 uint8_t* bp, double* mid, float* best_score, int32_t* tags, hipStream_t st,
                                 bool lanes = false, int lane_poll_limit = 1 << 16);

hipError_t launch_structured_max(const float* emit, const float* trans, const int32_t* lengths, int B, int N, int T,
                                 uint8_t* bp, double* mid, float* best_score, int32_t* tags, hipStream_t st,
                                 bool lanes = false, int lane_poll_limit = 1 << 16);

// Max-plus chunked scan (lccrf_scan.hip): the best score and the tag of the best path at the last
// position of every chunk (pin: [B][C] ints).  Mx: [B][C][256] doubles, K: [B][C][16] bytes of scratch.
struct MaxGroupBuffers {  // group level of the max-plus scan ([B][G]; many chunks only)
    double* Mx2;
    uint8_t* K2;
    int32_t* pin2;
};
hipError_t launch_scan_pins(int dtype, const void* phi, const int32_t* lengths, int B, int N, int T, int chunk,
                            double* Mx, uint8_t* K, int32_t* pin, const MaxGroupBuffers& gb, float* best_score,
                            hipStream_t st, const float* emit = nullptr, const float* trans = nullptr);
// Best path inside every chunk between those pinned tags (lccrf_viterbi.hip);
// mid: viterbi_mid_doubles(B, C, T) doubles of scratch.
hipError_t launch_chunked_max(int dtype, const void* phi, const int32_t* lengths, int B, int N, int T, uint8_t* bp,
                              double* mid, int32_t* tags, int chunk, const int32_t* pin, hipStream_t st,
                              const float* emit = nullptr, const float* trans = nullptr);

// Entropy H(p) [B] in one read of phi (lccrf_extras.hip, one-wave kernels for T <= 32).  ua / ub / Oa / Ob
// as for launch_sequential_sum (only the rows of the meeting positions are written); ha, hb: [B][T] floats.
hipError_t launch_entropy(int dtype, const void* phi, const int32_t* lengths, int B, int N, int T, float* ua, float* ub,
                          double* Oa, double* Ob, float* ha, float* hb, float* H, hipStream_t st);

// Cross-entropy H(p, q) (kl false) or KL(p || q) (kl true) [B]: the half chains of phi_p carry the expected
// score under phi_q (the expected score difference); logZq [B]: log Z of phi_q (natural logarithm); hoff: [B][2] doubles.
hipError_t launch_cross(bool kl, int dtype, const void* phi_p, const void* phi_q, const int32_t* lengths, int B, int N,
                        int T, float* ua, float* ub, double* Oa, double* Ob, float* ha, float* hb, double* hoff,
                        const double* logZq, float* out, hipStream_t st);

// Semi-Markov CRF forward (lccrf_semi.hip): logZ [B] from phi [B][N][K][T][T].
bool semi_markov_supported(int K, int T);
hipError_t launch_semi_markov_forward(int dtype, const void* phi, const int32_t* lengths, int B, int N, int K, int T,
                                      float* logZ, hipStream_t st);

}  // namespace lccrf
