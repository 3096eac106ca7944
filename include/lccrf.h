/*
 * lccrf.h - C ABI of the MI355X (gfx950) batched linear-chain CRF library.
 *
 * The model is the linear-chain CRF of the paper's section "Sequence Tagging": a
 * tag path y_0..y_{L-1} over T tags has log-potential
 *
 *     score(y) = phi[b][0][0][y_0] + sum_{i=1}^{L-1} phi[b][i][y_{i-1}][y_i]
 *
 * with a separate T x T matrix of log-potentials for every position (the paper's
 * per-time-step transition matrices), p(y) = exp(score(y) - logZ) (section
 * "Structured Distributions", Eq. 1-2).
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 *  - All data pointers are DEVICE pointers owned by the caller; the library never
 *    allocates, frees, synchronises or copies to the host.  Work is enqueued on
 *    `stream` (a hipStream_t passed as void*; NULL = the default stream) and the
 *    call returns at once.
 *  - phi: dense, contiguous, row-major [B][N][T][T], t fastest; element type by
 *    `dt` (LCCRF_F32: IEEE float; LCCRF_BF16: bfloat16, widened exactly to float
 *    before use).  s (third index) is the tag at position i-1, t the tag at
 *    position i.  Of the first matrix only row s = 0 is used: phi[b][0][0][t]
 *    scores starting in tag t.  Base address 16-byte aligned.
 *  - lengths: int32 [B] or NULL (= all N).  Values are clamped on the device to
 *    [0, N].  Positions i >= lengths[b] are never read.  lengths[b] = 0 is the empty
 *    chain: logZ = 0, marginals 0, score 0, tags -1.
 *  - -inf potentials are allowed (a forbidden edge; its marginal is 0).  If no path
 *    has a finite score, logZ = -inf and all marginals are 0.  +inf and NaN inputs
 *    are undefined.
 *  - workspace: device scratch of at least lccrf_workspace_bytes(op, ...) bytes,
 *    256-byte aligned, not shared by calls that may overlap in time.  Contents on
 *    entry are irrelevant; contents on exit are unspecified.
 *  - 1 <= T <= LCCRF_MAX_T, B >= 1, N >= 1, B*N*T*T < 2^62.
 *  - Return value: LCCRF_OK (0) or a negative lccrf_status.  Argument errors (every
 *    status but LCCRF_ELAUNCH) are found before anything is enqueued.  A query is
 *    several kernel launches; LCCRF_ELAUNCH means the HIP runtime refused one of
 *    them, and the launches before it are already enqueued: the outputs and the
 *    workspace are then unspecified, nothing else is harmed.
 *  - Thread safety: concurrent calls with distinct workspaces are safe.  The only
 *    mutable state in the library are three process-wide tuning knobs
 *    (lccrf_set_scan_chunk, lccrf_set_pair_poll_limit, lccrf_set_lane_poll_limit; atomic
 *    integers, meant to be
 *    set once at start-up) and caches of per-device constants.  A call reads the
 *    knobs once, at its start, so every call is consistent in itself; a workspace
 *    sized under one chunk setting and used under another is refused with
 *    LCCRF_EWORKSPACE if it is too small.
 *  - Repeat runs: results are bit-identical from run to run, with one exception:
 *    marginals at T = 128 in batches that fill at most a quarter of the chip's
 *    compute units are computed by pairs of workgroups (see
 *    lccrf_set_pair_poll_limit); a pair that gives its sequence up hands it to the
 *    one-workgroup kernel, which rounds differently, so where that hand-over depends
 *    on timing two runs may differ in the low-order bits (far inside the tolerance).
 *    LCCRF_ALGO_SEQUENTIAL never uses pairs.  Likewise a sum-product chain of LCCRF_ALGO_SEQUENTIAL_LANES
 *    (which AUTO takes for mid-sized batches of 17 .. 64 tags) whose producers fall behind its poll limit
 *    (lccrf_set_lane_poll_limit; milliseconds, not seen in practice) finishes in the log domain and
 *    rounds differently from a run in which they kept up.  (lccrf_argmax is bit-identical from run to run
 *    under every schedule: a max-plus chain that stops waiting computes the same sums and maxima alone.)
 */
#ifndef LCCRF_H
#define LCCRF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LCCRF_MAX_T 256

typedef enum { LCCRF_F32 = 0, LCCRF_BF16 = 1 } lccrf_dtype;

typedef enum {
    LCCRF_OP_LOGZ = 0,
    LCCRF_OP_MARGINALS = 1,
    LCCRF_OP_ARGMAX = 2,
    LCCRF_OP_LOG_PROB = 3,
    LCCRF_OP_ENTROPY = 4,
    LCCRF_OP_SAMPLE = 5,
    LCCRF_OP_CROSS_ENTROPY = 6, /* also the workspace of lccrf_kl_divergence */
} lccrf_op;

/* How the recursion over positions is scheduled.  Results are the same up to
 * rounding; AUTO picks by shape. */
typedef enum {
    LCCRF_ALGO_AUTO = 0,
    LCCRF_ALGO_SEQUENTIAL = 1, /* position by position (the forward algorithm as the paper uses it), one
                                  workgroup per chain; AUTO may instead split a chain over two workgroups */
    LCCRF_ALGO_SCAN = 2,       /* chunked associative scan over positions (the parallel variant the
                                  paper cites in "Sequence Tagging"): products of the T x T matrices
                                  of each chunk, a short serial pass over chunks, then every chunk
                                  on its own.  T <= 64 for the sum queries, T <= 32 for lccrf_argmax, else
                                  LCCRF_ENOTIMPL;
                                  AUTO takes it for long chains in small batches */
    LCCRF_ALGO_SEQUENTIAL_EXACT = 3, /* sequential, and every log-sum-exp shifted by its own maximum:
                                  the step that normally only replays rejected speculative steps
                                  is used for every position (same results up to rounding; slower) */
    LCCRF_ALGO_SEQUENTIAL_LANES = 4  /* sequential, the recursion in scaled probabilities by one wave per
                                  chain (a step is a vector-matrix product, one tag per lane) while the
                                  other waves of its workgroup stream and exponentiate the potentials and
                                  write the marginals; positions whose sums leave the range of single
                                  precision (or hold -inf) are taken in the log domain.  lccrf_log_partition
                                  and lccrf_marginals at 8 <= T <= 48, and at 52, 56, 60 and 64 tags.  For
                                  lccrf_argmax (any T <= 64) the same split in the max-plus
                                  semiring: one wave runs the scores in double precision, the others stream
                                  the potentials and find the pointers; tags and scores are those of
                                  LCCRF_ALGO_SEQUENTIAL bit for bit.  Other queries and tag counts:
                                  LCCRF_ENOTIMPL; AUTO takes it where the batch leaves the chip latency-bound */
} lccrf_algo;

typedef enum {
    LCCRF_OK = 0,
    LCCRF_EINVAL = -1,     /* bad B, N, T (1 <= T <= 256, B * N < 2e9), dtype, op or algo */
    LCCRF_ENULL = -2,      /* a required pointer is NULL */
    LCCRF_EWORKSPACE = -3, /* workspace NULL or smaller than lccrf_workspace_bytes */
    LCCRF_EALIGN = -4,     /* phi, an output or the workspace is misaligned */
    LCCRF_ELAUNCH = -5,    /* the HIP runtime refused a launch */
    LCCRF_ENOTIMPL = -6,   /* the requested algo does not exist for this shape */
    LCCRF_ETOOBIG = -7     /* lccrf_marginals_static: the shape needs more than the built-in scratch */
} lccrf_status;

/* Bytes of device scratch the given query needs (a multiple of 256); 0 on invalid
 * arguments.  Valid for every lccrf_algo. */
size_t lccrf_workspace_bytes(lccrf_op op, int B, int N, int T, lccrf_dtype dt);

/*
 * Log-partition function (paper: section "Computing Probability of a Structure and
 * Partition Function"; forward algorithm of section "Sequence Tagging", O(T^2 N)):
 *     logZ[b] = log sum_y exp(score_b(y)),   float [B] on the device.
 */
int lccrf_log_partition(const void* phi, lccrf_dtype dt, const int32_t* lengths,
                        int B, int N, int T,
                        float* logZ,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * Edge marginals (paper: section "Computing Marginals", Eq. 3 and Eq. 4: the
 * marginal of a part is the derivative of logZ with respect to its log-potential;
 * here computed by the hand-written forward-backward recursions):
 *     marginals[b][i][s][t] = p(y_{i-1} = s, y_i = t)        for 1 <= i < lengths[b]
 *     marginals[b][0][0][t] = p(y_0 = t)
 *     0 everywhere else (rows s > 0 of position 0, positions >= lengths[b]).
 * marginals: float [B][N][T][T], fully written.  logZ: float [B] or NULL.
 */
int lccrf_marginals(const void* phi, lccrf_dtype dt, const int32_t* lengths,
                    int B, int N, int T,
                    float* logZ, float* marginals,
                    void* workspace, size_t workspace_bytes, void* stream);

/*
 * Most probable tag path (paper: section "Computing Most Probable Structure": the
 * same recursion in the max-plus semiring; the path is what the gradient of the best
 * score with respect to the potentials marks):
 *     tags[b][i] in [0, T) for i < lengths[b], -1 for i >= lengths[b]; int32 [B][N].
 *     best_score[b] = score_b(tags[b]); float [B] or NULL.
 * Scores are accumulated in double precision.  Among exactly tied best paths the one
 * returned depends on the schedule.  The sequential schedule runs two chains that meet
 * at position h = lengths[b] / 2 and returns, of all best paths, the one with the
 * smallest tag at h, then the smallest tag at h-1, h-2, ..., 0 in that order (smallest
 * predecessor at every step down) and, independently, the smallest tag at h+1, ...,
 * L-1 (smallest successor at every step up).  The chunked scan returns some best path.
 */
int lccrf_argmax(const void* phi, lccrf_dtype dt, const int32_t* lengths,
                 int B, int N, int T,
                 float* best_score, int32_t* tags,
                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * lccrf_marginals for callers that cannot allocate device memory or bring a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same inputs, outputs, results
 * and errors as lccrf_marginals, but the scratch is a buffer built into the library
 * (lccrf_static_scratch_bytes() bytes, 64 MiB, on every GPU the library runs on, held until the
 * process ends); the call allocates and frees nothing.
 *   - A shape whose lccrf_workspace_bytes(LCCRF_OP_MARGINALS, ...) exceeds that size is refused with
 *     LCCRF_ETOOBIG before anything is enqueued (the headline shape B=64, N=512, T=128 needs 39 MB).
 *   - Every call on one GPU uses that GPU's one buffer: calls that may overlap in time on the same
 *     GPU (two streams, two threads) race and must not be made; calls on one stream are ordered.
 *     Nothing in the buffer has to be cleared between calls: every kernel writes what it later reads.
 *   - The first call on a device looks the buffer's address up (hipGetSymbolAddress); make it
 *     outside a stream capture.  LCCRF_ELAUNCH if that lookup fails.
 */
size_t lccrf_static_scratch_bytes(void);
int lccrf_marginals_static(const void* phi, lccrf_dtype dt, const int32_t* lengths,
                           int B, int N, int T,
                           float* logZ, float* marginals, void* stream);

/* The same three queries with the schedule chosen by the caller (tests, benchmarks).
 * LCCRF_ENOTIMPL if `algo` is not available for the shape. */
int lccrf_log_partition_algo(const void* phi, lccrf_dtype dt, const int32_t* lengths,
                             int B, int N, int T, float* logZ,
                             void* workspace, size_t workspace_bytes, void* stream, lccrf_algo algo);
int lccrf_marginals_algo(const void* phi, lccrf_dtype dt, const int32_t* lengths,
                         int B, int N, int T, float* logZ, float* marginals,
                         void* workspace, size_t workspace_bytes, void* stream, lccrf_algo algo);
int lccrf_argmax_algo(const void* phi, lccrf_dtype dt, const int32_t* lengths,
                      int B, int N, int T, float* best_score, int32_t* tags,
                      void* workspace, size_t workspace_bytes, void* stream, lccrf_algo algo);

/*
 * log p(y) = score(y) - logZ of one given tag path per sequence (paper, section "Structured
 * Distributions", Eq. 2: the probability of a structure; section "Computing Probability of a
 * Structure and Partition Function").
 *   tags      [B][N] int32 (device), tags[b][i] in [0, T) for i < length; entries past the length
 *             are ignored.  A tag out of range makes log_prob[b] NaN (nothing out of bounds is read).
 *   log_prob  [B] float32 (device).  Empty chain: 0.
 * The score and logZ are combined in double precision; one read of phi plus N gathers.
 * Workspace: lccrf_workspace_bytes(LCCRF_OP_LOG_PROB, ...).  Errors as lccrf_log_partition.
 */
int lccrf_log_prob(const void* phi, lccrf_dtype dt, const int32_t* lengths, const int32_t* tags,
                   int B, int N, int T, float* log_prob,
                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * Entropy H(p) = -sum_y p(y) log p(y) of every chain, in nats (paper, section "Entropy and KL
 * Divergence": H(p) = H(p, p) = logZ - sum_e p(e) phi(e)).  Computed in ONE read of phi and without
 * forming the marginals: the two half chains carry the conditional entropy of the path behind
 * them, and the meeting position combines them (the same value up to rounding).
 *   entropy   [B] float32 (device).  Empty chain: 0.  No finite path: NaN.
 * Workspace: lccrf_workspace_bytes(LCCRF_OP_ENTROPY, ...).  Errors as lccrf_log_partition.
 */
int lccrf_entropy(const void* phi, lccrf_dtype dt, const int32_t* lengths, int B, int N, int T,
                  float* entropy, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Cross-entropy H(p, q) = -sum_y p(y) log q(y) = logZ_q - sum_e p(e) phi_q(e) and Kullback-Leibler
 * divergence KL(p || q) = H(p, q) - H(p) of two chains over the same sequences, in nats (paper,
 * section "Entropy and KL Divergence").  phi_p and phi_q have the same shape, type and lengths.
 * Neither forms the marginals: one forward-backward read of phi_q gives logZ_q, then the two half
 * chains of p carry the expected score under phi_q (for KL: the expected score difference
 * phi_p - phi_q, formed per edge, so close chains lose no digits) while reading both tensors once.
 * An edge of probability zero under p contributes nothing whatever phi_q holds there; an edge
 * that p can take and q forbids (-inf) gives +inf.
 *   out       [B] float32 (device).  Empty chain: 0.  No finite path under p: NaN.
 * Workspace: lccrf_workspace_bytes(LCCRF_OP_CROSS_ENTROPY, ...).  Errors as lccrf_log_partition
 * (phi_q is checked like phi).
 */
int lccrf_cross_entropy(const void* phi_p, const void* phi_q, lccrf_dtype dt, const int32_t* lengths,
                        int B, int N, int T, float* out,
                        void* workspace, size_t workspace_bytes, void* stream);
int lccrf_kl_divergence(const void* phi_p, const void* phi_q, lccrf_dtype dt, const int32_t* lengths,
                        int B, int N, int T, float* out,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * One sample per sequence by forward-filtering backward-sampling (paper, section "Sampling a
 * Structure"): the forward algorithm, then y_{L-1} ~ exp(alpha_{L-1}(t)) and, going down,
 * y_i ~ exp(alpha_i(s) + phi[i+1][s][y_{i+1}]).  The randomness is the caller's: uniforms[b][i]
 * in [0, 1) decides position i by inversion of the cumulative weights over ascending tags (the
 * smallest tag whose cumulative weight exceeds u * total), so a call is reproducible and
 * samples are independent exactly as far as the uniforms are.
 *   uniforms  [B][N] float32 (device); entries past the lengths are ignored.
 *   tags      [B][N] int32 (device), -1 past the length; all 0 for a chain without a finite path.
 * Workspace: lccrf_workspace_bytes(LCCRF_OP_SAMPLE, ...).  Errors as lccrf_log_partition.
 */
int lccrf_sample(const void* phi, lccrf_dtype dt, const int32_t* lengths, const float* uniforms,
                 int B, int N, int T, int32_t* tags,
                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * lccrf_sample with the randomness drawn inside the library from an explicit key, as the paper asks of
 * sampling (section "Sampling a Structure": reproducible samples from explicit random keys): the uniform of
 * position i of sequence b is produced by the counter-based generator Philox4x32-10 (Salmon, Moraes, Dror
 * and Shaw, 2011: multipliers 0xD2511F53 and 0xCD9E8D57, key increments 0x9E3779B9 and 0xBB67AE85, ten
 * rounds) with key (seed mod 2^32, seed / 2^32) and counter (k mod 2^32, k / 2^32, 0, 0), k = b * N + i: the
 * upper 24 bits of the first output word times 2^-24.  Every draw depends on (seed, b, i) alone; the same
 * seed gives the same tags on every call, and lccrf_sample fed those uniforms gives the same tags too.
 * Other arguments, outputs, workspace and errors as lccrf_sample.
 */
int lccrf_sample_seeded(const void* phi, lccrf_dtype dt, const int32_t* lengths, uint64_t seed,
                        int B, int N, int T, int32_t* tags,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * Semi-Markov CRF, log-partition (paper, section "Segmentation with Semi-Markov CRF": the linear
 * chain's parametrisation with transition matrices, except that a transition may jump over
 * several positions; forward algorithm in O(K T^2 N)).  A structure splits positions 0..L-1 into
 * consecutive segments of 1..K positions, each carrying a tag.
 *   phi     [B][N][K][T][T] (device, dt, 16-byte aligned): phi[b][i][k][s][t] is the log-potential of
 *           a segment tagged t that ENDS at position i and covers k + 1 positions, after a
 *           segment tagged s; the first segment (k == i) reads row s = 0 only, the linear
 *           chain's convention for its first tag.  Entries with k > i, rows s > 0 of first
 *           segments and positions past the length are never used.  K = 1 is the linear chain.
 *   logZ    [B] float32 (device).  Empty sequence: 0.  No finite structure: -inf.
 * Needs no workspace.  Returns LCCRF_ENOTIMPL when the K most recent forward vectors do not fit
 * one workgroup's local memory (K * T above about 14000); other errors as lccrf_log_partition.
 */
int lccrf_semi_markov_log_partition(const void* phi, lccrf_dtype dt, const int32_t* lengths,
                                    int B, int N, int K, int T, float* logZ, void* stream);

/*
 * The three queries from STRUCTURED potentials: phi[b][i][s][t] = trans[s][t] + emit[b][i][t], the
 * usual tagging parameterisation (per-position emission scores plus one shared transition matrix;
 * the paper's linear-chain CRF takes the dense per-position matrices these stand for, section
 * "Sequence Tagging").  The dense tensor is never formed: the transition tile stays in registers
 * and a position brings T numbers instead of T*T, so log-partition and argmax read T times less
 * (marginals still write the dense [B,N,T,T] result).  Results equal those of the dense calls on
 * the materialised phi up to rounding; the first tag is scored trans[0][t] + emit[b][0][t].
 *   emit   [B][N][T] float32 (device), 16-byte aligned; trans [T][T] float32 (device), 16-byte aligned.
 * T <= 128 (else LCCRF_ENOTIMPL).  Workspace: lccrf_workspace_bytes of the matching op with LCCRF_F32.
 * The schedule is the one lccrf_auto_algo reports for the matching op and shape (long chains in small
 * batches take the chunked scan, mid-sized batches of up to 48 tags LCCRF_ALGO_SEQUENTIAL_LANES); there is no
 * per-call choice for these three.
 * Other arguments, outputs and errors as the dense calls.
 */
int lccrf_log_partition_structured(const float* emit, const float* trans, const int32_t* lengths,
                                   int B, int N, int T, float* logZ,
                                   void* workspace, size_t workspace_bytes, void* stream);
int lccrf_marginals_structured(const float* emit, const float* trans, const int32_t* lengths,
                               int B, int N, int T, float* logZ, float* marginals,
                               void* workspace, size_t workspace_bytes, void* stream);
int lccrf_argmax_structured(const float* emit, const float* trans, const int32_t* lengths,
                            int B, int N, int T, float* best_score, int32_t* tags,
                            void* workspace, size_t workspace_bytes, void* stream);

/* Positions per chunk of LCCRF_ALGO_SCAN: a process-wide tuning knob.  0 (the default) lets every
 * call choose by its shape (8, 16 or 32: the shortest chunks that the chip still holds all at
 * once); other values outside [4, 4096] return LCCRF_EINVAL and change nothing.  It enters
 * lccrf_workspace_bytes, so set it before sizing a workspace.  Every call reads it once at its start.
 * Results do not depend on it beyond rounding. */
int lccrf_set_scan_chunk(int chunk);

/* How many times a workgroup of the paired second pass of lccrf_marginals (T = 128, batches of at
 * most a quarter as many sequences as the chip has compute units: two workgroups per chain that swap
 * half vectors through device memory at every position) looks for its partner's words before it
 * gives the sequence up; the one-workgroup kernel then recomputes that sequence, so results never
 * depend on the limit beyond rounding.  A process-wide tuning knob.  Default 32768 polls (some tens
 * of milliseconds at worst; an exchange between resident partners takes under a microsecond), -1
 * restores it, 0 gives up without looking (every sequence then takes the one-workgroup kernel: for
 * tests of that path), more than 2^24 returns LCCRF_EINVAL. */
int lccrf_set_pair_poll_limit(int polls);

/* How many times the chain wave of LCCRF_ALGO_SEQUENTIAL_LANES looks for a matrix that its producer waves have
 * not delivered yet (one read of a word in LDS per look) before it stops waiting and finishes its half chain
 * alone in the log domain, straight from memory (the same path that serves -inf potentials), so results never
 * depend on the limit beyond rounding.  A process-wide tuning knob.  Default 65536 looks (a few milliseconds at
 * worst; a matrix is normally there before it is asked for), -1 restores it, 0 gives up at the first look that
 * fails (nearly every chain then runs in the log domain from its first position: for tests of that path), more
 * than 2^24 returns LCCRF_EINVAL.  The chain wave of lccrf_argmax under the same schedule waits for its helper
 * waves by the same limit, and then goes on alone with the same arithmetic: identical tags and scores. */
int lccrf_set_lane_poll_limit(int polls);

/* The schedule LCCRF_ALGO_AUTO takes for `op` at this shape under the current chunk size:
 * LCCRF_ALGO_SEQUENTIAL, LCCRF_ALGO_SEQUENTIAL_LANES or LCCRF_ALGO_SCAN.  Host-side arithmetic, nothing is launched;
 * LCCRF_EINVAL for a shape or op the library does not serve.  For callers that size or time a run
 * by the schedule it will take (the benchmark names its dominant kernel from it). */
int lccrf_auto_algo(lccrf_op op, int B, int N, int T);

/* Static, human-readable text for a status code. */
const char* lccrf_strerror(int code);

/* Library version: major * 10000 + minor * 100 + patch. */
int lccrf_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LCCRF_H */
