/*
 * CPU oracle for the batched linear-chain CRF.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, double-precision statement of what the GPU path must compute.
 * It is used by the tests, by the smoke check and by the benchmark's CPU-baseline
 * leg, and by nothing else: the product never routes through this file, and this
 * file shares no code, header, table or helper with the HIP sources.
 *
 * The model (paper, section "Structured Distributions", Eq. 1 and Eq. 2; section
 * "Sequence Tagging"): a tag path y_0..y_{L-1} over T tags has log-potential
 *
 *     score(y) = phi[0][0][y_0] + sum_{i=1}^{L-1} phi[i][y_{i-1}][y_i]
 *
 * with one T x T matrix of log-potentials per position.  Only row 0 of the
 * first matrix is used (it scores the first tag); phi at positions >= L is
 * never read.  p(y) = exp(score(y) - logZ), logZ = log sum_y exp(score(y)).
 *
 * What is computed, all by the textbook recursions the paper names:
 *   - forward algorithm in the log semiring            -> alpha, logZ
 *   - the matching backward recursion                   -> beta
 *   - edge marginals p(e) = d logZ / d phi(e) (section "Computing Marginals",
 *     Eq. 3 and Eq. 4) in their closed forward-backward form
 *   - the same recursion in the max-plus semiring (section "Computing Most
 *     Probable Structure")                              -> best path, its score,
 *     and the gap to the second-best path via max-marginals
 *   - log-probability of a given path (Eq. 2) and cross-entropy / entropy from the
 *     marginals (section "Entropy and KL Divergence"), as those formulas stand.
 *
 * No blocking, fusion or reordering: loops over b, i, s, t; every log-sum-exp is
 * shifted by its own maximum.  The only parallelism is an OpenMP loop over the
 * batch, whose sequences are independent.
 *
 * Storage types: dtype 0 = IEEE float32, dtype 1 = bfloat16 (upper 16 bits of a
 * float32); both are widened exactly to double before any arithmetic.
 *
 * Empty chain (L = 0): one empty structure of potential 1: logZ = 0, all
 * marginals 0, score 0, all tags -1.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static inline double phi_at(const void *phi, int dtype, size_t idx)
{
    if (dtype == 0) {
        return (double)((const float *)phi)[idx];
    } else {
        uint32_t bits = ((uint32_t)((const uint16_t *)phi)[idx]) << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    }
}

static inline int clamp_len(const int32_t *lengths, int b, int N)
{
    int L = lengths ? lengths[b] : N;
    if (L < 0) L = 0;
    if (L > N) L = N;
    return L;
}

/* log(sum_k exp(x[k])) with the maximum taken out; -inf when every x[k] is -inf. */
static double logsumexp(const double *x, int n)
{
    double m = -INFINITY;
    for (int k = 0; k < n; ++k)
        if (x[k] > m) m = x[k];
    if (m == -INFINITY) return -INFINITY;
    double s = 0.0;
    for (int k = 0; k < n; ++k) s += exp(x[k] - m);
    return m + log(s);
}

/* alpha[i][t] = log of the summed potential of all prefixes y_0..y_i that end in tag t. */
static void forward_one(const void *phi, int dtype, size_t base, int L, int T,
                        double *alpha /* [L][T] */, double *tmp /* [T] */)
{
    for (int t = 0; t < T; ++t) alpha[t] = phi_at(phi, dtype, base + (size_t)t);
    for (int i = 1; i < L; ++i) {
        size_t m = base + (size_t)i * T * T;
        for (int t = 0; t < T; ++t) {
            for (int s = 0; s < T; ++s)
                tmp[s] = alpha[(size_t)(i - 1) * T + s] + phi_at(phi, dtype, m + (size_t)s * T + t);
            alpha[(size_t)i * T + t] = logsumexp(tmp, T);
        }
    }
}

/* beta[i][s] = log of the summed potential of all suffixes y_{i+1}..y_{L-1} given y_i = s. */
static void backward_one(const void *phi, int dtype, size_t base, int L, int T,
                         double *beta /* [L][T] */, double *tmp /* [T] */)
{
    for (int t = 0; t < T; ++t) beta[(size_t)(L - 1) * T + t] = 0.0;
    for (int i = L - 1; i >= 1; --i) {
        size_t m = base + (size_t)i * T * T;
        for (int s = 0; s < T; ++s) {
            for (int t = 0; t < T; ++t)
                tmp[t] = phi_at(phi, dtype, m + (size_t)s * T + t) + beta[(size_t)i * T + t];
            beta[(size_t)(i - 1) * T + s] = logsumexp(tmp, T);
        }
    }
}

/* alpha, beta: [B][N][T] doubles, rows i >= L left untouched.  Either may be NULL. */
int lccrf_oracle_forward_backward(const void *phi, int dtype, const int32_t *lengths,
                                  int B, int N, int T,
                                  double *alpha, double *beta, double *logZ)
{
    if (!phi || B < 1 || N < 1 || T < 1 || (dtype != 0 && dtype != 1)) return -1;
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        int L = clamp_len(lengths, b, N);
        size_t base = (size_t)b * N * T * T;
        if (L == 0) {
            if (logZ) logZ[b] = 0.0;
            continue;
        }
        double *tmp = (double *)malloc(sizeof(double) * (size_t)T);
        double *a = alpha ? alpha + (size_t)b * N * T : (double *)malloc(sizeof(double) * (size_t)L * T);
        if (!tmp || !a) { err = 1; free(tmp); continue; }
        forward_one(phi, dtype, base, L, T, a, tmp);
        if (logZ) logZ[b] = logsumexp(a + (size_t)(L - 1) * T, T);
        if (beta) backward_one(phi, dtype, base, L, T, beta + (size_t)b * N * T, tmp);
        if (!alpha) free(a);
        free(tmp);
    }
    return err ? -2 : 0;
}

int lccrf_oracle_log_partition(const void *phi, int dtype, const int32_t *lengths,
                               int B, int N, int T, double *logZ)
{
    if (!logZ) return -1;
    return lccrf_oracle_forward_backward(phi, dtype, lengths, B, N, T, NULL, NULL, logZ);
}

/*
 * mu[b][i][s][t] = p(y_{i-1} = s, y_i = t) = exp(alpha[i-1][s] + phi[i][s][t] + beta[i][t] - logZ)
 * for 1 <= i < L; mu[b][0][0][t] = p(y_0 = t) = exp(alpha[0][t] + beta[0][t] - logZ);
 * every other entry (rows s > 0 of position 0, all positions >= L) is 0.
 * If no path has a finite score (logZ = -inf) all marginals are 0.
 */
int lccrf_oracle_marginals(const void *phi, int dtype, const int32_t *lengths,
                           int B, int N, int T, double *logZ /* may be NULL */, double *mu)
{
    if (!phi || !mu || B < 1 || N < 1 || T < 1 || (dtype != 0 && dtype != 1)) return -1;
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        int L = clamp_len(lengths, b, N);
        size_t base = (size_t)b * N * T * T;
        double *m = mu + base;
        memset(m, 0, sizeof(double) * (size_t)N * T * T);
        if (L == 0) {
            if (logZ) logZ[b] = 0.0;
            continue;
        }
        double *alpha = (double *)malloc(sizeof(double) * (size_t)L * T);
        double *beta = (double *)malloc(sizeof(double) * (size_t)L * T);
        double *tmp = (double *)malloc(sizeof(double) * (size_t)T);
        if (!alpha || !beta || !tmp) { err = 1; free(alpha); free(beta); free(tmp); continue; }
        forward_one(phi, dtype, base, L, T, alpha, tmp);
        backward_one(phi, dtype, base, L, T, beta, tmp);
        double lz = logsumexp(alpha + (size_t)(L - 1) * T, T);
        if (logZ) logZ[b] = lz;
        if (lz != -INFINITY) {
            for (int t = 0; t < T; ++t)
                m[t] = exp(alpha[t] + beta[t] - lz);
            for (int i = 1; i < L; ++i)
                for (int s = 0; s < T; ++s)
                    for (int t = 0; t < T; ++t) {
                        size_t k = (size_t)i * T * T + (size_t)s * T + t;
                        double e = alpha[(size_t)(i - 1) * T + s] + phi_at(phi, dtype, base + k)
                                   + beta[(size_t)i * T + t] - lz;
                        m[k] = exp(e);
                    }
        }
        free(alpha); free(beta); free(tmp);
    }
    return err ? -2 : 0;
}

/*
 * log p(y) = score(y) - logZ for one given tag path per sequence (section "Structured
 * Distributions", Eq. 2, numerator and denominator of the probability of a structure).
 * tags[b][i], i < L, must lie in [0, T); otherwise out[b] = NaN.  Empty chain: log p = 0.
 */
int lccrf_oracle_log_prob(const void *phi, int dtype, const int32_t *lengths, const int32_t *tags,
                          int B, int N, int T, double *out)
{
    if (!phi || !tags || !out || B < 1 || N < 1 || T < 1 || (dtype != 0 && dtype != 1)) return -1;
    double *logZ = (double *)malloc(sizeof(double) * (size_t)B);
    if (!logZ) return -2;
    int rc = lccrf_oracle_log_partition(phi, dtype, lengths, B, N, T, logZ);
    if (rc != 0) { free(logZ); return rc; }
    for (int b = 0; b < B; ++b) {
        int L = clamp_len(lengths, b, N);
        size_t base = (size_t)b * N * T * T;
        const int32_t *y = tags + (size_t)b * N;
        double sc = 0.0;
        int ok = 1;
        for (int i = 0; i < L; ++i)
            if (y[i] < 0 || y[i] >= T) ok = 0;
        if (ok && L > 0) {
            sc = phi_at(phi, dtype, base + (size_t)y[0]);
            for (int i = 1; i < L; ++i)
                sc += phi_at(phi, dtype, base + (size_t)i * T * T + (size_t)y[i - 1] * T + (size_t)y[i]);
        }
        out[b] = ok ? sc - logZ[b] : NAN;
    }
    free(logZ);
    return 0;
}

/*
 * Cross-entropy of two chains over the same edges (section "Entropy and KL Divergence"):
 *     H(p, q) = logZ_q - sum_e p(e) phi_q(e),
 * p(e) the edge marginals of p, the sum running over the first-tag "edges" (0, 0, t) and the
 * edges (i, s, t), 1 <= i < L.  Entropy is H(p, p); KL(p || q) = H(p, q) - H(p, p).
 * An edge with p(e) = 0 contributes nothing whatever phi_q(e) is.  If p has no finite path the
 * result is NaN.  Empty chain: 0.
 */
int lccrf_oracle_cross_entropy(const void *phi_p, const void *phi_q, int dtype, const int32_t *lengths,
                               int B, int N, int T, double *out)
{
    if (!phi_p || !phi_q || !out || B < 1 || N < 1 || T < 1 || (dtype != 0 && dtype != 1)) return -1;
    size_t esz = dtype == 0 ? 4 : 2;
    int err = 0;
    for (int b = 0; b < B; ++b) {   /* one sequence at a time: its marginals are N*T*T doubles */
        int L = clamp_len(lengths, b, N);
        if (L == 0) { out[b] = 0.0; continue; }
        size_t base = (size_t)b * N * T * T;
        int32_t len1 = L;
        double *mu = (double *)malloc(sizeof(double) * (size_t)N * T * T);
        double lzp, lzq;
        if (!mu) { err = 1; continue; }
        int rc = lccrf_oracle_marginals((const char *)phi_p + base * esz, dtype, &len1, 1, N, T, &lzp, mu);
        if (rc == 0) rc = lccrf_oracle_log_partition((const char *)phi_q + base * esz, dtype, &len1, 1, N, T, &lzq);
        if (rc != 0) { err = 1; free(mu); continue; }
        if (lzp == -INFINITY) { out[b] = NAN; free(mu); continue; }
        double acc = 0.0;
        for (int t = 0; t < T; ++t)
            if (mu[t] > 0.0) acc += mu[t] * phi_at(phi_q, dtype, base + (size_t)t);
        for (int i = 1; i < L; ++i)
            for (int s = 0; s < T; ++s)
                for (int t = 0; t < T; ++t) {
                    size_t k = (size_t)i * T * T + (size_t)s * T + t;
                    if (mu[k] > 0.0) acc += mu[k] * phi_at(phi_q, dtype, base + k);
                }
        out[b] = lzq - acc;
        free(mu);
    }
    return err ? -2 : 0;
}

/*
 * Forward-filtering backward-sampling (section "Sampling a Structure"): with alpha from the
 * forward algorithm, y_{L-1} is drawn from p(t) ~ exp(alpha_{L-1}(t)) and then, going down,
 * y_{i-1} from p(s | y_i) ~ exp(alpha_{i-1}(s) + phi[i][s][y_i]).  The randomness is an input:
 * uniforms[b][i] in [0, 1) decides position i by inversion of the cumulative distribution over
 * tags in ascending order: the chosen tag is the smallest t whose cumulative weight exceeds
 * u * (total weight); if rounding leaves none, the last tag of positive weight.
 *
 * margin[b] (optional): the smallest distance, over the positions of the chain, between
 * u * total and the nearest boundary of the chosen tag's interval, relative to the total: how
 * far the draw was from choosing a neighbouring tag.  A sequence without a finite path gets
 * tags 0 and margin 0.  tags[b][i] = -1 for i >= L.
 */
int lccrf_oracle_sample(const void *phi, int dtype, const int32_t *lengths, const float *uniforms,
                        int B, int N, int T, int32_t *tags, double *margin /* may be NULL */)
{
    if (!phi || !uniforms || !tags || B < 1 || N < 1 || T < 1 || (dtype != 0 && dtype != 1)) return -1;
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        int L = clamp_len(lengths, b, N);
        size_t base = (size_t)b * N * T * T;
        int32_t *y = tags + (size_t)b * N;
        for (int i = 0; i < N; ++i) y[i] = i < L ? 0 : -1;
        if (margin) margin[b] = L == 0 ? 1.0 : 0.0;
        if (L == 0) continue;
        double *alpha = (double *)malloc(sizeof(double) * (size_t)L * T);
        double *tmp = (double *)malloc(sizeof(double) * (size_t)T);
        double *w = (double *)malloc(sizeof(double) * (size_t)T);
        if (!alpha || !tmp || !w) { err = 1; free(alpha); free(tmp); free(w); continue; }
        forward_one(phi, dtype, base, L, T, alpha, tmp);
        if (logsumexp(alpha + (size_t)(L - 1) * T, T) == -INFINITY) { free(alpha); free(tmp); free(w); continue; }
        double worst = 1.0;
        for (int i = L - 1; i >= 0; --i) {
            /* log-weights of the tags of position i */
            for (int s = 0; s < T; ++s) {
                w[s] = alpha[(size_t)i * T + s];
                if (i < L - 1)
                    w[s] += phi_at(phi, dtype, base + (size_t)(i + 1) * T * T + (size_t)s * T + (size_t)y[i + 1]);
            }
            double m = -INFINITY, total = 0.0;
            for (int s = 0; s < T; ++s) if (w[s] > m) m = w[s];
            for (int s = 0; s < T; ++s) { w[s] = exp(w[s] - m); total += w[s]; }
            double target = (double)uniforms[(size_t)b * N + i] * total, cum = 0.0;
            int pick = -1, last_pos = 0;
            double lo = 0.0, hi = 0.0;
            for (int s = 0; s < T; ++s) {
                if (w[s] > 0.0) last_pos = s;
                if (pick < 0 && cum + w[s] > target) { pick = s; lo = cum; hi = cum + w[s]; }
                cum += w[s];
            }
            if (pick < 0) { pick = last_pos; lo = hi = target; }
            y[i] = pick;
            double d1 = (target - lo) / total, d2 = (hi - target) / total;
            if (pick == 0 || lo == 0.0) d1 = 1.0;           /* nothing below to fall into */
            if (d1 < worst) worst = d1;
            if (d2 < worst) worst = d2;
        }
        if (margin) margin[b] = worst;
        free(alpha); free(tmp); free(w);
    }
    return err ? -2 : 0;
}

/*
 * Max-plus semiring.  delta[i][t] = best score of a prefix ending in t;
 * bp[i][t] = smallest s attaining it.  The last tag is the smallest t attaining
 * max_t delta[L-1][t]; earlier tags follow the back-pointers.  tags[b][i] = -1 for
 * i >= L.
 *
 * gap[b] (optional) = best score minus the score of the best path that differs
 * from the returned one.  With eps the max-plus backward recursion,
 * mm[i][s][t] = delta[i-1][s] + phi[i][s][t] + eps[i][t] is the best score among
 * paths using edge (i, s, t) (and mm[0][t] = delta[0][t] + eps[0][t] among paths
 * starting in t).  Any other path uses at least one edge off the best path, so the
 * runner-up score is the largest mm over off-path edges.  +inf when there is no
 * other path (T = 1 or L = 0).
 */
int lccrf_oracle_viterbi(const void *phi, int dtype, const int32_t *lengths,
                         int B, int N, int T,
                         double *score /* may be NULL */, int32_t *tags, double *gap /* may be NULL */)
{
    if (!phi || !tags || B < 1 || N < 1 || T < 1 || (dtype != 0 && dtype != 1)) return -1;
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        int L = clamp_len(lengths, b, N);
        size_t base = (size_t)b * N * T * T;
        int32_t *y = tags + (size_t)b * N;
        for (int i = 0; i < N; ++i) y[i] = -1;
        if (L == 0) {
            if (score) score[b] = 0.0;
            if (gap) gap[b] = INFINITY;
            continue;
        }
        double *delta = (double *)malloc(sizeof(double) * (size_t)L * T);
        double *eps = (double *)malloc(sizeof(double) * (size_t)L * T);
        int32_t *bp = (int32_t *)malloc(sizeof(int32_t) * (size_t)L * T);
        if (!delta || !eps || !bp) { err = 1; free(delta); free(eps); free(bp); continue; }

        for (int t = 0; t < T; ++t) { delta[t] = phi_at(phi, dtype, base + (size_t)t); bp[t] = -1; }
        for (int i = 1; i < L; ++i) {
            size_t m = base + (size_t)i * T * T;
            for (int t = 0; t < T; ++t) {
                double best = -INFINITY; int arg = 0;
                for (int s = 0; s < T; ++s) {
                    double v = delta[(size_t)(i - 1) * T + s] + phi_at(phi, dtype, m + (size_t)s * T + t);
                    if (v > best) { best = v; arg = s; }
                }
                delta[(size_t)i * T + t] = best;
                bp[(size_t)i * T + t] = arg;
            }
        }
        double best = -INFINITY; int last = 0;
        for (int t = 0; t < T; ++t)
            if (delta[(size_t)(L - 1) * T + t] > best) { best = delta[(size_t)(L - 1) * T + t]; last = t; }
        if (score) score[b] = best;
        y[L - 1] = last;
        for (int i = L - 1; i >= 1; --i) y[i - 1] = bp[(size_t)i * T + y[i]];

        if (gap) {
            for (int t = 0; t < T; ++t) eps[(size_t)(L - 1) * T + t] = 0.0;
            for (int i = L - 1; i >= 1; --i) {
                size_t m = base + (size_t)i * T * T;
                for (int s = 0; s < T; ++s) {
                    double e = -INFINITY;
                    for (int t = 0; t < T; ++t) {
                        double v = phi_at(phi, dtype, m + (size_t)s * T + t) + eps[(size_t)i * T + t];
                        if (v > e) e = v;
                    }
                    eps[(size_t)(i - 1) * T + s] = e;
                }
            }
            double second = -INFINITY;
            for (int t = 0; t < T; ++t) {
                if (t == y[0]) continue;
                double v = delta[t] + eps[t];
                if (v > second) second = v;
            }
            for (int i = 1; i < L; ++i) {
                size_t m = base + (size_t)i * T * T;
                for (int s = 0; s < T; ++s)
                    for (int t = 0; t < T; ++t) {
                        if (s == y[i - 1] && t == y[i]) continue;
                        double v = delta[(size_t)(i - 1) * T + s] + phi_at(phi, dtype, m + (size_t)s * T + t)
                                   + eps[(size_t)i * T + t];
                        if (v > second) second = v;
                    }
            }
            if (best == -INFINITY) gap[b] = 0.0;           /* no finite path at all: nothing to separate */
            else gap[b] = best - second;                   /* +inf when no other finite path exists */
        }
        free(delta); free(eps); free(bp);
    }
    return err ? -2 : 0;
}

/* Number of OpenMP threads a parallel region would use (1 when built without OpenMP). */
#ifdef _OPENMP
#include <omp.h>
int lccrf_oracle_threads(void) { return omp_get_max_threads(); }
#else
int lccrf_oracle_threads(void) { return 1; }
#endif

/*
 * Semi-Markov CRF, log-partition (section "Segmentation with Semi-Markov CRF": the linear chain's
 * parametrisation with transition matrices, except that a transition may jump over several
 * positions; forward algorithm in O(K T^2 L) for segments of at most K positions).
 *
 * A structure is a split of positions 0..L-1 into consecutive segments of 1..K positions, each
 * carrying a tag.  phi[b][i][k][s][t] is the log-potential of a segment with tag t that ENDS at
 * position i and covers k + 1 positions, the segment before it carrying tag s; for the first
 * segment (k = i) row s = 0 is used, the linear chain's convention for its first tag.  With
 *     alpha_i(t) = log of the summed potential of all labelled splits of 0..i whose last
 *                  segment has tag t,
 *     alpha_i(t) = logsumexp over k = 0..min(K-1, i) and s of  alpha_{i-k-1}(s) + phi[i][k][s][t],
 *     alpha_{-1}(s) = 0 for s = 0 and -inf otherwise,
 * logZ = logsumexp_t alpha_{L-1}(t).  Entries with k > i, and rows s > 0 of the first segments,
 * are never read.  K = 1 is the linear chain.  Empty sequence: logZ = 0.
 */
int lccrf_oracle_semi_markov_log_partition(const void *phi, int dtype, const int32_t *lengths,
                                           int B, int N, int K, int T, double *logZ)
{
    if (!phi || !logZ || B < 1 || N < 1 || K < 1 || T < 1 || (dtype != 0 && dtype != 1)) return -1;
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        int L = clamp_len(lengths, b, N);
        if (L == 0) { logZ[b] = 0.0; continue; }
        size_t base = (size_t)b * N * K * T * T;
        double *alpha = (double *)malloc(sizeof(double) * (size_t)L * T);
        double *terms = (double *)malloc(sizeof(double) * (size_t)K * T);
        if (!alpha || !terms) { err = 1; free(alpha); free(terms); continue; }
        for (int i = 0; i < L; ++i)
            for (int t = 0; t < T; ++t) {
                int n = 0;
                for (int k = 0; k < K && k <= i; ++k) {
                    size_t m = base + (((size_t)i * K + k) * T) * T;
                    if (k == i) {               /* first segment: the empty prefix, row 0 */
                        terms[n++] = phi_at(phi, dtype, m + (size_t)t);
                    } else {
                        const double *prev = alpha + (size_t)(i - k - 1) * T;
                        for (int s2 = 0; s2 < T; ++s2)
                            terms[n++] = prev[s2] + phi_at(phi, dtype, m + (size_t)s2 * T + t);
                    }
                }
                alpha[(size_t)i * T + t] = logsumexp(terms, n);
            }
        logZ[b] = logsumexp(alpha + (size_t)(L - 1) * T, T);
        free(alpha); free(terms);
    }
    return err ? -2 : 0;
}
