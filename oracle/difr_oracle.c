/*
 * difr_oracle.c -- CPU oracle for the per-token verification scores.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * verifier's vocabulary pass computes.  It exists so that the GPU library can be
 * checked against something independent of it.  It shares no code, header,
 * table or constant generator with the HIP path, and nothing in the product
 * path may call it: only the tests, the smoke check and the benchmark's
 * cpu_baseline leg do.
 *
 * Everything is IEEE double, one row at a time, one vocabulary entry at a time,
 * in the order the paper states the steps.  Rows are independent, so the batch
 * entry points parallelise the OUTERMOST row loop with OpenMP and nothing else.
 *
 * What each function follows (paper: "Verifying LLM Inference to Detect Model
 * Weight Exfiltration"):
 *   - temperature softmax ................. Sec. 3.2, the softmax(z/T) equation
 *   - IPT sampler (CDF, first C_t > u) .... Sec. 3.2, Algorithm "IPT Sampler"
 *   - Gumbel-max sampler .................. Sec. 3.2, Algorithm "Gumbel-Max Sampler"
 *   - Token-IPT-DiFR interval and score ... Sec. 6.2 and the appendix algorithm
 *                                           "convolved Gaussian score"
 *   - Token-DiFR noise, ranking, A_{sigma,i}  Sec. 6.3 and the appendix algorithm
 *                                           for the Gumbel likelihood estimator
 *   - regenerate-and-compare per position . Sec. 5.1 and the appendix algorithm
 *                                           "verification via prefill"
 *   - Token-DiFR likelihood estimate ...... Sec. 6.3, appendix algorithm of the
 *                                           Gumbel-max FSSL estimator (active set,
 *                                           filter threshold, A, B, noise average)
 *   - Token-IPT-DiFR under the sampler's     Sec. 3.2 (filter policy), Sec. 6.2, appendix
 *     top-k / top-p filter .................  "convolved Gaussian score"
 *   - admissible set size ................. Sec. 7 (A_t(tau), log2 |A_t| bits per
 *                                           accepted token), appendix "Threshold
 *                                           selection and FPR-information trade-off"
 *   - logits from the final hidden state .. the Prefill step of the appendix
 *                                           algorithm "verification via prefill"
 *   - pooling and flagging ................ Sec. 5.2 (threshold rule), Sec. 6.4,
 *                                           appendix "Response to detecting
 *                                           exfiltration attempts" (score, pool, flag)
 *
 * Readings taken where the paper is silent or inconsistent:
 *   - H(seed || i) is Philox4x32-10 (Salmon et al., SC'11), key = the two halves
 *     of the 64-bit sequence seed, counter = (v >> 2, position, sequence, stream),
 *     output word v & 3.  stream 0 = Gumbel noise, stream 1 = the IPT uniform.
 *   - 32 bits r -> uniform: k = r >> 9, u = (2k + 1) * 2^-24, strictly inside (0,1)
 *     and exactly representable in single and double precision.
 *   - Gumbel: g = -ln(-ln u), natural logarithm.
 *   - the Gumbel-max sampler's printed "p_t + z_t" is read as log p_t + g_t, which
 *     has the same argmax as x_t / T + g_t (Sec. 3.2 text; Sec. 6.3 ranks by
 *     l_i + T G_i, again the same argmax for T > 0).
 *   - margin = max_v (x_v/T + g_v) - (x_t/T + g_t) for the claimed token t, i.e.
 *     -min_i A_{sigma,i} / T in the appendix algorithm's notation.
 *   - argmax ties go to the lowest index.
 *   - CDF in ascending vocabulary index, no sorting, no filtering; the claimed
 *     token's interval is [a, b) (sampler rule C_t > u).
 *   - Token-IPT-DiFR: mu = x = u in the printed algorithm; sigma is the Gaussian
 *     width, eps the small constant inside the logarithm.
 *   - pooling is the per-sequence mean; scores are suspiciousness, so a sequence
 *     is flagged unless mean <= tau (a NaN mean is flagged).
 *
 * Parity pins (tests/test_oracle_*.py): Philox known-answer vectors; closed forms
 * of the k -> u -> g map and its moments; brute force with exact rationals and
 * multi-precision on tiny vocabularies; library softmax / cumsum / searchsorted;
 * chi-square of sample frequencies; Gumbel max-stability; scipy / mpmath normal
 * CDF; the likelihood estimate against closed forms (no competitor, one competitor),
 * a direct simulation of the noisy race it describes, explicit Python sorting for the
 * active set and the filter threshold; the admissible-set count against explicit sorting and its geometric law;
 * the hidden-state-to-logits step against a library matrix product and
 * against the stored-logit entry points on inputs whose products are exact.
 * No function here is "parity unpinned".
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_DTYPE_BF16 0
#define ORACLE_DTYPE_F32 1

#define ORACLE_FLAG_MATCH 1u
#define ORACLE_FLAG_INVALID_CLAIM 2u
#define ORACLE_FLAG_NONFINITE 4u

#define ORACLE_STREAM_GUMBEL 0u
#define ORACLE_STREAM_IPT 1u

/* ------------------------------------------------------------------------- */
/* Philox4x32-10, from the published round definition.                        */
/* One round maps (c0,c1,c2,c3) with key (k0,k1) to                           */
/*   (hi(M1*c2)^c1^k0, lo(M1*c2), hi(M0*c0)^c3^k1, lo(M0*c0));                */
/* the key is bumped by the Weyl constants between rounds.                    */
/* ------------------------------------------------------------------------- */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        if (round > 0) {
            k0 += W0;
            k1 += W1;
        }
        uint64_t p0 = M0 * (uint64_t)c0;
        uint64_t p1 = M1 * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The 32 noise bits of vocabulary entry v at (seed, sequence, position, stream). */
uint32_t oracle_noise_word(uint64_t seed, uint32_t seq, uint32_t pos, uint32_t stream, uint64_t v)
{
    uint32_t ctr[4] = { (uint32_t)(v >> 2), pos, seq, stream };
    uint32_t key[2] = { (uint32_t)(seed & 0xFFFFFFFFu), (uint32_t)(seed >> 32) };
    uint32_t out[4];
    oracle_philox4x32_10(ctr, key, out);
    return out[v & 3u];
}

/* 32 bits -> uniform strictly inside (0,1): 23 bits, midpoint of each cell. */
double oracle_bits_to_uniform(uint32_t r)
{
    uint32_t k = r >> 9;
    return (2.0 * (double)k + 1.0) * 0x1p-24;
}

/* Standard Gumbel from a uniform: g = -ln(-ln u).  For u > 1/2 the inner
 * logarithm is taken as log1p(-(1-u)); 1-u is exact for the u above, so this is
 * the same real number evaluated without cancellation. */
double oracle_uniform_to_gumbel(double u)
{
    double t;
    if (u > 0.5)
        t = -log1p(-(1.0 - u));
    else
        t = -log(u);
    return -log(t);
}

/* The map above applied to n raw noise words (used to check a device map exhaustively). */
void oracle_gumbel_from_bits_array(const uint32_t *bits, int64_t n, double *g)
{
    for (int64_t i = 0; i < n; ++i) g[i] = oracle_uniform_to_gumbel(oracle_bits_to_uniform(bits[i]));
}

/* Exact value of a stored logit as a double. */
static double decode_bf16(uint16_t h)
{
    uint32_t w = (uint32_t)h << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

void oracle_decode_row(const void *row, int dtype, int64_t V, double *x)
{
    if (dtype == ORACLE_DTYPE_BF16) {
        const uint16_t *p = (const uint16_t *)row;
        for (int64_t v = 0; v < V; ++v) x[v] = decode_bf16(p[v]);
    } else {
        const float *p = (const float *)row;
        for (int64_t v = 0; v < V; ++v) x[v] = (double)p[v];
    }
}

/* Fill bits[v] with the raw noise words of one row (Gumbel or IPT stream). */
void oracle_noise_row(uint64_t seed, uint32_t seq, uint32_t pos, uint32_t stream, int64_t V, uint32_t *bits)
{
    for (int64_t v = 0; v < V; ++v) bits[v] = oracle_noise_word(seed, seq, pos, stream, (uint64_t)v);
}

/* ------------------------------------------------------------------------- */
/* Token-DiFR, one row.                                                       */
/*   y_v = x_v / T + g_v  for every v;  vhat = lowest index attaining max y;  */
/*   margin = y_vhat - y_t;  gap2 = y_vhat - (largest y over v != vhat).      */
/* claimed < 0 or >= V: margin and claimed_score are NaN, INVALID_CLAIM set   */
/* (claimed == -1 is how the sampler is asked for, see oracle_gumbel_score).  */
/* Optionally writes every y_v into y_out (tests use it).                     */
/* ------------------------------------------------------------------------- */
void oracle_gumbel_row(const double *x, int64_t V, double T, uint64_t seed, uint32_t seq, uint32_t pos,
                       int64_t claimed, double *margin, int32_t *argmax, double *max_score,
                       double *claimed_score, double *gap2, uint8_t *flags, double *y_out)
{
    double best = -INFINITY, second = -INFINITY, yt = NAN;
    int64_t best_v = -1;
    int nonfinite = 0;
    for (int64_t v = 0; v < V; ++v) {
        uint32_t r = oracle_noise_word(seed, seq, pos, ORACLE_STREAM_GUMBEL, (uint64_t)v);
        double u = oracle_bits_to_uniform(r);
        double g = oracle_uniform_to_gumbel(u);
        double y = x[v] / T + g;
        if (isnan(x[v]) || x[v] == INFINITY) nonfinite = 1;
        if (y_out) y_out[v] = y;
        if (v == claimed) yt = y;
        if (best_v < 0 || y > best) {
            second = best;
            best = y;
            best_v = v;
        } else if (y > second) {
            second = y;
        }
    }
    uint8_t f = 0;
    if (claimed < 0 || claimed >= V) {
        f |= ORACLE_FLAG_INVALID_CLAIM;
        *margin = NAN;
        *claimed_score = NAN;
    } else {
        *margin = best - yt;
        *claimed_score = yt;
        if (best_v == claimed) f |= ORACLE_FLAG_MATCH;
    }
    if (nonfinite) f |= ORACLE_FLAG_NONFINITE;
    *argmax = (int32_t)best_v;
    *max_score = best;
    *gap2 = best - second;
    *flags = f;
}

/* ------------------------------------------------------------------------- */
/* Gaussian log-mass of Token-IPT-DiFR:                                       */
/*   S = ln( Phi((b-u)/sigma) - Phi((a-u)/sigma) + eps ),                     */
/*   Phi(z) = (1 + erf(z / sqrt 2)) / 2.                                      */
/* The difference of the two normal CDF values is taken on the side where it  */
/* does not cancel (erfc in the tails); it is the same real number.           */
/* ------------------------------------------------------------------------- */
double oracle_gaussian_log_mass(double a, double b, double u, double sigma, double eps)
{
    double za = (a - u) / (sigma * M_SQRT2);
    double zb = (b - u) / (sigma * M_SQRT2);
    double mass;
    if (za >= 0.0)
        mass = 0.5 * (erfc(za) - erfc(zb));
    else if (zb <= 0.0)
        mass = 0.5 * (erfc(-zb) - erfc(-za));
    else
        mass = 0.5 * (erf(zb) + erf(-za));
    if (mass < 0.0) mass = 0.0;
    return log(mass + eps);
}

/* ------------------------------------------------------------------------- */
/* Token-IPT-DiFR, one row.                                                   */
/*   u from stream 1; p = softmax(x/T); Fbar = (0, cumsum p) in index order;  */
/*   a = Fbar[t], b = Fbar[t+1] (0-based t); d = max(a-u, u-b, 0);            */
/*   match = a <= u < b;  tok = first v with Fbar[v+1] > u.                   */
/* edge = min(|u-a|, |u-b|) is reported for the tests' near-tie rule.         */
/* ------------------------------------------------------------------------- */
void oracle_ipt_row(const double *x, int64_t V, double T, uint64_t seed, uint32_t seq, uint32_t pos,
                    int64_t claimed, double sigma, double eps, double *u_out, double *a_out, double *b_out,
                    double *dist, int32_t *tok, double *log_mass, double *edge, uint8_t *flags)
{
    uint32_t r = oracle_noise_word(seed, seq, pos, ORACLE_STREAM_IPT, 0);
    double u = oracle_bits_to_uniform(r);
    int nonfinite = 0;
    double m = -INFINITY;
    for (int64_t v = 0; v < V; ++v) {
        double s = x[v] / T;
        if (isnan(x[v]) || x[v] == INFINITY) nonfinite = 1;
        if (s > m) m = s;
    }
    double Z = 0.0;
    for (int64_t v = 0; v < V; ++v) Z += exp(x[v] / T - m);

    int valid = (claimed >= 0 && claimed < V);
    double c = 0.0, a = NAN, b = NAN;
    int64_t first = -1;
    for (int64_t v = 0; v < V; ++v) {
        double e = exp(x[v] / T - m);
        if (valid && v == claimed) {
            a = c / Z;
            b = a + e / Z;
        }
        c += e;
        if (first < 0 && c / Z > u) first = v;
    }
    if (first < 0) first = V - 1;

    uint8_t f = 0;
    if (!valid) {
        f |= ORACLE_FLAG_INVALID_CLAIM;
        *dist = NAN;
        *edge = NAN;
        *log_mass = NAN;
    } else {
        double d = 0.0;
        if (a - u > d) d = a - u;
        if (u - b > d) d = u - b;
        *dist = d;
        if (a <= u && u < b) f |= ORACLE_FLAG_MATCH;
        *edge = fmin(fabs(u - a), fabs(u - b));
        *log_mass = oracle_gaussian_log_mass(a, b, u, sigma, eps);
    }
    if (nonfinite) f |= ORACLE_FLAG_NONFINITE;
    *u_out = u;
    *a_out = a;
    *b_out = b;
    *tok = (int32_t)first;
    *flags = f;
}

/* ------------------------------------------------------------------------- */
/* Batch entry points: rows are independent; parallel over rows only.         */
/* logits: [N, ld] row-major host memory, dtype ORACLE_DTYPE_*.               */
/* temperatures may be NULL (then T = temperature for every row).             */
/* claimed may be NULL (every row is then treated as claimed = -1: sampling). */
/* ------------------------------------------------------------------------- */
static size_t elt_size(int dtype) { return dtype == ORACLE_DTYPE_BF16 ? 2u : 4u; }

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

int oracle_gumbel_score(const void *logits, int dtype, int64_t N, int64_t V, int64_t ld, double temperature,
                        const float *temperatures, const uint64_t *seeds, const int32_t *seq_ids,
                        const uint32_t *positions, const int32_t *claimed, double *margin, int32_t *argmax,
                        double *max_score, double *claimed_score, double *gap2, uint8_t *flags)
{
    int failed = 0;
#pragma omp parallel
    {
        double *x = (double *)malloc((size_t)(V > 0 ? V : 1) * sizeof(double));
        if (!x) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (int64_t n = 0; n < N; ++n) {
            if (!x) continue;
            const char *row = (const char *)logits + (size_t)n * (size_t)ld * elt_size(dtype);
            oracle_decode_row(row, dtype, V, x);
            double T = temperatures ? (double)temperatures[n] : temperature;
            int32_t s = seq_ids[n];
            int64_t t = claimed ? (int64_t)claimed[n] : -1;
            oracle_gumbel_row(x, V, T, seeds[s], (uint32_t)s, positions[n], t, &margin[n], &argmax[n],
                              &max_score[n], &claimed_score[n], &gap2[n], &flags[n], NULL);
        }
        free(x);
    }
    return failed;
}

int oracle_ipt_score(const void *logits, int dtype, int64_t N, int64_t V, int64_t ld, double temperature,
                     const float *temperatures, const uint64_t *seeds, const int32_t *seq_ids,
                     const uint32_t *positions, const int32_t *claimed, double sigma, double eps, double *u,
                     double *cdf_lo, double *cdf_hi, double *dist, int32_t *tok, double *log_mass, double *edge,
                     uint8_t *flags)
{
    int failed = 0;
#pragma omp parallel
    {
        double *x = (double *)malloc((size_t)(V > 0 ? V : 1) * sizeof(double));
        if (!x) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (int64_t n = 0; n < N; ++n) {
            if (!x) continue;
            const char *row = (const char *)logits + (size_t)n * (size_t)ld * elt_size(dtype);
            oracle_decode_row(row, dtype, V, x);
            double T = temperatures ? (double)temperatures[n] : temperature;
            int32_t s = seq_ids[n];
            int64_t t = claimed ? (int64_t)claimed[n] : -1;
            oracle_ipt_row(x, V, T, seeds[s], (uint32_t)s, positions[n], t, sigma, eps, &u[n], &cdf_lo[n],
                           &cdf_hi[n], &dist[n], &tok[n], &log_mass[n], &edge[n], &flags[n]);
        }
        free(x);
    }
    return failed;
}

/* ------------------------------------------------------------------------- */
/* Size of the admissible set of one position (Sec. 7: A_t(tau) = the tokens   */
/* the verifier would accept; an accepted token carries at most log2 |A_t|     */
/* bits).  With the Token-DiFR margin as the score, a token v is accepted when */
/* its margin  max_w y_w - y_v  is at most delta:                              */
/*   count = #{ v : max_w y_w - y_v <= delta }.                                */
/* The same count at delta - tol and delta + tol brackets what an evaluation   */
/* in lower precision may return.  y must hold V doubles of scratch.           */
/* ------------------------------------------------------------------------- */
void oracle_admissible_count_row(const double *x, int64_t V, double T, uint64_t seed, uint32_t seq, uint32_t pos,
                                 double delta, double tol, double *y, int32_t *count, int32_t *count_lo,
                                 int32_t *count_hi)
{
    double margin, max_score, claimed_score, gap2;
    int32_t argmax;
    uint8_t flags;
    oracle_gumbel_row(x, V, T, seed, seq, pos, -1, &margin, &argmax, &max_score, &claimed_score, &gap2, &flags, y);
    int32_t c = 0, lo = 0, hi = 0;
    for (int64_t v = 0; v < V; ++v) {
        double m = max_score - y[v];
        if (m <= delta) ++c;
        if (m <= delta - tol) ++lo;
        if (m <= delta + tol) ++hi;
    }
    *count = c;
    *count_lo = lo;
    *count_hi = hi;
}

int oracle_admissible_count(const void *logits, int dtype, int64_t N, int64_t V, int64_t ld, double temperature,
                            const float *temperatures, const uint64_t *seeds, const int32_t *seq_ids,
                            const uint32_t *positions, double delta, double tol, int32_t *count, int32_t *count_lo,
                            int32_t *count_hi)
{
    int failed = 0;
#pragma omp parallel
    {
        double *x = (double *)malloc((size_t)(V > 0 ? V : 1) * 2 * sizeof(double));
        if (!x) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (int64_t n = 0; n < N; ++n) {
            if (!x) continue;
            const char *row = (const char *)logits + (size_t)n * (size_t)ld * elt_size(dtype);
            oracle_decode_row(row, dtype, V, x);
            double T = temperatures ? (double)temperatures[n] : temperature;
            int32_t s = seq_ids[n];
            oracle_admissible_count_row(x, V, T, seeds[s], (uint32_t)s, positions[n], delta, tol, x + V, &count[n],
                                        &count_lo[n], &count_hi[n]);
        }
        free(x);
    }
    return failed;
}

/* ------------------------------------------------------------------------- */
/* Token-DiFR likelihood estimate of the claimed token (Sec. 6.3 and the        */
/* appendix algorithm of the Gumbel-max FSSL estimator), in the algorithm's     */
/* order and notation, Gaussian noise N(0, sigma^2) on every logit:             */
/*   1. G_i for every token (as everywhere in this file).                       */
/*   2. S = the s tokens with the largest l_i + T G_i, the claimed token left   */
/*      out (a factor for i = t* would compare t* with itself); ties to the     */
/*      lower index.                                                            */
/*   3. tau = the smallest logit the sampler's filter keeps: top-k first (the   */
/*      k largest logits), then top-p on the distribution renormalised over     */
/*      those k (the shortest prefix, in descending logit order, whose          */
/*      softmax(l/T) mass reaches p).  k <= 0: no top-k; p >= 1: no top-p;      */
/*      neither: tau = -inf.  With k <= 0 the nucleus is taken over the whole   */
/*      vocabulary.                                                             */
/*   4. A_i = l_t* - l_i + T (G_t* - G_i),  B_i = tau - l_i   for i in S.       */
/*   5. pi = (1/M) sum_j [l_t* + x_j > tau] prod_{i in S} Phi(max(x_j + A_i,    */
/*      B_i) / sigma),  x_j = sigma z_j, with the M standard normal draws z_j   */
/*      supplied by the caller (the algorithm samples them; drawing them is     */
/*      not part of what is checked here).                                      */
/* Outputs: pi, ln pi (-inf if pi = 0), tau, the set S (s indices, -1 padded,   */
/* in rank order) and two gaps for the tests' near-tie rule: gap_s = distance   */
/* between the last member of S and the best token left out, gap_p = distance   */
/* of the nucleus' cumulative mass from p at the two prefixes around the cut.   */
/* claimed outside [0,V): pi = NaN.                                             */
/* ------------------------------------------------------------------------- */
static double normal_cdf(double z) { return 0.5 * erfc(-z / M_SQRT2); }

typedef struct {
    double key;
    int64_t idx;
} keyed;

static int keyed_desc(const void *a, const void *b)
{
    const keyed *p = (const keyed *)a, *q = (const keyed *)b;
    if (p->key > q->key) return -1;
    if (p->key < q->key) return 1;
    return p->idx < q->idx ? -1 : (p->idx > q->idx ? 1 : 0);
}

/* The sampler's filter (Sec. 3.2 "temperature / top-k / nucleus policy"; the experiments use k = 50,     */
/* p = 0.95): tokens ranked by logit, descending, ties to the lower index; top-k keeps the first k;        */
/* top-p then keeps the shortest prefix of those whose softmax(l/T) mass, renormalised over the k, reaches */
/* p.  Fills order[0..V) with the ranking and returns the length of the kept prefix (>= 1).  gap_p: how    */
/* close the cumulative mass came to p on either side of the cut (for the tests' near-tie rule).           */
static int64_t filter_prefix(const double *x, int64_t V, double T, int64_t top_k, double top_p, keyed *order,
                             double *gap_p)
{
    for (int64_t v = 0; v < V; ++v) {
        order[v].key = x[v];
        order[v].idx = v;
    }
    qsort(order, (size_t)V, sizeof(keyed), keyed_desc);
    int64_t kept = (top_k > 0 && top_k < V) ? top_k : V;
    *gap_p = INFINITY;
    if (top_p < 1.0) {
        double Z = 0.0;
        for (int64_t r = 0; r < kept; ++r) Z += exp((order[r].key - order[0].key) / T);
        double cum = 0.0;
        for (int64_t r = 0; r < kept; ++r) {
            double before = cum;
            cum += exp((order[r].key - order[0].key) / T) / Z;
            if (cum >= top_p) {
                *gap_p = fmin(fabs(cum - top_p), fabs(top_p - before));
                kept = r + 1;
                break;
            }
        }
    }
    return kept;
}

int oracle_likelihood_row(const double *x, int64_t V, double T, uint64_t seed, uint32_t seq, uint32_t pos,
                          int64_t claimed, int64_t top_k, double top_p, int64_t s, double sigma, const double *z,
                          int64_t M, double *pi, double *log_pi, double *tau_out, int32_t *S_out, double *gap_s,
                          double *gap_p)
{
    keyed *a = (keyed *)malloc((size_t)(V > 0 ? V : 1) * sizeof(keyed));
    double *g = (double *)malloc((size_t)(V > 0 ? V : 1) * sizeof(double));
    if (!a || !g) {
        free(a);
        free(g);
        return 1;
    }
    /* 1. noise */
    for (int64_t v = 0; v < V; ++v)
        g[v] = oracle_uniform_to_gumbel(oracle_bits_to_uniform(oracle_noise_word(seed, seq, pos, ORACLE_STREAM_GUMBEL, (uint64_t)v)));
    const int valid = claimed >= 0 && claimed < V;
    /* 3. filter threshold (does not depend on the claim) */
    double tau = -INFINITY;
    *gap_p = INFINITY;
    if (top_k > 0 || top_p < 1.0) {
        int64_t kept = filter_prefix(x, V, T, top_k, top_p, a, gap_p);
        tau = a[kept - 1].key;
    }
    *tau_out = tau;
    for (int64_t j = 0; j < s; ++j) S_out[j] = -1;
    *gap_s = INFINITY;
    if (!valid) {
        *pi = NAN;
        *log_pi = NAN;
        free(a);
        free(g);
        return 0;
    }
    /* 2. active set */
    int64_t n = 0;
    for (int64_t v = 0; v < V; ++v) {
        if (v == claimed) continue;
        a[n].key = x[v] + T * g[v];
        a[n].idx = v;
        ++n;
    }
    qsort(a, (size_t)n, sizeof(keyed), keyed_desc);
    const int64_t ns = s < n ? s : n;
    if (ns > 0 && ns < n) *gap_s = (a[ns - 1].key - a[ns].key) / T; /* in units of l/T + G */
    /* 4. */
    double *A = (double *)malloc((size_t)(ns > 0 ? ns : 1) * 2 * sizeof(double)), *B = A + (ns > 0 ? ns : 1);
    if (!A) {
        free(a);
        free(g);
        return 1;
    }
    for (int64_t j = 0; j < ns; ++j) {
        const int64_t i = a[j].idx;
        S_out[j] = (int32_t)i;
        A[j] = x[claimed] - x[i] + T * (g[claimed] - g[i]);
        B[j] = tau - x[i];
    }
    /* 5. */
    double acc = 0.0;
    for (int64_t j = 0; j < M; ++j) {
        const double xj = sigma * z[j];
        if (x[claimed] + xj > tau) {
            double prod = 1.0;
            for (int64_t i = 0; i < ns; ++i) prod *= normal_cdf(fmax(xj + A[i], B[i]) / sigma);
            acc += prod;
        }
    }
    *pi = M > 0 ? acc / (double)M : NAN;
    *log_pi = log(*pi);
    free(A);
    free(a);
    free(g);
    return 0;
}

int oracle_likelihood(const void *logits, int dtype, int64_t N, int64_t V, int64_t ld, double temperature,
                      const float *temperatures, const uint64_t *seeds, const int32_t *seq_ids,
                      const uint32_t *positions, const int32_t *claimed, int64_t top_k, double top_p, int64_t s,
                      double sigma, const double *z, int64_t M, double *pi, double *log_pi, double *tau,
                      int32_t *S_out, double *gap_s, double *gap_p)
{
    int failed = 0;
#pragma omp parallel
    {
        double *x = (double *)malloc((size_t)(V > 0 ? V : 1) * sizeof(double));
        if (!x) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (int64_t n = 0; n < N; ++n) {
            if (!x) continue;
            const char *row = (const char *)logits + (size_t)n * (size_t)ld * elt_size(dtype);
            oracle_decode_row(row, dtype, V, x);
            double T = temperatures ? (double)temperatures[n] : temperature;
            int32_t sq = seq_ids[n];
            int64_t t = claimed ? (int64_t)claimed[n] : -1;
            if (oracle_likelihood_row(x, V, T, seeds[sq], (uint32_t)sq, positions[n], t, top_k, top_p, s, sigma, z, M,
                                      &pi[n], &log_pi[n], &tau[n], S_out + (size_t)n * (size_t)(s > 0 ? s : 0),
                                      &gap_s[n], &gap_p[n])) {
#pragma omp atomic write
                failed = 1;
            }
        }
        free(x);
    }
    return failed;
}

/* ------------------------------------------------------------------------- */
/* Token-IPT-DiFR when the sampler filters (Sec. 3.2 IPT sampler applied to the  */
/* filtered, renormalised distribution; appendix "convolved Gaussian score":     */
/* "token probabilities p" are the probabilities the sampler actually used).     */
/*   K = the kept prefix of filter_prefix();  p'_v = exp(x_v/T) / sum_K for      */
/*   v in K, 0 otherwise;  Fbar over ascending vocabulary index;  a, b, d, match */
/*   and the sampler's token as in oracle_ipt_row.  A claimed token outside K    */
/*   has an empty interval a = b (never a match, d = |u - a|).                   */
/* kept_out: |K|.  top_k <= 0 and top_p >= 1: identical to oracle_ipt_row.       */
/* ------------------------------------------------------------------------- */
int oracle_ipt_filtered_row(const double *x, int64_t V, double T, uint64_t seed, uint32_t seq, uint32_t pos,
                            int64_t claimed, int64_t top_k, double top_p, double sigma, double eps, double *u_out,
                            double *a_out, double *b_out, double *dist, int32_t *tok, double *log_mass, double *edge,
                            int32_t *kept_out, double *gap_p, uint8_t *flags)
{
    keyed *order = (keyed *)malloc((size_t)(V > 0 ? V : 1) * sizeof(keyed));
    unsigned char *in_K = (unsigned char *)calloc((size_t)(V > 0 ? V : 1), 1);
    if (!order || !in_K) {
        free(order);
        free(in_K);
        return 1;
    }
    const int64_t kept = filter_prefix(x, V, T, top_k, top_p, order, gap_p);
    for (int64_t r = 0; r < kept; ++r) in_K[order[r].idx] = 1;
    const double top = order[0].key;
    free(order);
    uint32_t r = oracle_noise_word(seed, seq, pos, ORACLE_STREAM_IPT, 0);
    double u = oracle_bits_to_uniform(r);
    int nonfinite = 0;
    double Z = 0.0;
    for (int64_t v = 0; v < V; ++v) {
        if (isnan(x[v]) || x[v] == INFINITY) nonfinite = 1;
        if (in_K[v]) Z += exp((x[v] - top) / T);
    }
    int valid = (claimed >= 0 && claimed < V);
    double c = 0.0, a = NAN, b = NAN;
    int64_t first = -1, last_kept = -1;
    for (int64_t v = 0; v < V; ++v) {
        double e = in_K[v] ? exp((x[v] - top) / T) : 0.0;
        if (valid && v == claimed) {
            a = c / Z;
            b = a + e / Z;
        }
        c += e;
        if (in_K[v]) last_kept = v;
        if (first < 0 && in_K[v] && c / Z > u) first = v;
    }
    if (first < 0) first = last_kept;
    free(in_K);
    uint8_t f = 0;
    if (!valid) {
        f |= ORACLE_FLAG_INVALID_CLAIM;
        *dist = NAN;
        *edge = NAN;
        *log_mass = NAN;
    } else {
        double d = 0.0;
        if (a - u > d) d = a - u;
        if (u - b > d) d = u - b;
        *dist = d;
        if (a <= u && u < b) f |= ORACLE_FLAG_MATCH;
        *edge = fmin(fabs(u - a), fabs(u - b));
        *log_mass = oracle_gaussian_log_mass(a, b, u, sigma, eps);
    }
    if (nonfinite) f |= ORACLE_FLAG_NONFINITE;
    *u_out = u;
    *a_out = a;
    *b_out = b;
    *tok = (int32_t)first;
    *kept_out = (int32_t)kept;
    *flags = f;
    return 0;
}

int oracle_ipt_filtered_score(const void *logits, int dtype, int64_t N, int64_t V, int64_t ld, double temperature,
                              const float *temperatures, const uint64_t *seeds, const int32_t *seq_ids,
                              const uint32_t *positions, const int32_t *claimed, int64_t top_k, double top_p,
                              double sigma, double eps, double *u, double *cdf_lo, double *cdf_hi, double *dist,
                              int32_t *tok, double *log_mass, double *edge, int32_t *kept, double *gap_p,
                              uint8_t *flags)
{
    int failed = 0;
#pragma omp parallel
    {
        double *x = (double *)malloc((size_t)(V > 0 ? V : 1) * sizeof(double));
        if (!x) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (int64_t n = 0; n < N; ++n) {
            if (!x) continue;
            const char *row = (const char *)logits + (size_t)n * (size_t)ld * elt_size(dtype);
            oracle_decode_row(row, dtype, V, x);
            double T = temperatures ? (double)temperatures[n] : temperature;
            int32_t s = seq_ids[n];
            int64_t t = claimed ? (int64_t)claimed[n] : -1;
            if (oracle_ipt_filtered_row(x, V, T, seeds[s], (uint32_t)s, positions[n], t, top_k, top_p, sigma, eps,
                                        &u[n], &cdf_lo[n], &cdf_hi[n], &dist[n], &tok[n], &log_mass[n], &edge[n],
                                        &kept[n], &gap_p[n], &flags[n])) {
#pragma omp atomic write
                failed = 1;
            }
        }
        free(x);
    }
    return failed;
}

/* ------------------------------------------------------------------------- */
/* Next-token logits of one position from its final hidden state: the last    */
/* step of the verifier's prefill (appendix algorithm "sampled token          */
/* verification via prefill": one forward pass yields the logits of every     */
/* position).  x_v = sum_k h_k * W[v,k], k ascending, every product and sum    */
/* in double from the exact values of the stored bf16 numbers.  No bias, no    */
/* rounding of x_v to a storage type.                                          */
/* ------------------------------------------------------------------------- */
void oracle_lmhead_row(const uint16_t *h, const uint16_t *W, int64_t V, int64_t d, int64_t ldw, double *x)
{
    for (int64_t v = 0; v < V; ++v) {
        const uint16_t *w = W + (size_t)v * (size_t)ldw;
        double acc = 0.0;
        for (int64_t k = 0; k < d; ++k) acc += decode_bf16(h[k]) * decode_bf16(w[k]);
        x[v] = acc;
    }
}

/* Both estimators on logits that are never stored: for each row n the logits  */
/* come from oracle_lmhead_row(hidden[n], weight), then Token-DiFR with the     */
/* claims claimed_gumbel and Token-IPT-DiFR with the claims claimed_ipt (either */
/* may be NULL = sampling).  Outputs as in the two batch entry points above;    */
/* x_out, if given, receives the logits ([N, V] doubles).                       */
int oracle_lmhead_score(const uint16_t *hidden, int64_t ldh, const uint16_t *weight, int64_t ldw, int64_t N,
                        int64_t V, int64_t d, double temperature, const float *temperatures,
                        const uint64_t *seeds, const int32_t *seq_ids, const uint32_t *positions,
                        const int32_t *claimed_gumbel, const int32_t *claimed_ipt, double sigma, double eps,
                        double *margin, int32_t *argmax, double *max_score, double *claimed_score, double *gap2,
                        uint8_t *flags_gumbel, double *u, double *cdf_lo, double *cdf_hi, double *dist,
                        int32_t *tok, double *log_mass, double *edge, uint8_t *flags_ipt, double *x_out)
{
    int failed = 0;
#pragma omp parallel
    {
        double *x = (double *)malloc((size_t)(V > 0 ? V : 1) * sizeof(double));
        if (!x) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (int64_t n = 0; n < N; ++n) {
            if (!x) continue;
            oracle_lmhead_row(hidden + (size_t)n * (size_t)ldh, weight, V, d, ldw, x);
            if (x_out) memcpy(x_out + (size_t)n * (size_t)V, x, (size_t)V * sizeof(double));
            double T = temperatures ? (double)temperatures[n] : temperature;
            int32_t s = seq_ids[n];
            int64_t tg = claimed_gumbel ? (int64_t)claimed_gumbel[n] : -1;
            int64_t ti = claimed_ipt ? (int64_t)claimed_ipt[n] : -1;
            oracle_gumbel_row(x, V, T, seeds[s], (uint32_t)s, positions[n], tg, &margin[n], &argmax[n],
                              &max_score[n], &claimed_score[n], &gap2[n], &flags_gumbel[n], NULL);
            oracle_ipt_row(x, V, T, seeds[s], (uint32_t)s, positions[n], ti, sigma, eps, &u[n], &cdf_lo[n],
                           &cdf_hi[n], &dist[n], &tok[n], &log_mass[n], &edge[n], &flags_ipt[n]);
        }
        free(x);
    }
    return failed;
}

/* ------------------------------------------------------------------------- */
/* Logit rank of the claimed token (Sec. 7.1: rank by raw logits, before        */
/* temperature and filtering; rank 0 = the highest logit):                      */
/*   rank = #{ v : x_v > x_t }.   Invalid claim: -1.                            */
/* ------------------------------------------------------------------------- */
int32_t oracle_logit_rank_row(const double *x, int64_t V, int64_t claimed)
{
    if (claimed < 0 || claimed >= V) return -1;
    int64_t r = 0;
    for (int64_t v = 0; v < V; ++v)
        if (x[v] > x[claimed]) ++r;
    return (int32_t)r;
}

int oracle_logit_rank(const void *logits, int dtype, int64_t N, int64_t V, int64_t ld, const int32_t *claimed,
                      int32_t *rank)
{
    int failed = 0;
#pragma omp parallel
    {
        double *x = (double *)malloc((size_t)(V > 0 ? V : 1) * sizeof(double));
        if (!x) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (int64_t n = 0; n < N; ++n) {
            if (!x) continue;
            const char *row = (const char *)logits + (size_t)n * (size_t)ld * elt_size(dtype);
            oracle_decode_row(row, dtype, V, x);
            rank[n] = oracle_logit_rank_row(x, V, claimed ? (int64_t)claimed[n] : -1);
        }
        free(x);
    }
    return failed;
}

/* ------------------------------------------------------------------------- */
/* Three-class token classification and per-token exfiltratable information    */
/* (Sec. 7.1 and the appendix algorithm "risk classification via score and      */
/* rank").  Scores here are suspiciousness, so "FSSL >= tau" reads score <= tau: */
/*   SAFE (0)        score <= tau                      bits = log2|A_t| if the   */
/*                                                     caller knows it, else 0   */
/*   SUSPICIOUS (1)  score >  tau and rank in [0, R)   bits = log2 R             */
/*   DANGEROUS (2)   otherwise (also NaN score, rank -1) bits = log2 V           */
/* R <= 0 means no rank tier (two-class baseline).                              */
/* ------------------------------------------------------------------------- */
void oracle_classify(const double *scores, const int32_t *ranks, int64_t N, double tau, int64_t R, int64_t V,
                     const double *log2_admissible, uint8_t *cls, double *bits)
{
    for (int64_t n = 0; n < N; ++n) {
        if (scores[n] <= tau) {
            cls[n] = 0;
            bits[n] = log2_admissible ? log2_admissible[n] : 0.0;
        } else if (scores[n] > tau && R > 0 && ranks[n] >= 0 && (int64_t)ranks[n] < R) {
            cls[n] = 1;
            bits[n] = log2((double)R);
        } else {
            cls[n] = 2;
            bits[n] = log2((double)V);
        }
    }
}

/* ------------------------------------------------------------------------- */
/* Pooling and flagging.  Rows of sequence s are [offsets[s], offsets[s+1]).  */
/*   mean_s = (1/L_s) sum score;  max_s;  mismatch_s = rows without MATCH;    */
/*   flag_s = !(mean_s <= tau).  An empty sequence has mean 0, max 0, flag 0. */
/* row_flags may be NULL (then mismatch_s = 0).                               */
/* ------------------------------------------------------------------------- */
void oracle_seq_reduce(const double *scores, const uint8_t *row_flags, const int64_t *offsets, int64_t S,
                       double tau, double *seq_mean, double *seq_max, int32_t *seq_mismatch, uint8_t *seq_flag)
{
    for (int64_t s = 0; s < S; ++s) {
        int64_t lo = offsets[s], hi = offsets[s + 1];
        if (hi <= lo) {
            seq_mean[s] = 0.0;
            seq_max[s] = 0.0;
            seq_mismatch[s] = 0;
            seq_flag[s] = 0;
            continue;
        }
        double sum = 0.0, mx = -INFINITY;
        int any_nan = 0;
        int32_t mis = 0;
        for (int64_t n = lo; n < hi; ++n) {
            sum += scores[n];
            if (isnan(scores[n])) any_nan = 1;
            if (scores[n] > mx) mx = scores[n];
            if (row_flags && !(row_flags[n] & ORACLE_FLAG_MATCH)) ++mis;
        }
        double mean = sum / (double)(hi - lo);
        seq_mean[s] = mean;
        seq_max[s] = any_nan ? NAN : mx;
        seq_mismatch[s] = mis;
        seq_flag[s] = (mean <= tau) ? 0 : 1;
    }
}
