/*
 * difr.h -- C ABI of the MI355X (gfx950) verifier scoring library, libdifr.so.
 *
 * The library scores claimed sampled tokens against verifier logits, one token
 * row (one position of one logged response) at a time, in a single streaming pass
 * over the row's full vocabulary:
 *
 *   difr_gumbel_score  Token-DiFR.  Regenerates the sampler's seeded Gumbel noise
 *                      g_v for every vocabulary entry, forms y_v = x_v / T + g_v,
 *                      and reports argmax_v y_v (the token the honest Gumbel-max
 *                      sampler would have produced) and the claimed token's margin
 *                      max_v y_v - y_t.           [Sec. 3.2 Gumbel-max sampler;
 *                      Sec. 6.3 and the appendix algorithm of the Gumbel likelihood
 *                      estimator: noise regeneration, ranking by l_i + T G_i, and
 *                      A_{sigma,i}, of which the margin is -min_i A_{sigma,i} / T]
 *   difr_ipt_score     Token-IPT-DiFR.  Regenerates the sampler's seeded uniform u,
 *                      forms p = softmax(x / T), the CDF in ascending token order,
 *                      the claimed token's interval [a, b) and the distance of u
 *                      from it; optionally the Gaussian log-mass score and the token
 *                      the honest inverse-CDF sampler would have produced.
 *                      [Sec. 3.2 IPT sampler; Sec. 6.2 and the appendix algorithm
 *                      "convolved Gaussian score"]
 *   difr_seq_reduce    Pools token scores per sequence (mean, max, mismatch count)
 *                      and flags sequences whose mean exceeds a threshold.
 *                      [Sec. 5.2 threshold rule; Sec. 6.4; appendix "Response to
 *                      detecting exfiltration attempts": score, pool, flag]
 *
 * The regenerate-and-compare form (one prefill gives logits at every position; each
 * position is sampled with the logged seed and compared with the logged token) is
 * the appendix algorithm "verification via prefill"; MATCH in the row flags is its
 * per-position comparison.
 *
 * Seeded randomness.  The paper's H(seed || i) is instantiated as Philox4x32-10:
 *   key     = (low 32 bits, high 32 bits) of the sequence's 64-bit seed
 *   counter = (v >> 2, position i, sequence id, stream)      output word v & 3
 *   stream 0: Gumbel noise of vocabulary entry v;  stream 1: the IPT uniform (v = 0)
 *   32 bits r -> u = (2 (r >> 9) + 1) * 2^-24  in (0,1);   g = -ln(-ln u).
 *
 * Conventions that hold for every entry point
 *   - Pointers documented DEVICE must be device pointers (HBM) valid on the current
 *     HIP device; the caller owns every buffer; the library allocates nothing and is
 *     thread-safe.  It keeps no state between calls but two per-device caches filled at
 *     the first call on a device: whether the device is gfx950 (asked of the runtime
 *     once) and, for difr_lmhead_score_static only, the address of its built-in buffer.
 *   - Work is enqueued on the given hipStream_t (passed as void*; NULL = the null
 *     stream) and the call returns without synchronising.  The return value reports
 *     host-side argument validation and the launch status only.
 *   - Return value: a difr_status (0 = DIFR_OK).  Nothing aborts or throws.  On an
 *     error return no kernel has been launched and no output has been touched.
 *   - Problems that are only visible on the device are reported per row in `flags`.
 *   - N == 0 (or S == 0 for difr_seq_reduce) is a successful no-op.
 */
#ifndef DIFR_H
#define DIFR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DIFR_OK = 0,
    DIFR_ERR_NULL = 1,        /* a required pointer is NULL                          */
    DIFR_ERR_SHAPE = 2,       /* N, V, S or ld negative, V == 0 with N > 0, ld < V,  */
                              /* V >= 2^31, or N >= 2^31                             */
    DIFR_ERR_DTYPE = 3,       /* dtype is not a difr_dtype                           */
    DIFR_ERR_TEMPERATURE = 4, /* temperature not finite or <= 0 (greedy T = 0 is a   */
                              /* different sampling rule and is not this path)       */
    DIFR_ERR_ALIGN = 5,       /* logits base not aligned to its element size         */
    DIFR_ERR_LAUNCH = 6,      /* the HIP runtime refused the launch                  */
    DIFR_ERR_UNSUPPORTED = 7, /* the current device is not gfx950                    */
    DIFR_ERR_ARGUMENT = 8,    /* sigma <= 0, eps < 0, NaN where a number is needed, or */
                              /* a top_k / top_p / s / M combination the call does not  */
                              /* take (stated at each call)                             */
    DIFR_ERR_CAPACITY = 9     /* the batch needs more scratch memory than the library's */
                              /* built-in buffer holds (difr_lmhead_score_static)       */
} difr_status;

typedef enum { DIFR_BF16 = 0, DIFR_F32 = 1 } difr_dtype;

/* Per-row flag bits written to `flags`. */
#define DIFR_FLAG_MATCH 1u         /* the regenerated token equals the claimed token  */
#define DIFR_FLAG_INVALID_CLAIM 2u /* claimed token outside [0, V) (or claimed==NULL): */
                                   /* scores of the claimed token are NaN; the         */
                                   /* regenerated token and its score are still valid  */
#define DIFR_FLAG_NONFINITE 4u     /* a NaN or +inf logit was seen in the row; the     */
                                   /* row's other outputs are unspecified.  -inf is    */
                                   /* a legal "masked" entry: zero probability, never  */
                                   /* the argmax.  difr_gumbel_score treats a NaN with */
                                   /* its sign bit set like -inf (masked, not flagged) */
#define DIFR_FLAG_SLOW_PATH 8u     /* informational: the row left the streaming fast   */
                                   /* path (re-read of the row)                        */

/*
 * One batch of token rows: "claimed token t*, verifier logits, seed, temperature"
 * (inputs of the appendix scoring algorithms) plus "context position i".
 * All pointers are DEVICE pointers owned by the caller.
 */
typedef struct {
    const void *logits;        /* [N, ld] row-major, element type `dtype`; base aligned to */
                               /* the element size.  Fast path: base and ld*sizeof(elt)    */
                               /* multiples of 16 bytes; otherwise a slower generic path   */
    int32_t dtype;             /* difr_dtype                                               */
    int64_t N;                 /* token rows, 0 <= N < 2^31                                */
    int64_t V;                 /* vocabulary size, 0 < V < 2^31                            */
    int64_t ld;                /* row pitch in elements, ld >= V                           */
    float temperature;         /* T > 0, finite; used when temperatures == NULL            */
    const float *temperatures; /* optional [N] per-row T (a row with T <= 0 or NaN gets    */
                               /* NaN scores and DIFR_FLAG_NONFINITE)                      */
    const uint64_t *seeds;     /* [S] one 64-bit sampling seed per sequence                */
    int64_t S;                 /* number of sequences, S >= 1 when N > 0                   */
    const int32_t *seq_ids;    /* [N] sequence of each row, in [0, S) (rows with an id     */
                               /* outside get NaN scores and DIFR_FLAG_INVALID_CLAIM)      */
    const uint32_t *positions; /* [N] response index i of the row's token                  */
    const int32_t *claimed;    /* [N] claimed token id; NULL = sampling mode (every row is */
                               /* treated as claimed = -1)                                 */
} difr_rows;

/*
 * Token-DiFR over a batch.  Outputs are DEVICE arrays of N elements; those marked
 * optional may be NULL.
 *   margin        max_v y_v - y_t >= 0, in units of x/T + g; exactly 0 when the claimed
 *                 token is the regenerated one; NaN for an invalid claim
 *   argmax        lowest index attaining max_v y_v (the regenerated token)
 *   max_score     (optional) max_v y_v
 *   claimed_score (optional) y_t, NaN for an invalid claim
 *   flags         DIFR_FLAG_* bits
 *   logit_rank    (optional) number of entries whose raw logit is strictly above the claimed
 *                 token's (rank 0 = the highest logit; the rank signal of Sec. 7.1, taken before
 *                 temperature and filtering); -1 for an invalid claim.  Asking for it costs
 *                 about one extra vector instruction per vocabulary entry
 * Arithmetic: fp32 on exact fp32 images of the stored logits; noise bits are
 * bit-identical to the definition above.
 */
int difr_gumbel_score(const difr_rows *in, float *margin, int32_t *argmax, float *max_score,
                      float *claimed_score, uint8_t *flags, int32_t *logit_rank, void *hip_stream);

/*
 * Token-IPT-DiFR over a batch.  Outputs are DEVICE arrays of N elements; those marked
 * optional may be NULL.
 *   dist       max(a - u, u - b, 0): distance of the seeded uniform from the claimed
 *              token's CDF interval; 0 when u lies in [a, b]; NaN for an invalid claim
 *   cdf_lo     (optional) a = sum_{v < t} p_v
 *   cdf_hi     (optional) b = a + p_t
 *   u          (optional) the regenerated uniform
 *   ipt_token  (optional) min{ v : sum_{w <= v} p_w > u }, the token the honest sampler
 *              draws.  Rows whose claim does not match take a second pass over the row
 *              (DIFR_FLAG_SLOW_PATH) when this output is requested
 *   log_mass   (optional) ln( Phi((b-u)/sigma) - Phi((a-u)/sigma) + eps ), evaluated in
 *              fp64 from the kernel's fp64 interval (a token whose probability is below
 *              fp32 resolution of its CDF position still has a non-zero width there);
 *              needs sigma > 0 and eps >= 0
 *   flags      DIFR_FLAG_* bits; MATCH means a <= u < b
 *   logit_rank (optional) as in difr_gumbel_score
 */
int difr_ipt_score(const difr_rows *in, float *dist, float *cdf_lo, float *cdf_hi, float *u,
                   int32_t *ipt_token, double sigma, double eps, float *log_mass, uint8_t *flags,
                   int32_t *logit_rank, void *hip_stream);

/*
 * Both estimators in one pass over the logits: difr_gumbel_score with the claims in->claimed and
 * difr_ipt_score with the claims claimed_ipt (DEVICE [N], or NULL for sampling mode), reading each
 * row from HBM once instead of twice.  Outputs have the meaning, layout and optionality of the
 * two single-estimator calls and are bit-identical to theirs; flags_gumbel and flags_ipt are the
 * two calls' `flags`.  logit_rank [N] int32 or NULL is the logit rank of the Token-DiFR claim
 * in->claimed as in difr_gumbel_score (counted in the same pass, only when asked for: it costs a few
 * per cent), so that one read of the logits feeds the score-and-rank classifier of difr_classify
 * [Sec. 7.1].  ipt_token, sigma, eps and log_mass are difr_ipt_score's (the sampler's own token costs its second,
 * early-exit pass on the rows whose claim does not match; log_mass is the paper's Token-IPT-DiFR score).  [Sec. 6.2 and Sec. 6.3 together: a verifier that does not know which sampler the server
 * ran, or that feeds both scores to one classifier.]
 */
int difr_score_both(const difr_rows *in, const int32_t *claimed_ipt, float *margin, int32_t *argmax, float *max_score,
                    float *claimed_score, uint8_t *flags_gumbel, int32_t *logit_rank, float *dist, float *cdf_lo,
                    float *cdf_hi, float *u, int32_t *ipt_token, double sigma, double eps, float *log_mass,
                    uint8_t *flags_ipt, void *hip_stream);

/*
 * difr_score_both for rows the caller knows to be concentrated (a confident model: most of a row's logits lie more
 * than 24 ln 2 = 16.6 score units below its best perturbed score).  Same arguments, same results bit for bit.  The
 * kernel tests each wave's 512 logits before it regenerates their noise and skips the noise where none of them can
 * reach the running maximum whatever its Gumbel variate [Sec. 6.3: the variates are bounded once the uniforms are
 * quantised]; on such rows the pass approaches the speed of reading them (a quarter to 40% faster when the logits fall
 * off as -3 ln rank or steeper), on flat rows (where the test never fires) it is 1-2% slower than difr_score_both.  With logit_rank != NULL, and for rows that are not 16-byte
 * aligned, it is difr_score_both.
 */
int difr_score_both_peaked(const difr_rows *in, const int32_t *claimed_ipt, float *margin, int32_t *argmax,
                           float *max_score, float *claimed_score, uint8_t *flags_gumbel, int32_t *logit_rank, float *dist,
                           float *cdf_lo, float *cdf_hi, float *u, int32_t *ipt_token, double sigma, double eps,
                           float *log_mass, uint8_t *flags_ipt, void *hip_stream);

/*
 * Token-IPT-DiFR on the distribution a filtering sampler used.  [Sec. 3.2: the IPT sampler applied under the
 * generation policy's top-k / top-p filter; Sec. 6.2 and the appendix "convolved Gaussian score", whose input p is
 * the probabilities the sampler actually used.]  The kept set K is a prefix of the tokens ranked by logit (ties to
 * the lower index): the first top_k, cut to the shortest prefix whose softmax(x/T) mass, renormalised over those
 * top_k, reaches top_p (top_p >= 1: no cut).  Inside K probabilities are renormalised, the CDF runs in ascending
 * vocabulary index, and everything else is as in difr_ipt_score: interval [a, b) of the claimed token, distance d,
 * MATCH, the sampler's own token, optional Gaussian log-mass.  A claimed token outside K has the empty interval
 * a = b (never a match; d = |u - a|).
 * 1 <= top_k <= 256; top_p > 0; rows 16-byte aligned (DIFR_ERR_ALIGN).  Outputs as difr_ipt_score (all
 * optional ones may be NULL) plus kept [N] int32 or NULL = |K|.  One pass over the logits.
 * top_k = 0 with top_p < 1 is the bare nucleus filter: the prefix is taken over the WHOLE vocabulary and may hold
 * tens of thousands of tokens.  The library then searches for the last (logit, index) pair inside K with a search
 * over the logit keys weighted by probability mass: three to five passes over the row instead of one.  The
 * marginal tokens of such a nucleus have probabilities around 1e-6, the accuracy of the fp32 exponentials the mass
 * is summed from, so kept[n] may differ from an evaluation in double by those few tokens; a, b and d keep the 1e-4
 * contract.  The sampler's own token, when asked for and not the claim, costs one more (early-exit) pass.
 * top_k = 0 with top_p >= 1 is refused (DIFR_ERR_ARGUMENT: no filter at all, call difr_ipt_score).
 */
int difr_ipt_score_filtered(const difr_rows *in, int32_t top_k, float top_p, float *dist, float *cdf_lo, float *cdf_hi,
                            float *u, int32_t *ipt_token, double sigma, double eps, float *log_mass, int32_t *kept,
                            uint8_t *flags, void *hip_stream);

/*
 * Token-DiFR likelihood estimate of the claimed token.  [Sec. 6.3; appendix algorithm of the Gumbel-max FSSL
 * estimator.]  Per row, with G the regenerated Gumbel noise and Gaussian noise N(0, sigma^2) on every logit:
 *   S     = the s tokens with the largest x_i + T G_i, the claimed token t left out (ties to the lower index);
 *   tau   = the smallest logit the sampler's filter keeps: top_k largest logits, then top_p on the distribution
 *           renormalised over those (shortest prefix in descending logit order whose softmax(x/T) mass reaches
 *           top_p).  top_k = 0: no top-k; top_p >= 1: no top-p; neither: tau = -inf.  top_k = 0 with top_p < 1
 *           is the bare nucleus over the whole vocabulary (see Limits);
 *   A_i   = x_t - x_i + T (G_t - G_i),  B_i = tau - x_i   for i in S;
 *   pi    = (1/M) sum_j [x_t + sigma z_j > tau] prod_{i in S} Phi(max(sigma z_j + A_i, B_i) / sigma).
 * p->z  DEVICE [M] fp32 standard normal draws, supplied by the caller and shared by all rows (the algorithm
 *       samples them; how is the caller's business: pseudo-random, stratified quantiles, a quadrature rule).
 * Limits: 0 <= s <= 256, 0 <= top_k <= 256, M >= 1, sigma > 0, top_p > 0 (else DIFR_ERR_ARGUMENT); rows must
 *       be 16-byte aligned (DIFR_ERR_ALIGN).  top_k = 0 with top_p < 1 (a nucleus over the whole vocabulary)
 *       runs the search described at difr_ipt_score_filtered first; it leaves the threshold in `tau`, which is
 *       then a required output (DIFR_ERR_NULL if NULL).
 * Outputs (DEVICE): pi [N] fp32; log_pi [N] fp32 or NULL (natural log, -inf if pi = 0; this is the FSSL score
 *       the paper thresholds); tau [N] fp32 or NULL; active [N, s] int32 or NULL (S in rank order of the fp32 scores, -1 padded);
 *       flags [N] (DIFR_FLAG_INVALID_CLAIM: pi NaN; DIFR_FLAG_NONFINITE).  Which tokens are in S is decided on
 *       fp32 scores; A_i, B_i and the average are then formed in fp64 / fp32 from exact logits and fp64 noise.
 * One pass over the logits.
 */
typedef struct {
    int32_t top_k;
    float top_p;
    int32_t s;
    float sigma;
    int32_t M;
    const float *z;
} difr_likelihood_params;

int difr_gumbel_likelihood(const difr_rows *in, const difr_likelihood_params *p, float *pi, float *log_pi, float *tau,
                           int32_t *active, uint8_t *flags, void *hip_stream);

/*
 * difr_gumbel_likelihood and difr_ipt_score_filtered in one pass over the logits, for the verifier that scores both
 * estimators under the sampler's top-k / top-p policy [Sec. 6.2 and Sec. 6.3 with the generation policy of Sec. 3.2]:
 * the k largest logits that fix the likelihood's threshold tau ARE the filtered distribution Token-IPT-DiFR works
 * on, so they are collected once and each row is read from HBM once instead of twice.  in->claimed are the
 * Token-DiFR claims, claimed_ipt (DEVICE [N] or NULL for sampling mode) the Token-IPT-DiFR claims; p as in
 * difr_gumbel_likelihood.  top_k = 0 with top_p < 1 (the bare nucleus) is served by the two single calls' kernels
 * one after the other on the stream - the nucleus search, which scores Token-IPT-DiFR and leaves the threshold in
 * tau (then required: DIFR_ERR_NULL if NULL), and the estimator's pass -; top_k = 0 with top_p >= 1 is no
 * filter at all and refused (DIFR_ERR_ARGUMENT).
 * Outputs have the meaning, layout and optionality of the two single calls and are bit-identical to theirs;
 * flags_gumbel and flags_ipt are the two calls' `flags`; sigma_ipt, eps belong to log_mass.
 */
int difr_score_both_filtered(const difr_rows *in, const int32_t *claimed_ipt, const difr_likelihood_params *p, float *pi,
                             float *log_pi, float *tau, int32_t *active, uint8_t *flags_gumbel, float *dist,
                             float *cdf_lo, float *cdf_hi, float *u, int32_t *ipt_token, double sigma_ipt, double eps,
                             float *log_mass, int32_t *kept, uint8_t *flags_ipt, void *hip_stream);

/*
 * Size of each row's admissible set.  [Sec. 7, "admissible set" A_t(tau) = { i : FSSL_t(i) >= tau }: an accepted
 * token carries at most log2 |A_t(tau)| bits, a sequence at most the sum; appendix "Threshold selection and
 * FPR-information trade-off".]  With the Token-DiFR margin as the score (suspiciousness, accepted when small):
 *     count[n] = #{ v in [0,V) : max_score[n] - y_v <= delta },   y_v = x_v / T + g_v  as in difr_gumbel_score,
 * i.e. the number of tokens that would have been scored margin <= delta had they been claimed at this position.
 * max_score  DEVICE [N]: the `max_score` output of difr_gumbel_score (or difr_score_both) for the same rows; the
 *            comparison is made in fp32, exactly as difr_gumbel_score forms margins, so the claimed token is
 *            counted if and only if its margin is <= delta.  delta >= 0, finite (else DIFR_ERR_ARGUMENT).
 * count      DEVICE [N] int32; log2_count DEVICE [N] fp32 or NULL (the per-token bit bound; it is the
 *            log2_admissible input of difr_classify).  A row with a NaN or infinite max_score, a bad sequence id
 *            or temperature gets count 0 and log2_count NaN.  in->claimed is not used.
 * One more pass over the logits (the row maximum has to be known first).
 */
int difr_admissible_count(const difr_rows *in, const float *max_score, float delta, int32_t *count, float *log2_count,
                          void *hip_stream);

/*
 * difr_score_both and the admissible-set size in ONE pass over the logits.  [Sec. 7: the score decides whether
 * a token is accepted, log2 |A_t| bounds what an accepted token can carry; a verifier wants both per position.]
 * The row maximum is only known at the end of the pass, so every score that may lie within delta of it is kept
 * in a short on-chip list while the running lower bound of the maximum rises, and the list is counted against
 * the true maximum after the row: count[n] is exactly what difr_admissible_count returns for max_score[n] and
 * the same delta.  If a row has more candidates than the list holds (a very large delta, or a row whose
 * bound stays far below its maximum for long), count[n] = -1 and log2_count[n] = NaN: call
 * difr_admissible_count for those rows.  With honest claims (the bound starts at the maximum) and delta up
 * to about 5 this does not happen.  Whether a crowded row ends as -1 can differ from run to run: a wavefront
 * prunes its list against the best bound it has seen, which includes bounds the other wavefronts of the row
 * publish, and when it sees them is a matter of timing.  A count that is not -1 is always the exact count.
 * delta >= 0, finite (else DIFR_ERR_ARGUMENT); rows must be 16-byte aligned (DIFR_ERR_ALIGN).
 * count DEVICE [N] int32 (required); log2_count DEVICE [N] fp32 or NULL.  All other arguments and outputs as
 * in difr_score_both, bit-identical to it.
 */
int difr_score_both_admissible(const difr_rows *in, const int32_t *claimed_ipt, float delta, float *margin,
                               int32_t *argmax, float *max_score, float *claimed_score, uint8_t *flags_gumbel,
                               float *dist, float *cdf_lo, float *cdf_hi, float *u, uint8_t *flags_ipt, int32_t *count,
                               float *log2_count, void *hip_stream);

/*
 * Fused LM head + scoring: both estimators on logits that are never stored.  The verifier's
 * prefill ends with the product of each position's final hidden state and the LM-head matrix
 * [appendix algorithm "sampled token verification via prefill": one forward pass yields the
 * next-token logits of every position]; here that product runs on the matrix cores tile by
 * tile and each tile of logits is scored in registers, so the 2 V bytes per token of the
 * stored-logit path are neither written nor read.
 *
 *   x[n][v] = sum_k hidden[n][k] * weight[v][k]      (bf16 inputs, fp32 accumulation; the
 *             logits are used as accumulated, without rounding to a storage type, no bias)
 *
 * hidden  DEVICE [N, ldh] bf16 row-major: final hidden state of each token position (after the
 *         model's last normalisation); weight  DEVICE [V, ldw] bf16 row-major: one row per
 *         vocabulary entry.  d % 64 == 0, ldh >= d, ldw >= d, ldh % 8 == ldw % 8 == 0, both bases
 *         16-byte aligned (else DIFR_ERR_SHAPE / DIFR_ERR_ALIGN).  N, V < 2^31; ldh, ldw < 2^23.
 * claimed_gumbel / claimed_ipt  DEVICE [N] or NULL: the claims scored by Token-DiFR and by
 *         Token-IPT-DiFR.  The remaining fields are those of difr_rows.
 * Outputs: those of difr_score_both, with the same optionality and flag bits.  Because
 *         the fp32 accumulation order of a matrix-core product is not the oracle's, logits carry
 *         an error of a few 1e-6 relative to sum_k |h_k w_k|; scores inherit it.
 *         ipt_token [N] int32 or NULL: the token the honest inverse-CDF sampler draws.  Its position
 *         needs the row's total mass, which is known only after the last tile of logits that are
 *         never stored: when asked for, the scoring pass also leaves the softmax mass of every half
 *         tile (128 entries) of every token in the workspace (16 bytes per token and 256 vocabulary
 *         entries: 156 MB at N = 16384, V = 151936), the merge finds the half tile in which the CDF
 *         passes u, and one more kernel forms that half tile's 128 logits again as plain dot products
 *         (DIFR_FLAG_SLOW_PATH; about 1 MB of LM-head rows read per token) and finds the entry.  Rows
 *         whose claim matches skip it: their token is the claim.
 *         logit_rank [N] int32 or NULL: entries whose logit exceeds the Token-DiFR claim's (Sec. 7.1),
 *         counted in the same pass against the claim's logit formed as a plain fp32 dot product (it has
 *         to be known before the first tile); the claimed entry is left out by index.  A logit within
 *         the accumulation error of the claim's may fall on either side: the count is exact up to
 *         those entries.  -1 for an invalid claim.  Asking for it costs a few per cent.
 *         sigma, eps, log_mass: as in difr_ipt_score (the paper's Token-IPT-DiFR score, fp64 from the
 *         fp64 interval).
 * workspace  DEVICE scratch of at least difr_lmhead_workspace_bytes(N, V, d, ipt_token != NULL)
 *         bytes, 8-byte aligned, owned by the caller, contents irrelevant before and after the call;
 *         calls that overlap in time need distinct workspaces.  Too small: DIFR_ERR_SHAPE.
 * Three kernels are enqueued on hip_stream (claim bound, GEMM + scoring, merge), four with ipt_token; no sync.
 */
typedef struct {
    const void *hidden;
    const void *weight;
    int64_t N, V, d, ldh, ldw;
    float temperature;
    const float *temperatures;
    const uint64_t *seeds;
    int64_t S;
    const int32_t *seq_ids;
    const uint32_t *positions;
    const int32_t *claimed_gumbel;
    const int32_t *claimed_ipt;
} difr_lmhead;

/* Host only, no device needed.  0 for N == 0 or arguments difr_lmhead_score would reject.
 * want_ipt_token != 0: with room for what the ipt_token output needs. */
size_t difr_lmhead_workspace_bytes(int64_t N, int64_t V, int64_t d, int32_t want_ipt_token);

int difr_lmhead_score(const difr_lmhead *in, float *margin, int32_t *argmax, float *max_score, float *claimed_score,
                      uint8_t *flags_gumbel, int32_t *logit_rank, float *dist, float *cdf_lo, float *cdf_hi, float *u,
                      int32_t *ipt_token, double sigma, double eps, float *log_mass, uint8_t *flags_ipt, void *workspace,
                      size_t workspace_bytes, void *hip_stream);

/*
 * difr_lmhead_score for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same inputs, same
 * outputs but ipt_token (what that output needs does not fit a built-in buffer), same kernels; the partial results of the vocabulary ranges go to a buffer that is part of
 * the library's device image (DIFR_LMHEAD_STATIC_SCRATCH_BYTES per GPU the library runs on, held until
 * the process ends) instead of a caller workspace.  The call allocates and frees nothing.
 *   - A batch with difr_lmhead_workspace_bytes(N, V, d, 0) > DIFR_LMHEAD_STATIC_SCRATCH_BYTES is refused
 *     with DIFR_ERR_CAPACITY and nothing is launched.  The 4 MiB hold every batch of up to 87,000
 *     tokens at any V (32 bytes per token and vocabulary range, at most 65,536 such pairs below
 *     65,536 tokens and one range per token above, plus 16 bytes per token).
 *   - Every call on a GPU uses that GPU's one buffer: calls that overlap in time on one GPU (two
 *     streams, two threads) race on it and give wrong results.  Calls in order on one stream are safe;
 *     nothing in the buffer has to survive from one call to the next and nothing has to be cleared.
 *   - The first call on a device resolves the buffer's address (hipGetSymbolAddress); make that call
 *     outside graph capture.  Later calls on that device only enqueue the three kernels.
 */
#define DIFR_LMHEAD_STATIC_SCRATCH_BYTES (4u << 20)
int difr_lmhead_score_static(const difr_lmhead *in, float *margin, int32_t *argmax, float *max_score,
                             float *claimed_score, uint8_t *flags_gumbel, int32_t *logit_rank, float *dist, float *cdf_lo,
                             float *cdf_hi, float *u, double sigma, double eps, float *log_mass, uint8_t *flags_ipt,
                             void *hip_stream);

/*
 * Three-class token classification and per-token exfiltratable information.  [Sec. 7.1 and the
 * appendix algorithm "per-token risk classification via score and rank".]  Scores are
 * suspiciousness (margin or dist), so the paper's "FSSL >= tau" reads score <= tau:
 *   class 0 SAFE        score <= tau                            bits = log2|A_t| if known, else 0
 *   class 1 SUSPICIOUS  score >  tau and 0 <= rank < rank_cutoff  bits = log2(rank_cutoff)
 *   class 2 DANGEROUS   otherwise (also a NaN score or rank -1)   bits = log2(V)
 * scores [N] fp32, ranks [N] int32 (logit_rank output above), log2_admissible [N] fp32 or NULL,
 * all DEVICE; outputs cls [N] uint8 and bits [N] fp32 (optional), DEVICE.  rank_cutoff <= 0
 * switches the rank tier off (two-class baseline).  V >= 1.
 */
int difr_classify(const float *scores, const int32_t *ranks, int64_t N, float tau, int64_t rank_cutoff, int64_t V,
                  const float *log2_admissible, uint8_t *cls, float *bits, void *hip_stream);

/*
 * Pooling and flagging.  scores [N] DEVICE fp32 token scores (margin or dist);
 * row_flags [N] DEVICE or NULL; seq_offsets [S+1] DEVICE, non-decreasing, rows of
 * sequence s are [seq_offsets[s], seq_offsets[s+1]) and seq_offsets[S] <= N.
 * Outputs are DEVICE arrays of S elements, each optional:
 *   seq_mean      mean of the sequence's scores (fp64 accumulation in a fixed order,
 *                 rounded to fp32); 0 for an empty sequence
 *   seq_max       maximum score (NaN if any score is NaN); 0 for an empty sequence
 *   seq_mismatch  rows of the sequence without DIFR_FLAG_MATCH (0 if row_flags == NULL)
 *   seq_flag      1 unless mean <= threshold (so a NaN mean is flagged); 0 if empty
 */
int difr_seq_reduce(const float *scores, const uint8_t *row_flags, const int64_t *seq_offsets, int64_t N,
                    int64_t S, float threshold, float *seq_mean, float *seq_max, int32_t *seq_mismatch,
                    uint8_t *seq_flag, void *hip_stream);

/*
 * Test and audit helper: difr_gumbel_score with the exact pre-filter switched off, so that
 * every vocabulary entry goes through both logarithms.  Same arguments, same outputs; the
 * two must agree bit for bit (the filter only skips entries that provably cannot reach the
 * row maximum).  Rows that are not 16-byte aligned always take this path.
 */
int difr_debug_gumbel_score_unfiltered(const difr_rows *in, float *margin, int32_t *argmax, float *max_score,
                                       float *claimed_score, uint8_t *flags, int32_t *logit_rank, void *hip_stream);

/*
 * Test and audit helper: writes the raw 32 noise bits of vocabulary entries
 * 0..V-1 of one row (`stream` 0 = Gumbel, 1 = IPT) to the DEVICE array bits[V],
 * using the same device code path as the scoring kernels.
 */
int difr_debug_noise(const difr_rows *in, int64_t row, int32_t stream, uint32_t *bits, void *hip_stream);

/*
 * Test and audit helper: evaluates the device's bits -> Gumbel map for the n raw
 * words in the DEVICE array bits[n] and writes g[n] (DEVICE, fp32).
 */
int difr_debug_gumbel_map(const uint32_t *bits, int64_t n, float *g, void *hip_stream);

/* Host-side helpers (no device access). */
void difr_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);
const char *difr_status_string(int status);
int difr_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DIFR_H */
