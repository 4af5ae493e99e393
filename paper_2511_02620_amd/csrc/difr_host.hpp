// Host-side launch functions implemented next to each kernel; called by the C ABI layer.
// Each returns 0 on success, non-zero if the HIP runtime refused the launch.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "difr_device.hpp"

namespace difr {

// filtered = false forces the unfiltered kernel (every entry evaluated exactly); unaligned rows always use it.
int launch_gumbel_score(const RowBatch &b, bool aligned, bool filtered, float *margin, int32_t *argmax,
                        float *max_score, float *claimed_score, uint8_t *flags, int32_t *logit_rank,
                        hipStream_t stream);
int launch_ipt_score(const RowBatch &b, bool aligned, float *dist, float *cdf_lo, float *cdf_hi, float *u,
                     int32_t *ipt_token, double sigma, double eps, float *log_mass, uint8_t *flags,
                     int32_t *logit_rank, hipStream_t stream);
// Size of each row's admissible set { v : max_score - y_v <= delta } (max_score from launch_gumbel_score).
int launch_admissible_count(const RowBatch &b, bool aligned, const float *max_score, float delta, int32_t *count,
                            float *log2_count, hipStream_t stream);
struct GumbelOutputs;
struct IptOutputs;
// Both estimators in one pass (aligned rows only).
int launch_ipt_nucleus(const RowBatch &b, float top_p, const IptOutputs &o, int32_t *kept, float *tau, hipStream_t stream);
int launch_score_both(const RowBatch &b, const int32_t *claimed_ipt, const GumbelOutputs &og, const IptOutputs &oi,
                      bool peaked, hipStream_t stream);
int launch_score_both_admissible(const RowBatch &b, const int32_t *claimed_ipt, const GumbelOutputs &og,
                                 const IptOutputs &oi, float delta, int32_t *count, float *log2_count, hipStream_t stream);
// Token-DiFR likelihood estimate (aligned rows only).
struct LikelihoodParams {
    int32_t top_k;   // 0 = no top-k
    float top_p;     // >= 1 = no top-p
    int32_t s;       // active-set size, 0 .. 256
    float sigma;     // standard deviation of the Gaussian logit noise
    int32_t M;       // number of draws
    const float *z;  // DEVICE [M] standard normal draws
    const float *tau_in;  // DEVICE [N] filter threshold found beforehand (nucleus over the whole vocabulary), or null
};
struct LikelihoodOutputs {
    float *pi, *log_pi, *tau;
    int32_t *active;  // [N, s] or null
    uint8_t *flags;
};
int launch_likelihood(const RowBatch &b, const LikelihoodParams &p, const LikelihoodOutputs &o, hipStream_t stream);
// The same pass with Token-IPT-DiFR under the same filter beside it (1 <= top_k <= 256); outputs as the two single calls.
int launch_score_both_filtered(const RowBatch &b, const LikelihoodParams &p, const LikelihoodOutputs &o,
                               const int32_t *claimed_ipt, const IptOutputs &oi, int32_t *kept, hipStream_t stream);
// Token-IPT-DiFR under the sampler's top-k / top-p filter (aligned rows only; 1 <= top_k <= 256).
int launch_ipt_filtered(const RowBatch &b, int top_k, float top_p, const IptOutputs &o, int32_t *kept, hipStream_t stream);
struct LmHeadBatch;
struct LmHeadWorkspace;
struct LmHeadPlan;
// Fused LM head + both estimators: claim bound, GEMM + scoring, merge.
int launch_lmhead_score(const LmHeadBatch &b, const LmHeadWorkspace &ws, const LmHeadPlan &plan, const GumbelOutputs &og,
                        const IptOutputs &oi, hipStream_t stream);
int launch_classify(const float *scores, const int32_t *ranks, int64_t N, float tau, int64_t R, int64_t V,
                    const float *log2_admissible, uint8_t *cls, float *bits, hipStream_t stream);
int launch_seq_reduce(const float *scores, const uint8_t *row_flags, const int64_t *seq_offsets, int64_t N,
                      int64_t S, float threshold, float *seq_mean, float *seq_max, int32_t *seq_mismatch,
                      uint8_t *seq_flag, hipStream_t stream);
int launch_debug_noise(const RowBatch &b, int64_t row, uint32_t stream_id, uint32_t *bits, hipStream_t stream);
int launch_debug_gumbel_map(const uint32_t *bits, int64_t n, float *g, hipStream_t stream);

}  // namespace difr
