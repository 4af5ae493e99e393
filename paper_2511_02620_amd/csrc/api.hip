// C ABI of libdifr.so: argument validation and kernel launches.  See include/difr.h for
// the meaning, layout and ownership of every argument.
#include <math.h>
#include <string.h>

#include <atomic>

#include "../../include/difr.h"
#include "difr_device.hpp"
#include "difr_host.hpp"
#include "gumbel_stream.hpp"
#include "ipt_stream.hpp"
#include "lmhead.hpp"

// Built-in workspace of difr_lmhead_score_static: every GPU the library runs on holds its own copy, at its own
// address, until the process ends.  In host code the name `scratch` is only a handle for hipGetSymbolAddress;
// the device address that call yields (one per device, cached below) is what kernels are given.
static __device__ __align__(256) unsigned char scratch[DIFR_LMHEAD_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
// 0 = not checked yet, 1 = gfx950, 2 = something else.  The one thing the library remembers between calls
// (include/difr.h says so): the answer for a device never changes, and asking the runtime costs microseconds.
std::atomic<int> g_arch_ok[kMaxDevices];

int check_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0) return DIFR_ERR_UNSUPPORTED;
    if (dev < kMaxDevices) {
        const int c = g_arch_ok[dev].load(std::memory_order_relaxed);
        if (c) return c == 1 ? DIFR_OK : DIFR_ERR_UNSUPPORTED;
    }
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return DIFR_ERR_UNSUPPORTED;
    const bool ok = strncmp(prop.gcnArchName, "gfx950", 6) == 0;
    if (dev < kMaxDevices) g_arch_ok[dev].store(ok ? 1 : 2, std::memory_order_relaxed);
    return ok ? DIFR_OK : DIFR_ERR_UNSUPPORTED;
}

constexpr size_t kStaticScratchBytes = DIFR_LMHEAD_STATIC_SCRATCH_BYTES;
// Device address of `scratch` per device, resolved at the first call of difr_lmhead_score_static on that device.
std::atomic<void *> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device, or null if the runtime cannot resolve it.
void *static_scratch()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0) return nullptr;
    if (dev < kMaxDevices) {
        void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
        if (p) return p;
    }
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
    if (dev < kMaxDevices) g_scratch_ptr[dev].store(p, std::memory_order_release);
    return p;
}

int validate_rows(const difr_rows *in, difr::RowBatch *b, bool *aligned)
{
    if (!in) return DIFR_ERR_NULL;
    if (in->N < 0 || in->V < 0 || in->ld < 0 || in->S < 0) return DIFR_ERR_SHAPE;
    if (in->N >= (int64_t)1 << 31 || in->V >= (int64_t)1 << 31) return DIFR_ERR_SHAPE;
    if (in->dtype != DIFR_BF16 && in->dtype != DIFR_F32) return DIFR_ERR_DTYPE;
    if (in->N > 0) {
        if (in->V == 0 || in->ld < in->V || in->S < 1) return DIFR_ERR_SHAPE;
        if (!in->logits || !in->seeds || !in->seq_ids || !in->positions) return DIFR_ERR_NULL;
        if (!in->temperatures && !(in->temperature > 0.0f && isfinite(in->temperature))) return DIFR_ERR_TEMPERATURE;
    }
    const uintptr_t esz = in->dtype == DIFR_BF16 ? 2u : 4u;
    const uintptr_t base = (uintptr_t)in->logits;
    if (base % esz) return DIFR_ERR_ALIGN;
    *aligned = (base % 16u == 0) && (((uint64_t)in->ld * esz) % 16u == 0);
    b->logits = in->logits;
    b->dtype = in->dtype;
    b->N = in->N;
    b->V = in->V;
    b->ld = in->ld;
    b->temperature = in->temperature;
    b->temperatures = in->temperatures;
    b->seeds = in->seeds;
    b->S = in->S;
    b->seq_ids = in->seq_ids;
    b->positions = in->positions;
    b->claimed = in->claimed;
    return DIFR_OK;
}

int validate_lmhead(const difr_lmhead *in, difr::LmHeadBatch *b)
{
    if (!in) return DIFR_ERR_NULL;
    if (in->N < 0 || in->V < 0 || in->d < 0 || in->ldh < 0 || in->ldw < 0 || in->S < 0) return DIFR_ERR_SHAPE;
    if (in->N >= (int64_t)1 << 31 || in->V >= (int64_t)1 << 31 || in->d >= (int64_t)1 << 31) return DIFR_ERR_SHAPE;
    // the kernel addresses the 256 rows of a tile with 32-bit byte offsets from the tile's first row
    if (in->ldh >= (int64_t)1 << 23 || in->ldw >= (int64_t)1 << 23) return DIFR_ERR_SHAPE;
    if (in->N > 0) {
        if (in->V == 0 || in->d == 0 || in->d % difr::kLmTileK || in->ldh < in->d || in->ldw < in->d || in->ldh % 8 ||
            in->ldw % 8 || in->S < 1)
            return DIFR_ERR_SHAPE;
        if (!in->hidden || !in->weight || !in->seeds || !in->seq_ids || !in->positions) return DIFR_ERR_NULL;
        if (!in->temperatures && !(in->temperature > 0.0f && isfinite(in->temperature))) return DIFR_ERR_TEMPERATURE;
        if ((uintptr_t)in->hidden % 16u || (uintptr_t)in->weight % 16u) return DIFR_ERR_ALIGN;
    }
    b->hidden = (const uint16_t *)in->hidden;
    b->weight = (const uint16_t *)in->weight;
    b->N = in->N;
    b->V = in->V;
    b->d = in->d;
    b->ldh = in->ldh;
    b->ldw = in->ldw;
    b->temperature = in->temperature;
    b->temperatures = in->temperatures;
    b->seeds = in->seeds;
    b->S = in->S;
    b->seq_ids = in->seq_ids;
    b->positions = in->positions;
    b->claimed_gumbel = in->claimed_gumbel;
    b->claimed_ipt = in->claimed_ipt;
    return DIFR_OK;
}

}  // namespace

extern "C" {

size_t difr_lmhead_workspace_bytes(int64_t N, int64_t V, int64_t d, int32_t want_ipt_token)
{
    if (N <= 0 || V <= 0 || d <= 0 || N >= (int64_t)1 << 31 || V >= (int64_t)1 << 31) return 0;
    const difr::LmHeadPlan plan = difr::lmhead_plan(N, V);
    return difr::lmhead_workspace_bytes(N, plan.splits, plan.n_vt, want_ipt_token != 0);
}

int difr_lmhead_score(const difr_lmhead *in, float *margin, int32_t *argmax, float *max_score, float *claimed_score,
                      uint8_t *flags_gumbel, int32_t *logit_rank, float *dist, float *cdf_lo, float *cdf_hi, float *u,
                      int32_t *ipt_token, double sigma, double eps, float *log_mass, uint8_t *flags_ipt, void *workspace,
                      size_t workspace_bytes, void *hip_stream)
{
    difr::LmHeadBatch b;
    int rc = validate_lmhead(in, &b);
    if (rc != DIFR_OK) return rc;
    if (log_mass && (!(sigma > 0.0) || !isfinite(sigma) || !(eps >= 0.0) || !isfinite(eps))) return DIFR_ERR_ARGUMENT;
    if (b.N == 0) return DIFR_OK;
    if (!margin || !argmax || !flags_gumbel || !dist || !flags_ipt || !workspace) return DIFR_ERR_NULL;
    const difr::LmHeadPlan plan = difr::lmhead_plan(b.N, b.V);
    if ((uintptr_t)workspace % 8u) return DIFR_ERR_ALIGN;
    const bool tok = ipt_token != nullptr;
    if (workspace_bytes < difr::lmhead_workspace_bytes(b.N, plan.splits, plan.n_vt, tok)) return DIFR_ERR_SHAPE;
    if ((rc = check_device()) != DIFR_OK) return rc;
    const difr::LmHeadWorkspace ws = difr::lmhead_carve(workspace, b.N, plan.splits, plan.n_vt, tok);
    const difr::GumbelOutputs og{margin, argmax, max_score, claimed_score, flags_gumbel, logit_rank};
    const difr::IptOutputs oi{dist, cdf_lo, cdf_hi, u, ipt_token, sigma, eps, log_mass, flags_ipt, nullptr};
    return difr::launch_lmhead_score(b, ws, plan, og, oi, (hipStream_t)hip_stream) ? DIFR_ERR_LAUNCH : DIFR_OK;
}

int difr_lmhead_score_static(const difr_lmhead *in, float *margin, int32_t *argmax, float *max_score,
                             float *claimed_score, uint8_t *flags_gumbel, int32_t *logit_rank, float *dist, float *cdf_lo,
                             float *cdf_hi, float *u, double sigma, double eps, float *log_mass, uint8_t *flags_ipt,
                             void *hip_stream)
{
    difr::LmHeadBatch b;
    int rc = validate_lmhead(in, &b);
    if (rc != DIFR_OK) return rc;
    if (log_mass && (!(sigma > 0.0) || !isfinite(sigma) || !(eps >= 0.0) || !isfinite(eps))) return DIFR_ERR_ARGUMENT;
    if (b.N == 0) return DIFR_OK;
    if (!margin || !argmax || !flags_gumbel || !dist || !flags_ipt) return DIFR_ERR_NULL;
    const difr::LmHeadPlan plan = difr::lmhead_plan(b.N, b.V);
    if (difr::lmhead_workspace_bytes(b.N, plan.splits) > kStaticScratchBytes) return DIFR_ERR_CAPACITY;
    if ((rc = check_device()) != DIFR_OK) return rc;
    void *ws_base = static_scratch();
    if (!ws_base) return DIFR_ERR_LAUNCH;
    const difr::LmHeadWorkspace ws = difr::lmhead_carve(ws_base, b.N, plan.splits);
    const difr::GumbelOutputs og{margin, argmax, max_score, claimed_score, flags_gumbel, logit_rank};
    const difr::IptOutputs oi{dist, cdf_lo, cdf_hi, u, nullptr, sigma, eps, log_mass, flags_ipt, nullptr};
    return difr::launch_lmhead_score(b, ws, plan, og, oi, (hipStream_t)hip_stream) ? DIFR_ERR_LAUNCH : DIFR_OK;
}

int difr_gumbel_score(const difr_rows *in, float *margin, int32_t *argmax, float *max_score, float *claimed_score,
                      uint8_t *flags, int32_t *logit_rank, void *hip_stream)
{
    difr::RowBatch b;
    bool aligned = false;
    int rc = validate_rows(in, &b, &aligned);
    if (rc != DIFR_OK) return rc;
    if (b.N == 0) return DIFR_OK;
    if (!margin || !argmax || !flags) return DIFR_ERR_NULL;
    if ((rc = check_device()) != DIFR_OK) return rc;
    return difr::launch_gumbel_score(b, aligned, true, margin, argmax, max_score, claimed_score, flags, logit_rank,
                                     (hipStream_t)hip_stream)
               ? DIFR_ERR_LAUNCH
               : DIFR_OK;
}

int difr_debug_gumbel_score_unfiltered(const difr_rows *in, float *margin, int32_t *argmax, float *max_score,
                                       float *claimed_score, uint8_t *flags, int32_t *logit_rank, void *hip_stream)
{
    difr::RowBatch b;
    bool aligned = false;
    int rc = validate_rows(in, &b, &aligned);
    if (rc != DIFR_OK) return rc;
    if (b.N == 0) return DIFR_OK;
    if (!margin || !argmax || !flags) return DIFR_ERR_NULL;
    if ((rc = check_device()) != DIFR_OK) return rc;
    return difr::launch_gumbel_score(b, aligned, false, margin, argmax, max_score, claimed_score, flags, logit_rank,
                                     (hipStream_t)hip_stream)
               ? DIFR_ERR_LAUNCH
               : DIFR_OK;
}

int difr_ipt_score(const difr_rows *in, float *dist, float *cdf_lo, float *cdf_hi, float *u, int32_t *ipt_token,
                   double sigma, double eps, float *log_mass, uint8_t *flags, int32_t *logit_rank, void *hip_stream)
{
    difr::RowBatch b;
    bool aligned = false;
    int rc = validate_rows(in, &b, &aligned);
    if (rc != DIFR_OK) return rc;
    if (log_mass && (!(sigma > 0.0) || !isfinite(sigma) || !(eps >= 0.0) || !isfinite(eps))) return DIFR_ERR_ARGUMENT;
    if (b.N == 0) return DIFR_OK;
    if (!dist || !flags) return DIFR_ERR_NULL;
    if ((rc = check_device()) != DIFR_OK) return rc;
    return difr::launch_ipt_score(b, aligned, dist, cdf_lo, cdf_hi, u, ipt_token, sigma, eps, log_mass, flags,
                                  logit_rank, (hipStream_t)hip_stream)
               ? DIFR_ERR_LAUNCH
               : DIFR_OK;
}

int difr_seq_reduce(const float *scores, const uint8_t *row_flags, const int64_t *seq_offsets, int64_t N, int64_t S,
                    float threshold, float *seq_mean, float *seq_max, int32_t *seq_mismatch, uint8_t *seq_flag,
                    void *hip_stream)
{
    if (N < 0 || S < 0 || S >= (int64_t)1 << 31) return DIFR_ERR_SHAPE;
    if (threshold != threshold) return DIFR_ERR_ARGUMENT;
    if (S == 0) return DIFR_OK;
    if (!seq_offsets || (N > 0 && !scores)) return DIFR_ERR_NULL;
    int rc = check_device();
    if (rc != DIFR_OK) return rc;
    return difr::launch_seq_reduce(scores, row_flags, seq_offsets, N, S, threshold, seq_mean, seq_max, seq_mismatch,
                                   seq_flag, (hipStream_t)hip_stream)
               ? DIFR_ERR_LAUNCH
               : DIFR_OK;
}

int difr_admissible_count(const difr_rows *in, const float *max_score, float delta, int32_t *count, float *log2_count,
                          void *hip_stream)
{
    difr::RowBatch b;
    bool aligned = false;
    int rc = validate_rows(in, &b, &aligned);
    if (rc != DIFR_OK) return rc;
    if (!(delta >= 0.0f) || !isfinite(delta)) return DIFR_ERR_ARGUMENT;
    if (b.N == 0) return DIFR_OK;
    if (!max_score || !count) return DIFR_ERR_NULL;
    if ((rc = check_device()) != DIFR_OK) return rc;
    return difr::launch_admissible_count(b, aligned, max_score, delta, count, log2_count, (hipStream_t)hip_stream)
               ? DIFR_ERR_LAUNCH
               : DIFR_OK;
}

int difr_ipt_score_filtered(const difr_rows *in, int32_t top_k, float top_p, float *dist, float *cdf_lo, float *cdf_hi,
                            float *u, int32_t *ipt_token, double sigma, double eps, float *log_mass, int32_t *kept,
                            uint8_t *flags, void *hip_stream)
{
    difr::RowBatch b;
    bool aligned = false;
    int rc = validate_rows(in, &b, &aligned);
    if (rc != DIFR_OK) return rc;
    if (top_k < 0 || top_k > 256 || !(top_p > 0.0f)) return DIFR_ERR_ARGUMENT;
    if (log_mass && (!(sigma > 0.0) || !isfinite(sigma) || !(eps >= 0.0) || !isfinite(eps))) return DIFR_ERR_ARGUMENT;
    // no top-k: a nucleus over the whole vocabulary (without top-p either there is no filter: difr_ipt_score)
    if (top_k == 0 && !(top_p < 1.0f)) return DIFR_ERR_ARGUMENT;
    if (b.N == 0) return DIFR_OK;
    if (!dist || !flags) return DIFR_ERR_NULL;
    if (!aligned) return DIFR_ERR_ALIGN;
    if ((rc = check_device()) != DIFR_OK) return rc;
    const difr::IptOutputs o{dist, cdf_lo, cdf_hi, u, ipt_token, sigma, eps, log_mass, flags, nullptr};
    if (top_k == 0) return difr::launch_ipt_nucleus(b, top_p, o, kept, nullptr, (hipStream_t)hip_stream) ? DIFR_ERR_LAUNCH : DIFR_OK;
    return difr::launch_ipt_filtered(b, top_k, top_p, o, kept, (hipStream_t)hip_stream) ? DIFR_ERR_LAUNCH : DIFR_OK;
}

int difr_gumbel_likelihood(const difr_rows *in, const difr_likelihood_params *p, float *pi, float *log_pi, float *tau,
                           int32_t *active, uint8_t *flags, void *hip_stream)
{
    difr::RowBatch b;
    bool aligned = false;
    int rc = validate_rows(in, &b, &aligned);
    if (rc != DIFR_OK) return rc;
    if (!p) return DIFR_ERR_NULL;
    if (p->s < 0 || p->s > 256 || p->top_k < 0 || p->top_k > 256 || p->M < 1) return DIFR_ERR_ARGUMENT;
    if (!(p->sigma > 0.0f) || !isfinite(p->sigma) || !(p->top_p > 0.0f)) return DIFR_ERR_ARGUMENT;
    // a nucleus over the whole vocabulary is found by a kernel of its own, which leaves the threshold in the
    // caller's tau array for the estimator to pick up: that output is then required
    const bool nucleus = p->top_k == 0 && p->top_p < 1.0f;
    if (nucleus && !tau) return DIFR_ERR_NULL;
    if (b.N == 0) return DIFR_OK;
    if (!pi || !flags || !p->z) return DIFR_ERR_NULL;
    if (!aligned) return DIFR_ERR_ALIGN;
    if ((rc = check_device()) != DIFR_OK) return rc;
    if (nucleus) {
        const difr::IptOutputs none{nullptr, nullptr, nullptr, nullptr, nullptr, 0.0, 0.0, nullptr, nullptr, nullptr};
        if (difr::launch_ipt_nucleus(b, p->top_p, none, nullptr, tau, (hipStream_t)hip_stream)) return DIFR_ERR_LAUNCH;
    }
    const difr::LikelihoodParams lp{p->top_k, p->top_p, p->s, p->sigma, p->M, p->z, nucleus ? tau : nullptr};
    const difr::LikelihoodOutputs lo{pi, log_pi, tau, active, flags};
    return difr::launch_likelihood(b, lp, lo, (hipStream_t)hip_stream) ? DIFR_ERR_LAUNCH : DIFR_OK;
}

int difr_score_both_filtered(const difr_rows *in, const int32_t *claimed_ipt, const difr_likelihood_params *p, float *pi,
                             float *log_pi, float *tau, int32_t *active, uint8_t *flags_gumbel, float *dist,
                             float *cdf_lo, float *cdf_hi, float *u, int32_t *ipt_token, double sigma_ipt, double eps,
                             float *log_mass, int32_t *kept, uint8_t *flags_ipt, void *hip_stream)
{
    difr::RowBatch b;
    bool aligned = false;
    int rc = validate_rows(in, &b, &aligned);
    if (rc != DIFR_OK) return rc;
    if (!p) return DIFR_ERR_NULL;
    if (p->s < 0 || p->s > 256 || p->top_k < 0 || p->top_k > 256 || p->M < 1) return DIFR_ERR_ARGUMENT;
    if (!(p->sigma > 0.0f) || !isfinite(p->sigma) || !(p->top_p > 0.0f)) return DIFR_ERR_ARGUMENT;
    if (log_mass && (!(sigma_ipt > 0.0) || !isfinite(sigma_ipt) || !(eps >= 0.0) || !isfinite(eps))) return DIFR_ERR_ARGUMENT;
    // no top-k: without top-p either there is no filter at all; with it, the nucleus over the whole vocabulary
    // is found by a kernel of its own (which scores Token-IPT-DiFR on it and leaves the threshold in the caller's
    // tau array, then a required output) and the estimator's pass follows on the same stream
    const bool nucleus = p->top_k == 0 && p->top_p < 1.0f;
    if (p->top_k == 0 && !nucleus) return DIFR_ERR_ARGUMENT;
    if (nucleus && !tau) return DIFR_ERR_NULL;
    if (b.N == 0) return DIFR_OK;
    if (!pi || !flags_gumbel || !p->z || !dist || !flags_ipt) return DIFR_ERR_NULL;
    if (!aligned) return DIFR_ERR_ALIGN;
    if ((rc = check_device()) != DIFR_OK) return rc;
    const difr::LikelihoodOutputs lo{pi, log_pi, tau, active, flags_gumbel};
    const difr::IptOutputs oi{dist, cdf_lo, cdf_hi, u, ipt_token, sigma_ipt, eps, log_mass, flags_ipt, nullptr};
    if (nucleus) {
        difr::RowBatch bi = b;
        bi.claimed = claimed_ipt;
        if (difr::launch_ipt_nucleus(bi, p->top_p, oi, kept, tau, (hipStream_t)hip_stream)) return DIFR_ERR_LAUNCH;
        const difr::LikelihoodParams ln{0, p->top_p, p->s, p->sigma, p->M, p->z, tau};
        return difr::launch_likelihood(b, ln, lo, (hipStream_t)hip_stream) ? DIFR_ERR_LAUNCH : DIFR_OK;
    }
    const difr::LikelihoodParams lp{p->top_k, p->top_p, p->s, p->sigma, p->M, p->z, nullptr};
    return difr::launch_score_both_filtered(b, lp, lo, claimed_ipt, oi, kept, (hipStream_t)hip_stream) ? DIFR_ERR_LAUNCH : DIFR_OK;
}

static int score_both_any(bool peaked, const difr_rows *in, const int32_t *claimed_ipt, float *margin, int32_t *argmax,
                          float *max_score, float *claimed_score, uint8_t *flags_gumbel, int32_t *logit_rank, float *dist,
                          float *cdf_lo, float *cdf_hi, float *u, int32_t *ipt_token, double sigma, double eps,
                          float *log_mass, uint8_t *flags_ipt, void *hip_stream)
{
    difr::RowBatch b;
    bool aligned = false;
    int rc = validate_rows(in, &b, &aligned);
    if (rc != DIFR_OK) return rc;
    if (log_mass && (!(sigma > 0.0) || !isfinite(sigma) || !(eps >= 0.0) || !isfinite(eps))) return DIFR_ERR_ARGUMENT;
    if (b.N == 0) return DIFR_OK;
    if (!margin || !argmax || !flags_gumbel || !dist || !flags_ipt) return DIFR_ERR_NULL;
    if ((rc = check_device()) != DIFR_OK) return rc;
    hipStream_t stream = (hipStream_t)hip_stream;
    if (aligned) {
        const difr::GumbelOutputs og{margin, argmax, max_score, claimed_score, flags_gumbel, logit_rank};
        const difr::IptOutputs oi{dist, cdf_lo, cdf_hi, u, ipt_token, sigma, eps, log_mass, flags_ipt, nullptr};
        return difr::launch_score_both(b, claimed_ipt, og, oi, peaked, stream) ? DIFR_ERR_LAUNCH : DIFR_OK;
    }
    // rows that are not 16-byte aligned: the two generic kernels, one after the other
    if (difr::launch_gumbel_score(b, false, true, margin, argmax, max_score, claimed_score, flags_gumbel, logit_rank, stream))
        return DIFR_ERR_LAUNCH;
    difr::RowBatch bi = b;
    bi.claimed = claimed_ipt;
    return difr::launch_ipt_score(bi, false, dist, cdf_lo, cdf_hi, u, ipt_token, sigma, eps, log_mass, flags_ipt, nullptr,
                                  stream)
               ? DIFR_ERR_LAUNCH
               : DIFR_OK;
}

int difr_score_both(const difr_rows *in, const int32_t *claimed_ipt, float *margin, int32_t *argmax, float *max_score,
                    float *claimed_score, uint8_t *flags_gumbel, int32_t *logit_rank, float *dist, float *cdf_lo,
                    float *cdf_hi, float *u, int32_t *ipt_token, double sigma, double eps, float *log_mass,
                    uint8_t *flags_ipt, void *hip_stream)
{
    return score_both_any(false, in, claimed_ipt, margin, argmax, max_score, claimed_score, flags_gumbel, logit_rank, dist,
                          cdf_lo, cdf_hi, u, ipt_token, sigma, eps, log_mass, flags_ipt, hip_stream);
}

int difr_score_both_peaked(const difr_rows *in, const int32_t *claimed_ipt, float *margin, int32_t *argmax,
                           float *max_score, float *claimed_score, uint8_t *flags_gumbel, int32_t *logit_rank, float *dist,
                           float *cdf_lo, float *cdf_hi, float *u, int32_t *ipt_token, double sigma, double eps,
                           float *log_mass, uint8_t *flags_ipt, void *hip_stream)
{
    return score_both_any(true, in, claimed_ipt, margin, argmax, max_score, claimed_score, flags_gumbel, logit_rank, dist,
                          cdf_lo, cdf_hi, u, ipt_token, sigma, eps, log_mass, flags_ipt, hip_stream);
}

int difr_score_both_admissible(const difr_rows *in, const int32_t *claimed_ipt, float delta, float *margin,
                               int32_t *argmax, float *max_score, float *claimed_score, uint8_t *flags_gumbel,
                               float *dist, float *cdf_lo, float *cdf_hi, float *u, uint8_t *flags_ipt, int32_t *count,
                               float *log2_count, void *hip_stream)
{
    difr::RowBatch b;
    bool aligned = false;
    int rc = validate_rows(in, &b, &aligned);
    if (rc != DIFR_OK) return rc;
    if (!(delta >= 0.0f) || !isfinite(delta)) return DIFR_ERR_ARGUMENT;
    if (b.N == 0) return DIFR_OK;
    if (!margin || !argmax || !flags_gumbel || !dist || !flags_ipt || !count) return DIFR_ERR_NULL;
    if (!aligned) return DIFR_ERR_ALIGN;
    if ((rc = check_device()) != DIFR_OK) return rc;
    const difr::GumbelOutputs og{margin, argmax, max_score, claimed_score, flags_gumbel, nullptr};
    const difr::IptOutputs oi{dist, cdf_lo, cdf_hi, u, nullptr, 0.0, 0.0, nullptr, flags_ipt, nullptr};
    return difr::launch_score_both_admissible(b, claimed_ipt, og, oi, delta, count, log2_count, (hipStream_t)hip_stream)
               ? DIFR_ERR_LAUNCH
               : DIFR_OK;
}

int difr_classify(const float *scores, const int32_t *ranks, int64_t N, float tau, int64_t rank_cutoff, int64_t V,
                  const float *log2_admissible, uint8_t *cls, float *bits, void *hip_stream)
{
    if (N < 0 || V < 1) return DIFR_ERR_SHAPE;
    if (tau != tau) return DIFR_ERR_ARGUMENT;
    if (N == 0) return DIFR_OK;
    if (!scores || !ranks || !cls) return DIFR_ERR_NULL;
    int rc = check_device();
    if (rc != DIFR_OK) return rc;
    return difr::launch_classify(scores, ranks, N, tau, rank_cutoff, V, log2_admissible, cls, bits,
                                 (hipStream_t)hip_stream)
               ? DIFR_ERR_LAUNCH
               : DIFR_OK;
}

int difr_debug_noise(const difr_rows *in, int64_t row, int32_t stream, uint32_t *bits, void *hip_stream)
{
    difr::RowBatch b;
    bool aligned = false;
    int rc = validate_rows(in, &b, &aligned);
    if (rc != DIFR_OK) return rc;
    if (row < 0 || row >= b.N || stream < 0) return DIFR_ERR_SHAPE;
    if (!bits) return DIFR_ERR_NULL;
    if ((rc = check_device()) != DIFR_OK) return rc;
    return difr::launch_debug_noise(b, row, (uint32_t)stream, bits, (hipStream_t)hip_stream) ? DIFR_ERR_LAUNCH
                                                                                            : DIFR_OK;
}

int difr_debug_gumbel_map(const uint32_t *bits, int64_t n, float *g, void *hip_stream)
{
    if (n < 0) return DIFR_ERR_SHAPE;
    if (n == 0) return DIFR_OK;
    if (!bits || !g) return DIFR_ERR_NULL;
    int rc = check_device();
    if (rc != DIFR_OK) return rc;
    return difr::launch_debug_gumbel_map(bits, n, g, (hipStream_t)hip_stream) ? DIFR_ERR_LAUNCH : DIFR_OK;
}

void difr_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    // Host copy of the block function (the kernels use the device version in difr_device.hpp).
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3], k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c0 = n0;
        c1 = (uint32_t)p1;
        c2 = n2;
        c3 = (uint32_t)p0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0;
    out[1] = c1;
    out[2] = c2;
    out[3] = c3;
}

const char *difr_status_string(int status)
{
    switch (status) {
        case DIFR_OK: return "ok";
        case DIFR_ERR_NULL: return "a required pointer is NULL";
        case DIFR_ERR_SHAPE: return "bad shape (N, V, S, ld or row index)";
        case DIFR_ERR_DTYPE: return "unknown logits dtype";
        case DIFR_ERR_TEMPERATURE: return "temperature must be finite and > 0";
        case DIFR_ERR_ALIGN: return "logits pointer not aligned to its element size";
        case DIFR_ERR_LAUNCH: return "HIP kernel launch failed";
        case DIFR_ERR_UNSUPPORTED: return "current device is not gfx950";
        case DIFR_ERR_ARGUMENT: return "bad scalar argument (sigma, eps, threshold, delta, or a top_k / top_p / s / M combination the call does not take)";
        case DIFR_ERR_CAPACITY: return "batch needs more scratch memory than the library's built-in buffer holds";
        default: return "unknown status";
    }
}

int difr_version(void) { return 100; }

}  // extern "C"
