// Token-DiFR likelihood estimate of the claimed token (Sec. 6.3; appendix algorithm of the Gumbel-max FSSL
// estimator): active set S = the s best perturbed scores, filter threshold tau from the sampler's top-k /
// top-p policy, A_i and B_i for i in S, and the average over the supplied normal draws of
//   [l_t* + x_j > tau] prod_{i in S} Phi(max(x_j + A_i, B_i) / sigma).
//
// One workgroup per row, one pass over the logits.  Two exact streaming selections run side by side
// (topn.hpp): the s largest y_v = x_v / T + g_v (claimed token left out), fed by the same gated Gumbel
// stream as the scoring kernels with the selection's threshold as the bound, and the k largest raw logits.
// Everything after the pass works on s + k + 1 tokens: their noise is recomputed in fp64, so A_i carries
// no fp32 error; only WHICH tokens are in S is decided in fp32.
#include "difr_device.hpp"
#include "difr_host.hpp"
#include "gumbel_stream.hpp"
#include "ipt_stream.hpp"
#include "logit_top.hpp"
#include "topn.hpp"

namespace difr {

// stream rounds per epoch once the thresholds have settled (vectors that trip a test only queue up, so a threshold that
// is an epoch old costs little; measured: 16, 24 and 32 alike, 8 slower by 4%)
constexpr int kLikEpoch = 16;

__device__ __forceinline__ double gumbel_f64(const RowInfo &ri, int32_t v)
{
    uint32_t r[4];
    noise_block(ri.key, ri.pos, ri.seq, kStreamGumbel, (uint32_t)v >> 2, r);
    const uint32_t rv = (v & 3) == 0 ? r[0] : (v & 3) == 1 ? r[1] : (v & 3) == 2 ? r[2] : r[3];
    const uint32_t k = rv >> 9;
    const double u = (double)(2u * k + 1u) * 0x1p-24;
    const double w = (double)(2u * (0x7FFFFFu - k) + 1u) * 0x1p-24;  // 1 - u, exact
    const double t = (u > 0.5) ? -log1p(-w) : -log(u);
    return -log(t);
}

__device__ __forceinline__ float normal_cdf_f32(float z) { return 0.5f * erfcf(-z * 0.70710678118654752f); }

// BOTH: the same pass also scores Token-IPT-DiFR on the distribution the filter leaves (the top-k logits are
// being collected anyway), with outputs identical to ipt_filtered_kernel's.
struct FilteredIptSide {
    const int32_t *claimed;  // [N] the Token-IPT-DiFR claims, or null
    IptOutputs o;
    int32_t *kept;
};

template <int DT, int CAP, bool BOTH>
__device__ __forceinline__ void likelihood_row(const RowBatch &b, const LikelihoodParams &p, const LikelihoodOutputs &o,
                                               const FilteredIptSide &ipt)
{
    typedef typename Elem<DT>::type elt_t;
    constexpr int E = Elem<DT>::kPerVec;
    __shared__ uint64_t buf_y[CAP];
    __shared__ uint64_t buf_x[CAP];
    __shared__ TopScratch scratch;
    __shared__ int32_t cnt_y, cnt_x;
    __shared__ uint32_t epoch_flags[3];
    __shared__ float lds_L[kWaves];
    __shared__ int32_t defer_q[kWaves * kDeferCap], defer_qx[kWaves * kDeferCap];
    __shared__ double lds_d[kWaves];
    __shared__ double sA[kTopMaxN], sB[kTopMaxN];
    __shared__ int32_t s_bad, s_tok;
    __shared__ double s_e[BOTH ? kTopMaxN : 1];     // the IPT side's kept set in ascending vocabulary index
    __shared__ int32_t s_idx[BOTH ? kTopMaxN : 1];

    const int64_t row = blockIdx.x;
    const RowInfo ri = load_row_info(b, row);
    const int tid = threadIdx.x;
    const float nan = __builtin_nanf("");
    const int64_t V = b.V;
    const int32_t t = ri.claimed;
    const bool valid = t >= 0 && (int64_t)t < V;
    if (!ri.seq_ok || !ri.temp_ok) {  // uniform over the workgroup
        if (tid == 0) {
            o.pi[row] = nan;
            if (o.log_pi) o.log_pi[row] = nan;
            if (o.tau) o.tau[row] = nan;
            o.flags[row] = (uint8_t)(ri.seq_ok ? kFlagNonfinite : kFlagInvalidClaim);
        }
        if (o.active)
            for (int j = tid; j < p.s; j += kBlock) o.active[row * p.s + j] = -1;
        if (BOTH) {
            RowInfo ri_ipt = ri;
            ri_ipt.claimed = ipt.claimed ? ipt.claimed[row] : -1;
            ipt_row_rejected(ri_ipt, row, ipt.o);
            if (ipt.kept && tid == 0) ipt.kept[row] = 0;
        }
        return;
    }
    const elt_t *x_row = reinterpret_cast<const elt_t *>(b.logits) + row * b.ld;

    GumbelStream<DT, false, false, true> g(ri, x_row, V, lds_L);
    g.arm_deferred(defer_q);
    TopN top_y;
    LogitTop<DT> lx;
    TopN &top_x = lx.top;
    top_y.init(buf_y, &cnt_y, valid ? p.s : 0, CAP);
    lx.init(buf_x, &cnt_x, p.top_k, CAP);
    lx.arm_deferred(defer_qx, x_row);
    if (tid == 0) {
        s_bad = 0;
        s_tok = -1;
        epoch_flags[0] = epoch_flags[1] = epoch_flags[2] = 0u;
    }
    __syncthreads();
    g.retarget(top_y);
    __syncthreads();

    // compaction of whichever buffer has reached its trigger (uniform decisions through the barrier
    // reduction, which returns a truth value: one call per buffer)
    auto settle = [&]() __attribute__((always_inline)) {
        if (__syncthreads_or((int)top_y.full)) {
            if (top_y.compact(scratch, true)) g.retarget(top_y);
        }
        if (p.top_k > 0 && __syncthreads_or((int)top_x.full)) {
            if (top_x.compact(scratch, true)) lx.retarget();
        }
    };

    const int64_t nvec = V / E;
    const int n_main = (int)(nvec / kBlock);                       // rounds in which every lane has a vector
    const int n_rounds = (int)((nvec + kBlock - 1) / kBlock);      // plus a last, partly filled one
    // one round, any gate mode, lanes past the end of the row idle (the priming run, the partly filled round, and
    // the careful mode below); what the round finds is looked at before it returns
    // (`only_wave` >= 0: only that wave's lanes take part)
    auto do_round = [&](int round, int only_wave = -1) __attribute__((always_inline)) {
        const int64_t vec = (int64_t)round * kBlock + tid;
        const bool in_row = vec < nvec;
        const bool active = in_row && (only_wave < 0 || (tid >> 6) == only_wave);
        u32x4 q = u32x4{0u, 0u, 0u, 0u};
        if (in_row) q = load_round(x_row, round);
        g.process_any(q, round, active, &top_y);
        g.drain(&top_y);
        if (p.top_k > 0) lx.push_vector(q, vec * E, active);
    };
    // full rounds [r0, r1) with the loop body instantiated for the gate's mode (it can only change at a
    // compaction, i.e. between epochs): one copy of the Philox + gate code per mode instead of one per
    // mode and unrolled round, which did not fit the instruction cache.  Vectors that trip a test wait in the
    // two per-wave queues, across epochs, until 64 of them make a look at them worth the wave's while.
    auto run_rounds = [&](auto mode_tag, int r0, int r1) __attribute__((always_inline)) {
        constexpr int MODE = decltype(mode_tag)::value;
        u32x4 q_next = load_round(x_row, r0);
#pragma nounroll
        for (int r = r0; r < r1; ++r) {
            const u32x4 q = q_next;
            if (r + 1 < r1) q_next = load_round(x_row, r + 1);  // keep one vector in flight
            g.template process<MODE>(q, r, true, &top_y);
            if (g.defer_n >= 64) g.drain(&top_y);
            if (p.top_k > 0) {
                lx.template note_vector<(DT == 0) ? ((MODE != 1 ? 1 : 0) | (MODE != 0 ? 2 : 0)) : 0>(q, r * kBlock + tid, g.seen_lo, g.seen_hi);
                if (lx.defer_n >= 64) lx.drain();
            }
        }
    };
    // priming run of the first round (topn.hpp): thresholds for both selections before anything is pushed
    if (n_rounds > 0) {
        top_y.begin_prime();
        top_x.begin_prime();
        do_round(0);
        if (top_y.end_prime(scratch)) g.retarget(top_y);
        if (top_x.end_prime(scratch)) lx.retarget();
    }
    // Epochs: the first round alone, then up to kLikEpoch rounds at a time without a barrier; the partly filled round is
    // an epoch of its own.  A push that finds a buffer full (data in ascending order, for instance) ends this mode.
    int round = 0, epoch = 0;
    bool ran_full = false;
    while (round < n_rounds) {
        // (the first epochs are 1, 1, 2 and 4 rounds long: the thresholds move only between epochs, and while little of
        // the row has been seen they move a lot - a threshold that is one doubling of the data behind lets twice as
        // many vectors through the tests)
        const int len = round < 2 ? 1 : (round < 4 ? 2 : (round < 8 ? 4 : kLikEpoch));
        const int r_end = round < n_main ? min(n_main, round + len) : n_rounds;
        if (round >= n_main)
            do_round(round);
        else if (g.gate.mode == 0)
            run_rounds(std::integral_constant<int, 0>(), round, r_end);
        else if (g.gate.mode == 1)
            run_rounds(std::integral_constant<int, 1>(), round, r_end);
        else
            run_rounds(std::integral_constant<int, 2>(), round, r_end);
        if (round >= n_main || r_end == n_rounds) {  // the row's last epoch: nothing may be left waiting
            g.drain(&top_y);
            lx.drain();
        }
        // one barrier per epoch: the workgroup's OR of "a push found a buffer full" and of the two compaction triggers.
        // (three words in turn: the word of the next epoch is cleared before this epoch's barrier, when every thread
        // has long read it for the last time, and is written only after that barrier)
        {
            const uint32_t mine = (uint32_t)(top_y.over || top_x.over) | ((uint32_t)top_y.full << 1) | ((uint32_t)top_x.full << 2);
            uint32_t *word = &epoch_flags[epoch % 3];
            if (mine) atomicOr(word, mine);
            if (tid == 0) epoch_flags[(epoch + 1) % 3] = 0u;
            __syncthreads();
            const uint32_t all = *word;
            ++epoch;
            if (all & 1u) {
                ran_full = true;
                break;
            }
            if (all & 2u) {
                if (top_y.compact(scratch, true)) g.retarget(top_y);
            }
            if (all & 4u) {
                if (top_x.compact(scratch, true)) lx.retarget();
            }
        }
        round = r_end;
    }
    if (ran_full) {
        // Careful mode: the row again from its start, one wave and one round at a time with a compaction check after
        // each step.  A step starts with fewer than kTopTrigger entries in a buffer and adds at most 8 per lane of one
        // wave, so the buffers cannot run full, whatever the order of the data.
        top_y.init(buf_y, &cnt_y, valid ? p.s : 0, CAP);
        lx.init(buf_x, &cnt_x, p.top_k, CAP);
        g.defer_n = 0;
        __syncthreads();
        g.retarget(top_y);
        __syncthreads();
        for (int r = 0; r < n_rounds; ++r) {
            for (int w = 0; w < kWaves; ++w) {
                do_round(r, w);
                settle();
            }
        }
    }
    top_y.new_epoch();  // the tail: at most one entry per thread
    top_x.new_epoch();
    // ragged tail: V % E entries, one lane each
    g.tail(&top_y);
    {
        const int64_t v = nvec * E + tid;
        if (v < V && p.top_k > 0) lx.push_entry(Elem<DT>::to_float(x_row[v]), (int32_t)v);
    }
    if (lx.bad) s_bad = 1;
    const int ns = top_y.finish_sorted(scratch);   // buf_y[0 .. ns): S in rank order
    const int nk = top_x.finish_sorted(scratch);   // buf_x[0 .. nk): the k largest logits, descending

    // filter threshold: top-k first, then top-p on the distribution renormalised over those k (fp64)
    double tau = -(double)__builtin_inff();
    int kc = 0;  // length of the filter's prefix of the ranked top-k logits
    if (p.top_k > 0) kc = filter_prefix_length(buf_x, nk, (double)ri.T, p.top_p, scratch);
    if (kc > 0) tau = (double)top_key(buf_x[kc - 1]);
    if (BOTH) {
        RowInfo ri_ipt = ri;
        ri_ipt.claimed = ipt.claimed ? ipt.claimed[row] : -1;
        __syncthreads();  // s_bad is final
        ipt_filtered_finish<DT>(ri_ipt, row, V, buf_x, kc, s_bad != 0, ipt.o, ipt.kept, s_e, s_idx, lds_d, &s_tok);
        __syncthreads();
    }
    if (p.tau_in) tau = (double)p.tau_in[row];  // found beforehand by the nucleus kernel (NaN if it could not: pi becomes NaN)
    double xt = 0.0, gt = 0.0;
    if (valid) {
        xt = (double)Elem<DT>::to_float(x_row[t]);
        gt = gumbel_f64(ri, t);
    }
    if (tid < ns) {
        const int32_t i = top_index(buf_y[tid]);
        const double xi = (double)Elem<DT>::to_float(x_row[i]);
        sA[tid] = xt - xi + (double)ri.T * (gt - gumbel_f64(ri, i));
        sB[tid] = tau - xi;
        if (o.active) o.active[row * p.s + tid] = i;
    } else if (o.active && tid < p.s) {
        o.active[row * p.s + tid] = -1;
    }
    if (o.active)
        for (int j = kBlock + tid; j < p.s; j += kBlock) o.active[row * p.s + j] = -1;  // (s <= 256: never runs)
    __syncthreads();

    // average over the supplied draws
    double acc = 0.0;
    if (valid) {
        const double sigma = (double)p.sigma, inv_sigma = 1.0 / sigma;
        for (int j = tid; j < p.M; j += kBlock) {
            const double xj = sigma * (double)p.z[j];
            if (xt + xj > tau) {
                float prod = 1.0f;
                for (int i = 0; i < ns; ++i) prod *= normal_cdf_f32((float)(fmax(xj + sA[i], sB[i]) * inv_sigma));
                acc += (double)prod;
            }
        }
    }
    const double total = block_sum_f64(acc, lds_d);
    if (tid == 0) {
        uint32_t f = s_bad ? kFlagNonfinite : 0u;
        float pi = nan, lp = nan;
        if (valid) {
            const double pd = total / (double)p.M;
            pi = (float)pd;
            lp = (float)log(pd);
        } else {
            f |= kFlagInvalidClaim;
        }
        o.pi[row] = pi;
        if (o.log_pi) o.log_pi[row] = lp;
        if (o.tau) o.tau[row] = (float)tau;
        o.flags[row] = (uint8_t)f;
    }
}

// Small selections (s and top_k up to kTopSmallN): 24 KB of LDS per workgroup, and the register budget of five
// waves per SIMD (the few spills that costs are worth the fifth workgroup: measured).  Large ones: big buffers.
template <int DT, bool BOTH>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(5))) void likelihood_small_kernel(RowBatch b, LikelihoodParams p,
                                                                                                         LikelihoodOutputs o,
                                                                                                         FilteredIptSide ipt)
{
    likelihood_row<DT, kTopCapSmall, BOTH>(b, p, o, ipt);
}
template <int DT, bool BOTH>
__global__ __launch_bounds__(kBlock) void likelihood_big_kernel(RowBatch b, LikelihoodParams p, LikelihoodOutputs o, FilteredIptSide ipt)
{
    likelihood_row<DT, kTopCapBig, BOTH>(b, p, o, ipt);
}

template <bool BOTH>
static int launch_likelihood_any(const RowBatch &b, const LikelihoodParams &p, const LikelihoodOutputs &o,
                                 const FilteredIptSide &ipt, hipStream_t stream)
{
    const dim3 grid((unsigned)b.N), block(kBlock);
    const bool small = p.s <= kTopSmallN && p.top_k <= kTopSmallN;
    if (b.dtype == 0) {
        if (small)
            likelihood_small_kernel<0, BOTH><<<grid, block, 0, stream>>>(b, p, o, ipt);
        else
            likelihood_big_kernel<0, BOTH><<<grid, block, 0, stream>>>(b, p, o, ipt);
    } else {
        if (small)
            likelihood_small_kernel<1, BOTH><<<grid, block, 0, stream>>>(b, p, o, ipt);
        else
            likelihood_big_kernel<1, BOTH><<<grid, block, 0, stream>>>(b, p, o, ipt);
    }
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

int launch_likelihood(const RowBatch &b, const LikelihoodParams &p, const LikelihoodOutputs &o, hipStream_t stream)
{
    const FilteredIptSide none{nullptr, IptOutputs{nullptr, nullptr, nullptr, nullptr, nullptr, 0.0, 0.0, nullptr, nullptr, nullptr}, nullptr};
    return launch_likelihood_any<false>(b, p, o, none, stream);
}

int launch_score_both_filtered(const RowBatch &b, const LikelihoodParams &p, const LikelihoodOutputs &o,
                               const int32_t *claimed_ipt, const IptOutputs &oi, int32_t *kept, hipStream_t stream)
{
    const FilteredIptSide side{claimed_ipt, oi, kept};
    return launch_likelihood_any<true>(b, p, o, side, stream);
}

}  // namespace difr
