// Both estimators in one pass over the row: Token-DiFR (Sec. 6.3) and Token-IPT-DiFR (Sec. 6.2)
// share the 16-byte vector each lane has just loaded, so the logits are read from HBM once for
// the two scores.  The two row streams are the ones the single-estimator kernels use
// (gumbel_stream.hpp, ipt_stream.hpp); outputs are bit-identical to theirs.
//
// RANK: the same pass also counts the entries whose raw logit exceeds the Token-DiFR claim's (logit rank, Sec. 7.1).
//
// ADM: the same pass also returns the size of the row's admissible set { v : max y - y_v <= delta } (Sec. 7),
// the count difr_admissible_count makes in a second pass once the maximum is known.
#include "difr_device.hpp"
#include "difr_host.hpp"
#include "gumbel_stream.hpp"
#include "ipt_stream.hpp"

namespace difr {

struct AdmissibleOutputs {
    float delta;
    int32_t *count;     // [N]; -1: not determined in one pass
    float *log2_count;  // [N] or null
};

// With the rank count the body needs 97 registers, one too many for five waves per SIMD; asked for five it fits in 96
// without spills and runs 5% faster.  The other variants ask for one wave, which is no constraint.
template <int DT, bool ADM, bool RANK, bool PEAKED = false>
__global__ __launch_bounds__(kBlock) __attribute__((amdgpu_waves_per_eu(RANK ? 5 : 1))) void score_both_kernel(
    RowBatch b, const int32_t *__restrict__ claimed_ipt, GumbelOutputs og, IptOutputs oi, AdmissibleOutputs oa)
{
    typedef typename Elem<DT>::type elt_t;
    constexpr int E = Elem<DT>::kPerVec;
    __shared__ float lds_y[kWaves];
    __shared__ int32_t lds_i[kWaves];
    __shared__ float lds_L[kWaves];
    __shared__ int32_t lds_rank[kWaves];
    __shared__ float lds_f[kWaves];
    __shared__ double lds_d[kWaves];
    __shared__ int32_t lds_tok;
    __shared__ float adm_lists[ADM ? kWaves * kAdmCap : 1];
    __shared__ int32_t adm_fills[kWaves];
    __shared__ int32_t lds_c[kWaves];

    const int64_t row = blockIdx.x;
    const RowInfo ri = load_row_info(b, row);
    RowInfo ri_ipt = ri;
    ri_ipt.claimed = claimed_ipt ? claimed_ipt[row] : -1;
    if (!ri.seq_ok || !ri.temp_ok) {  // uniform over the workgroup
        gumbel_row_rejected(ri, row, og);
        ipt_row_rejected(ri_ipt, row, oi);
        if (ADM && threadIdx.x == 0) {
            oa.count[row] = 0;
            if (oa.log2_count) oa.log2_count[row] = __builtin_nanf("");
        }
        return;
    }
    const int tid = threadIdx.x;
    const elt_t *x_row = reinterpret_cast<const elt_t *>(b.logits) + row * b.ld;
    const int64_t V = b.V;

    GumbelStream<DT, RANK, false, false, ADM, PEAKED> g(ri, x_row, V, lds_L);
    IptStream<DT> s(ri_ipt, x_row, V, false);
    __syncthreads();
    if (ADM) {
        g.arm_admissible(oa.delta, adm_lists, adm_fills);
        __syncthreads();
    }

    const int64_t nvec = V / E;                                      // complete vectors
    const int64_t nvec_total = (V + E - 1) / E;                      // the last vector may be partial
    const int full_rounds = (int)(nvec / kBlock);                    // rounds of 256 complete vectors
    const int n_rounds = (int)((nvec_total + kBlock - 1) / kBlock);  // full_rounds or full_rounds + 1
    const int round_t = s.valid ? (int)((s.t / E) / kBlock) : -1;    // round holding the IPT claim

    // Full rounds [round, r_end): Gumbel gates + IPT accumulation on the same vector.  The loop body is
    // instantiated once per Gumbel gate mode; a change of mode leaves the inner loop.
    int round = 0;
    auto run_rounds = [&](auto mode_tag, int r_end) {
        constexpr int MODE = decltype(mode_tag)::value;
        // one round; returns false when the loop must be left (end reached, or the gate changed mode)
        auto body = [&](const u32x4 &q) {
            g.template process<MODE>(q, round, true);
            s.fast_round(q);
            ++round;
            if ((round & 15) == 0) g.pickup();
            return round < r_end && g.gate.mode == MODE;
        };
        // one vector is kept in flight; two copies of the body, so that the vector being loaded and the one
        // being used simply swap roles instead of being copied from register to register every round
        u32x4 qa = load_round(x_row, round), qb = qa;
        while (true) {
            if (round + 1 < r_end) qb = load_round(x_row, round + 1);
            if (!body(qa)) break;
            if (round + 1 < r_end) qa = load_round(x_row, round + 1);
            if (!body(qb)) break;
        }
    };
    auto run_to = [&](int r_end) {
        while (round < r_end) {
            if (g.gate.mode == 0)
                run_rounds(std::integral_constant<int, 0>(), r_end);
            else if (g.gate.mode == 1)
                run_rounds(std::integral_constant<int, 1>(), r_end);
            else
                run_rounds(std::integral_constant<int, 2>(), r_end);
        }
    };
    // a round in which the IPT stream must look at indices (it holds the claimed token, or it is ragged)
    auto careful = [&](int r, bool prefix_open) {
        u32x4 q = u32x4{0u, 0u, 0u, 0u};
        if (s.has_vector(r)) q = load_round(x_row, r);
        g.process_any(q, r, (int64_t)r * kBlock + tid < nvec);
        s.careful_round(q, r, prefix_open);
    };

    if (s.valid && round_t < full_rounds) {
        run_to(round_t);
        careful(round_t, true);
        round = round_t + 1;
        run_to(full_rounds);
        if (n_rounds > full_rounds) careful(full_rounds, false);
    } else {
        run_to(full_rounds);
        if (s.valid) s.snapshot();  // everything so far lies below the IPT claim
        if (n_rounds > full_rounds) careful(full_rounds, s.valid);
    }
    g.tail();
    g.finish(row, og, lds_y, lds_i, lds_rank);
    if (ADM) {
        const float M = g.best_y;  // the row maximum, in every thread
        int32_t c = g.adm_count(lds_c);
        if (!(M == M) || !(fabsf(M) < __builtin_inff())) c = 0;  // as difr_admissible_count: no finite maximum
        if (tid == 0) {
            oa.count[row] = c;
            if (oa.log2_count) oa.log2_count[row] = c > 0 ? __log2f((float)c) : __builtin_nanf("");
        }
    }
    ipt_finish<DT, true>(b, ri_ipt, row, x_row, s.c, s.ref(), s.Z, s.P, s.refP(), 0, oi, lds_f, lds_d, &lds_tok);
}

int launch_score_both(const RowBatch &b, const int32_t *claimed_ipt, const GumbelOutputs &og, const IptOutputs &oi,
                      bool peaked, hipStream_t stream)
{
    const dim3 grid((unsigned)b.N), block(kBlock);
    const AdmissibleOutputs none{0.0f, nullptr, nullptr};
    const bool rank = og.logit_rank != nullptr;  // counted in the same stream, only when asked for
    if (peaked && !rank) {  // (with the rank count every round is looked at anyway: the ordinary kernel)
        if (b.dtype == 0)
            score_both_kernel<0, false, false, true><<<grid, block, 0, stream>>>(b, claimed_ipt, og, oi, none);
        else
            score_both_kernel<1, false, false, true><<<grid, block, 0, stream>>>(b, claimed_ipt, og, oi, none);
        return hipGetLastError() == hipSuccess ? 0 : 1;
    }
    if (b.dtype == 0) {
        if (rank)
            score_both_kernel<0, false, true><<<grid, block, 0, stream>>>(b, claimed_ipt, og, oi, none);
        else
            score_both_kernel<0, false, false><<<grid, block, 0, stream>>>(b, claimed_ipt, og, oi, none);
    } else {
        if (rank)
            score_both_kernel<1, false, true><<<grid, block, 0, stream>>>(b, claimed_ipt, og, oi, none);
        else
            score_both_kernel<1, false, false><<<grid, block, 0, stream>>>(b, claimed_ipt, og, oi, none);
    }
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

int launch_score_both_admissible(const RowBatch &b, const int32_t *claimed_ipt, const GumbelOutputs &og,
                                 const IptOutputs &oi, float delta, int32_t *count, float *log2_count, hipStream_t stream)
{
    const dim3 grid((unsigned)b.N), block(kBlock);
    const AdmissibleOutputs oa{delta, count, log2_count};
    if (b.dtype == 0)
        score_both_kernel<0, true, false><<<grid, block, 0, stream>>>(b, claimed_ipt, og, oi, oa);
    else
        score_both_kernel<1, true, false><<<grid, block, 0, stream>>>(b, claimed_ipt, og, oi, oa);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

}  // namespace difr
