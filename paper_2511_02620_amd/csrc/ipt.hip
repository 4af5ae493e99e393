// Token-IPT-DiFR row kernels: regenerate the seeded uniform u, form p = softmax(x / T)
// and its CDF in ascending token order, and report the claimed token's interval
// [a, b) = [Fbar_{t-1}, Fbar_t), the distance of u from it, and optionally the Gaussian
// log-mass and the honest sampler's token  min{ v : C_v > u }.
// (Sec. 3.2 softmax and IPT sampler; Sec. 6.2 and the appendix algorithm
// "convolved Gaussian score".)
//
// One workgroup per token row, one streaming pass; nothing of size V is stored.  Only when the
// honest sampler's token is asked for and differs from the claim is the row read a second time.
#include "difr_device.hpp"
#include "difr_host.hpp"
#include "ipt_stream.hpp"

namespace difr {

// Generic kernel: any alignment, element-wise loads.  Used for rows that are not 16-byte aligned.
template <int DT>
__global__ __launch_bounds__(kBlock) void ipt_score_generic_kernel(RowBatch b, IptOutputs o)
{
    typedef typename Elem<DT>::type elt_t;
    constexpr int E = Elem<DT>::kPerVec;
    __shared__ float lds_f[kWaves];
    __shared__ double lds_d[kWaves];
    __shared__ int32_t lds_tok;

    const int64_t row = blockIdx.x;
    const RowInfo ri = load_row_info(b, row);
    if (ipt_row_rejected(ri, row, o)) return;
    const int tid = threadIdx.x;
    const float ninf = -__builtin_inff();

    const elt_t *x_row = reinterpret_cast<const elt_t *>(b.logits) + row * b.ld;
    const int64_t V = b.V;
    const float c = kLog2e / ri.T;  // exponent scale: exp(x/T) = 2^(x c)
    const int64_t t = ri.claimed;
    const int64_t tcut = (t >= 0 && t < V) ? t : 0;  // prefix is over v < tcut
    const float xt = (t >= 0 && t < V) ? Elem<DT>::to_float(x_row[t]) : __builtin_nanf("");
    __shared__ int32_t lds_rank[kWaves];
    int32_t above = 0;  // entries whose raw logit exceeds the claimed token's (logit rank)

    float m = ninf, neg_mc = __builtin_inff(), neg_mcP = __builtin_inff();  // (+inf: no reference yet)
    double Z = 0.0, P = 0.0;
    for (int64_t base = (int64_t)tid * E; base < V; base += (int64_t)kBlock * E) {
        float x[E], e[E];
        load_elems<DT, false>(x_row, base, V, x);
#pragma unroll
        for (int j = 0; j < E; ++j) above += (int32_t)(x[j] > xt);
        float m8 = x[0];
#pragma unroll
        for (int j = 1; j < E; ++j) m8 = fmaxf(m8, x[j]);
        if (m8 > m) {  // rebase the running sum (m = -inf: Z is still 0 and stays 0)
            const float moved = -(m8 * c);
            Z *= (double)fast_exp2(moved - neg_mc);  // between the two rounded references (see ipt_finish)
            m = m8;
            neg_mc = moved;
        }
#pragma unroll
        for (int j = 0; j < E; ++j) e[j] = fast_exp2(__fmaf_rn(x[j], c, neg_mc));
        float pre = 0.0f;
#pragma unroll
        for (int j = 0; j < E; ++j)
            if (base + j < tcut) pre += e[j];
        if (base < tcut) {
            P = Z + (double)pre;
            neg_mcP = neg_mc;
        }
        Z += (double)tree_sum<E>(e);
    }
    above = block_sum_i32(above, lds_rank);
    ipt_finish<DT, false>(b, ri, row, x_row, c, -neg_mc, Z, P, -neg_mcP, above, o, lds_f, lds_d, &lds_tok);
}

// Streaming kernel for 16-byte aligned rows (the streaming state is described in ipt_stream.hpp).
template <int DT>
__global__ __launch_bounds__(kBlock) void ipt_score_kernel(RowBatch b, IptOutputs o)
{
    typedef typename Elem<DT>::type elt_t;
    constexpr int E = Elem<DT>::kPerVec;
    __shared__ float lds_f[kWaves];
    __shared__ double lds_d[kWaves];
    __shared__ int32_t lds_tok;
    __shared__ int32_t lds_rank[kWaves];

    const int64_t row = blockIdx.x;
    const RowInfo ri = load_row_info(b, row);
    if (ipt_row_rejected(ri, row, o)) return;
    const elt_t *x_row = reinterpret_cast<const elt_t *>(b.logits) + row * b.ld;
    const int64_t V = b.V;

    IptStream<DT> s(ri, x_row, V, o.logit_rank != nullptr);

    auto load = [&](int round) {
        const char *p = reinterpret_cast<const char *>(x_row) + (size_t)round * (kBlock * 16) + threadIdx.x * 16u;
        return __builtin_nontemporal_load(reinterpret_cast<const ipt_u32x4 *>(p));
    };
    auto stream = [&](int r0, int r1) {  // full rounds [r0, r1) with one vector kept in flight
        if (r0 >= r1) return;
        ipt_u32x4 q_next = load(r0);
        for (int round = r0; round < r1; ++round) {
            const ipt_u32x4 q = q_next;
            if (round + 1 < r1) q_next = load(round + 1);
            s.fast_round(q);
        }
    };
    auto careful = [&](int round, bool prefix_open) {
        ipt_u32x4 q = ipt_u32x4{0u, 0u, 0u, 0u};
        if (s.has_vector(round)) q = load(round);
        s.careful_round(q, round, prefix_open);
    };

    const int64_t nvec_total = (V + E - 1) / E;                      // the last vector may be partial
    const int full_rounds = (int)((V / E) / kBlock);                 // rounds of 256 complete vectors
    const int n_rounds = (int)((nvec_total + kBlock - 1) / kBlock);  // full_rounds or full_rounds + 1
    const int round_t = s.valid ? (int)((s.t / E) / kBlock) : -1;

    if (s.valid && round_t < full_rounds) {
        stream(0, round_t);
        careful(round_t, true);
        stream(round_t + 1, full_rounds);
        if (n_rounds > full_rounds) careful(full_rounds, false);
    } else {
        stream(0, full_rounds);
        if (s.valid) s.snapshot();  // everything so far lies below the claimed token
        if (n_rounds > full_rounds) careful(full_rounds, s.valid);
    }
    const int32_t above = s.total_above(lds_rank);
    ipt_finish<DT, true>(b, ri, row, x_row, s.c, s.ref(), s.Z, s.P, s.refP(), above, o, lds_f, lds_d, &lds_tok);
}

int launch_ipt_score(const RowBatch &b, bool aligned, float *dist, float *cdf_lo, float *cdf_hi, float *u,
                     int32_t *ipt_token, double sigma, double eps, float *log_mass, uint8_t *flags,
                     int32_t *logit_rank, hipStream_t stream)
{
    const dim3 grid((unsigned)b.N), block(kBlock);
    const IptOutputs o{dist, cdf_lo, cdf_hi, u, ipt_token, sigma, eps, log_mass, flags, logit_rank};
    if (b.dtype == 0) {
        if (aligned)
            ipt_score_kernel<0><<<grid, block, 0, stream>>>(b, o);
        else
            ipt_score_generic_kernel<0><<<grid, block, 0, stream>>>(b, o);
    } else {
        if (aligned)
            ipt_score_kernel<1><<<grid, block, 0, stream>>>(b, o);
        else
            ipt_score_generic_kernel<1><<<grid, block, 0, stream>>>(b, o);
    }
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

}  // namespace difr
