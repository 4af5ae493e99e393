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
#include "topn.hpp"

namespace difr {

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

template <int DT>
__global__ __launch_bounds__(kBlock) void likelihood_kernel(RowBatch b, LikelihoodParams p, LikelihoodOutputs o)
{
    typedef typename Elem<DT>::type elt_t;
    constexpr int E = Elem<DT>::kPerVec;
    __shared__ uint64_t buf_y[kTopCap];
    __shared__ uint64_t buf_x[kTopCap];
    __shared__ TopScratch scratch;
    __shared__ int32_t cnt_y, cnt_x, snap_y, snap_x;
    __shared__ float lds_L[kWaves];
    __shared__ double lds_d[kWaves];
    __shared__ double sA[kTopMaxN], sB[kTopMaxN];
    __shared__ double s_tau;
    __shared__ int32_t s_bad;

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
        return;
    }
    const elt_t *x_row = reinterpret_cast<const elt_t *>(b.logits) + row * b.ld;

    TopN top_y, top_x;
    top_y.init(buf_y, &cnt_y, valid ? p.s : 0);
    top_x.init(buf_x, &cnt_x, p.top_k);
    if (tid == 0) {
        s_bad = 0;
        snap_y = snap_x = 0;
    }
    GumbelStream<DT, false, false, true> g(ri, x_row, V, lds_L);
    __syncthreads();
    g.arm_topn(&top_y);
    __syncthreads();
    uint32_t bad = 0;

    // raw-logit candidates of one vector.  First a test of the whole vector against the selection's threshold
    // (bf16: packed 16-bit min / max on the raw bit patterns, as in the Gumbel gates; a NaN with the sign bit
    // clear passes it and is flagged below, one with the sign bit set counts as -inf), then the 64-bit
    // composite only for the entries that pass.
    float x_floor = -__builtin_inff();
    uint32_t x_floor16 = cap_bits(x_floor, true);
    bool x_floor_pos = false;
    auto set_x_floor = [&](float f) {
        x_floor = f;
        x_floor_pos = f > 0.0f;
        x_floor16 = cap_bits(f, !x_floor_pos);
    };
    auto push_logits = [&](u32x4 q, int64_t v0, bool active) {
        bool hit;
        if (DT == 0) {
            if (x_floor_pos) {
                i16x2 m = __builtin_elementwise_max(as_i16x2(q.x), as_i16x2(q.y));
                m = __builtin_elementwise_max(m, as_i16x2(q.z));
                m = __builtin_elementwise_max(m, as_i16x2(q.w));
                hit = (int16_t)(m.x > m.y ? m.x : m.y) >= (int16_t)x_floor16;
            } else {
                u16x2 m = __builtin_elementwise_min(as_u16x2(q.x), as_u16x2(q.y));
                m = __builtin_elementwise_min(m, as_u16x2(q.z));
                m = __builtin_elementwise_min(m, as_u16x2(q.w));
                hit = (uint16_t)(m.x < m.y ? m.x : m.y) <= (uint16_t)x_floor16;
            }
        } else {
            hit = !(__uint_as_float(q.x) < x_floor) || !(__uint_as_float(q.y) < x_floor) ||
                  !(__uint_as_float(q.z) < x_floor) || !(__uint_as_float(q.w) < x_floor);
        }
        hit = hit && active;
        if (__builtin_amdgcn_ballot_w64(hit) != 0ull) {
            if (hit) {
                const uint32_t qw[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
                for (int j = 0; j < E; ++j) {
                    const uint32_t w = qw[DT == 0 ? j >> 1 : j];
                    const float xv = DT == 0 ? __uint_as_float((j & 1) ? (w & 0xFFFF0000u) : (w << 16)) : __uint_as_float(w);
                    bad |= (uint32_t)!(xv < __builtin_inff());
                    if (xv >= x_floor) top_x.push(top_composite(xv, (int32_t)(v0 + j)));
                }
            }
        }
    };
    // compaction of whichever buffer has reached its trigger (uniform decisions through the barrier
    // reduction, which returns a truth value: one call per buffer)
    auto settle = [&]() {
        if (__syncthreads_or((int)top_y.full)) {
            if (top_y.compact(scratch, true)) g.retarget();
        }
        if (p.top_k > 0 && __syncthreads_or((int)top_x.full)) {
            top_x.compact(scratch, true);
            set_x_floor(top_key(top_x.theta));
        }
    };

    const int64_t nvec = V / E;
    const int n_rounds = (int)((nvec + kBlock - 1) / kBlock);
    auto fetch = [&](int round) {
        u32x4 q = u32x4{0u, 0u, 0u, 0u};
        if ((int64_t)round * kBlock + tid < nvec) q = load_round(x_row, round);
        return q;
    };
    auto do_round = [&](u32x4 q, int round) {
        const int64_t vec = (int64_t)round * kBlock + tid;
        const bool active = vec < nvec;
        g.process_any(q, round, active);
        if (p.top_k > 0) push_logits(q, vec * E, active);
    };
    // Epochs: the first round alone (every entry is a candidate while there is no threshold: exactly the
    // quota), then eight rounds at a time without a barrier.
    int round = 0;
    while (round < n_rounds) {
        const int r_end = min(n_rounds, round + (round == 0 ? 1 : 8));
        top_y.new_epoch(kTopQuota);
        top_x.new_epoch(kTopQuota);
        u32x4 q_next = fetch(round);
        for (int r = round; r < r_end; ++r) {
            const u32x4 q = q_next;
            if (r + 1 < r_end) q_next = fetch(r + 1);  // keep one vector in flight
            do_round(q, r);
        }
        if (__syncthreads_or((int)(top_y.over || top_x.over))) {
            // some thread had more candidates than its quota (data in ascending order, for instance):
            // forget the epoch and repeat it round by round, compacting whenever a trigger is reached
            if (tid == 0) {
                cnt_y = snap_y;
                cnt_x = snap_x;
            }
            top_y.new_epoch(0x7FFFFFFF);
            top_x.new_epoch(0x7FFFFFFF);
            top_y.full = top_x.full = false;
            __syncthreads();
            for (int r = round; r < r_end; ++r) {
                do_round(fetch(r), r);
                settle();
            }
        } else {
            settle();
        }
        if (tid == 0) {
            snap_y = cnt_y;
            snap_x = cnt_x;
        }
        __syncthreads();
        round = r_end;
    }
    top_y.new_epoch(kTopQuota);  // the tail: at most one entry per thread
    top_x.new_epoch(kTopQuota);
    // ragged tail: V % E entries, one lane each
    g.tail();
    {
        const int64_t v = nvec * E + tid;
        if (v < V && p.top_k > 0) {
            const float xv = Elem<DT>::to_float(x_row[v]);
            bad |= (uint32_t)!(xv < __builtin_inff());
            if (xv >= x_floor) top_x.push(top_composite(xv, (int32_t)v));
        }
    }
    if (bad) s_bad = 1;
    const int ns = top_y.finish_sorted(scratch);   // buf_y[0 .. ns): S in rank order
    const int nk = top_x.finish_sorted(scratch);   // buf_x[0 .. nk): the k largest logits, descending

    // filter threshold: top-k first, then top-p on the distribution renormalised over those k (fp64, one thread)
    if (tid == 0) {
        double tau = -(double)__builtin_inff();
        if (p.top_k > 0 && nk > 0) {
            int kept = nk;
            if (p.top_p < 1.0f) {
                const double x0 = (double)top_key(buf_x[0]);
                const double T = (double)ri.T;
                double Z = 0.0;
                for (int r = 0; r < nk; ++r) Z += exp(((double)top_key(buf_x[r]) - x0) / T);
                double cum = 0.0;
                for (int r = 0; r < nk; ++r) {
                    cum += exp(((double)top_key(buf_x[r]) - x0) / T) / Z;
                    if (cum >= (double)p.top_p) {
                        kept = r + 1;
                        break;
                    }
                }
            }
            tau = (double)top_key(buf_x[kept - 1]);
        }
        s_tau = tau;
    }
    __syncthreads();
    const double tau = s_tau;
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

int launch_likelihood(const RowBatch &b, const LikelihoodParams &p, const LikelihoodOutputs &o, hipStream_t stream)
{
    const dim3 grid((unsigned)b.N), block(kBlock);
    if (b.dtype == 0)
        likelihood_kernel<0><<<grid, block, 0, stream>>>(b, p, o);
    else
        likelihood_kernel<1><<<grid, block, 0, stream>>>(b, p, o);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

}  // namespace difr
