// Token-IPT-DiFR on the distribution a filtering sampler used (Sec. 3.2: IPT sampler under the generation
// policy's top-k / top-p filter; Sec. 6.2 and the appendix "convolved Gaussian score" with p = those
// probabilities).  The kept set K is a prefix of the tokens ranked by logit (ties to the lower index):
// the first top_k, cut further to the shortest prefix whose softmax(x / T) mass, renormalised over the
// top_k, reaches top_p.  Inside K the probabilities are renormalised and the CDF runs in ascending
// vocabulary index; a claimed token outside K has an empty interval.
//
// One workgroup per row, one pass over the logits that keeps the top_k largest (logit_top.hpp); no noise
// is generated per entry, so the pass runs at streaming speed.  Everything else works on <= 256 tokens in fp64.
#include "difr_device.hpp"
#include "difr_host.hpp"
#include "gumbel_stream.hpp"
#include "ipt_stream.hpp"
#include "logit_top.hpp"
#include "topn.hpp"

namespace difr {

template <int DT, int CAP>
__global__ __launch_bounds__(kBlock) void ipt_filtered_kernel(RowBatch b, int top_k, float top_p, IptOutputs o,
                                                              int32_t *__restrict__ kept_out)
{
    typedef typename Elem<DT>::type elt_t;
    constexpr int E = Elem<DT>::kPerVec;
    __shared__ uint64_t buf_x[CAP];
    __shared__ TopScratch scratch;
    __shared__ int32_t cnt_x, s_bad, s_tok;
    __shared__ uint32_t epoch_flags[3];
    __shared__ int32_t defer_q[kWaves * kDeferCap];
    __shared__ double lds_d[kWaves];
    __shared__ double s_e[kTopMaxN];     // unnormalised probabilities of K in ascending vocabulary index
    __shared__ int32_t s_idx[kTopMaxN];  // and those indices

    const int64_t row = blockIdx.x;
    const RowInfo ri = load_row_info(b, row);
    const int tid = threadIdx.x;
    if (ipt_row_rejected(ri, row, o)) {
        if (kept_out && tid == 0) kept_out[row] = 0;
        return;
    }
    const int64_t V = b.V;
    const elt_t *x_row = reinterpret_cast<const elt_t *>(b.logits) + row * b.ld;

    LogitTop<DT> lx;
    lx.init(buf_x, &cnt_x, top_k, CAP);
    lx.arm_deferred(defer_q, x_row);
    if (tid == 0) {
        s_bad = 0;
        s_tok = -1;
        epoch_flags[0] = epoch_flags[1] = epoch_flags[2] = 0u;
    }
    __syncthreads();
    const int64_t nvec = V / E;
    const int n_main = (int)(nvec / kBlock);                   // rounds in which every lane has a vector
    const int n_rounds = (int)((nvec + kBlock - 1) / kBlock);  // plus a last, partly filled one
    auto fetch = [&](int round) {
        u32x4 q = u32x4{0u, 0u, 0u, 0u};
        if ((int64_t)round * kBlock + tid < nvec) q = load_round(x_row, round);
        return q;
    };
    // one round looked at on the spot (the priming run, the partly filled round, the careful mode below);
    // `only_wave` >= 0: only that wave's lanes take part
    auto do_round = [&](u32x4 q, int round, int only_wave = -1) {
        const int64_t vec = (int64_t)round * kBlock + tid;
        lx.push_vector(q, vec * E, vec < nvec && (only_wave < 0 || (tid >> 6) == only_wave));
    };
    // priming run of the first round (topn.hpp): a threshold before anything is pushed
    if (n_rounds > 0) {
        lx.top.begin_prime();
        do_round(fetch(0), 0);
        if (lx.top.end_prime(scratch)) lx.retarget();
    }
    // Epochs without barriers, as in the likelihood kernel: vectors that hold a candidate wait in the wave's queue until
    // 64 of them make the look at their entries worth the wave's while; one barrier per epoch combines "a push found
    // the buffer full" and the compaction trigger.
    int round = 0, epoch = 0;
    bool ran_full = false;
    while (round < n_rounds) {
        // epochs of 1, 1, 2, 4 rounds, then 8 at a time: the threshold moves only between epochs, and while little
        // of the row has been seen it moves a lot (each doubling of what has been seen brings about top_k pushes)
        const int len = round < 2 ? 1 : (round < 4 ? 2 : (round < 8 ? 4 : kTopEpoch));
        const int r_end = round < n_main ? min(n_main, round + len) : n_rounds;
        if (round >= n_main) {
            do_round(fetch(round), round);
        } else {
            // all vectors of the epoch are requested before the first is used: with a handful of workgroups per CU
            // nothing else would hide the load latency
            u32x4 qv[kTopEpoch];
#pragma unroll
            for (int i = 0; i < kTopEpoch; ++i) qv[i] = (round + i < r_end) ? load_round(x_row, round + i) : u32x4{0u, 0u, 0u, 0u};
#pragma unroll
            for (int i = 0; i < kTopEpoch; ++i) {
                if (round + i < r_end) {
                    lx.note_vector(qv[i], (round + i) * kBlock + tid);
                    if (lx.defer_n >= 64) lx.drain();
                }
            }
        }
        if (r_end == n_rounds) lx.drain();  // the row's last epoch: nothing may be left waiting
        {
            const uint32_t mine = (uint32_t)lx.top.over | ((uint32_t)lx.top.full << 1);
            uint32_t *word = &epoch_flags[epoch % 3];  // (three words in turn, see the likelihood kernel)
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
                if (lx.top.compact(scratch, true)) lx.retarget();
            }
        }
        round = r_end;
    }
    if (ran_full) {
        // Careful mode (data in ascending order, for instance): the row again from its start, one wave and one round
        // at a time with a compaction check after each step, so that the buffer cannot run full (topn.hpp).
        lx.init(buf_x, &cnt_x, top_k, CAP);
        __syncthreads();
        for (int r = 0; r < n_rounds; ++r) {
            const u32x4 q = fetch(r);
            for (int w = 0; w < kWaves; ++w) {
                do_round(q, r, w);
                if (__syncthreads_or((int)lx.top.full)) {
                    if (lx.top.compact(scratch, true)) lx.retarget();
                }
            }
        }
    }
    lx.top.new_epoch();
    {
        const int64_t v = nvec * E + tid;  // ragged tail: V % E entries
        if (v < V) lx.push_entry(Elem<DT>::to_float(x_row[v]), (int32_t)v);
    }
    if (lx.bad) s_bad = 1;
    const int nk = lx.top.finish_sorted(scratch);  // buf_x[0 .. nk): the top_k logits in rank order
    const int kc = filter_prefix_length(buf_x, nk, (double)ri.T, top_p, scratch);
    ipt_filtered_finish<DT>(ri, row, V, buf_x, kc, s_bad != 0, o, kept_out, s_e, s_idx, lds_d, &s_tok);
}

int launch_ipt_filtered(const RowBatch &b, int top_k, float top_p, const IptOutputs &o, int32_t *kept, hipStream_t stream)
{
    const dim3 grid((unsigned)b.N), block(kBlock);
    const bool small = top_k <= kTopSmallN;
    if (b.dtype == 0) {
        if (small)
            ipt_filtered_kernel<0, kTopCapSmall><<<grid, block, 0, stream>>>(b, top_k, top_p, o, kept);
        else
            ipt_filtered_kernel<0, kTopCapBig><<<grid, block, 0, stream>>>(b, top_k, top_p, o, kept);
    } else {
        if (small)
            ipt_filtered_kernel<1, kTopCapSmall><<<grid, block, 0, stream>>>(b, top_k, top_p, o, kept);
        else
            ipt_filtered_kernel<1, kTopCapBig><<<grid, block, 0, stream>>>(b, top_k, top_p, o, kept);
    }
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

}  // namespace difr
