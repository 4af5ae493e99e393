// Token-DiFR row kernels: regenerate the seeded Gumbel noise over the whole vocabulary,
// rank by y_v = x_v / T + g_v, report the regenerated token (argmax) and the claimed
// token's margin  max_v y_v - y_t  (= -min_i A_{sigma,i} / T in the notation of the
// appendix algorithm of the Gumbel likelihood estimator; Sec. 6.3, Sec. 3.2).
//
// One workgroup (4 wavefronts) per token row; the row is streamed exactly once with
// 128-bit loads; noise is generated in registers, four vocabulary entries per Philox
// block; nothing of size V is ever stored.
#include "difr_device.hpp"
#include "difr_host.hpp"
#include "gumbel_stream.hpp"

namespace difr {

// Unfiltered kernel: every entry goes through both logarithms.  Any alignment.  The reference
// for the filtered kernel and the path for rows that are not 16-byte aligned.
template <int DT, bool ALIGNED>
__global__ __launch_bounds__(kBlock) void gumbel_score_kernel(RowBatch b, float *__restrict__ margin,
                                                              int32_t *__restrict__ argmax,
                                                              float *__restrict__ max_score,
                                                              float *__restrict__ claimed_score,
                                                              uint8_t *__restrict__ flags,
                                                              int32_t *__restrict__ logit_rank)
{
    typedef typename Elem<DT>::type elt_t;
    constexpr int E = Elem<DT>::kPerVec;
    __shared__ float lds_y[kWaves];
    __shared__ int32_t lds_i[kWaves];
    __shared__ int32_t lds_rank[kWaves];

    const int64_t row = blockIdx.x;
    const RowInfo ri = load_row_info(b, row);
    const int tid = threadIdx.x;
    const float nan = __builtin_nanf("");

    if (!ri.seq_ok || !ri.temp_ok) {  // uniform over the workgroup
        if (tid == 0) {
            margin[row] = nan;
            argmax[row] = -1;
            if (max_score) max_score[row] = nan;
            if (claimed_score) claimed_score[row] = nan;
            if (logit_rank) logit_rank[row] = -1;
            flags[row] = (uint8_t)(ri.seq_ok ? kFlagNonfinite : kFlagInvalidClaim);
        }
        return;
    }

    const elt_t *x_row = reinterpret_cast<const elt_t *>(b.logits) + row * b.ld;
    const int64_t V = b.V;
    const float inv_T = 1.0f / ri.T;
    const bool claim_ok = ri.claimed >= 0 && (int64_t)ri.claimed < V;
    const float xt = claim_ok ? Elem<DT>::to_float(x_row[ri.claimed]) : nan;

    float best_y = -__builtin_inff();
    int32_t best_v = 0x7FFFFFFF;
    uint32_t bad = 0;
    int32_t above = 0;  // entries whose raw logit exceeds the claimed token's

    for (int64_t base = (int64_t)tid * E; base < V; base += (int64_t)kBlock * E) {
        float x[E];
        load_elems<DT, ALIGNED>(x_row, base, V, x);
#pragma unroll
        for (int q = 0; q < E / 4; ++q) {
            uint32_t r[4];
            noise_block(ri.key, ri.pos, ri.seq, kStreamGumbel, (uint32_t)((base >> 2) + q), r);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float xv = x[4 * q + j];
                const float y = perturbed_score(xv, inv_T, r[j]);
                bad |= (uint32_t)!(xv < __builtin_inff());  // NaN or +inf
                above += (int32_t)(xv > xt);
                if (y > best_y) {
                    best_y = y;
                    best_v = (int32_t)(base + 4 * q + j);
                }
            }
        }
    }

    block_argmax(best_y, best_v, lds_y, lds_i);
    const int any_bad = __syncthreads_or((int)bad);
    above = block_sum_i32(above, lds_rank);

    if (tid == 0) {
        if (best_v == 0x7FFFFFFF) best_v = 0;  // every entry masked: all scores are -inf
        uint32_t f = any_bad ? kFlagNonfinite : 0u;
        float yt = nan, mg = nan;
        const int32_t t = ri.claimed;
        if (t >= 0 && (int64_t)t < V) {
            uint32_t r[4];
            noise_block(ri.key, ri.pos, ri.seq, kStreamGumbel, (uint32_t)t >> 2, r);
            const uint32_t rt = (t & 3) == 0 ? r[0] : (t & 3) == 1 ? r[1] : (t & 3) == 2 ? r[2] : r[3];
            yt = perturbed_score(Elem<DT>::to_float(x_row[t]), inv_T, rt);
            mg = best_y - yt;
            if (best_v == t) f |= kFlagMatch;
        } else {
            f |= kFlagInvalidClaim;
        }
        margin[row] = mg;
        argmax[row] = best_v;
        if (max_score) max_score[row] = best_y;
        if (claimed_score) claimed_score[row] = yt;
        if (logit_rank) logit_rank[row] = claim_ok ? above : -1;
        flags[row] = (uint8_t)f;
    }
}

// Filtered streaming kernel for 16-byte aligned rows (the filter is described in gumbel_stream.hpp).
template <int DT, bool RANK>
__global__ __launch_bounds__(kBlock) void gumbel_score_filtered_kernel(RowBatch b, GumbelOutputs o)
{
    typedef typename Elem<DT>::type elt_t;
    constexpr int E = Elem<DT>::kPerVec;
    __shared__ float lds_y[kWaves];
    __shared__ int32_t lds_i[kWaves];
    __shared__ float lds_L[kWaves];
    __shared__ int32_t lds_rank[kWaves];

    const int64_t row = blockIdx.x;
    const RowInfo ri = load_row_info(b, row);
    if (gumbel_row_rejected(ri, row, o)) return;
    const int tid = threadIdx.x;
    const elt_t *x_row = reinterpret_cast<const elt_t *>(b.logits) + row * b.ld;
    const int64_t V = b.V;

    GumbelStream<DT, RANK> g(ri, x_row, V, lds_L);
    __syncthreads();

    const int64_t nvec = V / E;               // full vectors; the last V % E entries are the tail
    const int n_main = (int)(nvec / kBlock);  // rounds in which every lane of every wave has a vector

    // Full rounds.  The loop body is instantiated once per gate mode; a change of mode (only
    // possible when the bound L moves) leaves the inner loop.
    int round = 0;
    auto run_rounds = [&](auto mode_tag) {
        constexpr int MODE = decltype(mode_tag)::value;
        // one round; returns false when the loop must be left (end reached, or the gate changed mode)
        auto body = [&](const u32x4 &q) {
            g.template process<MODE>(q, round, true);
            ++round;
            if ((round & 15) == 0) g.pickup();
            return round < n_main && g.gate.mode == MODE;
        };
        // one vector is kept in flight; two copies of the body, so that the vector being loaded and the one
        // being used swap roles instead of being copied from register to register every round
        u32x4 qa = load_round(x_row, round), qb = qa;
        while (true) {
            if (round + 1 < n_main) qb = load_round(x_row, round + 1);
            if (!body(qa)) break;
            if (round + 1 < n_main) qa = load_round(x_row, round + 1);
            if (!body(qb)) break;
        }
    };
    while (round < n_main) {
        if (g.gate.mode == 0)
            run_rounds(std::integral_constant<int, 0>());
        else if (g.gate.mode == 1)
            run_rounds(std::integral_constant<int, 1>());
        else
            run_rounds(std::integral_constant<int, 2>());
    }
    if ((int64_t)n_main * kBlock < nvec) {  // last, partly filled round of vectors
        const bool active = (int64_t)n_main * kBlock + tid < nvec;
        u32x4 q = u32x4{0u, 0u, 0u, 0u};
        if (active) q = load_round(x_row, n_main);
        g.process_any(q, n_main, active);
    }
    g.tail();
    g.finish(row, o, lds_y, lds_i, lds_rank);
}

// Size of the admissible set of each row (Sec. 7: A_t(tau) = tokens whose score passes the threshold; here
// the score is the margin, so A_t = { v : max_score - y_v <= delta }).  Second pass over the row with the
// row maximum known: the same exact pre-filter with the fixed bound M - delta, and a count instead of an
// argmax.  Any alignment is accepted; unaligned rows evaluate every entry.
template <int DT, bool ALIGNED>
__global__ __launch_bounds__(kBlock) void admissible_count_kernel(RowBatch b, const float *__restrict__ max_score,
                                                                  float delta, int32_t *__restrict__ count,
                                                                  float *__restrict__ log2_count)
{
    typedef typename Elem<DT>::type elt_t;
    constexpr int E = Elem<DT>::kPerVec;
    __shared__ float lds_L[kWaves];
    __shared__ int32_t lds_c[kWaves];
    const int64_t row = blockIdx.x;
    RowInfo ri = load_row_info(b, row);
    ri.claimed = -1;
    const int tid = threadIdx.x;
    const float M = max_score[row];
    const float nan = __builtin_nanf("");
    if (!ri.seq_ok || !ri.temp_ok || !(M == M) || !(fabsf(M) < __builtin_inff())) {  // uniform over the workgroup
        if (tid == 0) {
            count[row] = 0;
            if (log2_count) log2_count[row] = nan;
        }
        return;
    }
    const elt_t *x_row = reinterpret_cast<const elt_t *>(b.logits) + row * b.ld;
    const int64_t V = b.V;
    int32_t c = 0;
    if (ALIGNED) {
        GumbelStream<DT, false, true> g(ri, x_row, V, lds_L);
        __syncthreads();
        g.arm_count(M, delta);
        __syncthreads();
        const int64_t nvec = V / E;
        const int n_main = (int)(nvec / kBlock);
        int round = 0;
        auto run_rounds = [&](auto mode_tag) {  // the bound never moves, so neither does the gate mode
            constexpr int MODE = decltype(mode_tag)::value;
            u32x4 q_next = load_round(x_row, round);
            while (round < n_main) {
                const u32x4 q = q_next;
                if (round + 1 < n_main) q_next = load_round(x_row, round + 1);
                g.template process<MODE>(q, round, true);
                ++round;
            }
        };
        if (n_main > 0) {
            if (g.gate.mode == 0)
                run_rounds(std::integral_constant<int, 0>());
            else if (g.gate.mode == 1)
                run_rounds(std::integral_constant<int, 1>());
            else
                run_rounds(std::integral_constant<int, 2>());
        }
        if ((int64_t)n_main * kBlock < nvec) {
            const bool active = (int64_t)n_main * kBlock + tid < nvec;
            u32x4 q = u32x4{0u, 0u, 0u, 0u};
            if (active) q = load_round(x_row, n_main);
            g.process_any(q, n_main, active);
        }
        g.tail();
        c = (int32_t)g.count;
    } else {
        const float inv_T = 1.0f / ri.T;
        for (int64_t base = (int64_t)tid * E; base < V; base += (int64_t)kBlock * E) {
            float x[E];
            load_elems<DT, false>(x_row, base, V, x);
#pragma unroll
            for (int q = 0; q < E / 4; ++q) {
                uint32_t r[4];
                noise_block(ri.key, ri.pos, ri.seq, kStreamGumbel, (uint32_t)((base >> 2) + q), r);
#pragma unroll
                for (int j = 0; j < 4; ++j) c += (int32_t)(M - perturbed_score(x[4 * q + j], inv_T, r[j]) <= delta);
            }
        }
    }
    c = block_sum_i32(c, lds_c);
    if (tid == 0) {
        count[row] = c;
        if (log2_count) log2_count[row] = c > 0 ? __log2f((float)c) : nan;
    }
}

// Raw noise words of one row, through the same device code as the scoring kernels.
__global__ __launch_bounds__(kBlock) void debug_noise_kernel(RowBatch b, int64_t row, uint32_t stream,
                                                             uint32_t *__restrict__ bits)
{
    const RowInfo ri = load_row_info(b, row);
    const int64_t nq = (b.V + 3) >> 2;
    for (int64_t q = (int64_t)blockIdx.x * kBlock + threadIdx.x; q < nq; q += (int64_t)gridDim.x * kBlock) {
        uint32_t r[4];
        noise_block(ri.key, ri.pos, ri.seq, stream, (uint32_t)q, r);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (4 * q + j < b.V) bits[4 * q + j] = r[j];
    }
}

__global__ __launch_bounds__(kBlock) void debug_gumbel_map_kernel(const uint32_t *__restrict__ bits, int64_t n,
                                                                  float *__restrict__ g)
{
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (int64_t)gridDim.x * kBlock)
        g[i] = gumbel_from_bits(bits[i]);
}

int launch_gumbel_score(const RowBatch &b, bool aligned, bool filtered, float *margin, int32_t *argmax,
                        float *max_score, float *claimed_score, uint8_t *flags, int32_t *logit_rank,
                        hipStream_t stream)
{
    const dim3 grid((unsigned)b.N), block(kBlock);
    const GumbelOutputs o{margin, argmax, max_score, claimed_score, flags, logit_rank};
#define DIFR_ARGS b, margin, argmax, max_score, claimed_score, flags, logit_rank
    if (aligned && filtered) {
        if (b.dtype == 0) {
            if (logit_rank)
                gumbel_score_filtered_kernel<0, true><<<grid, block, 0, stream>>>(b, o);
            else
                gumbel_score_filtered_kernel<0, false><<<grid, block, 0, stream>>>(b, o);
        } else {
            if (logit_rank)
                gumbel_score_filtered_kernel<1, true><<<grid, block, 0, stream>>>(b, o);
            else
                gumbel_score_filtered_kernel<1, false><<<grid, block, 0, stream>>>(b, o);
        }
    } else if (b.dtype == 0) {
        if (aligned)
            gumbel_score_kernel<0, true><<<grid, block, 0, stream>>>(DIFR_ARGS);
        else
            gumbel_score_kernel<0, false><<<grid, block, 0, stream>>>(DIFR_ARGS);
    } else {
        if (aligned)
            gumbel_score_kernel<1, true><<<grid, block, 0, stream>>>(DIFR_ARGS);
        else
            gumbel_score_kernel<1, false><<<grid, block, 0, stream>>>(DIFR_ARGS);
    }
#undef DIFR_ARGS
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

int launch_admissible_count(const RowBatch &b, bool aligned, const float *max_score, float delta, int32_t *count,
                            float *log2_count, hipStream_t stream)
{
    const dim3 grid((unsigned)b.N), block(kBlock);
    if (b.dtype == 0) {
        if (aligned)
            admissible_count_kernel<0, true><<<grid, block, 0, stream>>>(b, max_score, delta, count, log2_count);
        else
            admissible_count_kernel<0, false><<<grid, block, 0, stream>>>(b, max_score, delta, count, log2_count);
    } else {
        if (aligned)
            admissible_count_kernel<1, true><<<grid, block, 0, stream>>>(b, max_score, delta, count, log2_count);
        else
            admissible_count_kernel<1, false><<<grid, block, 0, stream>>>(b, max_score, delta, count, log2_count);
    }
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

int launch_debug_noise(const RowBatch &b, int64_t row, uint32_t stream_id, uint32_t *bits, hipStream_t stream)
{
    const int64_t nq = (b.V + 3) >> 2;
    int64_t blocks = (nq + kBlock - 1) / kBlock;
    if (blocks > 4096) blocks = 4096;
    debug_noise_kernel<<<dim3((unsigned)blocks), dim3(kBlock), 0, stream>>>(b, row, stream_id, bits);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

int launch_debug_gumbel_map(const uint32_t *bits, int64_t n, float *g, hipStream_t stream)
{
    int64_t blocks = (n + kBlock - 1) / kBlock;
    if (blocks > 8192) blocks = 8192;
    debug_gumbel_map_kernel<<<dim3((unsigned)blocks), dim3(kBlock), 0, stream>>>(bits, n, g);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

}  // namespace difr
