// Token-DiFR row kernel: regenerate the seeded Gumbel noise over the whole vocabulary,
// rank by y_v = x_v / T + g_v, report the regenerated token (argmax) and the claimed
// token's margin  max_v y_v - y_t  (= -min_i A_{sigma,i} / T in the notation of the
// appendix algorithm of the Gumbel likelihood estimator; Sec. 6.3, Sec. 3.2).
//
// One workgroup (4 wavefronts) per token row; the row is streamed exactly once with
// 128-bit loads; noise is generated in registers, four vocabulary entries per Philox
// block; nothing of size V is ever stored.
#include <type_traits>

#include "difr_device.hpp"
#include "difr_host.hpp"

namespace difr {

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

// ---------------------------------------------------------------------------------
// Filtered streaming kernel (aligned rows only).
//
// The row maximum is bounded from below by L: the claimed token's own score at first
// (for an honest claim that IS the maximum), then the best score seen so far.  An entry
// can only matter if y_v = x_v / T + g_v >= L.  Cheap tests per 16-byte vector, none of
// which needs a logarithm, rule that out for almost every entry.  With two noise levels
// G_lo < G_hi (top 8 / top 13 bits of the word all ones) and the Gumbel bounds
// g < g_lo for r < G_lo, g < g_hi for r < G_hi:
//   A  some word r >= G_hi                                   (very large noise)
//   B  some logit x >= T (L - g_lo - slack)                  (very heavy logit)
//   C  some word r >= G_lo  and  some logit x >= T (L - g_hi - slack)   (both moderate)
// An entry of a vector that trips none of A, B, C has y_v < L.  A uses the maximum of the
// eight words; B and C use packed 16-bit min / max of the raw bf16 bit patterns (for a
// cap <= 0, "x >= cap" is "bits <= bits(cap)" as unsigned 16-bit; for a cap > 0 it is
// "bits >= bits(cap)" as signed 16-bit).  Entries of a vector that trips a test get a
// per-entry bound g_v <= (151 - bits(float(q_v)) 2^-23) ln 2, q_v = (~r_v) >> 8  (from
// -ln(-ln(1-w)) <= -ln w and log2(1+m) >= m), and only those whose bound still reaches L
// are evaluated exactly, with the same arithmetic as the unfiltered kernel.  Every noise
// word is still generated; the outputs are identical to the unfiltered kernel's, bit for
// bit, because L never exceeds the true maximum.
// ---------------------------------------------------------------------------------
constexpr int kGateLoBits = 8, kGateHiBits = 13;  // best pair of a sweep on the Zipf-profile workload
constexpr uint32_t kGateLo = 0xFFFFFFFFu << (32 - kGateLoBits);  // r >= kGateLo: top 8 bits are ones
constexpr uint32_t kGateHi = 0xFFFFFFFFu << (32 - kGateHiBits);  // r >= kGateHi: top 13 bits are ones
// sup of g over r < gate, -ln(-ln(1 - (2^(24-bits)+1) 2^-24)), rounded up: 8 bits 5.543206, 13 bits 9.010365
constexpr float kGumbelLo = 5.5433f, kGumbelHi = 9.0104f;

typedef uint16_t u16x2 __attribute__((ext_vector_type(2)));
typedef int16_t i16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ u16x2 as_u16x2(uint32_t w) { return __builtin_bit_cast(u16x2, w); }
__device__ __forceinline__ i16x2 as_i16x2(uint32_t w) { return __builtin_bit_cast(i16x2, w); }

// Upper bound on the Gumbel variate of noise word r (see the comment above); error of the
// float conversions is below 1e-5 and is covered by the caller's slack.
__device__ __forceinline__ float gumbel_upper_bound(uint32_t r)
{
    const float f = (float)((~r) >> 8);
    const float bits = (float)__float_as_int(f);
    return __fmaf_rn(bits, -kLn2 * 0x1p-23f, 151.0f * kLn2);
}

// bf16 bit pattern of a logit cap, rounded so that the 16-bit test never misses an entry:
// cap <= 0: sign bit forced (+0 counts as -0) and magnitude rounded up; cap > 0: truncated.
__device__ __forceinline__ uint32_t cap_bits(float cap, bool neg)
{
    const uint32_t b = __float_as_uint(cap);
    uint32_t c = b >> 16;
    if (neg) {
        c |= 0x8000u;
        if ((b & 0xFFFFu) != 0u && c < 0xFF80u) c += 1u;
    }
    return c;
}

struct Gate {
    float L;          // lower bound on the row maximum (wave-uniform)
    float Lgate;      // L minus slack: an entry whose upper bound is below this cannot reach L
    float xcap_hi;    // test B: T (L - g_lo - slack), in logit units
    float xcap_lo;    // test C: T (L - g_hi - slack)
    uint32_t cap16_hi, cap16_lo;  // their bf16 bit patterns
    int mode;         // 0: both caps <= 0 (unsigned min test); 1: both > 0 (signed max test); 2: hi > 0 >= lo
};

__device__ __forceinline__ Gate make_gate(float L, float T)
{
    Gate g;
    L = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, L)));
    const float slack = 0.01f + 1e-5f * fabsf(L);
    g.L = L;
    g.Lgate = L - slack;
    float hi = (L - kGumbelLo - slack) * T, lo = (L - kGumbelHi - slack) * T;
    if (!(hi == hi)) hi = -__builtin_inff();  // L = +-inf arithmetic: gate everything in
    if (!(lo == lo)) lo = -__builtin_inff();
    g.xcap_hi = hi;
    g.xcap_lo = lo;
    const bool hi_neg = !(hi > 0.0f), lo_neg = !(lo > 0.0f);
    g.cap16_hi = cap_bits(hi, hi_neg);
    g.cap16_lo = cap_bits(lo, lo_neg);
    g.mode = hi_neg ? 0 : (lo_neg ? 2 : 1);
    return g;
}

// RANK: also count the entries whose raw logit exceeds the claimed token's (logit rank, Sec. 7.1).
// For bf16 the count works on the raw bit patterns, two per dword, without unpacking: for a claimed
// logit >= +0 "x > x_t" is "bits > bits(x_t)" as signed 16-bit, for a negative one it is
// "bits < bits(x_t)" as unsigned 16-bit (a claimed -0 is treated as +0).
template <int DT, bool RANK>
__global__ __launch_bounds__(kBlock) void gumbel_score_filtered_kernel(RowBatch b, float *__restrict__ margin,
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
    __shared__ float lds_L[kWaves];
    __shared__ int32_t lds_rank[kWaves];

    const int64_t row = blockIdx.x;
    const RowInfo ri = load_row_info(b, row);
    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const float nan = __builtin_nanf("");
    const float ninf = -__builtin_inff();

    if (!ri.seq_ok || !ri.temp_ok) {  // uniform over the workgroup
        if (tid == 0) {
            margin[row] = nan;
            argmax[row] = -1;
            if (max_score) max_score[row] = nan;
            if (claimed_score) claimed_score[row] = nan;
            if (RANK) logit_rank[row] = -1;
            flags[row] = (uint8_t)(ri.seq_ok ? kFlagNonfinite : kFlagInvalidClaim);
        }
        return;
    }

    const elt_t *x_row = reinterpret_cast<const elt_t *>(b.logits) + row * b.ld;
    const int64_t V = b.V;
    const float T = ri.T;
    const float inv_T = 1.0f / T;

    // The claimed token's score, by the same function the stream uses: the first lower bound.
    const int32_t t = ri.claimed;
    const bool valid = (t >= 0 && (int64_t)t < V);
    float yt = nan, xt = nan;
    if (valid) {
        uint32_t r[4];
        noise_block(ri.key, ri.pos, ri.seq, kStreamGumbel, (uint32_t)t >> 2, r);
        const uint32_t rt = (t & 3) == 0 ? r[0] : (t & 3) == 1 ? r[1] : (t & 3) == 2 ? r[2] : r[3];
        xt = Elem<DT>::to_float(x_row[t]);
        yt = perturbed_score(xt, inv_T, rt);
    }
    // logit rank: wave-uniform count of entries above the claimed logit
    uint32_t above = 0;
    const uint32_t xt_bits = (xt == 0.0f) ? 0u : __float_as_uint(xt);  // -0 counts as +0
    const bool xt_pos = (xt_bits >> 31) == 0u;
    const uint32_t xt16 = xt_bits >> 16;
    auto count_above = [&](u32x4 q, bool active) {
        const uint32_t qw[4] = {q.x, q.y, q.z, q.w};
        uint32_t n = 0;
        if (DT == 0) {
            if (xt_pos) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    n += __builtin_popcountll(__builtin_amdgcn_ballot_w64(active && (int16_t)(qw[j] & 0xFFFFu) > (int16_t)xt16));
                    n += __builtin_popcountll(__builtin_amdgcn_ballot_w64(active && (int16_t)(qw[j] >> 16) > (int16_t)xt16));
                }
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    n += __builtin_popcountll(__builtin_amdgcn_ballot_w64(active && (uint16_t)(qw[j] & 0xFFFFu) < (uint16_t)xt16));
                    n += __builtin_popcountll(__builtin_amdgcn_ballot_w64(active && (uint16_t)(qw[j] >> 16) < (uint16_t)xt16));
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                n += __builtin_popcountll(__builtin_amdgcn_ballot_w64(active && __uint_as_float(qw[j]) > xt));
        }
        above += n;
    };
    Gate gate = make_gate((yt == yt) ? yt : ninf, T);
    if ((tid & 63) == 0) lds_L[wave] = gate.L;

    float best_y = ninf;
    int32_t best_v = 0x7FFFFFFF;
    uint32_t bad = 0;

    // Exact evaluation of one entry (same arithmetic as the unfiltered kernel), ties to the lowest index.
    auto evaluate = [&](float xv, uint32_t rv, int32_t v) {
        const float y = perturbed_score(xv, inv_T, rv);
        bad |= (uint32_t)!(xv < __builtin_inff());
        if (y > best_y || (y == best_y && v < best_v)) {
            best_y = y;
            best_v = v;
        }
    };
    // Entry-level test: can this entry still reach the lower bound?
    auto consider = [&](float xv, uint32_t rv, int32_t v) {
        if (!(__fmaf_rn(xv, inv_T, gumbel_upper_bound(rv)) < gate.Lgate)) evaluate(xv, rv, v);
    };

    const int64_t nvec = V / E;                 // full vectors; the last V % E entries are the tail
    const int n_main = (int)(nvec / kBlock);    // rounds in which every lane of every wave has a vector
    __syncthreads();

    // One 16-byte vector per lane.  `round` is the vector round (vector index = round * 256 + tid).
    // M0 * (Philox counter word 0) = M0 * (round's first block) + M0 * (lane's block offset): the
    // second term never changes, the first is scalar, and the sum cannot wrap (counter < 2^29).
    uint64_t lane_prod = (uint64_t)kPhiloxM0 * (uint32_t)(tid * (E / 4));
    asm volatile("" : "+v"(lane_prod));  // keep it a loop-invariant register pair
    auto process = [&](auto mode_tag, u32x4 q, int round, bool active) {
        constexpr int MODE = decltype(mode_tag)::value;  // the gate's mode, fixed for this instantiation
        const uint64_t round_prod = (uint64_t)kPhiloxM0 * (uint32_t)(round * kBlock * (E / 4));
        const uint64_t p0 = round_prod + lane_prod;
        uint32_t r[E];
        philox4x32_10_from_product(p0, ri.pos, ri.seq, kStreamGumbel, ri.key, r);
        if (E == 8) philox4x32_10_from_product(p0 + kPhiloxM0, ri.pos, ri.seq, kStreamGumbel, ri.key, r + 4);
        // the largest of the words, for tests A and C
        uint32_t rmax = r[0];
#pragma unroll
        for (int j = 1; j < E; ++j) rmax = max(rmax, r[j]);
        // wave-wide masks of the lanes whose vector trips A, B, or both halves of C
        const uint64_t amask = __builtin_amdgcn_ballot_w64(active && rmax >= kGateHi);
        const uint64_t cnmask = __builtin_amdgcn_ballot_w64(active && rmax >= kGateLo);
        uint64_t bmask, cxmask;
        if (DT == 0) {
            uint16_t lo = 0, hi = 0;
            if (MODE != 1) {  // smallest bit pattern as unsigned: the largest logit if it is <= 0 ...
                u16x2 m = __builtin_elementwise_min(as_u16x2(q.x), as_u16x2(q.y));
                m = __builtin_elementwise_min(m, as_u16x2(q.z));
                m = __builtin_elementwise_min(m, as_u16x2(q.w));
                lo = m.x < m.y ? m.x : m.y;
            }
            if (MODE != 0) {  // ... largest bit pattern as signed: the largest logit if it is > 0
                i16x2 m = __builtin_elementwise_max(as_i16x2(q.x), as_i16x2(q.y));
                m = __builtin_elementwise_max(m, as_i16x2(q.z));
                m = __builtin_elementwise_max(m, as_i16x2(q.w));
                hi = (uint16_t)(m.x > m.y ? m.x : m.y);
            }
            const bool b_hit = MODE == 0 ? lo <= (uint16_t)gate.cap16_hi : (int16_t)hi >= (int16_t)gate.cap16_hi;
            const bool c_hit = MODE == 1 ? (int16_t)hi >= (int16_t)gate.cap16_lo : lo <= (uint16_t)gate.cap16_lo;
            bmask = __builtin_amdgcn_ballot_w64(active && b_hit);
            cxmask = __builtin_amdgcn_ballot_w64(active && c_hit);
        } else {  // fp32 logits: plain compares (a NaN counts as gated in)
            const float x0 = __uint_as_float(q.x), x1 = __uint_as_float(q.y), x2 = __uint_as_float(q.z),
                        x3 = __uint_as_float(q.w);
            bmask = __builtin_amdgcn_ballot_w64(active && (!(x0 < gate.xcap_hi) || !(x1 < gate.xcap_hi) ||
                                                           !(x2 < gate.xcap_hi) || !(x3 < gate.xcap_hi)));
            cxmask = __builtin_amdgcn_ballot_w64(active && (!(x0 < gate.xcap_lo) || !(x1 < gate.xcap_lo) ||
                                                            !(x2 < gate.xcap_lo) || !(x3 < gate.xcap_lo)));
        }
        const uint64_t hitmask = amask | bmask | (cnmask & cxmask);
        if (RANK) count_above(q, active);
        if (__builtin_expect(hitmask != 0ull, 0)) {
            if ((hitmask >> (tid & 63)) & 1ull) {
                // Entries that could matter are those with moderate noise or a moderate logit; each of
                // them is then tested against its own noise bound before anything exact is computed.
                const int32_t v0 = (round * kBlock + tid) * E;
                const uint32_t qw[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
                for (int j = 0; j < E; ++j) {
                    const uint32_t w = qw[DT == 0 ? j >> 1 : j];
                    const float xv = DT == 0 ? __uint_as_float((j & 1) ? (w & 0xFFFF0000u) : (w << 16))
                                             : __uint_as_float(w);
                    if (r[j] >= kGateLo || !(xv < gate.xcap_lo)) consider(xv, r[j], v0 + j);
                }
            }
            // a better score raises the lower bound for this wave; other waves pick it up from LDS
            if (__builtin_amdgcn_ballot_w64(best_y > gate.L) != 0ull) {
                float L = fmaxf(wave_max(best_y), gate.L);
                L = fmaxf(fmaxf(L, lds_L[0]), fmaxf(lds_L[1], fmaxf(lds_L[2], lds_L[3])));
                gate = make_gate(L, T);
                if ((tid & 63) == 0) lds_L[wave] = gate.L;
            }
        }
    };

    const char *row_bytes = reinterpret_cast<const char *>(x_row);
    const uint32_t lane_off = (uint32_t)tid * 16u;
    auto load_round = [&](int round) {
        return __builtin_nontemporal_load(
            reinterpret_cast<const u32x4 *>(row_bytes + (size_t)round * (kBlock * 16) + lane_off));
    };

    // Full rounds.  The loop body is instantiated once per gate mode so that it carries no mode
    // branches; a change of mode (only possible when the bound L moves) leaves the inner loop.
    int round = 0;
    auto run_rounds = [&](auto mode_tag) {
        constexpr int MODE = decltype(mode_tag)::value;
        u32x4 q_next = load_round(round);
        while (round < n_main) {
            const u32x4 q = q_next;
            if (round + 1 < n_main) q_next = load_round(round + 1);  // keep one vector in flight
            process(mode_tag, q, round, true);
            ++round;
            if ((round & 15) == 0) {  // pick up a bound another wave has raised
                const float L = fmaxf(fmaxf(lds_L[0], lds_L[1]), fmaxf(lds_L[2], lds_L[3]));
                if (L > gate.L) gate = make_gate(L, T);
            }
            if (gate.mode != MODE) break;
        }
    };
    while (round < n_main) {
        if (gate.mode == 0)
            run_rounds(std::integral_constant<int, 0>());
        else if (gate.mode == 1)
            run_rounds(std::integral_constant<int, 1>());
        else
            run_rounds(std::integral_constant<int, 2>());
    }
    if ((int64_t)n_main * kBlock < nvec) {  // last, partly filled round of vectors
        const bool active = (int64_t)n_main * kBlock + tid < nvec;
        u32x4 q;
        if (active) {
            q = load_round(n_main);
        } else {  // a lane without a vector: -inf entries and no noise
            const uint32_t pad = DT == 0 ? 0xFF80FF80u : 0xFF800000u;
            q = u32x4{pad, pad, pad, pad};
        }
        if (gate.mode == 0)
            process(std::integral_constant<int, 0>(), q, n_main, active);
        else if (gate.mode == 1)
            process(std::integral_constant<int, 1>(), q, n_main, active);
        else
            process(std::integral_constant<int, 2>(), q, n_main, active);
    }
    // the ragged tail: V % E entries, one lane each, evaluated exactly
    {
        const int64_t v = nvec * E + tid;
        if (v < V) {
            uint32_t r[4];
            noise_block(ri.key, ri.pos, ri.seq, kStreamGumbel, (uint32_t)(v >> 2), r);
            const uint32_t rv = (v & 3) == 0 ? r[0] : (v & 3) == 1 ? r[1] : (v & 3) == 2 ? r[2] : r[3];
            evaluate(Elem<DT>::to_float(x_row[v]), rv, (int32_t)v);
        }
        if (RANK) above += __builtin_popcountll(__builtin_amdgcn_ballot_w64(v < V && Elem<DT>::to_float(x_row[v < V ? v : 0]) > xt));
    }

    block_argmax(best_y, best_v, lds_y, lds_i);
    if (RANK && (tid & 63) == 0) lds_rank[wave] = (int32_t)above;
    const int any_bad = __syncthreads_or((int)bad);

    if (tid == 0) {
        if (RANK) logit_rank[row] = valid ? lds_rank[0] + lds_rank[1] + lds_rank[2] + lds_rank[3] : -1;
        if (best_v == 0x7FFFFFFF) best_v = 0;  // every entry masked: all scores are -inf
        uint32_t f = any_bad ? kFlagNonfinite : 0u;
        float mg = nan;
        if (valid) {
            mg = best_y - yt;
            if (best_v == t) f |= kFlagMatch;
        } else {
            f |= kFlagInvalidClaim;
        }
        margin[row] = mg;
        argmax[row] = best_v;
        if (max_score) max_score[row] = best_y;
        if (claimed_score) claimed_score[row] = yt;
        flags[row] = (uint8_t)f;
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
#define DIFR_ARGS b, margin, argmax, max_score, claimed_score, flags, logit_rank
    if (aligned && filtered) {
        if (b.dtype == 0) {
            if (logit_rank)
                gumbel_score_filtered_kernel<0, true><<<grid, block, 0, stream>>>(DIFR_ARGS);
            else
                gumbel_score_filtered_kernel<0, false><<<grid, block, 0, stream>>>(DIFR_ARGS);
        } else {
            if (logit_rank)
                gumbel_score_filtered_kernel<1, true><<<grid, block, 0, stream>>>(DIFR_ARGS);
            else
                gumbel_score_filtered_kernel<1, false><<<grid, block, 0, stream>>>(DIFR_ARGS);
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
