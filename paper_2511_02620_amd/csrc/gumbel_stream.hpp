// Row-streaming state of the filtered Token-DiFR kernel (Sec. 6.3; appendix algorithm of the Gumbel
// likelihood estimator: noise regeneration, ranking by l_i + T G_i, A_{sigma,i}), kept as a struct
// so that the Gumbel-only kernel and the kernel that scores both estimators in one pass share it.
#pragma once

#include <type_traits>

#include "difr_device.hpp"
#include "topn.hpp"

namespace difr {

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
// sup of g over all words: -ln(-ln(1 - 2^-24)) = 24 ln 2 - O(2^-25), rounded up (PEAKED streams, see GumbelStream)
constexpr float kGumbelMax = 16.6356f;

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

// `reach`: how far below L a score may lie and still matter (0 for the argmax; delta when the entries within
// delta of the row maximum are wanted as well).  All tests are made against L - reach.
__device__ __forceinline__ Gate make_gate(float L, float T, float reach = 0.0f)
{
    Gate g;
    L = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, L)));
    const float Lr = L - reach;
    const float slack = 0.01f + 1e-5f * fabsf(Lr);
    g.L = L;
    g.Lgate = Lr - slack;
    float hi = (Lr - kGumbelLo - slack) * T, lo = (Lr - kGumbelHi - slack) * T;
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

struct GumbelOutputs {
    float *margin;
    int32_t *argmax;
    float *max_score;
    float *claimed_score;
    uint8_t *flags;
    int32_t *logit_rank;
};

// Rows whose sequence id or temperature is unusable get NaN scores and a flag; uniform per workgroup.
__device__ __forceinline__ bool gumbel_row_rejected(const RowInfo &ri, int64_t row, const GumbelOutputs &o)
{
    if (ri.seq_ok && ri.temp_ok) return false;
    if (threadIdx.x == 0) {
        const float nan = __builtin_nanf("");
        o.margin[row] = nan;
        o.argmax[row] = -1;
        if (o.max_score) o.max_score[row] = nan;
        if (o.claimed_score) o.claimed_score[row] = nan;
        if (o.logit_rank) o.logit_rank[row] = -1;
        o.flags[row] = (uint8_t)(ri.seq_ok ? kFlagNonfinite : kFlagInvalidClaim);
    }
    return true;
}

// RANK: also count the entries whose raw logit exceeds the claimed token's (logit rank, Sec. 7.1).
// For bf16 the count works on the raw bit patterns, two per dword, without unpacking: for a claimed
// logit >= +0 "x > x_t" is "bits > bits(x_t)" as signed 16-bit, for a negative one it is
// "bits < bits(x_t)" as unsigned 16-bit (a claimed -0 is treated as +0).
//
// COUNT: instead of tracking the best score, count the entries whose score is within `delta` of a
// maximum that is already known (the admissible set of Sec. 7: tokens the verifier would accept).
// The same gates apply with the fixed bound M - delta; nothing ever raises it.
//
// TOPN: instead of tracking the best score, push every score that may belong to the n largest of the
// row (the claimed token left out) into a TopN buffer; the gates use the buffer's threshold as the bound.
// That bound lies well below the row maximum (the n-th best score, not the best), so a wave meets a vector
// that trips a test in about every second round - in one or two of its 64 lanes.  Looking at those entries
// on the spot would make the whole wave walk the per-entry code for them.  Instead the lane only notes the
// vector's number in a per-wave LDS queue; once 64 are waiting (and at the end of every epoch of the caller)
// the wave drains the queue with one vector per lane: the vector is read again, its noise is generated again,
// and the per-entry tests run with all lanes busy.  Which entries end up in the selection does not depend on
// when they are pushed, so the result is the same.
//
// ADM: the argmax as usual and, in the same pass, the size of the admissible set { v : max y - y_v <= delta }
// although the maximum is only known at the end.  The gates test against L - delta instead of L (L = the
// running lower bound of the maximum), every score evaluated that may lie within delta of the final maximum
// is kept in a per-wave LDS list, and the list is counted against the true maximum after the row.  Since
// L <= max y at all times, nothing within delta of the maximum is ever skipped or dropped.  A wave prunes
// its own list against its current L - delta whenever it is half full (wave-synchronous, no barrier); if
// pruning cannot get it below half, the row is reported as undetermined (count -1) rather than risk a miss.
//
// PEAKED: one more test, in FRONT of the noise generation: no noise word lifts an entry by more than g_max, so a
// wave none of whose logits reaches T (L - g_max) skips the round without running Philox at all.  On rows much more
// concentrated than a Zipf profile (a confident model's) most rounds go that way and the stream runs at the speed
// of reading them; on flat rows the test never fires and costs a few per cent (the noise generation can no longer
// start before the vector has arrived), which is why it is a variant the caller asks for.  Same outputs, bit for bit.
constexpr int kAdmCap = 1024;  // list entries per wave
constexpr int kDeferCap = 128; // TOPN streams: queue slots per wave (fewer than 64 waiting + at most 64 new ones)

template <int DT, bool RANK, bool COUNT = false, bool TOPN = false, bool ADM = false, bool PEAKED = false>
struct GumbelStream {
    static_assert(!PEAKED || (!COUNT && !TOPN && !ADM), "the early test is kept up to date for the plain argmax stream only");
    typedef typename Elem<DT>::type elt_t;
    static constexpr int E = Elem<DT>::kPerVec;

    // row constants
    const RowInfo &ri;
    const elt_t *x_row;
    int64_t V;
    float T, inv_T;
    int tid, wave;
    float *lds_L;  // kWaves floats: each wave publishes its lower bound here
    int32_t t;
    bool valid;
    float yt, xt;
    uint32_t xt16;
    bool xt_pos;
    uint64_t lane_prod;
    // running state
    Gate gate;
    float best_y;
    int32_t best_v;
    uint32_t bad, above;
    // COUNT mode
    float count_M, count_delta;
    uint32_t count;
    // ADM mode
    float adm_delta;    // 0 in every other mode
    float *adm_list;    // this wave's kAdmCap floats in LDS
    int32_t *adm_fill;  // this wave's fill counter in LDS
    uint32_t adm_over;  // the list could not be kept below half: the count is not to be trusted
    // TOPN mode: this wave's queue of vectors waiting for the per-entry look, and how many wait (wave-uniform)
    int32_t *defer_q;
    int defer_n;
    uint32_t seen_lo, seen_hi;  // the last vector's extreme bf16 patterns, as far as process<MODE>() formed them
    // PEAKED streams: T (L - g_max - slack), no entry below it can reach L whatever its noise; its bf16 pattern;
    // whether it is <= 0 (always so in gate modes 0 and 2).  Follows the gate: peak_cap() after every change of it.
    float xcap_max;
    uint32_t cap16_max;
    bool max_neg;

    // Computes the claimed token's score with the same function the stream uses (the first lower
    // bound) and publishes it.  The caller must __syncthreads() before the first process().
    __device__ __forceinline__ GumbelStream(const RowInfo &ri_, const elt_t *x_row_, int64_t V_, float *lds_L_)
        : ri(ri_), x_row(x_row_), V(V_), T(ri_.T), inv_T(1.0f / ri_.T), tid((int)threadIdx.x),
          wave((int)threadIdx.x >> 6), lds_L(lds_L_), t(ri_.claimed)
    {
        const float nan = __builtin_nanf("");
        valid = (t >= 0 && (int64_t)t < V);
        yt = nan;
        xt = nan;
        if (valid) {
            uint32_t r[4];
            noise_block(ri.key, ri.pos, ri.seq, kStreamGumbel, (uint32_t)t >> 2, r);
            const uint32_t rt = (t & 3) == 0 ? r[0] : (t & 3) == 1 ? r[1] : (t & 3) == 2 ? r[2] : r[3];
            xt = Elem<DT>::to_float(x_row[t]);
            yt = perturbed_score(xt, inv_T, rt);
        }
        const uint32_t xt_bits = (xt == 0.0f) ? 0u : __float_as_uint(xt);  // -0 counts as +0
        xt_pos = (xt_bits >> 31) == 0u;
        xt16 = xt_bits >> 16;
        above = 0;
        gate = make_gate((yt == yt) ? yt : -__builtin_inff(), T);
        if ((tid & 63) == 0) lds_L[wave] = gate.L;
        best_y = -__builtin_inff();
        best_v = 0x7FFFFFFF;
        bad = 0;
        // M0 * (Philox counter word 0) = M0 * (round's first block) + M0 * (lane's block offset): the
        // second term never changes, the first is scalar, and the sum cannot wrap (counter < 2^29).
        lane_prod = (uint64_t)kPhiloxM0 * (uint32_t)(tid * (E / 4));
        asm volatile("" : "+v"(lane_prod));  // keep it a loop-invariant register pair
        count_M = count_delta = 0.0f;
        count = 0;
        adm_delta = 0.0f;
        adm_list = nullptr;
        adm_fill = nullptr;
        adm_over = 0;
        defer_q = nullptr;
        defer_n = 0;
        seen_lo = seen_hi = 0u;
        if (PEAKED) peak_cap();
    }

    __device__ __forceinline__ void peak_cap()
    {
        const float Lr = gate.L - adm_delta;
        const float slack = 0.01f + 1e-5f * fabsf(Lr);
        float mx = (Lr - kGumbelMax - slack) * T;
        if (!(mx == mx)) mx = -__builtin_inff();
        xcap_max = mx;
        max_neg = !(mx > 0.0f);
        cap16_max = cap_bits(mx, max_neg);
    }

    // ADM mode: lists = kWaves * kAdmCap floats, fills = kWaves counters, both in LDS.  Call after the
    // constructor's publication has been separated by a __syncthreads(); synchronise again before process().
    __device__ __forceinline__ void arm_admissible(float delta, float *lists, int32_t *fills)
    {
        adm_delta = delta;
        adm_list = lists + wave * kAdmCap;
        adm_fill = fills + wave;
        if ((tid & 63) == 0) *adm_fill = 0;
        gate = make_gate(gate.L, T, adm_delta);
    }

    // TOPN mode: queues = kWaves * kDeferCap vector numbers in LDS.  Before the first process(); nothing to synchronise
    // (a wave only ever touches its own queue).
    __device__ __forceinline__ void arm_deferred(int32_t *queues)
    {
        defer_q = queues + wave * kDeferCap;
        defer_n = 0;
    }

    // TOPN mode, whole wave (call from wave-uniform code): the per-entry look at every waiting vector, one vector per
    // lane, against the gate as it stands now (it only ever rises, so nothing that still matters is missed).  The
    // queue persists across the caller's epochs; the caller drains it before the selection is finished.
    __device__ __forceinline__ void drain(TopN *top)
    {
        const int lane = tid & 63;
        while (defer_n > 0) {
            const int take = defer_n < 64 ? defer_n : 64;
            defer_n -= take;
            if (lane < take) {
                const int32_t vec = defer_q[defer_n + lane];
                const u32x4 q = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const char *>(x_row) + (size_t)vec * 16u);
                uint32_t r[E];
                const uint64_t p0 = (uint64_t)kPhiloxM0 * (uint32_t)(vec * (E / 4));
                philox4x32_10_from_product(p0, ri.pos, ri.seq, kStreamGumbel, ri.key, r);
                if (E == 8) philox4x32_10_from_product(p0 + kPhiloxM0, ri.pos, ri.seq, kStreamGumbel, ri.key, r + (E - 4));
                const int32_t v0 = vec * E;
                const uint32_t qw[4] = {q.x, q.y, q.z, q.w};
                float xs[E];
                uint32_t cand = 0;  // the entries whose own noise bound still reaches the gate
#pragma unroll
                for (int j = 0; j < E; ++j) {
                    const uint32_t w = qw[DT == 0 ? j >> 1 : j];
                    xs[j] = DT == 0 ? __uint_as_float((j & 1) ? (w & 0xFFFF0000u) : (w << 16)) : __uint_as_float(w);
                    if (!(__fmaf_rn(xs[j], inv_T, gumbel_upper_bound(r[j])) < gate.Lgate)) cand |= 1u << j;
                }
                // a lane has few of them, at scattered positions: each lane takes its own next one per turn (walking
                // the eight positions in step would run the exact evaluation once for every position any lane has one at)
                while (cand != 0u) {
                    const int j = __builtin_ctz(cand);
                    cand &= cand - 1u;
                    float xv = xs[0];
                    uint32_t rv = r[0];
#pragma unroll
                    for (int k = 1; k < E; ++k) {
                        xv = j == k ? xs[k] : xv;
                        rv = j == k ? r[k] : rv;
                    }
                    evaluate(xv, rv, v0 + j, top);
                }
            }
        }
    }

    // TOPN mode: scores go to the selection handed to process() / tail() (by pointer argument, never stored:
    // the selection must stay in registers); the bound is its threshold (call retarget() whenever that
    // moves).  Same synchronisation rules as arm_count().
    __device__ __forceinline__ void retarget(const TopN &top)
    {
        const float bound = top.theta == 0ull ? -__builtin_inff() : (top.theta == ~0ull ? 3.0e38f : top_key(top.theta));
        gate = make_gate(bound, T);
        if ((tid & 63) == 0) lds_L[wave] = gate.L;
    }

    // COUNT mode: fix the bound at M - delta.  Call after the constructor's publication has been
    // separated by a __syncthreads(); the caller synchronises again before the first process().
    __device__ __forceinline__ void arm_count(float M, float delta)
    {
        count_M = M;
        count_delta = delta;
        float Lc = M - delta;
        if (!(Lc == Lc)) Lc = -__builtin_inff();
        gate = make_gate(Lc, T);
        if ((tid & 63) == 0) lds_L[wave] = gate.L;
    }

    // Exact evaluation of one entry (same arithmetic as the unfiltered kernel), ties to the lowest index.
    __device__ __forceinline__ void evaluate(float xv, uint32_t rv, int32_t v, TopN *top = nullptr)
    {
        const float y = perturbed_score(xv, inv_T, rv);
        bad |= (uint32_t)!(xv < __builtin_inff());
        if (COUNT) {
            count += (uint32_t)(count_M - y <= count_delta);  // the margin of entry v, in the kernel's precision
            return;
        }
        if (TOPN) {
            if (y == y && v != t) top->push(top_composite(y, v));
            return;
        }
        if (y > best_y || (y == best_y && v < best_v)) {
            best_y = y;
            best_v = v;
        }
        if (ADM) {
            if (!(y < gate.Lgate)) {  // may lie within delta of the final maximum
                const int32_t i = atomicAdd(adm_fill, 1);
                if (i < kAdmCap)
                    adm_list[i] = y;
                else
                    adm_over = 1;
            }
        }
    }

    // ADM mode, whole wave (call from wave-uniform code): drop what the current bound has ruled out once the
    // list is half full.  A call of process() adds at most 512 entries, so a list that starts below half
    // cannot overflow.
    __device__ __forceinline__ void adm_prune()
    {
        const int lane = tid & 63;
        const int32_t fill = __builtin_amdgcn_readfirstlane(*adm_fill);
        if (fill <= kAdmCap / 2) return;
        const int32_t c = min(fill, kAdmCap);
        int32_t out = 0;
        for (int32_t base = 0; base < c; base += 64) {
            const bool have = base + lane < c;
            const float y = have ? adm_list[base + lane] : 0.0f;
            const bool keep = have && !(y < gate.Lgate);
            const uint64_t m = __builtin_amdgcn_ballot_w64(keep);
            const int32_t pos = out + (int32_t)__builtin_popcountll(m & ((1ull << lane) - 1ull));
            if (keep) adm_list[pos] = y;  // pos <= base + lane: nothing unread is overwritten
            out += (int32_t)__builtin_popcountll(m);
        }
        if (lane == 0) *adm_fill = out;
        if (out > kAdmCap / 2) adm_over = 1;
    }

    // ADM mode, all 256 threads, after finish() (best_y is then the row maximum in every thread): the number
    // of listed scores within delta of it, by the expression that forms margins; -1 if undetermined.
    __device__ __forceinline__ int32_t adm_count(int32_t *lds_c)
    {
        const int lane = tid & 63;
        const int32_t c = min(__builtin_amdgcn_readfirstlane(*adm_fill), kAdmCap);
        int32_t n = 0;
        for (int32_t base = 0; base < c; base += 64) {
            const bool in = base + lane < c && (best_y - adm_list[base + lane < c ? base + lane : 0] <= adm_delta);
            n += (int32_t)__builtin_popcountll(__builtin_amdgcn_ballot_w64(in));
        }
        const int any_over = __syncthreads_or((int)adm_over);
        if (lane == 0) lds_c[wave] = n;
        __syncthreads();
        n = lds_c[0] + lds_c[1] + lds_c[2] + lds_c[3];
        return any_over ? -1 : n;
    }

    // Entry-level test: can this entry still reach the lower bound?
    __device__ __forceinline__ void consider(float xv, uint32_t rv, int32_t v, TopN *top = nullptr)
    {
        if (!(__fmaf_rn(xv, inv_T, gumbel_upper_bound(rv)) < gate.Lgate)) evaluate(xv, rv, v, top);
    }

    __device__ __forceinline__ void count_above(u32x4 q, bool active)
    {
        const uint32_t qw[4] = {q.x, q.y, q.z, q.w};
        uint32_t n = 0;
        if (DT == 0) {
            if (xt_pos) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    n += __builtin_popcountll(
                        __builtin_amdgcn_ballot_w64(active && (int16_t)(qw[j] & 0xFFFFu) > (int16_t)xt16));
                    n += __builtin_popcountll(
                        __builtin_amdgcn_ballot_w64(active && (int16_t)(qw[j] >> 16) > (int16_t)xt16));
                }
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    n += __builtin_popcountll(
                        __builtin_amdgcn_ballot_w64(active && (uint16_t)(qw[j] & 0xFFFFu) < (uint16_t)xt16));
                    n += __builtin_popcountll(
                        __builtin_amdgcn_ballot_w64(active && (uint16_t)(qw[j] >> 16) < (uint16_t)xt16));
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                n += __builtin_popcountll(__builtin_amdgcn_ballot_w64(active && __uint_as_float(qw[j]) > xt));
        }
        above += n;
    }

    // Upper bound of the logits of one vector from its extreme bf16 bit patterns (lo: smallest as unsigned, known
    // unless MODE == 1; hi: largest as signed, known unless MODE == 0): the largest signed pattern if it is a positive
    // number (a NaN with its sign clear stays a NaN and passes every "<" test), else the smallest unsigned pattern
    // if all are negative, else something that passes.
    template <int MODE>
    __device__ __forceinline__ static float vector_upper_bound(uint16_t lo, uint16_t hi)
    {
        const float f_hi = __uint_as_float((uint32_t)hi << 16), f_lo = __uint_as_float((uint32_t)lo << 16);
        if (MODE == 0) return lo < 0x8000u ? __builtin_inff() : f_lo;  // a positive entry: not bounded by lo
        if (MODE == 1) return (int16_t)hi >= 0 ? f_hi : -0.0f;         // all negative: bounded by zero
        return (int16_t)hi >= 0 ? f_hi : f_lo;
    }
    __device__ __forceinline__ static float vector_upper_bound_f32(u32x4 q)
    {
        const float x0 = __uint_as_float(q.x), x1 = __uint_as_float(q.y), x2 = __uint_as_float(q.z), x3 = __uint_as_float(q.w);
        float xub = fmaxf(fmaxf(x0, x1), fmaxf(x2, x3));
        if (!(x0 + x1 + x2 + x3 == x0 + x1 + x2 + x3)) xub = __builtin_inff();  // a NaN among them (or both infinities)
        return xub;
    }

    // One 16-byte vector per lane; `round` is the vector round (vector index = round * 256 + tid).
    // MODE is the gate's mode, fixed per instantiation so that the loop body carries no mode branches.
    template <int MODE>
    __device__ __forceinline__ void process(u32x4 q, int round, bool active, TopN *top = nullptr)
    {
        if (PEAKED) {
            bool reach;
            if (DT == 0) {
                if (MODE == 1 && !max_neg) {
                    i16x2 m = __builtin_elementwise_max(as_i16x2(q.x), as_i16x2(q.y));
                    m = __builtin_elementwise_max(m, as_i16x2(q.z));
                    m = __builtin_elementwise_max(m, as_i16x2(q.w));
                    reach = (int16_t)(m.x > m.y ? m.x : m.y) >= (int16_t)cap16_max;
                } else {
                    u16x2 m = __builtin_elementwise_min(as_u16x2(q.x), as_u16x2(q.y));
                    m = __builtin_elementwise_min(m, as_u16x2(q.z));
                    m = __builtin_elementwise_min(m, as_u16x2(q.w));
                    reach = (uint16_t)(m.x < m.y ? m.x : m.y) <= (uint16_t)cap16_max;
                }
            } else {
                reach = !(__uint_as_float(q.x) < xcap_max) || !(__uint_as_float(q.y) < xcap_max) ||
                        !(__uint_as_float(q.z) < xcap_max) || !(__uint_as_float(q.w) < xcap_max);
            }
            if (__builtin_amdgcn_ballot_w64(active && reach) == 0ull) {
                if (RANK) count_above(q, active);
                return;
            }
        }
        const uint64_t round_prod = (uint64_t)kPhiloxM0 * (uint32_t)(round * kBlock * (E / 4));
        const uint64_t p0 = round_prod + lane_prod;
        uint32_t r[E];
        philox4x32_10_from_product(p0, ri.pos, ri.seq, kStreamGumbel, ri.key, r);
        if (E == 8) philox4x32_10_from_product(p0 + kPhiloxM0, ri.pos, ri.seq, kStreamGumbel, ri.key, r + (E - 4));
        // the largest of the words, for tests A and C
        uint32_t rmax = r[0];
#pragma unroll
        for (int j = 1; j < E; ++j) rmax = max(rmax, r[j]);
        if (TOPN) {
            // The selection's bound lies several units below the row maximum, where tests A, B and C trip for a fifth
            // of all vectors and filter nothing.  One test takes their place: y_v <= x_max / T + bound(r_max) for every
            // entry of the vector (both terms are monotone, and so is the rounding of the sum) - the expression of the
            // per-entry test, on the vector's largest logit and largest word.  A vector that passes is only noted.
            float xub;
            if (DT == 0) {
                uint16_t lo = 0, hi = 0;
                if (MODE != 1) {
                    u16x2 m = __builtin_elementwise_min(as_u16x2(q.x), as_u16x2(q.y));
                    m = __builtin_elementwise_min(m, as_u16x2(q.z));
                    m = __builtin_elementwise_min(m, as_u16x2(q.w));
                    lo = m.x < m.y ? m.x : m.y;
                }
                if (MODE != 0) {
                    i16x2 m = __builtin_elementwise_max(as_i16x2(q.x), as_i16x2(q.y));
                    m = __builtin_elementwise_max(m, as_i16x2(q.z));
                    m = __builtin_elementwise_max(m, as_i16x2(q.w));
                    hi = (uint16_t)(m.x > m.y ? m.x : m.y);
                }
                seen_lo = lo;  // (a selection of raw logits that runs beside this stream tests the same extremes)
                seen_hi = hi;
                xub = vector_upper_bound<MODE>(lo, hi);
            } else {
                xub = vector_upper_bound_f32(q);
            }
            const uint64_t hitmask =
                __builtin_amdgcn_ballot_w64(active && !(__fmaf_rn(xub, inv_T, gumbel_upper_bound(rmax)) < gate.Lgate));
            if (hitmask != 0ull) {
                const uint32_t before = __builtin_amdgcn_mbcnt_hi((uint32_t)(hitmask >> 32),
                                                                  __builtin_amdgcn_mbcnt_lo((uint32_t)hitmask, 0u));
                if ((hitmask >> (tid & 63)) & 1ull) defer_q[defer_n + (int)before] = round * kBlock + tid;
                defer_n += (int)__builtin_popcountll(hitmask);
            }
            return;
        }
        // wave-wide masks of the lanes whose vector trips A, B, or both halves of C
        const uint64_t amask = __builtin_amdgcn_ballot_w64(active && rmax >= kGateHi);
        const uint64_t cnmask = __builtin_amdgcn_ballot_w64(active && rmax >= kGateLo);
        uint64_t bmask, cxmask;
        uint16_t lo = 0, hi = 0;  // bf16: extreme bit patterns of the vector (see below)
        if (DT == 0) {
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
                // The three tests look at the largest word and the largest logit of the vector separately.  Taken
                // together they bound every entry of it: y_v <= x_max / T + bound(r_max) (both terms are monotone,
                // and so is the rounding of the sum), so one more test per vector, with the expression the
                // per-entry test uses, rules out most vectors that tripped a test: the per-entry test below would
                // fail for each of their entries.  x_max from the extreme bit patterns: the largest signed
                // pattern if it is a positive number (a NaN with its sign clear stays a NaN and passes), else the
                // smallest unsigned pattern if all are negative, else something that passes.
                const float xub = DT == 0 ? vector_upper_bound<MODE>(lo, hi) : vector_upper_bound_f32(q);
                if (!(__fmaf_rn(xub, inv_T, gumbel_upper_bound(rmax)) < gate.Lgate)) {
                    // Entries that could matter are those with moderate noise or a moderate logit; each of
                    // them is then tested against its own noise bound before anything exact is computed.
                    const int32_t v0 = (round * kBlock + tid) * E;
                    const uint32_t qw[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
                    for (int j = 0; j < E; ++j) {
                        const uint32_t w = qw[DT == 0 ? j >> 1 : j];
                        const float xv = DT == 0 ? __uint_as_float((j & 1) ? (w & 0xFFFF0000u) : (w << 16))
                                                 : __uint_as_float(w);
                        if (r[j] >= kGateLo || !(xv < gate.xcap_lo)) consider(xv, r[j], v0 + j, top);
                    }
                }
            }
            // a better score raises the lower bound for this wave; other waves pick it up from LDS
            if (__builtin_amdgcn_ballot_w64(best_y > gate.L) != 0ull) {
                float L = fmaxf(wave_max(best_y), gate.L);
                L = fmaxf(fmaxf(L, lds_L[0]), fmaxf(lds_L[1], fmaxf(lds_L[2], lds_L[3])));
                gate = make_gate(L, T, ADM ? adm_delta : 0.0f);
                if (PEAKED) peak_cap();
                if ((tid & 63) == 0) lds_L[wave] = gate.L;
            }
            if (ADM) adm_prune();
        }
    }

    // process() for whatever mode the gate is in right now (used outside the hot loop)
    __device__ __forceinline__ void process_any(u32x4 q, int round, bool active, TopN *top = nullptr)
    {
        if (gate.mode == 0)
            process<0>(q, round, active, top);
        else if (gate.mode == 1)
            process<1>(q, round, active, top);
        else
            process<2>(q, round, active, top);
    }

    // pick up a bound another wave has raised
    __device__ __forceinline__ void pickup()
    {
        const float L = fmaxf(fmaxf(lds_L[0], lds_L[1]), fmaxf(lds_L[2], lds_L[3]));
        if (L > gate.L) {
            gate = make_gate(L, T, ADM ? adm_delta : 0.0f);
            if (PEAKED) peak_cap();
        }
    }

    // the ragged tail: V % E entries, one lane each, evaluated exactly
    __device__ __forceinline__ void tail(TopN *top = nullptr)
    {
        const int64_t v = (V / E) * E + tid;
        if (v < V) {
            uint32_t r[4];
            noise_block(ri.key, ri.pos, ri.seq, kStreamGumbel, (uint32_t)(v >> 2), r);
            const uint32_t rv = (v & 3) == 0 ? r[0] : (v & 3) == 1 ? r[1] : (v & 3) == 2 ? r[2] : r[3];
            evaluate(Elem<DT>::to_float(x_row[v]), rv, (int32_t)v, top);
        }
        if (RANK)
            above += __builtin_popcountll(
                __builtin_amdgcn_ballot_w64(v < V && Elem<DT>::to_float(x_row[v < V ? v : 0]) > xt));
    }

    // block reduction and outputs
    __device__ __forceinline__ void finish(int64_t row, const GumbelOutputs &o, float *lds_y, int32_t *lds_i,
                                           int32_t *lds_rank)
    {
        block_argmax(best_y, best_v, lds_y, lds_i);
        if (RANK && (tid & 63) == 0) lds_rank[wave] = (int32_t)above;
        const int any_bad = __syncthreads_or((int)bad);
        if (tid == 0) {
            const float nan = __builtin_nanf("");
            if (RANK) o.logit_rank[row] = valid ? lds_rank[0] + lds_rank[1] + lds_rank[2] + lds_rank[3] : -1;
            if (best_v == 0x7FFFFFFF) best_v = 0;  // every entry masked: all scores are -inf
            uint32_t f = any_bad ? kFlagNonfinite : 0u;
            float mg = nan;
            if (valid) {
                mg = best_y - yt;
                if (best_v == t) f |= kFlagMatch;
            } else {
                f |= kFlagInvalidClaim;
            }
            o.margin[row] = mg;
            o.argmax[row] = best_v;
            if (o.max_score) o.max_score[row] = best_y;
            if (o.claimed_score) o.claimed_score[row] = yt;
            o.flags[row] = (uint8_t)f;
        }
    }
};

// 16-byte non-temporal load of lane `tid`'s vector in vector round `round` of a row.
__device__ __forceinline__ u32x4 load_round(const void *x_row, int round)
{
    const char *p = reinterpret_cast<const char *>(x_row) + (size_t)round * (kBlock * 16) + threadIdx.x * 16u;
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
}

}  // namespace difr
