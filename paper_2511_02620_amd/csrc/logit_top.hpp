// Streaming selection of the k largest raw logits of a row (the sampler's top-k set; Sec. 3.2 filter
// policy), on top of topn.hpp: a cheap test of a whole 16-byte vector against the selection's threshold
// first, the 64-bit composite only for the entries that pass.
#pragma once

#include "gumbel_stream.hpp"
#include "ipt_stream.hpp"
#include "topn.hpp"

namespace difr {

template <int DT>
struct LogitTop {
    static constexpr int E = Elem<DT>::kPerVec;
    TopN top;
    float floor;       // no logit below this can still belong to the k largest (wave-uniform)
    uint32_t floor16;  // its bf16 bit pattern, rounded so that the packed test never misses an entry
    bool floor_pos;
    uint32_t bad;      // a NaN (sign bit clear) or +inf logit was seen
    // note_vector() / drain(): this wave's queue of vectors that hold a candidate (kDeferCap vector numbers in LDS),
    // how many wait (wave-uniform), and the row they are read from again
    int32_t *defer_q;
    int defer_n;
    const void *defer_row;

    __device__ __forceinline__ void init(uint64_t *buf, int32_t *count, int k, int cap)
    {
        top.init(buf, count, k, cap);
        bad = 0;
        defer_n = 0;
        set_floor(-__builtin_inff());
    }
    // queues = kWaves * kDeferCap ints in LDS (a wave only ever touches its own part)
    __device__ __forceinline__ void arm_deferred(int32_t *queues, const void *x_row)
    {
        defer_q = queues + ((int)threadIdx.x >> 6) * kDeferCap;
        defer_n = 0;
        defer_row = x_row;
    }
    __device__ __forceinline__ void set_floor(float f)
    {
        floor = f;
        floor_pos = f > 0.0f;
        floor16 = cap_bits(f, !floor_pos);
    }
    // call after a compaction of `top`.  (A coarse compaction leaves a threshold whose low key bits are zero; when the
    // n-th largest logit so far is a masked entry, -inf, that image is not a number: nothing is below the floor then.)
    __device__ __forceinline__ void retarget()
    {
        float f = top.theta == 0ull ? -__builtin_inff() : top_key(top.theta);
        if (!(f == f)) f = -__builtin_inff();
        set_floor(f);
    }

    __device__ __forceinline__ void push_entry(float xv, int32_t v)
    {
        bad |= (uint32_t)!(xv < __builtin_inff());
        if (xv >= floor) top.push(top_composite(xv, v));
    }

    // The test of push_vector() on vector number `vec` of the row, but a vector that passes is only noted in the
    // wave's queue: a wave in which one or two lanes hold a candidate does not walk the entries for them.  The caller
    // keeps defer_n below 64 between calls (drain() once it is not) and drains before the selection is finished.
    // HAVE: which of the vector's extreme bf16 patterns the caller has at hand (bit 0: `lo`, the smallest as
    // unsigned; bit 1: `hi`, the largest as signed) - the Gumbel stream beside this selection forms them for its own
    // test; the other one, if needed, is formed here.
    template <int HAVE = 0>
    __device__ __forceinline__ void note_vector(u32x4 q, int32_t vec, uint32_t lo = 0u, uint32_t hi = 0u)
    {
        bool hit;
        if (DT == 0) {
            if (floor_pos) {
                if (!(HAVE & 2)) {
                    i16x2 m = __builtin_elementwise_max(as_i16x2(q.x), as_i16x2(q.y));
                    m = __builtin_elementwise_max(m, as_i16x2(q.z));
                    m = __builtin_elementwise_max(m, as_i16x2(q.w));
                    hi = (uint16_t)(m.x > m.y ? m.x : m.y);
                }
                hit = (int16_t)hi >= (int16_t)floor16;
            } else {
                if (!(HAVE & 1)) {
                    u16x2 m = __builtin_elementwise_min(as_u16x2(q.x), as_u16x2(q.y));
                    m = __builtin_elementwise_min(m, as_u16x2(q.z));
                    m = __builtin_elementwise_min(m, as_u16x2(q.w));
                    lo = m.x < m.y ? m.x : m.y;
                }
                hit = (uint16_t)lo <= (uint16_t)floor16;
            }
        } else {
            hit = !(__uint_as_float(q.x) < floor) || !(__uint_as_float(q.y) < floor) ||
                  !(__uint_as_float(q.z) < floor) || !(__uint_as_float(q.w) < floor);
        }
        const uint64_t m = __builtin_amdgcn_ballot_w64(hit);
        if (m == 0ull) return;
        const uint32_t before = __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
        if (hit) defer_q[defer_n + (int)before] = vec;
        defer_n += (int)__builtin_popcountll(m);
    }

    // Whole wave, from wave-uniform code: every waiting vector is read again, one per lane, and its entries that
    // reach the floor as it stands now are pushed.  (+inf and NaNs with the sign bit clear always pass the vector
    // test, so they are seen - and flagged - here.)
    __device__ __forceinline__ void drain()
    {
        const int lane = (int)threadIdx.x & 63;
        while (defer_n > 0) {
            const int take = defer_n < 64 ? defer_n : 64;
            defer_n -= take;
            if (lane < take) {
                const int32_t vec = defer_q[defer_n + lane];
                const u32x4 q = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const char *>(defer_row) + (size_t)vec * 16u);
                const uint32_t qw[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
                for (int j = 0; j < E; ++j) {
                    const uint32_t w = qw[DT == 0 ? j >> 1 : j];
                    const float xv = DT == 0 ? __uint_as_float((j & 1) ? (w & 0xFFFF0000u) : (w << 16)) : __uint_as_float(w);
                    if (DT == 0)
                        bad |= (uint32_t)((int32_t)__float_as_uint(xv) >= (int32_t)0x7F800000);
                    else
                        bad |= (uint32_t)!(xv < __builtin_inff());
                    if (xv >= floor) top.push(top_composite(xv, vec * E + j));
                }
            }
        }
    }

    // One 16-byte vector (entries v0 .. v0 + E - 1).  bf16: packed 16-bit min / max on the raw bit patterns, as
    // in the Gumbel gates; a NaN with the sign bit clear passes the test and is flagged, one with the sign bit
    // set counts as -inf.
    __device__ __forceinline__ void push_vector(u32x4 q, int64_t v0, bool active)
    {
        bool hit;
        if (DT == 0) {
            if (floor_pos) {
                i16x2 m = __builtin_elementwise_max(as_i16x2(q.x), as_i16x2(q.y));
                m = __builtin_elementwise_max(m, as_i16x2(q.z));
                m = __builtin_elementwise_max(m, as_i16x2(q.w));
                hit = (int16_t)(m.x > m.y ? m.x : m.y) >= (int16_t)floor16;
            } else {
                u16x2 m = __builtin_elementwise_min(as_u16x2(q.x), as_u16x2(q.y));
                m = __builtin_elementwise_min(m, as_u16x2(q.z));
                m = __builtin_elementwise_min(m, as_u16x2(q.w));
                hit = (uint16_t)(m.x < m.y ? m.x : m.y) <= (uint16_t)floor16;
            }
        } else {
            hit = !(__uint_as_float(q.x) < floor) || !(__uint_as_float(q.y) < floor) ||
                  !(__uint_as_float(q.z) < floor) || !(__uint_as_float(q.w) < floor);
        }
        hit = hit && active;
        const uint64_t m = __builtin_amdgcn_ballot_w64(hit);
        if (m == 0ull) return;
        const uint32_t qw[4] = {q.x, q.y, q.z, q.w};
        if (hit && DT == 0) {
            // +inf or a NaN with the sign bit clear: the largest pattern, as signed 16-bit, is >= 0x7F80
            i16x2 mx = __builtin_elementwise_max(as_i16x2(q.x), as_i16x2(q.y));
            mx = __builtin_elementwise_max(mx, as_i16x2(q.z));
            mx = __builtin_elementwise_max(mx, as_i16x2(q.w));
            bad |= (uint32_t)((mx.x > mx.y ? mx.x : mx.y) >= (int16_t)0x7F80);
        }
        if (top.priming) {  // every lane has a vector to look at and a push is a comparison: each lane its own
            if (hit) {
#pragma unroll
                for (int j = 0; j < E; ++j) {
                    const uint32_t w = qw[DT == 0 ? j >> 1 : j];
                    const float xv = DT == 0 ? __uint_as_float((j & 1) ? (w & 0xFFFF0000u) : (w << 16)) : __uint_as_float(w);
                    if (DT != 0) bad |= (uint32_t)!(xv < __builtin_inff());
                    if (xv >= floor) top.push(top_composite(xv, (int32_t)(v0 + j)));
                }
            }
            return;
        }
        // A few lanes have a vector with a candidate in it.  Left to themselves they would walk their E entries
        // while the rest of the wave waits, and the wave would run the push once for every entry position at
        // which any of them has a candidate.  Instead the wave shares the work: the lanes with a hit are numbered
        // (their lane ids gathered into lanes 0, 1, ...), and in each pass 64 / E of them are served, lane L
        // looking at entry L % E of the (L / E)-th of them - one test and one push per pass for the whole wave.
        const int lane = (int)threadIdx.x & 63;
        const int rank = (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
        const int nh = (int)__builtin_popcountll(m);
        // a permutation of the lanes: those with a hit first, in lane order
        const int ids = __builtin_amdgcn_ds_permute((hit ? rank : nh + lane - rank) << 2, lane);
        const int e = lane & (E - 1), g = lane / E;
        for (int base = 0; base < nh; base += 64 / E) {  // (wave-uniform)
            const int k = base + g;
            const int src = __builtin_amdgcn_ds_bpermute((k & 63) << 2, ids);
            const uint32_t w0 = (uint32_t)__builtin_amdgcn_ds_bpermute(src << 2, (int)qw[0]);
            const uint32_t w1 = (uint32_t)__builtin_amdgcn_ds_bpermute(src << 2, (int)qw[1]);
            const uint32_t w2 = (uint32_t)__builtin_amdgcn_ds_bpermute(src << 2, (int)qw[2]);
            const uint32_t w3 = (uint32_t)__builtin_amdgcn_ds_bpermute(src << 2, (int)qw[3]);
            const int d = DT == 0 ? e >> 1 : e;
            const uint32_t w = d == 0 ? w0 : (d == 1 ? w1 : (d == 2 ? w2 : w3));
            const float xv = DT == 0 ? __uint_as_float((e & 1) ? (w & 0xFFFF0000u) : (w << 16)) : __uint_as_float(w);
            const bool have = k < nh;
            if (DT != 0) bad |= (uint32_t)(have && !(xv < __builtin_inff()));
            if (have && xv >= floor) top.push(top_composite(xv, (int32_t)v0 + (src - lane) * E + e));
        }
    }
};

// The filter's kept prefix from the k largest logits in rank order (buf[0 .. nk), descending): top-k is the whole
// list, top-p cuts it to the shortest prefix whose softmax(x / T) mass, renormalised over the list, reaches
// top_p.  All 256 threads call it (nk <= kTopMaxN, `s` idle): the exponentials are taken in parallel, one per
// thread, and one thread then adds them up in rank order in fp64.  Returns the prefix length (>= 1 if nk >= 1) to
// every thread; ends with a __syncthreads().
__device__ __forceinline__ int filter_prefix_length(const uint64_t *buf, int nk, double T, float top_p, TopScratch &s)
{
    if (nk <= 0 || !(top_p < 1.0f)) return nk;
    const int tid = threadIdx.x;
    double *e = reinterpret_cast<double *>(s.tmp);
    if (tid < nk) e[tid] = exp(((double)top_key(buf[tid]) - (double)top_key(buf[0])) / T);
    __syncthreads();
    if (tid == 0) {
        double Z = 0.0;
        for (int r = 0; r < nk; ++r) Z += e[r];
        // (the cumulative mass against top_p Z: the same cut as the cumulative probability against top_p, except
        // within a rounding of the boundary, and no division per entry on the one thread everybody waits for)
        const double target = (double)top_p * Z;
        double cum = 0.0;
        int kept = nk;
        for (int r = 0; r < nk; ++r) {
            cum += e[r];
            if (cum >= target) {
                kept = r + 1;
                break;
            }
        }
        s.kept = kept;
    }
    __syncthreads();
    const int kept = s.kept;
    __syncthreads();
    return kept;
}

// Token-IPT-DiFR on the kept set K = buf[0 .. kc) (the filter's prefix of the top-k logits, in rank order): the
// members are put in ascending vocabulary index, their renormalised CDF is formed in fp64, and the claimed
// token's interval, the distance of the regenerated uniform from it, the sampler's own token and the
// Gaussian log-mass are written (Sec. 3.2, Sec. 6.2, appendix "convolved Gaussian score").  All 256 threads;
// s_e / s_idx: kTopMaxN entries of LDS each, lds_d: kWaves doubles, s_tok: one int preset to -1.
template <int DT>
__device__ __forceinline__ void ipt_filtered_finish(const RowInfo &ri, int64_t row, int64_t V, const uint64_t *buf, int kc,
                                                    bool bad_seen, const IptOutputs &o, int32_t *kept_out, double *s_e,
                                                    int32_t *s_idx, double *lds_d, int32_t *s_tok)
{
    const int tid = threadIdx.x;
    const float nan = __builtin_nanf("");
    const int64_t t = ri.claimed;
    const bool valid = t >= 0 && t < V;
    // K in ascending vocabulary index: each member finds its place by counting the members with a smaller index
    const double x0 = kc > 0 ? (double)top_key(buf[0]) : 0.0;
    if (tid < kc) {
        const int32_t mine = top_index(buf[tid]);
        int place = 0;
        for (int r = 0; r < kc; ++r) place += (int)(top_index(buf[r]) < mine);
        s_idx[place] = mine;
        s_e[place] = exp(((double)top_key(buf[tid]) - x0) / (double)ri.T);
    }
    __syncthreads();
    const double e = tid < kc ? s_e[tid] : 0.0;
    const int32_t idx = tid < kc ? s_idx[tid] : 0x7FFFFFFF;
    double Z;
    const double incl = block_inclusive_scan(e, lds_d, Z);  // CDF numerators in index order

    uint32_t r4[4];
    noise_block(ri.key, ri.pos, ri.seq, kStreamIpt, 0u, r4);
    const float u = uniform_from_bits(r4[0]);
    const double ud = (double)u;
    const bool bad = bad_seen || !(Z > 0.0) || !(Z < (double)__builtin_inff());

    // the sampler's token: the first member whose cumulative mass exceeds u (the last member if rounding leaves none)
    if (tid < kc && !bad) {
        const double before = incl - e;
        if (incl / Z > ud && !(before / Z > ud)) *s_tok = idx;
    }
    // the claimed token's interval
    const double below = block_sum_f64((tid < kc && (int64_t)idx < t) ? e : 0.0, lds_d);
    const double own = block_sum_f64((tid < kc && (int64_t)idx == t) ? e : 0.0, lds_d);
    __syncthreads();
    if (tid == 0) {
        float a = nan, bb = nan, d = nan;
        double ad = 0.0, bd = 0.0;
        bool match = false;
        if (valid && !bad) {
            ad = below / Z;
            bd = ad + own / Z;
            a = (float)ad;
            bb = (float)bd;
            d = (float)fmax(fmax(ad - ud, ud - bd), 0.0);
            match = (ad <= ud) && (ud < bd);
        }
        uint32_t f = 0;
        if (!valid) f |= kFlagInvalidClaim;
        if (bad) f |= kFlagNonfinite;
        if (match) f |= kFlagMatch;
        int32_t tok = *s_tok;
        if (tok < 0 && kc > 0) tok = s_idx[kc - 1];
        o.dist[row] = d;
        if (o.cdf_lo) o.cdf_lo[row] = a;
        if (o.cdf_hi) o.cdf_hi[row] = bb;
        if (o.u) o.u[row] = u;
        if (o.ipt_token) o.ipt_token[row] = bad ? -1 : tok;
        if (o.log_mass) o.log_mass[row] = (valid && !bad) ? (float)gaussian_log_mass(ad, bd, ud, o.sigma, o.eps) : nan;
        if (kept_out) kept_out[row] = kc;
        o.flags[row] = (uint8_t)f;
    }
}

}  // namespace difr
