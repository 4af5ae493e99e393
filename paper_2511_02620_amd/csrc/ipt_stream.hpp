// Row-streaming state of the Token-IPT-DiFR kernel (Sec. 3.2 softmax and IPT sampler; Sec. 6.2 and
// the appendix algorithm "convolved Gaussian score"), kept as a struct so that the IPT-only kernel
// and the kernel that scores both estimators in one pass share it.
#pragma once

#include "difr_device.hpp"

namespace difr {

typedef uint32_t ipt_u32x4 __attribute__((ext_vector_type(4)));

// Inclusive scan (fp64) over the 256 threads in thread order; returns the inclusive value and
// the block total.  Fixed shape.
__device__ __forceinline__ double block_inclusive_scan(double v, double *lds /* kWaves */, double &total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const double o = __shfl_up(v, off, 64);
        if (lane >= off) v += o;
    }
    __syncthreads();
    if (lane == 63) lds[wave] = v;
    __syncthreads();
    double before = 0.0, tot = 0.0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const double s = lds[w];
        if (w < wave) before += s;
        tot += s;
    }
    total = tot;
    return v + before;
}

__device__ __forceinline__ double block_sum_f64(double v, double *lds /* kWaves */)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = v;
    __syncthreads();
    double s = lds[0];
#pragma unroll
    for (int i = 1; i < kWaves; ++i) s += lds[i];
    return s;
}

// max(a, b, c) as the bare three-input instruction (a NaN operand is ignored; NaNs are caught
// later through the sum of exponentials, not here).
__device__ __forceinline__ float max3_raw(float a, float b, float c)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// Sum of the E exponentials of one vector as a fixed binary tree in fp32.
template <int E>
__device__ __forceinline__ float tree_sum(const float e[E])
{
    float t[E];
#pragma unroll
    for (int j = 0; j < E; ++j) t[j] = e[j];
#pragma unroll
    for (int w = E / 2; w >= 1; w >>= 1) {
#pragma unroll
        for (int j = 0; j < w; ++j) t[j] += t[j + w];
    }
    return t[0];
}

// Gaussian log-mass of [a,b] under N(u, sigma^2), fp64:
//   ln( Phi((b-u)/sigma) - Phi((a-u)/sigma) + eps ),
// with the difference taken on the non-cancelling side (erfc in the tails).
__device__ double gaussian_log_mass(double a, double b, double u, double sigma, double eps)
{
    const double s = 1.0 / (sigma * 1.4142135623730951);
    const double za = (a - u) * s, zb = (b - u) * s;
    double mass;
    if (za >= 0.0)
        mass = 0.5 * (erfc(za) - erfc(zb));
    else if (zb <= 0.0)
        mass = 0.5 * (erfc(-zb) - erfc(-za));
    else
        mass = 0.5 * (erf(zb) + erf(-za));
    if (mass < 0.0) mass = 0.0;
    return log(mass + eps);
}

// Everything after the streaming pass: combine the 256 partial (max, sum) pairs, regenerate u,
// form the interval and the distance, optionally search the honest sampler's token, write outputs.
struct IptOutputs {
    float *dist, *cdf_lo, *cdf_hi, *u;
    int32_t *ipt_token;
    double sigma, eps;
    float *log_mass;
    uint8_t *flags;
    int32_t *logit_rank;
};

template <int DT, bool ALIGNED>
__device__ __forceinline__ void ipt_finish(const RowBatch &b, const RowInfo &ri, int64_t row,
                                           const typename Elem<DT>::type *x_row, float c, float ref, double Z,
                                           double P, float refP, int32_t above, const IptOutputs &o, float *lds_f,
                                           double *lds_d, int32_t *lds_tok)
{
    constexpr int E = Elem<DT>::kPerVec;
    const int tid = threadIdx.x;
    const float nan = __builtin_nanf("");
    const float ninf = -__builtin_inff();
    const int64_t V = b.V;
    const int64_t t = ri.claimed;
    const bool valid = (t >= 0 && t < V);

    // Combine the 256 partial (reference, sum) pairs in a fixed order.  `ref` is the exponent a thread's terms were
    // taken against: they are 2^(x c - ref), with ref the ROUNDED product of the thread's reference logit and c.  The
    // common reference is the largest of them, and a thread's scale is 2^(ref - M) from the difference of the two
    // rounded numbers: forming it from the reference logits instead, as 2^((m - M) c), would be off by the rounding
    // of m c - half a unit in its last place, 1e-5 when |m| / T runs into the hundreds, a different amount in every
    // thread.
    const float M = block_max(ref, lds_f);  // (-inf: every entry masked; +inf or NaN: a +inf or NaN logit)
    const float neg_Mc = -M;
    // a thread that saw only masked entries has ref = -inf and Z = 0: its scale is 2^-inf = 0
    const double Zs = Z * (double)fast_exp2(ref - M);
    const double Ps = (refP > ninf) ? P * (double)fast_exp2(refP - M) : 0.0;
    const double Ztot = block_sum_f64(Zs, lds_d);
    const double Ptot = block_sum_f64(Ps, lds_d);

    // Regenerated uniform: stream 1, vocabulary index 0.
    uint32_t r[4];
    noise_block(ri.key, ri.pos, ri.seq, kStreamIpt, 0u, r);
    const float u = uniform_from_bits(r[0]);

    // Z is NaN if a NaN logit was seen, +inf if a +inf logit was (then M = +inf); M = -inf if every
    // entry is masked.  All of these make the distribution undefined.
    const bool bad = !(Ztot > 0.0) || !(Ztot < (double)__builtin_inff()) || !(M < __builtin_inff()) || !(M > ninf);

    float a = nan, bb = nan, d = nan;
    double ad = 0.0, bd = 0.0;
    bool match = false;
    if (valid && !bad) {
        const double et = (double)fast_exp2(__fmaf_rn(Elem<DT>::to_float(x_row[t]), c, neg_Mc));
        const double ud = (double)u;
        ad = Ptot / Ztot;
        bd = (Ptot + et) / Ztot;
        a = (float)ad;
        bb = (float)bd;
        d = (float)fmax(fmax(ad - ud, ud - bd), 0.0);
        match = (ad <= ud) && (ud < bd);
    }

    uint32_t f = 0;
    if (!valid) f |= kFlagInvalidClaim;
    if (bad) f |= kFlagNonfinite;
    if (match) f |= kFlagMatch;

    int32_t tok = match ? (int32_t)t : -1;
    if (o.ipt_token != nullptr && !match && !bad) {
        // Second pass: walk the CDF in token order until it exceeds u * Z.
        f |= kFlagSlowPath;
        const double target = (double)u * Ztot;
        double before = 0.0;  // mass of all entries before the current step
        if (tid == 0) *lds_tok = -1;
        __syncthreads();
        for (int64_t step0 = 0; step0 < V; step0 += (int64_t)kBlock * E) {
            const int64_t base = step0 + (int64_t)tid * E;
            float e[E];
            if (base < V) {
                float x[E];
                load_elems<DT, ALIGNED>(x_row, base, V, x);
#pragma unroll
                for (int j = 0; j < E; ++j) e[j] = fast_exp2(__fmaf_rn(x[j], c, neg_Mc));
            } else {
#pragma unroll
                for (int j = 0; j < E; ++j) e[j] = 0.0f;
            }
            const double ls = (double)tree_sum<E>(e);
            double total;
            const double incl = block_inclusive_scan(ls, lds_d, total);
            if (before + total > target) {  // uniform: the token is inside this step
                const double excl = before + (incl - ls);
                if (excl <= target && before + incl > target) {  // exactly one thread
                    double cacc = excl;
                    int32_t found = -1;
#pragma unroll
                    for (int j = 0; j < E; ++j) {
                        cacc += (double)e[j];
                        if (found < 0 && cacc > target) found = (int32_t)(base + j);
                    }
                    if (found < 0) found = (int32_t)((base + E - 1 < V) ? base + E - 1 : V - 1);
                    *lds_tok = found;
                }
                break;
            }
            before += total;
        }
        __syncthreads();
        tok = *lds_tok;
        if (tok < 0) tok = (int32_t)(V - 1);  // u * Z at or beyond the accumulated total
    }

    if (tid == 0) {
        o.dist[row] = d;
        if (o.cdf_lo) o.cdf_lo[row] = a;
        if (o.cdf_hi) o.cdf_hi[row] = bb;
        if (o.u) o.u[row] = u;
        if (o.ipt_token) o.ipt_token[row] = bad ? -1 : tok;
        if (o.log_mass)
            o.log_mass[row] =
                (valid && !bad) ? (float)gaussian_log_mass(ad, bd, (double)u, o.sigma, o.eps) : nan;
        if (o.logit_rank) o.logit_rank[row] = valid ? above : -1;
        o.flags[row] = (uint8_t)f;
    }
}

__device__ __forceinline__ bool ipt_row_rejected(const RowInfo &ri, int64_t row, const IptOutputs &o)
{
    if (ri.seq_ok && ri.temp_ok) return false;
    if (threadIdx.x == 0) {
        const float nan = __builtin_nanf("");
        o.dist[row] = nan;
        if (o.cdf_lo) o.cdf_lo[row] = nan;
        if (o.cdf_hi) o.cdf_hi[row] = nan;
        if (o.u) o.u[row] = nan;
        if (o.ipt_token) o.ipt_token[row] = -1;
        if (o.log_mass) o.log_mass[row] = nan;
        if (o.logit_rank) o.logit_rank[row] = -1;
        o.flags[row] = (uint8_t)(ri.seq_ok ? kFlagNonfinite : kFlagInvalidClaim);
    }
    return true;
}

// Online softmax statistics per thread: m = the lane's reference logit (see terms()), Z = sum of 2^((x - m) c).  Each
// vector's terms are summed as an fp32 tree and the vector sums are accumulated in fp64, so the CDF
// values are good to fp32 rounding.  (P, with its own reference) is the same sum restricted to v < t.  Vector rounds
// that lie wholly below the claimed token, wholly above it, and are full need no per-entry test:
// the prefix is simply a snapshot of Z taken between the two groups of rounds.  Only the round
// that holds the claimed token and the last, partly filled round look at indices.
constexpr float kRefLift = 16.0f;  // see IptStream::terms()

template <int DT>
struct IptStream {
    typedef typename Elem<DT>::type elt_t;
    static constexpr int E = Elem<DT>::kPerVec;

    const elt_t *x_row;
    int64_t V, t;
    bool valid, want_rank;
    float c;   // exponent scale: exp(x/T) = 2^(x c)
    float xt;  // claimed token's raw logit (for the logit rank)
    int tid;
    // running state
    float m, neg_mc, neg_mcP;
    double Z, P;
    uint32_t above;       // wave-uniform ballot counts (full rounds)
    uint32_t lane_above;  // per-lane counts (careful rounds)

    __device__ __forceinline__ IptStream(const RowInfo &ri, const elt_t *x_row_, int64_t V_, bool want_rank_)
        : x_row(x_row_), V(V_), t(ri.claimed), want_rank(want_rank_), c(kLog2e / ri.T), tid((int)threadIdx.x)
    {
        valid = (t >= 0 && t < V);
        xt = valid ? Elem<DT>::to_float(x_row[t]) : __builtin_nanf("");
        m = -__builtin_inff();
        neg_mc = __builtin_inff();  // no reference yet: see terms()
        neg_mcP = __builtin_inff();
        Z = 0.0;
        P = 0.0;
        above = 0;
        lane_above = 0;
    }

    static __device__ __forceinline__ void unpack(ipt_u32x4 q, float x[E])
    {
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
        if (DT == 0) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                x[2 * j] = __uint_as_float(w[j] << 16);
                x[2 * j + 1] = __uint_as_float(w[j] & 0xFFFF0000u);
            }
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) x[j] = __uint_as_float(w[j]);
        }
    }

    // Exponentials of one vector relative to the lane's reference point m.  The reference is the maximum of the
    // first vector the lane met and moves only when it has to: the sum of the eight terms is needed anyway,
    // and as long as it stays below 2^64 no term has overflowed (an entry more than 64 / c above m, or a lane
    // that has no reference yet -- neg_mc = +inf makes every term inf or NaN -- sends the sum over the limit).
    // Nothing is lost by a reference below the running maximum: fp32 terms keep their relative precision at any
    // scale, the sums are fp64, and every lane's sum is rescaled to the row's common reference at the end.
    // Returns the sum of the terms.
    __device__ __forceinline__ float terms(const float x[E], float e[E])
    {
#pragma unroll
        for (int j = 0; j < E; ++j) e[j] = fast_exp2(__fmaf_rn(x[j], c, neg_mc));
        float sum = tree_sum<E>(e);
        if (__builtin_amdgcn_ballot_w64(!(sum <= 0x1p64f)) != 0ull) {
            asm volatile("" ::: "memory");  // keep this a real, rarely taken branch
            if (!(sum <= 0x1p64f)) {
                float m8;
                if (E == 8)
                    m8 = max3_raw(max3_raw(x[0], x[1], x[2]), max3_raw(x[3], x[4], x[5]), max3_raw(x[6 % E], x[7 % E], x[7 % E]));
                else
                    m8 = max3_raw(max3_raw(x[0], x[1], x[2]), x[3], x[3]);
                if (m8 > m) {  // (m = -inf: Z is still 0 and stays 0)
                    // The reference exponent is put kRefLift above the vector's largest: an fp32 exponent is good to
                    // half a unit in its last place, 1e-6 at 16 and beyond, and the entries that lie far above a
                    // lane's first vector - the few tokens that carry the mass of a peaked row - are the ones whose
                    // terms have to be exact; the many small ones below average their roundings out.
                    const float moved = -(m8 * c + kRefLift);
                    Z *= (double)fast_exp2(moved - neg_mc);  // from the old rounded reference to the new one (see ipt_finish)
                    m = m8;
                    neg_mc = moved;
                }
                // a lane that has met only masked entries keeps m = -inf; its terms are 2^(-inf + 0) = 0
                const float shift = (m > -__builtin_inff()) ? neg_mc : 0.0f;
#pragma unroll
                for (int j = 0; j < E; ++j) e[j] = fast_exp2(__fmaf_rn(x[j], c, shift));
                sum = tree_sum<E>(e);
            }
        }
        return sum;
    }

    // a full round: every lane holds a complete vector, no index tests
    __device__ __forceinline__ void fast_round(ipt_u32x4 q)
    {
        float x[E], e[E];
        unpack(q, x);
        if (want_rank) {  // logit rank: one compare per entry, counted with ballots
            uint32_t n = 0;
#pragma unroll
            for (int j = 0; j < E; ++j) n += __builtin_popcountll(__builtin_amdgcn_ballot_w64(x[j] > xt));
            above += n;
        }
        Z += (double)terms(x, e);
    }

    // everything seen so far lies below the claimed token
    __device__ __forceinline__ void snapshot()
    {
        P = Z;
        neg_mcP = neg_mc;
    }

    // the exponents the sums Z and P were taken against (-inf: no reference yet, the sum is 0), for ipt_finish
    __device__ __forceinline__ float ref() const { return -neg_mc; }
    __device__ __forceinline__ float refP() const { return -neg_mcP; }

    // a round that needs index tests: the one holding the claimed token and the last, ragged one.
    // `q` must have been loaded for every lane whose first entry v0 is below V.
    __device__ __forceinline__ void careful_round(ipt_u32x4 q, int round, bool prefix_open)
    {
        const int64_t v0 = ((int64_t)round * kBlock + tid) * E;
        if (v0 < V) {
            float x[E], e[E];
            unpack(q, x);
#pragma unroll
            for (int j = 0; j < E; ++j)
                if (v0 + j >= V) x[j] = -__builtin_inff();
            if (want_rank) {  // divergent here: this lane's own count, the wave sums come at the end
                uint32_t n = 0;
#pragma unroll
                for (int j = 0; j < E; ++j) n += (uint32_t)(x[j] > xt);
                lane_above += n;
            }
            const float sum = terms(x, e);
            if (prefix_open) {
                float pre = 0.0f;
#pragma unroll
                for (int j = 0; j < E; ++j)
                    if (v0 + j < t) pre += e[j];
                P = Z + (double)pre;
                neg_mcP = neg_mc;
            }
            Z += (double)sum;
        } else if (prefix_open) {
            P = Z;
            neg_mcP = neg_mc;
        }
    }

    // does lane `tid` have a vector (possibly partial) in this round?
    __device__ __forceinline__ bool has_vector(int round) const
    {
        return ((int64_t)round * kBlock + tid) * E < V;
    }

    __device__ __forceinline__ int32_t total_above(int32_t *lds_rank)
    {
        if (!want_rank) return 0;
        const int32_t mine = (int32_t)lane_above + ((tid & 63) == 0 ? (int32_t)above : 0);
        return block_sum_i32(mine, lds_rank);
    }
};

}  // namespace difr
