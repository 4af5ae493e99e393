// Token-IPT-DiFR row kernel: regenerate the seeded uniform u, form p = softmax(x / T)
// and its CDF in ascending token order, and report the claimed token's interval
// [a, b) = [Fbar_{t-1}, Fbar_t), the distance of u from it, and optionally the Gaussian
// log-mass and the honest sampler's token  min{ v : C_v > u }.
// (Sec. 3.2 softmax and IPT sampler; Sec. 6.2 and the appendix algorithm
// "convolved Gaussian score".)
//
// One workgroup per token row, one streaming pass: every thread keeps an online
// (max, sum) pair for the exponentials it has seen, plus a snapshot of its sum at the
// point where its walk crosses the claimed token, which is its share of the prefix
// sum_{v < t} e_v.  Nothing of size V is stored.  Only when the honest sampler's token
// is asked for and differs from the claim is the row read a second time (block scan).
#include "difr_device.hpp"
#include "difr_host.hpp"

namespace difr {

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
                                           const typename Elem<DT>::type *x_row, float c, float m, double Z,
                                           double P, float mP, int32_t above, const IptOutputs &o, float *lds_f,
                                           double *lds_d, int32_t *lds_tok)
{
    constexpr int E = Elem<DT>::kPerVec;
    const int tid = threadIdx.x;
    const float nan = __builtin_nanf("");
    const float ninf = -__builtin_inff();
    const int64_t V = b.V;
    const int64_t t = ri.claimed;
    const bool valid = (t >= 0 && t < V);

    // Combine the 256 partial (max, sum) pairs in a fixed order.
    const float M = block_max(m, lds_f);
    const float neg_Mc = -(M * c);
    // a thread that saw only masked entries has m = -inf and Z = 0: its scale is 2^-inf = 0
    const double Zs = Z * (double)fast_exp2((m - M) * c);
    const double Ps = (mP > ninf) ? P * (double)fast_exp2((mP - M) * c) : 0.0;
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

    float m = ninf, neg_mc = 0.0f, mP = ninf;
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
            Z *= (double)fast_exp2((m - m8) * c);
            m = m8;
            neg_mc = -(m8 * c);
        }
#pragma unroll
        for (int j = 0; j < E; ++j) e[j] = fast_exp2(__fmaf_rn(x[j], c, neg_mc));
        float pre = 0.0f;
#pragma unroll
        for (int j = 0; j < E; ++j)
            if (base + j < tcut) pre += e[j];
        if (base < tcut) {
            P = Z + (double)pre;
            mP = m;
        }
        Z += (double)tree_sum<E>(e);
    }
    above = block_sum_i32(above, lds_rank);
    ipt_finish<DT, false>(b, ri, row, x_row, c, m, Z, P, mP, above, o, lds_f, lds_d, &lds_tok);
}

// Streaming kernel for 16-byte aligned rows.
//
// Online softmax statistics per thread: m = running maximum logit, Z = sum of 2^((x - m) c).  Each
// vector's terms are summed as an fp32 tree and the vector sums are accumulated in fp64, so the CDF
// values are good to fp32 rounding.  (P, mP) is the same sum restricted to v < t.  Vector rounds
// that lie wholly below the claimed token, wholly above it, and are full need no per-entry test:
// the prefix is simply a snapshot of Z taken between the two groups of rounds.  Only the round
// that holds the claimed token and the last, partly filled round look at indices.
template <int DT>
__global__ __launch_bounds__(kBlock) void ipt_score_kernel(RowBatch b, IptOutputs o)
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
    const bool valid = (t >= 0 && t < V);

    float m = ninf, neg_mc = 0.0f, mP = ninf;
    double Z = 0.0, P = 0.0;
    // logit rank (Sec. 7.1): entries whose raw logit exceeds the claimed token's, counted per wave
    // with ballots so that it costs one compare per entry and only when asked for
    __shared__ int32_t lds_rank[kWaves];
    const bool want_rank = o.logit_rank != nullptr;
    const float xt = valid ? Elem<DT>::to_float(x_row[t]) : __builtin_nanf("");
    uint32_t above = 0;

    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const char *row_bytes = reinterpret_cast<const char *>(x_row);
    const uint32_t lane_off = (uint32_t)tid * 16u;
    auto load_round = [&](int round) {
        return __builtin_nontemporal_load(
            reinterpret_cast<const u32x4 *>(row_bytes + (size_t)round * (kBlock * 16) + lane_off));
    };
    auto unpack = [&](u32x4 q, float x[E]) {
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
    };
    // exponentials of one vector relative to the (possibly raised) running maximum
    auto terms = [&](const float x[E], float e[E]) {
        float m8;
        if (E == 8)
            m8 = max3_raw(max3_raw(x[0], x[1], x[2]), max3_raw(x[3], x[4], x[5]), max3_raw(x[6], x[7], x[7]));
        else
            m8 = max3_raw(max3_raw(x[0], x[1], x[2]), x[3], x[3]);
        // Rebase the running sum when a lane meets a new maximum (m = -inf: Z is still 0 and stays 0).
        // After the first few vectors no lane does, so the test is one compare and a scalar branch.
        if (__builtin_amdgcn_ballot_w64(m8 > m) != 0ull) {
            asm volatile("" ::: "memory");  // keep this a real branch: the body must not be speculated
            if (m8 > m) {
                Z *= (double)fast_exp2((m - m8) * c);
                m = m8;
                neg_mc = -(m8 * c);
            }
        }
        // while only masked entries have been seen neg_mc is 0, so the exponent stays -inf, not NaN
#pragma unroll
        for (int j = 0; j < E; ++j) e[j] = fast_exp2(__fmaf_rn(x[j], c, neg_mc));
    };
    auto count_above = [&](const float x[E]) {
        uint32_t n = 0;
#pragma unroll
        for (int j = 0; j < E; ++j) n += __builtin_popcountll(__builtin_amdgcn_ballot_w64(x[j] > xt));
        above += n;
    };
    auto fast_round = [&](u32x4 q) {
        float x[E], e[E];
        unpack(q, x);
        if (want_rank) count_above(x);
        terms(x, e);
        Z += (double)tree_sum<E>(e);
    };
    // a round that needs index tests: the one holding the claimed token and the last, ragged one
    uint32_t lane_above = 0;
    auto careful_round = [&](int round, bool prefix_open) {
        const int64_t v0 = ((int64_t)round * kBlock + tid) * E;
        if (v0 < V) {
            float x[E], e[E];
            unpack(load_round(round), x);
#pragma unroll
            for (int j = 0; j < E; ++j)
                if (v0 + j >= V) x[j] = ninf;
            if (want_rank) {  // divergent here: add this lane's own count, the wave sum comes at the end
                uint32_t n = 0;
#pragma unroll
                for (int j = 0; j < E; ++j) n += (uint32_t)(x[j] > xt);
                lane_above += n;
            }
            terms(x, e);
            if (prefix_open) {
                float pre = 0.0f;
#pragma unroll
                for (int j = 0; j < E; ++j)
                    if (v0 + j < t) pre += e[j];
                P = Z + (double)pre;
                mP = m;
            }
            Z += (double)tree_sum<E>(e);
        } else if (prefix_open) {
            P = Z;
            mP = m;
        }
    };
    auto stream = [&](int r0, int r1) {  // full rounds [r0, r1) with one vector kept in flight
        if (r0 >= r1) return;
        u32x4 q_next = load_round(r0);
        for (int round = r0; round < r1; ++round) {
            const u32x4 q = q_next;
            if (round + 1 < r1) q_next = load_round(round + 1);
            fast_round(q);
        }
    };

    const int64_t nvec_total = (V + E - 1) / E;                       // the last vector may be partial
    const int full_rounds = (int)((V / E) / kBlock);                  // rounds of 256 complete vectors
    const int n_rounds = (int)((nvec_total + kBlock - 1) / kBlock);   // full_rounds or full_rounds + 1
    const int round_t = valid ? (int)((t / E) / kBlock) : -1;

    if (valid && round_t < full_rounds) {
        stream(0, round_t);
        careful_round(round_t, true);
        stream(round_t + 1, full_rounds);
        if (n_rounds > full_rounds) careful_round(full_rounds, false);
    } else {
        stream(0, full_rounds);
        if (valid) {  // everything so far lies below the claimed token
            P = Z;
            mP = m;
        }
        if (n_rounds > full_rounds) careful_round(full_rounds, valid);
    }
    int32_t total_above = 0;
    if (want_rank) {  // wave-uniform ballot counts (lane 0 carries them) plus the per-lane counts of careful rounds
        const int32_t mine = (int32_t)lane_above + ((tid & 63) == 0 ? (int32_t)above : 0);
        total_above = block_sum_i32(mine, lds_rank);
    }
    ipt_finish<DT, true>(b, ri, row, x_row, c, m, Z, P, mP, total_above, o, lds_f, lds_d, &lds_tok);
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
