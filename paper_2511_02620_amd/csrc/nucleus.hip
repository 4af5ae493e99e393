// The nucleus (top-p) filter over the WHOLE vocabulary, and Token-IPT-DiFR on the distribution it leaves
// (Sec. 3.2: the sampler's filter policy and the IPT sampler; Sec. 6.2; appendix "convolved Gaussian
// score").  K is the shortest prefix of the tokens ranked by logit (ties to the lower index) whose
// softmax(x / T) mass reaches top_p.  With no top-k in front of it K can hold tens of thousands of tokens,
// so it is not collected: the kernel finds the CUT, the last (logit, index) pair that still belongs to K,
// and membership of any token is one comparison against it.
//
// One workgroup per row, several passes over the row (it is read from HBM again each time).  Throughout, a
// token's KEY is the order-preserving integer image of its logit at the storage type's resolution (16 bits for
// bf16, formed on the packed patterns), and a bracket is a range of keys [klo, khi].
//   0    a look at the first 256 vectors: their largest entry R (the exponent reference for every mass
//        2^((x - R) c): any finite reference serves) and their smallest finite one;
//   B1   every thread adds the mass of its entries to 16 private LDS bins (no atomics, no conflicts) that divide
//        the span of LOGIT VALUES seen in step 0 evenly, values outside falling into the end bins; the same pass
//        finds the smallest and largest key of the row (NaN / +inf check, the maximum M).  The bins are combined
//        in a fixed order in fp64, their total Z fixes the target top_p * Z, and the bin in which the cumulative
//        mass from the top reaches it becomes the bracket: bin1 is monotone in the logit, so its first key is
//        found by bisection.  (If M lies so far above R that terms could overflow, the pass is repeated with
//        R = M.)
//   BC   bf16 rows whose bracket is now at most 16 logit values with many entries each (the usual case when K is
//        large: near the cut a bf16 value is shared by thousands of tokens) are finished by one counting pass:
//        per value of the bracket and per thread the number of entries, and of entries below the claimed token's
//        index; entries of equal value have equal mass, which is taken per value in fp64.  Two reads in all.
//        Every other row goes on with B2 and C:
//   B2.. the bracket's key range is divided evenly into at most 16 bins and searched in the same way, until it
//        is a single key - one logit value - or provably holds at most kNucCap entries (its mass divided by the
//        weight of its smallest key bounds their number).  Typically one or two passes;
//   C    the bracket is gathered as 64-bit composites (topn.hpp), sorted, and walked in rank order with an fp64
//        scan until the mass is reached: that entry is the cut.  A single-value bracket needs no sorting: the
//        ties enter K in index order with equal mass, so their number is a division.  The same pass sums what
//        lies above the bracket and below the claimed token's index.
// Why the first bins are laid over logit values and not over the leading key bits: the mass is spread over
// logit values, while key bits spend most of their range on exponents near zero - a search by key digits takes
// three passes in which nine entries in ten are still inside the bracket.
// Masses are fp32 terms accumulated per thread in fp32 and combined in fp64; whether a token whose
// probability is 1e-6 still falls inside K is decided with a relative accuracy of about 1e-6 of the total
// mass, which is the accuracy of the fp32 exponentials themselves.
#include "difr_device.hpp"
#include "difr_host.hpp"
#include "ipt_stream.hpp"
#include "topn.hpp"

namespace difr {

constexpr int kNucBins = 16;    // 4 key bits per pass
constexpr int kNucCap = 2048;   // entries gathered and sorted at the end

constexpr int kNucRawBytes = kNucBins * kBlock * 4;  // LDS the multi-pass search needs from its caller
static_assert(kNucRawBytes >= kNucCap * (int)sizeof(uint64_t), "gather buffer must fit the bin memory");

// One row by the multi-pass search described above.  `raw`: kNucRawBytes of LDS, 16-byte aligned (mass bins
// [bin][thread] during the search; the gather buffer afterwards).  All 256 threads of the workgroup call it.
template <int DT>
__device__ __forceinline__ void nucleus_row_multipass(const RowBatch &b, float top_p, const IptOutputs &o,
                                                      int32_t *__restrict__ kept_out, float *__restrict__ tau_out,
                                                      unsigned char *raw)
{
    typedef typename Elem<DT>::type elt_t;
    constexpr int E = Elem<DT>::kPerVec;
    __shared__ double part_m[16][kNucBins];
    __shared__ double bin_m[kNucBins];
    __shared__ float lds_f[kWaves];
    __shared__ double lds_d[kWaves];
    __shared__ int32_t lds_i[kWaves];
    __shared__ int32_t s_fill;
    __shared__ float s_xtau;
    __shared__ double s_mass_in;
    __shared__ uint64_t s_cut;
    float *mass = reinterpret_cast<float *>(raw);
    uint64_t *buf = reinterpret_cast<uint64_t *>(raw);

    const int64_t row = blockIdx.x;
    const RowInfo ri = load_row_info(b, row);
    const int tid = threadIdx.x;
    const float nan = __builtin_nanf("");
    const float ninf = -__builtin_inff();
    const bool want_ipt = o.dist != nullptr;
    auto give_up = [&](uint32_t flag, int32_t kept) __attribute__((always_inline)) {  // uniform over the workgroup
        if (tid == 0) {
            if (want_ipt) {
                o.dist[row] = nan;
                if (o.cdf_lo) o.cdf_lo[row] = nan;
                if (o.cdf_hi) o.cdf_hi[row] = nan;
                if (o.u) o.u[row] = nan;
                if (o.log_mass) o.log_mass[row] = nan;
                o.flags[row] = (uint8_t)flag;
            }
            if (kept_out) kept_out[row] = kept;
            if (tau_out) tau_out[row] = nan;
        }
    };
    if (!ri.seq_ok || !ri.temp_ok) {
        give_up(ri.seq_ok ? kFlagNonfinite : kFlagInvalidClaim, 0);
        return;
    }
    const int64_t V = b.V;
    const int64_t t = ri.claimed;
    const bool valid = t >= 0 && t < V;
    const elt_t *x_row = reinterpret_cast<const elt_t *>(b.logits) + row * b.ld;
    const float c = kLog2e / ri.T;

    // One pass over the row: f(q, base) for every 16-byte vector of this thread, with the next vector already
    // requested while the current one is worked on.  Entries past the end of the row read as -inf.
    const int32_t nvec = (int32_t)((V + E - 1) / E);  // V < 2^31
    const uint32_t V32 = (uint32_t)V;
    auto fetch = [&](int32_t vec) { return *reinterpret_cast<const ipt_u32x4 *>(x_row + (size_t)vec * E); };
    // the last vector of a ragged row: entries past the end become -inf
    auto ragged_patched = [&](ipt_u32x4 q, uint32_t base) __attribute__((always_inline)) {
        if (base + E > V32) {
            uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
            for (int j = 0; j < E; ++j) {
                if (base + j < V32) continue;
                if (DT == 0)
                    w[j >> 1] = (j & 1) ? ((w[j >> 1] & 0x0000FFFFu) | 0xFF800000u) : ((w[j >> 1] & 0xFFFF0000u) | 0x0000FF80u);
                else
                    w[j] = 0xFF800000u;
            }
            q = ipt_u32x4{w[0], w[1], w[2], w[3]};
        }
        return q;
    };
    auto for_each_vector = [&](auto &&f) __attribute__((always_inline)) {
        int32_t vec = tid;
        ipt_u32x4 q_next = ipt_u32x4{0u, 0u, 0u, 0u};
        if (vec < nvec) q_next = fetch(vec);
        while (vec < nvec) {
            ipt_u32x4 q = q_next;
            const int32_t next = vec + kBlock;
            if (next < nvec) q_next = fetch(next);
            const uint32_t base = (uint32_t)vec * E;
            q = ragged_patched(q, base);
            f(q, base);
            vec = next;
        }
    };
    // Order keys of a vector at the resolution the storage type has: equal logits have equal keys, a larger logit
    // a larger key.  -0 and +0 are the same logit (ties go by index, not by sign), so they share a key.
    // bf16: two 16-bit keys per dword, formed on the packed patterns: 0x8000 + magnitude for a clear sign bit,
    // 0x8000 - magnitude for a set one.  fp32: float_order_bits of the value with -0 read as +0.
    auto keys_of = [&](const ipt_u32x4 &q, uint32_t (&kw)[4]) __attribute__((always_inline)) {
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (DT == 0) {
                typedef int16_t i16x2_t __attribute__((ext_vector_type(2)));
                typedef uint16_t u16x2_t __attribute__((ext_vector_type(2)));
                const uint32_t sg = __builtin_bit_cast(uint32_t, __builtin_bit_cast(i16x2_t, w[i]) >> 15);  // 0xFFFF where the sign bit is set
                const uint32_t a = (w[i] & 0x7FFF7FFFu) ^ sg ^ 0x80008000u;  // 0x8000 + m, or 0x7FFF - m
                kw[i] = __builtin_bit_cast(uint32_t, __builtin_bit_cast(u16x2_t, a) - __builtin_bit_cast(u16x2_t, sg));  // (- 0xFFFF = + 1)
            } else {
                kw[i] = float_order_bits(__uint_as_float(w[i]) + 0.0f);
            }
        }
    };
    auto key_of_value = [&](float x) __attribute__((always_inline)) {  // the same key from a single value
        if (DT != 0) return float_order_bits(x + 0.0f);
        const uint32_t b = __float_as_uint(x) >> 16, m = b & 0x7FFFu;
        return (b & 0x8000u) ? 0x8000u - m : 0x8000u + m;
    };
    auto value_of = [&](const ipt_u32x4 &q, int j) __attribute__((always_inline)) {
        const uint32_t w[4] = {q.x, q.y, q.z, q.w};
        if (DT == 0) return __uint_as_float((j & 1) ? (w[j >> 1] & 0xFFFF0000u) : (w[j >> 1] << 16));
        return __uint_as_float(w[j]);
    };

    // ---- a look at the first 256 vectors: their largest entry R and their smallest finite one.  R is the exponent
    //      reference: any finite reference serves (fp32 terms keep their relative precision at every scale, the sums
    //      are fp64); the row maximum M itself comes out of the first search pass, and that pass is repeated with
    //      R = M in the rare case that M lies so far above R that terms could overflow.  The two together tell the
    //      first search pass where to put its bins.  A first round without a usable value takes a pass of its own. ----
    float R = ninf, lo_s = __builtin_inff();
    auto look = [&](const ipt_u32x4 &q) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < E; ++j) {
            const float v = value_of(q, j);
            R = fmaxf(R, v);  // NaNs drop out; the first search pass finds them
            if (v > ninf) lo_s = fminf(lo_s, v);
        }
    };
    if (tid < nvec) {
        look(ragged_patched(fetch(tid), (uint32_t)tid * E));  // (ragged only in a row shorter than one round)
    }
    R = block_max(R, lds_f);
    if (!(R > ninf && R < __builtin_inff())) {  // uniform
        R = ninf;
        lo_s = __builtin_inff();
        for_each_vector([&](const ipt_u32x4 &q, uint32_t) { look(q); });
        R = block_max(R, lds_f);
        if (!(R > ninf && R < __builtin_inff())) {  // every entry masked, or a +inf
            give_up(kFlagNonfinite | (valid ? 0u : kFlagInvalidClaim), 0);
            return;
        }
    }
    lo_s = -block_max(-lo_s, lds_f);  // finite and <= R, since R is
    // A mass is 2^((x - R) c64), c64 = log2(e) / T.  The difference x - R comes first: for the entries that carry the
    // mass it is small and exact, so what the fp32 exponent loses is in proportion to it (an exponent formed as
    // x c - R c would carry the rounding of two products of the size of R c, 1e-5 and more when |R| / T is in the
    // hundreds, and the masses that decide the cut - fp32 in the search, fp64 in its last step - would disagree by
    // as much).  The constant is taken in two fp32 pieces, so that what an exponent loses to ITS rounding (a tilt of
    // up to 6e-8 |x - R| c over the whole row, all to one side) is gone as well; the large piece is rounded DOWN, which
    // makes the small one positive: a masked entry, -inf, then gives -inf in both products and a mass of zero with no
    // special case.
    const double c64 = 1.4426950408889634074 / (double)ri.T;
    float c_hi = (float)c64;
    if ((double)c_hi >= c64 && c_hi > 1.0e-30f) c_hi = __uint_as_float(__float_as_uint(c_hi) - 1u);
    const float c_lo = fmaxf((float)(c64 - (double)c_hi), 1.1754944e-38f);
    auto mass_of = [&](float x) __attribute__((always_inline)) {
        const float d = x - R;
        return fast_exp2(__fmaf_rn(d, c_hi, d * c_lo));
    };
    // (the same real number in fp64: for the few masses of the last step)
    auto mass_of_f64 = [&](float x) __attribute__((always_inline)) { return exp2(((double)x - (double)R) * c64); };

    // ---- passes B: search for the bracket [klo, khi] of keys that holds the cut ----
    // Keys are the order-preserving images of the logits at the storage type's resolution (16 bits for bf16).
    constexpr uint32_t kKeyPosInf = DT == 0 ? 0xFF80u : 0xFF800000u;  // keys >= this: +inf or a NaN, sign clear
    constexpr uint32_t kKeyNegInf = DT == 0 ? 0x0080u : 0x007FFFFFu;  // -inf; keys < this: a NaN with the sign bit set
    auto value_of_key = [&](uint32_t k) __attribute__((always_inline)) {
        if (DT != 0) return float_from_order_bits(k);
        return __uint_as_float((k >= 0x8000u ? k - 0x8000u : 0x8000u | (0x8000u - k)) << 16);
    };
    auto key_of = [&](const uint32_t (&kw)[4], int j) __attribute__((always_inline)) {
        if (DT == 0) return (j & 1) ? (kw[j >> 1] >> 16) : (kw[j >> 1] & 0xFFFFu);
        return kw[j];
    };
    // block-wide maximum / minimum of a key
    auto block_max_key = [&](uint32_t k) __attribute__((always_inline)) {
        uint32_t m = k;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, off, 64));
        __syncthreads();
        if ((tid & 63) == 0) lds_i[tid >> 6] = (int32_t)m;
        __syncthreads();
        return max(max((uint32_t)lds_i[0], (uint32_t)lds_i[1]), max((uint32_t)lds_i[2], (uint32_t)lds_i[3]));
    };
    auto block_min_key = [&](uint32_t k) __attribute__((always_inline)) {
        uint32_t m = k;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) m = min(m, (uint32_t)__shfl_xor((int)m, off, 64));
        __syncthreads();
        if ((tid & 63) == 0) lds_i[tid >> 6] = (int32_t)m;
        __syncthreads();
        return min(min((uint32_t)lds_i[0], (uint32_t)lds_i[1]), min((uint32_t)lds_i[2], (uint32_t)lds_i[3]));
    };
    // the 256 x 16 per-thread bins -> bin_m[16], in a fixed order, fp64; ends with a barrier
    auto combine_bins = [&]() __attribute__((always_inline)) {
        __syncthreads();
        {
            const int k = tid & 15, grp = tid >> 4;
            double sm = 0.0;
#pragma unroll
            for (int i = 0; i < 16; ++i) sm += (double)mass[k * kBlock + grp * 16 + i];
            part_m[grp][k] = sm;
        }
        __syncthreads();
        if (tid < kNucBins) {
            double sm = 0.0;
#pragma unroll
            for (int grp = 0; grp < 16; ++grp) sm += part_m[grp][tid];
            bin_m[tid] = sm;
        }
        __syncthreads();
    };
    // a thread's bins are its own: plain read-modify-write (LDS float atomics run many times slower here)
    auto add_mass = [&](uint32_t bin, float e) __attribute__((always_inline)) { mass[(int)bin * kBlock + tid] += e; };
    auto clear_bins = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int k = 0; k < kNucBins; ++k) mass[k * kBlock + tid] = 0.0f;
    };
    double mass_above = 0.0, target = 0.0;
    // from the top: the first bin in which the cumulative mass reaches the target (every thread walks the same 16
    // values in the same order); what lies above it is added to mass_above
    auto select_bin = [&]() __attribute__((always_inline)) {
        int sel = 0;
        for (int k = kNucBins - 1; k >= 0; --k) {
            if (mass_above + bin_m[k] >= target || k == 0) {
                sel = k;
                break;
            }
            mass_above += bin_m[k];
        }
        return sel;
    };

    // First pass: every entry counts (the total mass Z fixes the target), and the 16 bins divide the span of
    // LOGIT VALUES seen in the first round evenly - the mass is spread over logit values, not over key bits, which
    // spend most of their range on exponents near zero.  bin1 is monotone in the logit, so each bin is a range of
    // keys; values outside the span seen in the first round fall into the end bins.
    uint32_t klo, khi;
    double bracket_mass;  // mass of the entries with keys in [klo, khi]
    while (true) {
        float sc = (R > lo_s) ? 16.0f / (R - lo_s) : 0.0f;
        if (!(sc > 0.0f && sc < 1.0e30f)) sc = 1.0e-30f;  // no span to divide: every finite value lands in bin 0
        const float off = -(lo_s * sc);
        auto bin1 = [&](float x) __attribute__((always_inline)) {  // (clamped before the conversion: always in range)
            return (uint32_t)(int)__builtin_amdgcn_fmed3f(__fmaf_rn(x, sc, off), 0.0f, 15.0f);
        };
        clear_bins();
        // Largest and smallest key met.  bf16: three packed extremes of the raw bit patterns (of the even and of the
        // odd entries) tell as much, at three instructions per two entries: the largest pattern as signed 16-bit is
        // the largest entry that is not negative (or +inf, or a NaN with the sign clear), the largest as unsigned the
        // most negative one (or -inf, or a NaN with the sign set), the smallest as unsigned the negative entry nearest
        // to zero if all are negative, else the smallest non-negative one.
        typedef uint16_t u16x2_t __attribute__((ext_vector_type(2)));
        typedef int16_t i16x2_t __attribute__((ext_vector_type(2)));
        uint32_t kmax = 0u, kmin = 0xFFFFFFFFu;
        uint32_t smax = 0x80008000u, umax = 0u, umin = 0xFFFFFFFFu;
        for_each_vector([&](const ipt_u32x4 &q, uint32_t) {
            if (DT == 0) {
                const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    smax = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(i16x2_t, smax), __builtin_bit_cast(i16x2_t, w[i])));
                    umax = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(u16x2_t, umax), __builtin_bit_cast(u16x2_t, w[i])));
                    umin = __builtin_bit_cast(uint32_t, __builtin_elementwise_min(__builtin_bit_cast(u16x2_t, umin), __builtin_bit_cast(u16x2_t, w[i])));
                }
            } else {
                uint32_t kw[4];
                keys_of(q, kw);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    kmax = max(kmax, kw[i]);
                    kmin = min(kmin, kw[i]);
                }
            }
#pragma unroll
            for (int j = 0; j < E; ++j) {
                const float x = value_of(q, j);
                add_mass(bin1(x), mass_of(x));
            }
        });
        bool sign_set_nan = false;
        if (DT == 0) {
            // (signed maximum through the unsigned reduction: flip the sign bit)
            const uint32_t sm = block_max_key(max((smax & 0xFFFFu) ^ 0x8000u, (smax >> 16) ^ 0x8000u)) ^ 0x8000u;
            const uint32_t um = block_max_key(max(umax & 0xFFFFu, umax >> 16));
            const uint32_t un = block_min_key(min(umin & 0xFFFFu, umin >> 16));
            auto key_of_pattern = [&](uint32_t p) __attribute__((always_inline)) {
                return (p & 0x8000u) ? 0x8000u - (p & 0x7FFFu) : 0x8000u + p;
            };
            sign_set_nan = um > 0xFF80u;
            kmax = key_of_pattern(sm < 0x8000u ? sm : un);  // a non-negative entry exists: the largest of them
            kmin = key_of_pattern(um >= 0x8000u ? um : un);  // a negative entry exists: the most negative of them
        } else {
            kmax = block_max_key(kmax);  // (a thread without a vector still holds the neutral values)
            kmin = block_min_key(kmin);
        }
        if (kmax >= kKeyPosInf || kmin < kKeyNegInf || sign_set_nan) {  // uniform: NaN or +inf somewhere, no distribution
            give_up(kFlagNonfinite | (valid ? 0u : kFlagInvalidClaim), 0);
            return;
        }
        const float M = value_of_key(kmax);
        if ((M - R) * c > 96.0f) {  // uniform; terms of 2^96 and more: start again from M
            R = M;
            continue;
        }
        combine_bins();
        double Z = 0.0;
        for (int k = 0; k < kNucBins; ++k) Z += bin_m[k];
        target = (double)top_p * Z;
        const uint32_t sel = (uint32_t)select_bin();
        // the keys of bin `sel`: bin1 is monotone over the keys from -inf to the largest finite one, so the first
        // key of a bin is found by bisection (every thread runs the same search)
        auto first_key_of_bin = [&](uint32_t b) __attribute__((always_inline)) {  // smallest key k with bin1 >= b
            uint32_t a = kKeyNegInf, z = kKeyPosInf;                              // answer in [a, z]
            while (a < z) {
                const uint32_t mid = a + ((z - a) >> 1);
                if (bin1(value_of_key(mid)) >= b)
                    z = mid;
                else
                    a = mid + 1;
            }
            return a;
        };
        klo = sel == 0 ? kKeyNegInf : first_key_of_bin(sel);
        khi = sel == 15 ? kKeyPosInf - 1u : first_key_of_bin(sel + 1u) - 1u;
        klo = max(klo, kmin);
        khi = min(khi, kmax);
        bracket_mass = bin_m[sel];  // clipping to [kmin, kmax] removes no entry
        __syncthreads();            // the bins are cleared or reused next
        break;
    }
    double Zk = 0.0, below = 0.0;  // mass of K; mass of the members of K below the claimed token's index
    int64_t kept = 0;
    float tau_val = nan;
    uint64_t cut = 0ull;   // sorted path: the last member of K in rank order
    int64_t n_tie = 0;     // tie path: how many of the ties belong to K
    int32_t tb = 0;        //           and how many ties lie below the claimed token's index
    bool many_ties = false;
    const uint32_t t32 = valid ? (uint32_t)t : 0u;  // an invalid claim has nothing below it (its outputs are NaN anyway)

    // bf16 rows whose bracket is a handful of logit values with many entries each (the usual case when K is large:
    // near the cut a bf16 value is shared by thousands of tokens): ONE more pass finishes the row.  Entries of equal
    // value have equal mass, so the pass only counts, per value of the bracket and per thread, the entries and those
    // of them below the claimed token's index (16 + 16 bits in one private LDS word), and sums what lies above the
    // bracket as the last pass of the general path does.  The values' masses are then taken in fp64, the value at
    // which the cumulative mass reaches the target is found by walking at most 16 of them, and it is treated as the
    // general path treats a single-value bracket: its ties enter K in index order.
    bool provably_small = false;
    {
        const double e_lo = (double)mass_of(value_of_key(klo));
        provably_small = e_lo > 0.0 && e_lo < (double)__builtin_inff() && bracket_mass <= e_lo * (double)(kNucCap - 48);
    }
    const bool by_counts = DT == 0 && khi > klo && khi - klo < (uint32_t)kNucBins && !provably_small && V <= (int64_t)(1 << 24);
    if (by_counts) {  // uniform
        const uint32_t span = khi - klo;
        uint32_t *cnt = reinterpret_cast<uint32_t *>(raw);  // [key - klo][thread]; a thread meets fewer than 2^16 entries
#pragma unroll
        for (int k = 0; k < kNucBins; ++k) cnt[k * kBlock + tid] = 0u;
        double below_above = 0.0;
        int32_t n_above = 0;
        for_each_vector([&](const ipt_u32x4 &q, uint32_t base) {
            uint32_t kw[4];
            keys_of(q, kw);
            float below_vec = 0.0f;
            // whether an entry lies below the claimed token's index is the same for a whole vector, but for the one
            // vector of the row that holds the claim (and a ragged last one is looked at entry by entry as well)
            const bool all_below = base + E <= t32;
            const bool mixed = (!all_below && base < t32) || base + E > V32;
            if (__builtin_amdgcn_ballot_w64(mixed) == 0ull) {
                const uint32_t inc = all_below ? 0x10001u : 1u;
#pragma unroll
                for (int j = 0; j < E; ++j) {
                    const uint32_t key = key_of(kw, j);
                    const uint32_t d = key - klo;
                    if (d <= span) {
                        cnt[(int)d * kBlock + tid] += inc;
                    } else if (key > khi) {
                        n_above += 1;
                        if (all_below) below_vec += mass_of(value_of(q, j));
                    }
                }
            } else {
#pragma unroll
                for (int j = 0; j < E; ++j) {
                    if (base + E > V32 && base + j >= V32) continue;  // (a ragged last vector)
                    const uint32_t key = key_of(kw, j);
                    const uint32_t d = key - klo;
                    if (d <= span) {
                        cnt[(int)d * kBlock + tid] += (base + j < t32) ? 0x10001u : 1u;
                    } else if (key > khi) {
                        n_above += 1;
                        if (base + j < t32) below_vec += mass_of(value_of(q, j));
                    }
                }
            }
            below_above += (double)below_vec;
        });
        // the 256 x 16 counters -> 16 totals of each kind (exact), through the memory of part_m
        int32_t(*part_c)[kNucBins][2] = reinterpret_cast<int32_t(*)[kNucBins][2]>(&part_m[0][0]);
        int32_t *key_cnt = reinterpret_cast<int32_t *>(&bin_m[0]);  // [16][2]
        __syncthreads();
        {
            const int k = tid & 15, grp = tid >> 4;
            int32_t all = 0, low = 0;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const uint32_t v = cnt[k * kBlock + grp * 16 + i];
                all += (int32_t)(v & 0xFFFFu);
                low += (int32_t)(v >> 16);
            }
            part_c[grp][k][0] = all;
            part_c[grp][k][1] = low;
        }
        __syncthreads();
        if (tid < 2 * kNucBins) {
            int32_t sm = 0;
#pragma unroll
            for (int grp = 0; grp < 16; ++grp) sm += part_c[grp][tid >> 1][tid & 1];
            key_cnt[tid] = sm;
        }
        __syncthreads();
        const int64_t cnt_above = (int64_t)block_sum_i32(n_above, lds_i);
        // from the top: the first value at which the cumulative mass reaches the target (every thread walks the
        // same values in the same order); the values above it belong to K whole
        double ma = mass_above, below_hi = 0.0, e_cut = 0.0;
        int64_t cnt_hi = 0;
        int jcut = -1, jlast = -1;
        for (int j = (int)span; j >= 0; --j) {
            const int64_t na = key_cnt[2 * j];
            if (na == 0) continue;
            const double e = mass_of_f64(value_of_key(klo + (uint32_t)j));
            jlast = j;
            e_cut = e;
            if (ma + e * (double)na >= target) {
                jcut = j;
                break;
            }
            ma += e * (double)na;
            cnt_hi += na;
            below_hi += e * (double)key_cnt[2 * j + 1];
        }
        many_ties = true;
        if (jcut < 0 && jlast >= 0) {  // rounding left the target just out of reach: the whole bracket
            jcut = jlast;
            const int64_t na = key_cnt[2 * jcut];
            ma -= e_cut * (double)na;
            cnt_hi -= na;
            below_hi -= e_cut * (double)key_cnt[2 * jcut + 1];
        }
        const int64_t bracket = jcut >= 0 ? (int64_t)key_cnt[2 * jcut] : 0;
        tb = jcut >= 0 ? key_cnt[2 * jcut + 1] : 0;
        n_tie = e_cut > 0.0 ? (int64_t)ceil((target - ma) / e_cut) : bracket;
        n_tie = n_tie < 1 ? 1 : n_tie;
        n_tie = n_tie > bracket ? bracket : n_tie;
        klo = khi = klo + (uint32_t)(jcut >= 0 ? jcut : 0);
        tau_val = value_of_key(klo);
        below = block_sum_f64(below_above, lds_d) + below_hi + e_cut * (double)((int64_t)tb < n_tie ? (int64_t)tb : n_tie);
        Zk = ma + e_cut * (double)n_tie;
        kept = cnt_above + cnt_hi + n_tie;
        mass_above = ma;
    } else {
    // Further passes: the bracket's key range divided evenly into at most 16 bins, until it is a single key (one
    // logit value) or provably small enough to sort.  No counts are kept: every entry of the bracket weighs at
    // least as much as the bracket's smallest key would, so mass / that weight bounds the number of entries.
    bool single_value = false;
    while (true) {
        if (khi <= klo) {  // (khi < klo cannot happen: the selected bin holds mass)
            khi = klo;
            single_value = true;
            break;
        }
        {  // (a bracket whose lower edge is -inf gives no bound)
            const double e_lo = (double)mass_of(value_of_key(klo));
            if (e_lo > 0.0 && e_lo < (double)__builtin_inff() && bracket_mass <= e_lo * (double)(kNucCap - 48)) break;
        }
        const uint32_t span = khi - klo;
        const int sh = max(0, 28 - (int)__builtin_clz(span));  // span >> sh <= 15
        clear_bins();
        for_each_vector([&](const ipt_u32x4 &q, uint32_t) {
            uint32_t kw[4];
            keys_of(q, kw);
#pragma unroll
            for (int j = 0; j < E; ++j) {
                const uint32_t d = key_of(kw, j) - klo;
                if (d <= span) add_mass(d >> sh, mass_of(value_of(q, j)));
            }
        });
        combine_bins();
        const uint32_t sel = (uint32_t)select_bin();
        bracket_mass = bin_m[sel];
        klo = klo + (sel << sh);
        khi = min(khi, klo + ((1u << sh) - 1u));
        __syncthreads();  // the bins are cleared or reused next
    }
    // A single logit value shared by the whole bracket (possibly thousands of tokens) needs no sorting: the ties
    // enter K in index order, each with the same mass, and how many of them do is a division.
    many_ties = single_value;

    // ---- pass C: gather the bracket (or count the ties below the claimed token), and sum what lies above the
    //      bracket and below the claimed token's index ----
    if (tid == 0) s_fill = 0;
    __syncthreads();
    double below_above = 0.0;  // mass of entries above the bracket with index < t
    int32_t ties_below = 0;    // many_ties: bracket entries with index < t ...
    int32_t ties = 0;          // ... and all of them
    int32_t n_above = 0;       // entries above the bracket
    const uint32_t span_c = khi - klo;
    for_each_vector([&](const ipt_u32x4 &q, uint32_t base) {
        uint32_t kw[4];
        keys_of(q, kw);
        float below_vec = 0.0f;
#pragma unroll
        for (int j = 0; j < E; ++j) {
            if (base + E > V32 && base + j >= V32) continue;  // (false for every vector but a ragged last one)
            const uint32_t key = key_of(kw, j);
            if (key - klo <= span_c) {
                if (many_ties) {
                    ties += 1;
                    ties_below += (int32_t)(base + j < t32);
                    s_xtau = value_of(q, j);  // the same value from every thread that writes it
                } else {
                    const int32_t i = atomicAdd(&s_fill, 1);
                    if (i < kNucCap) buf[i] = top_composite(value_of(q, j), (int32_t)(base + j));
                }
            } else if (key > khi) {
                n_above += 1;
                if (base + j < t32) below_vec += mass_of(value_of(q, j));
            }
        }
        below_above += (double)below_vec;
    });
    __syncthreads();
    const int64_t cnt_above = (int64_t)block_sum_i32(n_above, lds_i);

    if (many_ties) {
        tau_val = s_xtau;
        const double e_tau = mass_of_f64(tau_val);
        const int64_t bracket = (int64_t)block_sum_i32(ties, lds_i);
        n_tie = e_tau > 0.0 ? (int64_t)ceil((target - mass_above) / e_tau) : bracket;
        n_tie = n_tie < 1 ? 1 : (n_tie > bracket ? bracket : n_tie);
        tb = block_sum_i32(ties_below, lds_i);
        below = block_sum_f64(below_above, lds_d) + e_tau * (double)((int64_t)tb < n_tie ? (int64_t)tb : n_tie);
        Zk = mass_above + e_tau * (double)n_tie;
        kept = cnt_above + n_tie;
    } else {
        const int n = min(s_fill, kNucCap);
        int P = 256;
        while (P < n) P <<= 1;
        for (int i = n + tid; i < P; i += kBlock) buf[i] = 0ull;  // below every real composite
        __syncthreads();
        // bitonic sort, descending: rank order (larger logit first, then the smaller index)
        for (int k = 2; k <= P; k <<= 1) {
            for (int j = k >> 1; j > 0; j >>= 1) {
                for (int i = tid; i < P; i += kBlock) {
                    const int l = i ^ j;
                    if (l > i) {
                        const uint64_t a = buf[i], bb = buf[l];
                        const bool desc = (i & k) == 0;
                        if (desc ? (a < bb) : (a > bb)) {
                            buf[i] = bb;
                            buf[l] = a;
                        }
                    }
                }
                __syncthreads();
            }
        }
        // walk the sorted bracket: thread `tid` owns positions [tid * per, tid * per + per)
        const int per = P / kBlock;
        auto term = [&](int q) {  // mass of the thread's q-th position (0 past the end)
            const int i = tid * per + q;
            return (q < per && i < n) ? mass_of_f64(top_key(buf[i])) : 0.0;
        };
        double run = 0.0;
#pragma unroll
        for (int q = 0; q < kNucCap / kBlock; ++q) run += term(q);
        double total;
        const double before = block_inclusive_scan(run, lds_d, total) - run;
        // the first position at which the cumulative mass reaches the target: in the thread, then over the workgroup
        int32_t my_pos = 0x7FFFFFFF;
        double my_mass = 0.0, acc = before;
#pragma unroll
        for (int q = 0; q < kNucCap / kBlock; ++q) {
            acc += term(q);
            if (q < per && tid * per + q < n && my_pos == 0x7FFFFFFF && mass_above + acc >= target) {
                my_pos = tid * per + q;
                my_mass = acc;
            }
        }
        int32_t pos = my_pos;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) pos = min(pos, __shfl_xor(pos, off, 64));
        if ((tid & 63) == 0) lds_i[tid >> 6] = pos;
        __syncthreads();
        pos = min(min(lds_i[0], lds_i[1]), min(lds_i[2], lds_i[3]));
        if (pos == 0x7FFFFFFF) {  // rounding left the target just out of reach: the whole bracket
            pos = n - 1;
            if (n > 0 && pos >= tid * per && pos < tid * per + per) {
                s_mass_in = before + run;
                s_cut = buf[pos];
            }
        } else if (pos == my_pos) {
            s_mass_in = my_mass;
            s_cut = buf[pos];
        }
        if (n == 0 && tid == 0) {  // cannot happen for top_p > 0 (the selected bin is never empty); be safe
            s_mass_in = 0.0;
            s_cut = ~0ull;
        }
        __syncthreads();
        cut = s_cut;
        Zk = mass_above + s_mass_in;
        // included bracket entries below the claimed token's index
        double mine_below = 0.0;
#pragma unroll
        for (int q = 0; q < kNucCap / kBlock; ++q) {
            const int i = tid * per + q;
            if (q < per && i <= pos && i < n && (int64_t)top_index(buf[i]) < t) mine_below += term(q);
        }
        below = block_sum_f64(below_above + mine_below, lds_d);
        kept = cnt_above + (int64_t)(n > 0 ? pos + 1 : 0);
        tau_val = n > 0 ? top_key(cut) : nan;
    }
    }  // (the general path)
    const uint32_t span_c = khi - klo;  // for the sampler's token below

    if (tid == 0) {
        if (kept_out) kept_out[row] = (int32_t)kept;
        if (tau_out) tau_out[row] = tau_val;
    }
    if (!want_ipt) return;

    // ---- the interval of the claimed token (every thread forms it: whether the sampler's token has to be
    //      searched is decided by all of them) ----
    uint32_t r[4];
    noise_block(ri.key, ri.pos, ri.seq, kStreamIpt, 0u, r);
    const float u = uniform_from_bits(r[0]);
    const double ud = (double)u;
    float a = nan, bb = nan, d = nan;
    double ad = 0.0, bd = 0.0;
    bool match = false;
    const bool ok = Zk > 0.0 && Zk < (double)__builtin_inff();
    if (valid && ok) {
        const float xt = Elem<DT>::to_float(x_row[t]);
        bool in_K;
        if (many_ties) {
            const uint32_t kt = key_of_value(xt);
            in_K = kt > khi || (kt == klo && (int64_t)tb < n_tie);
        } else {
            in_K = top_composite(xt, (int32_t)t) >= cut;
        }
        const double own = in_K ? (double)mass_of(xt) : 0.0;
        ad = below / Zk;
        bd = ad + own / Zk;
        a = (float)ad;
        bb = (float)bd;
        d = (float)fmax(fmax(ad - ud, ud - bd), 0.0);
        match = (ad <= ud) && (ud < bd);
    }
    uint32_t f = 0;
    if (!valid) f |= kFlagInvalidClaim;
    if (!ok) f |= kFlagNonfinite;
    if (match) f |= kFlagMatch;

    // ---- the sampler's own token, when asked for and the claim is not it: one more pass, in vocabulary order, over
    //      the masses of the members of K until their running sum exceeds u Z_K.  A token above the bracket is a
    //      member, one inside it is if it ranks no lower than the cut (sorted bracket) or is among the first n_tie
    //      of the ties in index order; the pass ends with the step that holds the token. ----
    int32_t tok = match ? (int32_t)t : -1;
    if (o.ipt_token != nullptr && ok && !match) {  // uniform
        f |= kFlagSlowPath;
        const double goal = ud * Zk;
        double before = 0.0;       // mass of the members in the steps already walked
        int64_t ties_before = 0;   // many_ties: bracket entries in those steps
        int32_t last_member = -1;  // the thread's last member so far (rounding can leave the goal just out of reach)
        if (tid == 0) s_fill = -1;
        __syncthreads();
        for (int32_t vec0 = 0; vec0 < nvec; vec0 += kBlock) {
            const int32_t vec = vec0 + tid;
            const uint32_t base = (uint32_t)vec * E;
            ipt_u32x4 q = ipt_u32x4{0u, 0u, 0u, 0u};
            uint32_t kw[4] = {0u, 0u, 0u, 0u};
            int32_t my_ties = 0;
            if (vec < nvec) {
                q = ragged_patched(fetch(vec), base);
                keys_of(q, kw);
                if (many_ties) {
#pragma unroll
                    for (int j = 0; j < E; ++j) my_ties += (int32_t)(key_of(kw, j) - klo <= span_c);
                }
            }
            int64_t tie_rank = 0;  // many_ties: bracket entries with a smaller index than this thread's first
            if (many_ties) {       // uniform
                double tie_total;
                const double incl = block_inclusive_scan((double)my_ties, lds_d, tie_total);  // (exact: small integers)
                tie_rank = ties_before + (int64_t)(incl - (double)my_ties);
                ties_before += (int64_t)tie_total;
            }
            float e[E];
#pragma unroll
            for (int j = 0; j < E; ++j) {
                e[j] = 0.0f;
                if (vec >= nvec) continue;
                const uint32_t key = key_of(kw, j);
                bool member = key > khi;
                if (key - klo <= span_c)
                    member = many_ties ? (tie_rank++ < n_tie) : (top_composite(value_of(q, j), (int32_t)(base + j)) >= cut);
                if (member) {
                    e[j] = mass_of(value_of(q, j));
                    last_member = (int32_t)(base + j);
                }
            }
            const double ls = (double)tree_sum<E>(e);
            double total;
            const double incl = block_inclusive_scan(ls, lds_d, total);
            if (before + total > goal) {  // uniform: the token is inside this step
                const double excl = before + (incl - ls);
                if (excl <= goal && before + incl > goal) {  // exactly one thread
                    double cacc = excl;
                    int32_t found = -1;
#pragma unroll
                    for (int j = 0; j < E; ++j) {
                        cacc += (double)e[j];
                        if (found < 0 && e[j] > 0.0f && cacc > goal) found = (int32_t)(base + j);
                    }
                    s_fill = found >= 0 ? found : last_member;  // (found < 0: rounding between the two sums)
                }
                break;
            }
            before += total;
        }
        __syncthreads();
        tok = s_fill;
        if (tok < 0) {  // u Z_K at or beyond the accumulated total: the last member of K in vocabulary order
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) last_member = max(last_member, __shfl_xor(last_member, off, 64));
            __syncthreads();
            if ((tid & 63) == 0) lds_i[tid >> 6] = last_member;
            __syncthreads();
            tok = max(max(lds_i[0], lds_i[1]), max(lds_i[2], lds_i[3]));
        }
    }

    if (tid == 0) {
        o.dist[row] = d;
        if (o.cdf_lo) o.cdf_lo[row] = a;
        if (o.cdf_hi) o.cdf_hi[row] = bb;
        if (o.u) o.u[row] = u;
        if (o.ipt_token) o.ipt_token[row] = ok ? tok : -1;
        if (o.log_mass) o.log_mass[row] = (valid && ok) ? (float)gaussian_log_mass(ad, bd, ud, o.sigma, o.eps) : nan;
        o.flags[row] = (uint8_t)f;
    }
}

template <int DT>
__global__ __launch_bounds__(kBlock) void ipt_nucleus_kernel(RowBatch b, float top_p, IptOutputs o,
                                                             int32_t *__restrict__ kept_out, float *__restrict__ tau_out)
{
    __shared__ __attribute__((aligned(16))) unsigned char raw[kNucRawBytes];
    nucleus_row_multipass<DT>(b, top_p, o, kept_out, tau_out, raw);
}

int launch_ipt_nucleus(const RowBatch &b, float top_p, const IptOutputs &o, int32_t *kept, float *tau, hipStream_t stream)
{
    const dim3 grid((unsigned)b.N), block(kBlock);
    if (b.dtype == 0)
        ipt_nucleus_kernel<0><<<grid, block, 0, stream>>>(b, top_p, o, kept, tau);
    else
        ipt_nucleus_kernel<1><<<grid, block, 0, stream>>>(b, top_p, o, kept, tau);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

}  // namespace difr
