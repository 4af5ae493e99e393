// Fused LM head + scoring: the logits x[n][v] = <hidden[n], weight[v]> (the last step of the
// verifier's prefill; appendix algorithm "sampled token verification via prefill") are produced
// tile by tile on the matrix cores and scored in registers by both estimators (Token-DiFR,
// Sec. 6.3; Token-IPT-DiFR, Sec. 6.2) without ever being written to memory.
//
// Work split: a workgroup owns 256 token rows and a contiguous range of 256-entry vocabulary
// tiles.  Per tile it runs a bf16 MFMA GEMM over the hidden dimension (W tile as the A operand,
// H tile as the B operand, both staged through LDS in 64-deep slabs, double buffered), so that in
// the 32x32 accumulator blocks a lane holds 16 vocabulary entries of ONE token, four consecutive
// entries per register group: exactly the granularity of one Philox4x32 block.  The epilogue
// then updates, per lane and token, the running best perturbed score and the online softmax sums,
// and the next tile starts.  Partial results of the vocabulary ranges are merged by a last kernel.
#include <type_traits>
#include <utility>

#include "difr_device.hpp"
#include "difr_host.hpp"
#include "gumbel_stream.hpp"
#include "ipt_stream.hpp"
#include "lmhead.hpp"

namespace difr {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// When the 16 copies of a slab are issued: copy c goes out after matrix instruction kCopySlot[c] of the 48
// issued in the fourth k step of one slab and the first two of the next.  Spaced out because the memory
// pipeline accepts a 1 KB copy only every so often, and a wave whose copy is not accepted cannot issue its
// next matrix instruction either (measured: all 16 in one k step cost 11% of the kernel's time).
__host__ __device__ constexpr int copy_at_slot(int n)
{
    constexpr int kCopySlot[16] = {0, 3, 5, 8, 10, 13, 15, 18, 20, 23, 25, 28, 30, 33, 35, 38};
    for (int c = 0; c < 16; ++c)
        if (kCopySlot[c] == n) return c;
    return -1;
}

// f(integral_constant<int, 0>()), ..., f(integral_constant<int, N - 1>()): a loop whose index is a compile-time
// constant in the body (register numbers and instruction immediates depend on it)
template <int... Is, class F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, Is...>, F &&f)
{
    (f(std::integral_constant<int, Is>()), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(std::make_integer_sequence<int, N>(), f);
}

struct TokInfo {
    PhiloxKey key;
    uint32_t pos, seq;
    float inv_T;
    int32_t tg, ti;  // claims of the two estimators, -1 if absent or out of range
    bool ok;         // sequence id and temperature usable
    bool seq_ok;
};

__device__ __forceinline__ TokInfo load_tok(const LmHeadBatch &b, int64_t n)
{
    TokInfo t;
    const int32_t s = b.seq_ids[n];
    t.seq_ok = (s >= 0 && (int64_t)s < b.S);
    const uint64_t seed = t.seq_ok ? b.seeds[s] : 0ull;
    t.key.k0 = (uint32_t)seed;
    t.key.k1 = (uint32_t)(seed >> 32);
    t.seq = (uint32_t)s;
    t.pos = b.positions[n];
    const float T = b.temperatures ? b.temperatures[n] : b.temperature;
    t.ok = t.seq_ok && (T > 0.0f) && (T < __builtin_inff());
    t.inv_T = t.ok ? 1.0f / T : 1.0f;
    const int32_t tg = b.claimed_gumbel ? b.claimed_gumbel[n] : -1;
    const int32_t ti = b.claimed_ipt ? b.claimed_ipt[n] : -1;
    t.tg = (tg >= 0 && (int64_t)tg < b.V) ? tg : -1;
    t.ti = (ti >= 0 && (int64_t)ti < b.V) ? ti : -1;
    return t;
}

__device__ __forceinline__ uint32_t noise_word_of(const TokInfo &t, uint32_t stream, int32_t v)
{
    uint32_t r[4];
    noise_block(t.key, t.pos, t.seq, stream, (uint32_t)v >> 2, r);
    return (v & 3) == 0 ? r[0] : (v & 3) == 1 ? r[1] : (v & 3) == 2 ? r[2] : r[3];
}

// ---------------------------------------------------------------------------------
// Before the GEMM: a lower bound on each row's best perturbed score, from the Token-DiFR claim.
// For an honest claim the claimed token IS the row maximum, so almost every other entry can be
// ruled out by its noise word alone.  The claimed logit is a plain fp32 dot product here; it
// differs from the matrix-core value of the same logit by accumulation order only, and the bound
// is lowered by a rigorous estimate of that difference, so it never exceeds the true maximum.
// One wave per token.
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void lmhead_prepare_kernel(LmHeadBatch b, LmHeadWorkspace ws)
{
    const int lane = threadIdx.x & 63;
    const int64_t n = (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6);
    if (n >= b.N) return;  // uniform per wave
    const TokInfo t = load_tok(b, n);
    float L0 = -__builtin_inff(), x_ref = __builtin_nanf("");
    if (t.ok && t.tg >= 0) {
        const uint16_t *h = b.hidden + n * b.ldh;
        const uint16_t *w = b.weight + (int64_t)t.tg * b.ldw;
        float dot = 0.0f, mag = 0.0f;
        for (int64_t c = lane; c < b.d / 8; c += 64) {
            const uint4 hv = *reinterpret_cast<const uint4 *>(h + 8 * c);
            const uint4 wv = *reinterpret_cast<const uint4 *>(w + 8 * c);
            const uint32_t hw[4] = {hv.x, hv.y, hv.z, hv.w}, ww[4] = {wv.x, wv.y, wv.z, wv.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float h0 = __uint_as_float(hw[j] << 16), h1 = __uint_as_float(hw[j] & 0xFFFF0000u);
                const float w0 = __uint_as_float(ww[j] << 16), w1 = __uint_as_float(ww[j] & 0xFFFF0000u);
                dot = __fmaf_rn(h0, w0, dot);
                dot = __fmaf_rn(h1, w1, dot);
                mag = __fmaf_rn(fabsf(h0), fabsf(w0), mag);
                mag = __fmaf_rn(fabsf(h1), fabsf(w1), mag);
            }
        }
        dot = wave_sum(dot);
        mag = wave_sum(mag);
        x_ref = dot;
        const float y = perturbed_score(dot, t.inv_T, noise_word_of(t, kStreamGumbel, t.tg));
        // any two fp32 summation orders of d products differ by at most ~2 d 2^-24 sum|h w|; twice that here
        const float slack = 1e-3f + 1e-5f * fabsf(y) + t.inv_T * mag * (float)b.d * 0x1p-22f;
        L0 = y - slack;
        if (!(L0 == L0) || !(L0 < __builtin_inff())) L0 = -__builtin_inff();
    }
    if (lane == 0) {
        ws.L0[n] = L0;
        ws.x_claim_ref[n] = x_ref;
        ws.x_claim_gumbel[n] = __builtin_nanf("");
        ws.x_claim_ipt[n] = __builtin_nanf("");
    }
}

// ---------------------------------------------------------------------------------
// Per-lane, per-token running state of the epilogue.
// ---------------------------------------------------------------------------------
// The exponent a partial softmax sum with reference logit m is taken against: terms are 2^(x c - ref_exp(m, c)).  A
// whole number, so that moving a sum from one reference to another is a multiplication by an exact power of two
// and the many partial sums of a token (lanes, half tiles, vocabulary ranges) stay consistent to the last bit;
// with m c itself, rounded, every partial sum would sit on a reference that is off by the rounding of ITS product -
// 1e-6 and more once |m| / T reaches a few tens.
__device__ __forceinline__ float ref_exp(float m, float c) { return ceilf(m * c); }

struct Slot {
    float best_y;
    int32_t best_v;
    float L;      // lower bound on the row's best score: max(bound from the claim, best seen by this lane)
    float m;      // largest logit seen by this lane for this token
    double Z, P;  // sum of 2^((x - m) c) over all entries seen / over those below the IPT claim
    uint32_t above;  // RANK: entries seen whose logit exceeds the reference value of the Token-DiFR claim's
};

// Noise gate: an entry with noise word r < rgate cannot reach L whatever its logit (all logits seen
// are <= m).  g(r) <= c  <=>  u(r) <= exp(-exp(-c)); the threshold is lowered by 64 cells of the 23-bit
// uniform, far more than the fp32 error of the two exponentials.  Anything doubtful gives 0 (no skipping).
__device__ __forceinline__ uint32_t noise_gate(float L, float cap)
{
    const float c = L - cap - (0.01f + 1e-5f * (fabsf(L) + fabsf(cap)));
    const float t = fast_exp2(-c * kLog2e);
    const float kf = fast_exp2(-t * kLog2e) * 0x1p23f;
    const uint32_t kg = (kf > 64.0f) ? (uint32_t)kf - 64u : 0u;
    return kg << 9;
}

struct BlockCtx {
    const TokInfo &t;
    float c;       // log2(e) / T
    float neg_mc;  // -ref_exp(m, c)
    float Lgate;   // L minus slack
    uint32_t rgate;
    bool live;     // the lane's token row exists (n < N)
    float x_ref;   // RANK: the Token-DiFR claim's logit as a plain dot product (NaN: no claim, nothing counts)
};

__device__ __forceinline__ void refresh_gates(const Slot &s, BlockCtx &k)
{
    k.Lgate = s.L - (0.01f + 1e-5f * fabsf(s.L));
    k.rgate = noise_gate(s.L, s.m * k.t.inv_T);
}

// Score one 32x32 accumulator block: this lane's 16 entries are the logits of ONE token at
// vocabulary rows v(r) = vlane + 8 (r / 4) + (r % 4).
//
// RANK: also count the entries whose logit exceeds the Token-DiFR claim's (logit rank, Sec. 7.1).  The claim's
// logit must be known before the first tile, so the count is made against its plain fp32 dot product from the
// preparation kernel; the claimed entry itself is left out by index (its matrix-core value may differ from that
// reference in the last bits).
template <bool RANK>
__device__ __forceinline__ void score_block(const f32x16 acc, Slot &s, BlockCtx &k, int32_t vlane, int32_t V,
                                            bool ragged, int64_t n, const LmHeadWorkspace &ws)
{
    const float ninf = -__builtin_inff();
    // the accumulators live in the accumulation registers; fetch them one by one (left to itself the
    // register allocator moves whole blocks through scratch memory instead)
    float x[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) asm("v_accvgpr_read_b32 %0, %1" : "=v"(x[r]) : "a"(acc[r]));
    if (ragged) {  // uniform: the tile runs past the end of the vocabulary
#pragma unroll
        for (int r = 0; r < 16; ++r)
            if (vlane + 8 * (r >> 2) + (r & 3) >= V) x[r] = ninf;
    }
    if (RANK) {
#pragma unroll
        for (int r = 0; r < 16; ++r) s.above += (uint32_t)(x[r] > k.x_ref);  // rows past V are -inf, a NaN counts nothing
    }
    // ---- Token-IPT-DiFR: online softmax sums ----
    float bm = max3_raw(x[0], x[1], x[2]);
#pragma unroll
    for (int r = 3; r < 15; r += 2) bm = max3_raw(bm, x[r], x[r + 1]);
    bm = fmaxf(bm, x[15]);
    if (__builtin_amdgcn_ballot_w64(bm > s.m) != 0ull) {
        asm volatile("" ::: "memory");  // keep this a real, rarely taken branch
        if (bm > s.m) {
            const double f = (s.m > ninf) ? (double)fast_exp2(ref_exp(s.m, k.c) - ref_exp(bm, k.c)) : 0.0;
            s.Z *= f;
            s.P *= f;
            s.m = bm;
            k.neg_mc = -ref_exp(bm, k.c);
            refresh_gates(s, k);  // the logit cap of the noise gate has moved
        }
    }
    float e[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) e[r] = fast_exp2(__fmaf_rn(x[r], k.c, k.neg_mc));
    if (ragged) {
#pragma unroll
        for (int r = 0; r < 16; ++r)
            if (vlane + 8 * (r >> 2) + (r & 3) >= V) e[r] = 0.0f;
    }
    const float bs = tree_sum<16>(e);
    float ps = (vlane + 27 < k.t.ti) ? bs : 0.0f;  // all 16 rows lie below the IPT claim
    // a claimed token inside this lane's rows: exact prefix, and keep the claimed logits (rare)
    const bool near = (uint32_t)(k.t.ti - vlane) < 28u || (uint32_t)(k.t.tg - vlane) < 28u;
    if (__builtin_amdgcn_ballot_w64(near) != 0ull) {
        asm volatile("" ::: "memory");
        if (near) {
            const bool straddle = (uint32_t)(k.t.ti - vlane) < 28u;
            if (straddle) ps = 0.0f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int32_t v = vlane + 8 * (r >> 2) + (r & 3);
                if (straddle && v < k.t.ti) ps += e[r];
                if (k.live && v == k.t.ti) ws.x_claim_ipt[n] = x[r];
                if (k.live && v == k.t.tg) ws.x_claim_gumbel[n] = x[r];
                if (RANK && v == k.t.tg && x[r] > k.x_ref) s.above -= 1u;  // the claim does not outrank itself
            }
        }
    }
    s.Z += (double)bs;
    s.P += (double)ps;

    // ---- Token-DiFR: noise for all 16 entries, exact score only where the gates allow ----
    uint32_t rw[16];
#pragma unroll
    for (int g = 0; g < 4; ++g) noise_block(k.t.key, k.t.pos, k.t.seq, kStreamGumbel, (uint32_t)(vlane + 8 * g) >> 2, rw + 4 * g);
    uint32_t rmax = rw[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) rmax = max(rmax, rw[r]);
    if (__builtin_amdgcn_ballot_w64(rmax >= k.rgate) != 0ull) {
        asm volatile("" ::: "memory");
        if (rmax >= k.rgate) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int32_t v = vlane + 8 * (r >> 2) + (r & 3);
                if (rw[r] >= k.rgate && !(ragged && v >= V) &&
                    !(__fmaf_rn(x[r], k.t.inv_T, gumbel_upper_bound(rw[r])) < k.Lgate)) {
                    const float y = perturbed_score(x[r], k.t.inv_T, rw[r]);
                    if (y > s.best_y || (y == s.best_y && v < s.best_v)) {
                        s.best_y = y;
                        s.best_v = v;
                    }
                }
            }
            if (s.best_y > s.L) {
                s.L = s.best_y;
                refresh_gates(s, k);
            }
        }
    }
}

__device__ __forceinline__ void merge_softmax(float &m, double &Z, double &P, float om, double oZ, double oP, float c)
{
    const float ninf = -__builtin_inff();
    const float M = fmaxf(m, om);
    const double f = (m > ninf) ? (double)fast_exp2(ref_exp(m, c) - ref_exp(M, c)) : 0.0;
    const double of = (om > ninf) ? (double)fast_exp2(ref_exp(om, c) - ref_exp(M, c)) : 0.0;
    Z = Z * f + oZ * of;
    P = P * f + oP * of;
    m = M;
}

// ---------------------------------------------------------------------------------
// The GEMM + epilogue kernel.  256 threads = 4 waves in a 2 (vocabulary) x 2 (tokens) arrangement;
// each wave owns a 128 x 128 sub-tile = 4 x 4 accumulator blocks of 32 x 32.
// LDS: two stages of [256 rows][64 k] bf16 for each operand; the eight 16-byte chunks of a row are
// permuted by (row / 2) % 8 so that both the 16-byte slab writes and the fragment reads of 16
// consecutive rows spread over all 64 banks.
// ---------------------------------------------------------------------------------
//
// TOK: also leave, per token and half tile (the 128 vocabulary entries of a tile that one wave scores), the softmax
// mass of that half tile with its exponent reference.  The sampler's own Token-IPT-DiFR token is the first entry
// at which the CDF passes u; the CDF needs the row's total mass, known only after the last tile, so the search is
// made afterwards: over these masses for the half tile, and inside it by forming its 128 logits again.
template <bool RANK, bool TOK>
__global__ __launch_bounds__(kBlock, 1) void lmhead_score_kernel(LmHeadBatch b, LmHeadWorkspace ws, LmHeadPlan plan)
{
    __shared__ __attribute__((aligned(16))) uint16_t lds_w[2][kLmTileV * kLmTileK];  // 32 KB per stage
    __shared__ __attribute__((aligned(16))) uint16_t lds_h[2][kLmTileT * kLmTileK];
    // per-token constants of the workgroup's 256 token rows (one wave per SIMD cannot hide a global load
    // in the epilogue, an LDS read it can): key, position, sequence, 1/T, the two claims
    __shared__ uint32_t lds_tok[RANK ? 8 : 7][kLmTileT];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wv = wave >> 1, wt = wave & 1;  // vocabulary half, token half
    const int l32 = lane & 31, lh = lane >> 5;

    // Workgroup -> (token block, vocabulary range).  Consecutive workgroup ids go to different XCDs;
    // remap so that each XCD works on a compact set of token blocks across all ranges and its L2
    // sees each weight tile and each hidden-state tile from several workgroups at about the same time.
    const int G = plan.n_tb * plan.splits;
    int q = blockIdx.x;
    if (G % 8 == 0) q = (q % 8) * (G / 8) + q / 8;
    const int tb = q / plan.splits, sp = q % plan.splits;
    const int vt0 = (int)((int64_t)sp * plan.n_vt / plan.splits), vt1 = (int)((int64_t)(sp + 1) * plan.n_vt / plan.splits);
    const int64_t n0 = (int64_t)tb * kLmTileT;
    const int32_t V = (int32_t)b.V;
    const int nk = (int)(b.d / kLmTileK);

    // Slab copy, global memory straight into LDS (no registers in between): a slab is 256 rows x 64 k of
    // each operand, i.e. whole 128-byte lines.  One wave-wide 16-byte-per-lane load fills 1 KB of LDS in
    // lane order = 8 rows; lane i lands in 16-byte position i % 8 of row i / 8, so it fetches the k chunk
    // that the permutation of the LDS layout puts there.  Thread -> rows (tid / 8) + 32 p, p = 0 .. 7.
    const int crow = tid >> 3;
    const int cchunk = (tid & 7) ^ ((crow >> 1) & 7);
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    // Addresses are a wave-uniform base (scalar registers, moved by scalar arithmetic) plus a 32-bit
    // per-lane byte offset that never changes, so a load costs no vector arithmetic.
    uint32_t hoff[8];  // hidden-state rows: offset from the first row of the token block
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        int64_t r = crow + 32 * p;
        if (n0 + r > b.N - 1) r = b.N - 1 - n0;
        hoff[p] = (uint32_t)(r * b.ldh + cchunk * 8) * 2u;
    }
    const char *const hbase = reinterpret_cast<const char *>(b.hidden + n0 * b.ldh);
    const uint32_t wrow_bytes = (uint32_t)b.ldw * 2u;
    uint32_t woff[8];  // weight rows: offset from the first row of the vocabulary tile
    // rows past the end of the vocabulary (last tile only) re-read the last row
    auto set_woff = [&](int vt) {
        const int64_t tile_v0 = (int64_t)vt * kLmTileV;
        const int32_t last = (int32_t)((b.V - tile_v0 < kLmTileV ? b.V - tile_v0 : kLmTileV) - 1);  // uniform
#pragma unroll
        for (int p = 0; p < 8; ++p) woff[p] = (uint32_t)min(crow + 32 * p, last) * wrow_bytes + (uint32_t)cchunk * 16u;
    };
    set_woff(vt0);
    // load cursor: the next slab to fetch is slab l_kt of vocabulary tile l_vt; once past the end it stays
    // on the last tile (harmless reloads keep the loop free of special cases)
    int l_vt = vt0, l_kt = 0;
    auto advance_cursor = [&]() {
        const bool wrap = (l_kt + 1 == nk);
        l_kt = wrap ? 0 : l_kt + 1;
        if (wrap && l_vt + 1 < vt1) {
            ++l_vt;
            if ((int64_t)(l_vt + 1) * kLmTileV > b.V) set_woff(l_vt);  // the ragged tile, at most once
        }
    };
    // Chunk i (0-7: weight rows, 8-15: hidden-state rows) of the cursor's slab -> LDS stage buf.
    // The register M0 carries the LDS address of lane 0; lane i writes 16 i bytes further on.  Written as
    // assembly for two reasons: the compiler would make every later LDS read wait for the copies in flight (it
    // cannot tell the stages apart; the waits are placed by hand, see copies_landed), and a wave that runs
    // alone on its SIMD can issue only a handful of instructions between two matrix instructions, so a copy
    // must cost no address arithmetic: scalar base, invariant lane offset, M0 = stage base + constant.
    auto copy_chunk = [&](auto I, int buf) {
        constexpr int i = decltype(I)::value;
        const char *sbase = i < 8 ? reinterpret_cast<const char *>(b.weight + (int64_t)l_vt * kLmTileV * b.ldw + l_kt * kLmTileK)
                                  : hbase + (size_t)l_kt * (kLmTileK * 2);
        const uint32_t voff = i < 8 ? woff[i & 7] : hoff[i & 7];
        const uint16_t *stage = (i < 8 ? &lds_w[buf][0] : &lds_h[buf][0]) + 8 * wave_u * kLmTileK;
        const uint32_t lds_base = (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) void *)stage;
        // (M0 is set and consumed inside the one statement and declared clobbered; the compiler's remark that
        // it is a reserved register does not apply to that use)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
        asm volatile("s_add_u32 m0, %2, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %0"
                     :
                     : "s"(sbase), "v"(voff), "s"(lds_base), "n"(32 * (i & 7) * kLmTileK * 2)
                     : "memory", "m0", "scc");
#pragma clang diagnostic pop
    };
    // every copy this wave has issued has landed in LDS, and every LDS read it has issued is complete
    auto copies_landed = [&]() { asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory"); };
    auto barrier = [&]() {
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };

    // fragment reads: lane -> row l32 of a 32-row block, 16-byte k chunk 2 kk + lh (permuted like the copy)
    const int sw = (l32 >> 1) & 7;
    const int a_row_off = (wv * 128 + l32) * kLmTileK;
    const int b_row_off = (wt * 128 + l32) * kLmTileK;
    struct Frag {
        bf16x8 a[4], b[4];
    };
    // fragment i (0-3: weight blocks, 4-7: hidden-state blocks) of k step kk from LDS stage buf
    auto read_frag = [&](Frag &f, int i, int buf, int kk) {
        const int coff = ((2 * kk + lh) ^ sw) * 8;
        if (i < 4)
            f.a[i] = *reinterpret_cast<const bf16x8 *>(&lds_w[buf][a_row_off + i * 32 * kLmTileK + coff]);
        else
            f.b[i - 4] = *reinterpret_cast<const bf16x8 *>(&lds_h[buf][b_row_off + (i - 4) * 32 * kLmTileK + coff]);
    };

    {
        int64_t n = n0 + tid;
        if (n > b.N - 1) n = b.N - 1;
        const TokInfo t = load_tok(b, n);
        lds_tok[0][tid] = t.key.k0;
        lds_tok[1][tid] = t.key.k1;
        lds_tok[2][tid] = t.pos;
        lds_tok[3][tid] = t.seq;
        lds_tok[4][tid] = __float_as_uint(t.inv_T);
        lds_tok[5][tid] = (uint32_t)t.tg;
        lds_tok[6][tid] = (uint32_t)t.ti;
        if (RANK) lds_tok[7][tid] = __float_as_uint(ws.x_claim_ref[n]);
    }
    auto tok_from_lds = [&](int i) {
        TokInfo t;
        t.key.k0 = lds_tok[0][i];
        t.key.k1 = lds_tok[1][i];
        t.pos = lds_tok[2][i];
        t.seq = lds_tok[3][i];
        t.inv_T = __uint_as_float(lds_tok[4][i]);
        t.tg = (int32_t)lds_tok[5][i];
        t.ti = (int32_t)lds_tok[6][i];
        t.ok = t.seq_ok = true;  // not used by the epilogue
        return t;
    };

    // per-lane state of the lane's four tokens
    Slot slot[4];
    const int64_t tok_first = n0 + wt * 128 + l32;  // the lane's tokens are tok_first + 32 jb
    auto tok_row = [&](int jb) { return tok_first + 32 * jb < b.N ? tok_first + 32 * jb : b.N - 1; };
    auto tok_is_live = [&](int jb) { return tok_first + 32 * jb < b.N; };
#pragma unroll
    for (int jb = 0; jb < 4; ++jb) {
        const int64_t n = tok_row(jb);
        slot[jb].best_y = -__builtin_inff();
        slot[jb].best_v = 0x7FFFFFFF;
        slot[jb].L = ws.L0[n];
        slot[jb].m = -__builtin_inff();
        slot[jb].Z = 0.0;
        slot[jb].P = 0.0;
        slot[jb].above = 0u;
    }

    // ---- main loop ----
    // One wave per SIMD: nothing else hides latency, so copies and fragment reads are interleaved with the
    // matrix instructions by hand and the order is pinned with scheduling fences.  Per 64-deep slab, four
    // k steps of 16 MFMAs each:
    //   steps 0-1: + fragment reads for the next step, + the rest of the copies of the next slab
    //   step 2:    + fragment reads for step 3
    //   wait for this wave's copies, barrier
    //   step 3:    + fragment reads for step 0 of the next slab (from the other LDS stage), + the first copies
    //              of the slab after that into the stage just released
    f32x16 acc[4][4];
    Frag F0, F1;
    auto kstep = [&](const Frag &cur, Frag &nxt, int buf_next, int kk_next, auto READ, auto &&extra) {
        static_for<8>([&](auto I) {
            constexpr int i = decltype(I)::value, e0 = 2 * i, e1 = 2 * i + 1;
            acc[e0 >> 2][e0 & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur.a[e0 >> 2], cur.b[e0 & 3], acc[e0 >> 2][e0 & 3], 0, 0, 0);
            extra(std::integral_constant<int, e0>());
            acc[e1 >> 2][e1 & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur.a[e1 >> 2], cur.b[e1 & 3], acc[e1 >> 2][e1 & 3], 0, 0, 0);
            extra(std::integral_constant<int, e1>());
            if (decltype(READ)::value) read_frag(nxt, i, buf_next, kk_next);
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    int par = 0;  // LDS stage of the slab being multiplied
    // Two LDS stages.  The stage of slab g is last read during its third k step (fragments are read one
    // step ahead), so after the barrier that follows that step it is free until the same barrier of slab
    // g + 1, and the 16 copies of slab g + 2 are issued into it during the fourth step of slab g and the
    // first two of slab g + 1 (copy_at_slot).  Each wave waits for its own copies before the barrier of
    // slab g + 1; the last of them has had a whole k step to land by then.  The LAST slab of a tile does
    // not read fragments ahead, so the epilogue has those 64 registers for itself.
    const std::true_type yes;
    const std::false_type no;
    // the copy (if any) that goes out at slot E of phase PH (0: fourth k step, 1 and 2: first and second of the next slab)
    auto cp = [&](auto PH, int buf) {
        return [&, buf](auto E) {
            constexpr int c = copy_at_slot(16 * decltype(PH)::value + decltype(E)::value);
            if constexpr (c >= 0) copy_chunk(std::integral_constant<int, c>(), buf);
        };
    };
    auto slab = [&](auto LAST) {
        kstep(F0, F1, par, 1, yes, cp(std::integral_constant<int, 1>(), par ^ 1));
        kstep(F1, F0, par, 2, yes, cp(std::integral_constant<int, 2>(), par ^ 1));
        advance_cursor();
        kstep(F0, F1, par, 3, yes, [&](auto) {});
        copies_landed();
        barrier();
        if (decltype(LAST)::value)
            kstep(F1, F0, par ^ 1, 0, no, cp(std::integral_constant<int, 0>(), par));
        else
            kstep(F1, F0, par ^ 1, 0, yes, cp(std::integral_constant<int, 0>(), par));
        par ^= 1;
    };

    // prologue: slab 0 whole, and of slab 1 what the fourth k step of a slab before it would have issued
    static_for<16>([&](auto I) { copy_chunk(I, 0); });
    advance_cursor();
    static_for<16>([&](auto E) { cp(std::integral_constant<int, 0>(), 1)(E); });
    copies_landed();
    __syncthreads();

    for (int vt = vt0; vt < vt1; ++vt) {
        const int64_t v0 = (int64_t)vt * kLmTileV;
        const f32x16 zero = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int ib = 0; ib < 4; ++ib)
#pragma unroll
            for (int jb = 0; jb < 4; ++jb) acc[ib][jb] = zero;
#pragma unroll
        for (int i = 0; i < 8; ++i) read_frag(F0, i, par, 0);
        for (int kt = 1; kt < nk; ++kt) slab(no);
        slab(yes);

        // ---- epilogue: score the 256 x 256 logits of this tile ----
        const bool ragged = v0 + kLmTileV > b.V;
        // (explicit instantiation per block: the accumulator indices must be compile-time constants)
        auto score_token = [&](auto JB) {
            constexpr int jb = decltype(JB)::value;
            const TokInfo t = tok_from_lds(wt * 128 + jb * 32 + l32);
            BlockCtx k{t, t.inv_T * kLog2e, 0.0f, 0.0f, 0u, tok_is_live(jb),
                       RANK ? __uint_as_float(lds_tok[RANK ? 7 : 0][wt * 128 + jb * 32 + l32]) : 0.0f};
            k.neg_mc = (slot[jb].m > -__builtin_inff()) ? -ref_exp(slot[jb].m, k.c) : 0.0f;
            refresh_gates(slot[jb], k);
            const int32_t vl = (int32_t)v0 + wv * 128 + 4 * lh;
            const double Z_before = slot[jb].Z;
            const float m_before = slot[jb].m;
            score_block<RANK>(acc[0][jb], slot[jb], k, vl, V, ragged, tok_row(jb), ws);
            score_block<RANK>(acc[1][jb], slot[jb], k, vl + 32, V, ragged, tok_row(jb), ws);
            score_block<RANK>(acc[2][jb], slot[jb], k, vl + 64, V, ragged, tok_row(jb), ws);
            score_block<RANK>(acc[3][jb], slot[jb], k, vl + 96, V, ragged, tok_row(jb), ws);
            if (TOK) {
                // what this lane's 64 entries of the half tile added to its sum, relative to its reference now;
                // then the two lanes that share the token (rows 0-3 and 4-7 mod 8) combined
                const float ninf = -__builtin_inff();
                const Slot &s = slot[jb];
                double mine = s.Z;
                if (m_before > ninf)
                    mine -= Z_before * (s.m == m_before ? 1.0 : (double)fast_exp2(ref_exp(m_before, k.c) - ref_exp(s.m, k.c)));
                const float ms = mine > 0.0 ? (float)mine : 0.0f, mm = s.m;
                const float os = __shfl_xor(ms, 32, 64), om = __shfl_xor(mm, 32, 64);
                const float M = fmaxf(mm, om);
                const float both = (mm > ninf ? ms * fast_exp2(ref_exp(mm, k.c) - ref_exp(M, k.c)) : 0.0f) +
                                   (om > ninf ? os * fast_exp2(ref_exp(om, k.c) - ref_exp(M, k.c)) : 0.0f);
                if (lh == 0 && tok_is_live(jb)) ws.half_sum[(int64_t)(2 * vt + wv) * b.N + tok_row(jb)] = make_float2(both, M);
            }
        };
        score_token(std::integral_constant<int, 0>());
        score_token(std::integral_constant<int, 1>());
        score_token(std::integral_constant<int, 2>());
        score_token(std::integral_constant<int, 3>());
    }

    // ---- merge the four lanes/waves that share a token and write this range's partial ----
    float *ex_y = reinterpret_cast<float *>(&lds_w[0][0]);  // [2][128] each, in the (now idle) tile memory
    int32_t *ex_v = reinterpret_cast<int32_t *>(ex_y + 256);
    float *ex_m = reinterpret_cast<float *>(ex_v + 256);
    double *ex_Z = reinterpret_cast<double *>(ex_m + 256);
    double *ex_P = ex_Z + 256;
    uint32_t *ex_a = reinterpret_cast<uint32_t *>(ex_P + 256);
    float tok_c[4];
#pragma unroll
    for (int jb = 0; jb < 4; ++jb) {
        Slot &s = slot[jb];
        tok_c[jb] = __uint_as_float(lds_tok[4][wt * 128 + jb * 32 + l32]) * kLog2e;
        const float oy = __shfl_xor(s.best_y, 32, 64);
        const int32_t ov = __shfl_xor(s.best_v, 32, 64);
        const float om = __shfl_xor(s.m, 32, 64);
        const double oZ = __shfl_xor(s.Z, 32, 64), oP = __shfl_xor(s.P, 32, 64);
        if (RANK) s.above += (uint32_t)__shfl_xor((int)s.above, 32, 64);
        if (lh == 0) {  // rows 0-3 (mod 8) first, then rows 4-7: a fixed order
            argmax_combine(s.best_y, s.best_v, oy, ov);
            merge_softmax(s.m, s.Z, s.P, om, oZ, oP, tok_c[jb]);
        }
    }
    copies_landed();  // the tile memory is reused below: nothing may still be on its way into it
    __syncthreads();
    if (wv == 1 && lh == 0) {
#pragma unroll
        for (int jb = 0; jb < 4; ++jb) {
            const int i = wt * 128 + jb * 32 + l32;
            ex_y[i] = slot[jb].best_y;
            ex_v[i] = slot[jb].best_v;
            ex_m[i] = slot[jb].m;
            ex_Z[i] = slot[jb].Z;
            ex_P[i] = slot[jb].P;
            if (RANK) ex_a[i] = slot[jb].above;
        }
    }
    __syncthreads();
    if (wv == 0 && lh == 0) {
#pragma unroll
        for (int jb = 0; jb < 4; ++jb) {
            if (!tok_is_live(jb)) continue;
            Slot &s = slot[jb];
            const int i = wt * 128 + jb * 32 + l32;
            argmax_combine(s.best_y, s.best_v, ex_y[i], ex_v[i]);
            merge_softmax(s.m, s.Z, s.P, ex_m[i], ex_Z[i], ex_P[i], tok_c[jb]);
            const int64_t o = (int64_t)sp * b.N + tok_row(jb);
            ws.best_y[o] = s.best_y;
            ws.best_v[o] = s.best_v;
            ws.m[o] = s.m;
            ws.Z[o] = s.Z;
            ws.P[o] = s.P;
            if (RANK) ws.above[o] = (int32_t)(s.above + ex_a[i]);
        }
    }
}

// ---------------------------------------------------------------------------------
// Merge the vocabulary ranges of each token (ascending) and form every output.  One thread per token.
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void lmhead_finalize_kernel(LmHeadBatch b, LmHeadWorkspace ws, int splits, int n_vt,
                                                                 GumbelOutputs og, IptOutputs oi)
{
    const int64_t n = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (n >= b.N) return;
    const float nan = __builtin_nanf("");
    const float ninf = -__builtin_inff();
    const TokInfo t = load_tok(b, n);
    const int32_t tg_raw = b.claimed_gumbel ? b.claimed_gumbel[n] : -1;
    (void)tg_raw;
    if (!t.ok) {
        const uint8_t f = (uint8_t)(t.seq_ok ? kFlagNonfinite : kFlagInvalidClaim);
        og.margin[n] = nan;
        og.argmax[n] = -1;
        if (og.max_score) og.max_score[n] = nan;
        if (og.claimed_score) og.claimed_score[n] = nan;
        og.flags[n] = f;
        if (og.logit_rank) og.logit_rank[n] = -1;
        oi.dist[n] = nan;
        if (oi.cdf_lo) oi.cdf_lo[n] = nan;
        if (oi.cdf_hi) oi.cdf_hi[n] = nan;
        if (oi.u) oi.u[n] = nan;
        if (oi.log_mass) oi.log_mass[n] = nan;
        if (oi.ipt_token) {
            oi.ipt_token[n] = -1;
            ws.cross_half[n] = -1;
        }
        oi.flags[n] = f;
        return;
    }
    const float c = t.inv_T * kLog2e;
    float best_y = ninf, m = ninf;
    int32_t best_v = 0x7FFFFFFF;
    double Z = 0.0, P = 0.0;
    int32_t above = 0;
    for (int sp = 0; sp < splits; ++sp) {
        const int64_t o = (int64_t)sp * b.N + n;
        argmax_combine(best_y, best_v, ws.best_y[o], ws.best_v[o]);
        merge_softmax(m, Z, P, ws.m[o], ws.Z[o], ws.P[o], c);
        if (og.logit_rank) above += ws.above[o];
    }
    if (best_v == 0x7FFFFFFF) best_v = 0;
    const bool ipt_bad = !(Z > 0.0) || !(Z < (double)__builtin_inff()) || !(m < __builtin_inff()) || !(m > ninf);
    const bool nonfinite = !(Z == Z) || !(Z < (double)__builtin_inff()) || !(m < __builtin_inff());

    // Token-DiFR
    uint32_t fg = nonfinite ? kFlagNonfinite : 0u;
    float yt = nan, mg = nan;
    if (t.tg >= 0) {
        yt = perturbed_score(ws.x_claim_gumbel[n], t.inv_T, noise_word_of(t, kStreamGumbel, t.tg));
        mg = best_y - yt;
        if (best_v == t.tg) fg |= kFlagMatch;
    } else {
        fg |= kFlagInvalidClaim;
    }
    og.margin[n] = mg;
    og.argmax[n] = best_v;
    if (og.max_score) og.max_score[n] = best_y;
    if (og.claimed_score) og.claimed_score[n] = yt;
    og.flags[n] = (uint8_t)fg;
    if (og.logit_rank) og.logit_rank[n] = t.tg >= 0 ? above : -1;

    // Token-IPT-DiFR
    uint32_t r[4];
    noise_block(t.key, t.pos, t.seq, kStreamIpt, 0u, r);
    const float u = uniform_from_bits(r[0]);
    float a = nan, bb = nan, dd = nan, lm = nan;
    bool match = false;
    if (t.ti >= 0 && !ipt_bad) {
        const double et = (double)fast_exp2(__fmaf_rn(ws.x_claim_ipt[n], c, -ref_exp(m, c)));
        const double ud = (double)u;
        const double ad = P / Z, bd = (P + et) / Z;
        a = (float)ad;
        bb = (float)bd;
        dd = (float)fmax(fmax(ad - ud, ud - bd), 0.0);
        match = (ad <= ud) && (ud < bd);
        if (oi.log_mass) lm = (float)gaussian_log_mass(ad, bd, ud, oi.sigma, oi.eps);
    }
    uint32_t fi = 0;
    if (t.ti < 0) fi |= kFlagInvalidClaim;
    if (ipt_bad) fi |= kFlagNonfinite;
    if (match) fi |= kFlagMatch;
    oi.dist[n] = dd;
    if (oi.cdf_lo) oi.cdf_lo[n] = a;
    if (oi.cdf_hi) oi.cdf_hi[n] = bb;
    if (oi.u) oi.u[n] = u;
    if (oi.log_mass) oi.log_mass[n] = lm;
    if (oi.ipt_token) {
        // The sampler's own token: the claim if it matches; else the first entry at which the CDF passes u.  The
        // half tile in which that happens is found from the masses the scoring pass left (vocabulary order, each
        // brought to the row's final reference); the entry inside it by the kernel that follows.
        int32_t tok = -1, half = -1;
        double rest = 0.0;
        if (ipt_bad) {
            tok = -1;
        } else if (match) {
            tok = t.ti;
        } else {
            const double target = (double)u * Z;
            double cum = 0.0;
            int32_t last = -1;  // last half tile with any mass: where rounding puts a u beyond the summed total
            double cum_last = 0.0;
            for (int h = 0; h < 2 * n_vt; ++h) {
                const float2 p = ws.half_sum[(int64_t)h * b.N + n];
                if (!(p.x > 0.0f)) continue;
                const double w = (double)p.x * (double)fast_exp2(ref_exp(p.y, c) - ref_exp(m, c));
                if (cum + w > target) {
                    half = h;
                    rest = target - cum;
                    break;
                }
                if (w > 0.0) {
                    last = h;
                    cum_last = cum;
                }
                cum += w;
            }
            if (half < 0) {
                half = last;
                rest = target - cum_last;
            }
            if (half >= 0) fi |= kFlagSlowPath;
        }
        oi.ipt_token[n] = tok;
        ws.cross_half[n] = half;
        ws.cross_rest[n] = rest;
        ws.final_m[n] = m;
    }
    oi.flags[n] = (uint8_t)fi;
}

// ---------------------------------------------------------------------------------
// The sampler's own Token-IPT-DiFR token inside the half tile the merge kernel found: the 128 logits of that
// half tile are formed again as plain fp32 dot products (one wave per 32 of them, a row of the LM-head matrix
// read by the whole wave at a time), turned into softmax terms relative to the row's final reference and scanned
// in vocabulary order for the first entry at which the running sum passes what was left to cover.  One workgroup
// per token; tokens that are already known (matching or missing claims, rejected rows) leave at once.
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void lmhead_ipt_token_kernel(LmHeadBatch b, LmHeadWorkspace ws, IptOutputs oi)
{
    __shared__ float lds_e[128];
    const int64_t n = blockIdx.x;
    const int32_t half = ws.cross_half[n];
    if (half < 0) return;  // uniform
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const TokInfo t = load_tok(b, n);
    const float c = t.inv_T * kLog2e, m = ws.final_m[n];
    const int64_t v0 = (int64_t)half * 128;
    const uint16_t *h = b.hidden + n * b.ldh;
    for (int r = wave * 32; r < wave * 32 + 32; ++r) {
        const int64_t v = v0 + r;
        float e = 0.0f;
        if (v < b.V) {  // uniform per wave
            const uint16_t *w = b.weight + v * b.ldw;
            float dot = 0.0f;
            for (int64_t q = lane; q < b.d / 8; q += 64) {
                const uint4 hv = *reinterpret_cast<const uint4 *>(h + 8 * q);
                const uint4 wv = *reinterpret_cast<const uint4 *>(w + 8 * q);
                const uint32_t hw[4] = {hv.x, hv.y, hv.z, hv.w}, ww[4] = {wv.x, wv.y, wv.z, wv.w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    dot = __fmaf_rn(__uint_as_float(hw[j] << 16), __uint_as_float(ww[j] << 16), dot);
                    dot = __fmaf_rn(__uint_as_float(hw[j] & 0xFFFF0000u), __uint_as_float(ww[j] & 0xFFFF0000u), dot);
                }
            }
            dot = wave_sum(dot);
            e = fast_exp2(__fmaf_rn(dot, c, -ref_exp(m, c)));
            if (!(e == e)) e = 0.0f;
        }
        if (lane == 0) lds_e[r] = e;
    }
    __syncthreads();
    if (wave == 0) {
        // inclusive scan over the 128 terms in vocabulary order: lane l holds entries 2l and 2l + 1
        const double e0 = (double)lds_e[2 * lane], e1 = (double)lds_e[2 * lane + 1];
        double incl = e0 + e1;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const double o = __shfl_up(incl, off, 64);
            if (lane >= off) incl += o;
        }
        const double before = incl - (e0 + e1), rest = ws.cross_rest[n];
        int32_t idx = 0x7FFFFFFF;
        if (e0 > 0.0 && before + e0 > rest)
            idx = 2 * lane;
        else if (e1 > 0.0 && before + e0 + e1 > rest)
            idx = 2 * lane + 1;
        int32_t last = e1 > 0.0 ? 2 * lane + 1 : (e0 > 0.0 ? 2 * lane : -1);  // rounding may leave `rest` uncovered
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            idx = min(idx, __shfl_xor(idx, off, 64));
            last = max(last, __shfl_xor(last, off, 64));
        }
        if (lane == 0) {
            if (idx == 0x7FFFFFFF) idx = last >= 0 ? last : 0;
            oi.ipt_token[n] = (int32_t)(v0 + idx);
        }
    }
}

int launch_lmhead_score(const LmHeadBatch &b, const LmHeadWorkspace &ws, const LmHeadPlan &plan, const GumbelOutputs &og,
                        const IptOutputs &oi, hipStream_t stream)
{
    lmhead_prepare_kernel<<<dim3((unsigned)((b.N + kWaves - 1) / kWaves)), dim3(kBlock), 0, stream>>>(b, ws);
    if (hipGetLastError() != hipSuccess) return 1;
    // the logit rank and the masses behind the sampler's own token are produced in the scoring pass, only when asked for
    const dim3 grid((unsigned)(plan.n_tb * plan.splits)), block(kBlock);
    const bool rank = og.logit_rank != nullptr, tok = oi.ipt_token != nullptr;
    if (rank && tok)
        lmhead_score_kernel<true, true><<<grid, block, 0, stream>>>(b, ws, plan);
    else if (rank)
        lmhead_score_kernel<true, false><<<grid, block, 0, stream>>>(b, ws, plan);
    else if (tok)
        lmhead_score_kernel<false, true><<<grid, block, 0, stream>>>(b, ws, plan);
    else
        lmhead_score_kernel<false, false><<<grid, block, 0, stream>>>(b, ws, plan);
    if (hipGetLastError() != hipSuccess) return 1;
    lmhead_finalize_kernel<<<dim3((unsigned)((b.N + kBlock - 1) / kBlock)), block, 0, stream>>>(b, ws, plan.splits, plan.n_vt,
                                                                                            og, oi);
    if (hipGetLastError() != hipSuccess) return 1;
    if (tok) {
        lmhead_ipt_token_kernel<<<dim3((unsigned)b.N), block, 0, stream>>>(b, ws, oi);
        if (hipGetLastError() != hipSuccess) return 1;
    }
    return 0;
}

}  // namespace difr
