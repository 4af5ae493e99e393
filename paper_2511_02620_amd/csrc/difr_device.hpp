// Device-side building blocks shared by the scoring kernels (gfx950, wave64).
//
//  - Philox4x32-10 noise keyed on (seed, sequence, position, vocabulary index): the
//    instantiation of the paper's H(seed || i) (Sec. 3.2, "Sampling multiple tokens").
//  - the bits -> uniform -> Gumbel map  u = (2 (r >> 9) + 1) 2^-24,  g = -ln(-ln u)
//    (Sec. 3.2 Gumbel-max sampler; Sec. 6.3 noise regeneration).
//  - 128-bit row loads of bf16 / fp32 logits and fixed-shape block reductions.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace difr {

constexpr int kBlock = 256;          // threads per workgroup: 4 wavefronts of 64
constexpr int kWaves = kBlock / 64;
constexpr uint32_t kStreamGumbel = 0u;
constexpr uint32_t kStreamIpt = 1u;

constexpr uint32_t kFlagMatch = 1u;
constexpr uint32_t kFlagInvalidClaim = 2u;
constexpr uint32_t kFlagNonfinite = 4u;
constexpr uint32_t kFlagSlowPath = 8u;

constexpr float kLn2 = 0.693147180559945309417f;
constexpr float kLog2e = 1.44269504088896340736f;

// Kernel-side image of difr_rows.
struct RowBatch {
    const void *logits;
    int32_t dtype;
    int64_t N, V, ld;
    float temperature;
    const float *temperatures;
    const uint64_t *seeds;
    int64_t S;
    const int32_t *seq_ids;
    const uint32_t *positions;
    const int32_t *claimed;
};

// ---------------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11).  One round:
//   (c0,c1,c2,c3) <- (hi(M1 c2)^c1^k0, lo(M1 c2), hi(M0 c0)^c3^k1, lo(M0 c0)),
// key bumped by the Weyl constants between rounds.
// ---------------------------------------------------------------------------------
struct PhiloxKey {
    uint32_t k0, k1;
};

// a ^ b ^ c in one instruction (three-input bitwise op, truth table 0x96).
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c)
{
    return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

constexpr uint32_t kPhiloxM0 = 0xD2511F53u, kPhiloxM1 = 0xCD9E8D57u;
constexpr uint32_t kPhiloxW0 = 0x9E3779B9u, kPhiloxW1 = 0xBB67AE85u;

// The ten rounds, with the first round's product M0 * c0 supplied by the caller.  In the
// streaming kernels c0 = (uniform base) + (per-lane constant), so that product is one
// 64-bit add of a scalar and a loop-invariant vector value instead of a multiply.
__device__ __forceinline__ void philox4x32_10_from_product(uint64_t p0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                           PhiloxKey key, uint32_t out[4])
{
    uint32_t k0 = key.k0, k1 = key.k1;
    uint32_t c0;
    {
        const uint64_t p1 = (uint64_t)kPhiloxM1 * c2;
        c0 = xor3((uint32_t)(p1 >> 32), c1, k0);
        c1 = (uint32_t)p1;
        c2 = xor3((uint32_t)(p0 >> 32), c3, k1);
        c3 = (uint32_t)p0;
    }
#pragma unroll
    for (int r = 1; r < 10; ++r) {
        k0 += kPhiloxW0;
        k1 += kPhiloxW1;
        const uint64_t q0 = (uint64_t)kPhiloxM0 * c0;  // one 32x32->64 multiply gives hi and lo
        const uint64_t q1 = (uint64_t)kPhiloxM1 * c2;
        const uint32_t n0 = xor3((uint32_t)(q1 >> 32), c1, k0);
        const uint32_t n2 = xor3((uint32_t)(q0 >> 32), c3, k1);
        c0 = n0;
        c1 = (uint32_t)q1;
        c2 = n2;
        c3 = (uint32_t)q0;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, PhiloxKey key,
                                              uint32_t out[4])
{
    philox4x32_10_from_product((uint64_t)kPhiloxM0 * c0, c1, c2, c3, key, out);
}

// Noise words of the four vocabulary entries 4*q .. 4*q+3 of one row.
__device__ __forceinline__ void noise_block(PhiloxKey key, uint32_t pos, uint32_t seq, uint32_t stream, uint32_t q,
                                            uint32_t out[4])
{
    philox4x32_10(q, pos, seq, stream, key, out);
}

// ---------------------------------------------------------------------------------
// 32 noise bits -> standard Gumbel variate, fp32.
//   k = r >> 9;  u = (2k+1) 2^-24;  w = 1 - u = (2k'+1) 2^-24 with k' = 2^23-1-k (both exact).
//   t = -ln u:  u <= 1/2 : hardware log2 of u;
//               u  > 1/2 : -log1p(-w); series for w < 2^-5 (truncation < 2^-27 relative),
//                          hardware log2 of 1-w otherwise (|log2| >= 0.045, so its absolute
//                          error of ~1 ulp stays ~1e-6 relative).
//   g = -ln t.
// ---------------------------------------------------------------------------------
__device__ __forceinline__ float gumbel_from_bits(uint32_t r)
{
    const uint32_t k = r >> 9;
    const uint32_t kc = 0x7FFFFFu - k;
    const float u = (float)(2u * k + 1u) * 0x1p-24f;
    const float w = (float)(2u * kc + 1u) * 0x1p-24f;
    const float t_log = -kLn2 * __log2f(u);
    const float t_ser = w * (1.0f + w * (0.5f + w * (0.333333343f + w * (0.25f + w * 0.2f))));
    const float t = (w < 0x1p-5f) ? t_ser : t_log;
    return -kLn2 * __log2f(t);
}

// Perturbed score of one vocabulary entry: y = x / T + g, with 1/T pre-rounded to fp32.
__device__ __forceinline__ float perturbed_score(float x, float inv_T, uint32_t r)
{
    return __fmaf_rn(x, inv_T, gumbel_from_bits(r));
}

// 2^x by the hardware instruction: results below 2^-126 flush to zero, which is what a
// softmax term that small should contribute.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ float uniform_from_bits(uint32_t r)
{
    return (float)(2u * (r >> 9) + 1u) * 0x1p-24f;
}

// ---------------------------------------------------------------------------------
// Row loads.  ELEMS consecutive logits starting at element `base` of a row, as fp32.
// Entries at or beyond V read as -inf (zero probability, never the argmax).
// ---------------------------------------------------------------------------------
template <int DT>
struct Elem;
template <>
struct Elem<0> {  // bf16
    typedef uint16_t type;
    static constexpr int kPerVec = 8;
    static __device__ __forceinline__ float to_float(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }
};
template <>
struct Elem<1> {  // fp32
    typedef float type;
    static constexpr int kPerVec = 4;
    static __device__ __forceinline__ float to_float(float f) { return f; }
};

template <int DT, bool ALIGNED>
__device__ __forceinline__ void load_elems(const typename Elem<DT>::type *row, int64_t base, int64_t V,
                                           float x[Elem<DT>::kPerVec])
{
    constexpr int E = Elem<DT>::kPerVec;
    const float ninf = -__builtin_inff();
    if (ALIGNED) {
        const uint4 q = *reinterpret_cast<const uint4 *>(row + base);
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
        if (base + E > V) {
#pragma unroll
            for (int j = 0; j < E; ++j)
                if (base + j >= V) x[j] = ninf;
        }
    } else {
#pragma unroll
        for (int j = 0; j < E; ++j) x[j] = (base + j < V) ? Elem<DT>::to_float(row[base + j]) : ninf;
    }
}

// ---------------------------------------------------------------------------------
// Fixed-shape reductions over the 256 threads of a workgroup.  The shape never depends
// on data, so results are bit-reproducible run to run.
// ---------------------------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

__device__ __forceinline__ float block_sum(float v, float *lds /* >= kWaves floats */)
{
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = v;
    __syncthreads();
    float s = lds[0];
#pragma unroll
    for (int i = 1; i < kWaves; ++i) s += lds[i];
    return s;
}

__device__ __forceinline__ int32_t block_sum_i32(int32_t v, int32_t *lds /* >= kWaves ints */)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = v;
    __syncthreads();
    int32_t s = lds[0];
#pragma unroll
    for (int i = 1; i < kWaves; ++i) s += lds[i];
    return s;
}

__device__ __forceinline__ float block_max(float v, float *lds /* >= kWaves floats */)
{
    v = wave_max(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = v;
    __syncthreads();
    float s = lds[0];
#pragma unroll
    for (int i = 1; i < kWaves; ++i) s = fmaxf(s, lds[i]);
    return s;
}

// (value, index) maximum with ties to the lowest index.
__device__ __forceinline__ void argmax_combine(float &y, int32_t &i, float oy, int32_t oi)
{
    if (oy > y || (oy == y && oi < i)) {
        y = oy;
        i = oi;
    }
}

__device__ __forceinline__ void block_argmax(float &y, int32_t &i, float *lds_y, int32_t *lds_i)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float oy = __shfl_xor(y, off, 64);
        const int32_t oi = __shfl_xor(i, off, 64);
        argmax_combine(y, i, oy, oi);
    }
    __syncthreads();
    if ((threadIdx.x & 63) == 0) {
        lds_y[threadIdx.x >> 6] = y;
        lds_i[threadIdx.x >> 6] = i;
    }
    __syncthreads();
    y = lds_y[0];
    i = lds_i[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) argmax_combine(y, i, lds_y[w], lds_i[w]);
}

// Per-row scalars every kernel needs.  `ok` is false for a sequence id outside [0,S)
// or a temperature that is not a positive finite number.
struct RowInfo {
    PhiloxKey key;
    uint32_t pos, seq;
    float T;
    int32_t claimed;
    bool seq_ok, temp_ok;
};

__device__ __forceinline__ RowInfo load_row_info(const RowBatch &b, int64_t row)
{
    RowInfo r;
    const int32_t s = b.seq_ids[row];
    r.seq_ok = (s >= 0 && (int64_t)s < b.S);
    const uint64_t seed = r.seq_ok ? b.seeds[s] : 0ull;
    r.key.k0 = (uint32_t)seed;
    r.key.k1 = (uint32_t)(seed >> 32);
    r.seq = (uint32_t)s;
    r.pos = b.positions[row];
    r.T = b.temperatures ? b.temperatures[row] : b.temperature;
    r.temp_ok = (r.T > 0.0f) && (r.T < __builtin_inff());
    r.claimed = b.claimed ? b.claimed[row] : -1;
    return r;
}

}  // namespace difr
