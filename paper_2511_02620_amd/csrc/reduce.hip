// Pooling and flagging: per-sequence mean / max / mismatch count of token scores and
// the threshold decision (Sec. 5.2 threshold rule; Sec. 6.4 pooling; appendix
// "Response to detecting exfiltration attempts": score, pool, flag).
//
// One workgroup per sequence.  Each thread accumulates a strided share in fp64, then a
// fixed binary tree over the 256 partials: no atomics, so the result is reproducible.
#include <math.h>

#include "difr_device.hpp"
#include "difr_host.hpp"

namespace difr {

__global__ __launch_bounds__(kBlock) void seq_reduce_kernel(const float *__restrict__ scores,
                                                            const uint8_t *__restrict__ row_flags,
                                                            const int64_t *__restrict__ seq_offsets, int64_t N,
                                                            float threshold, float *__restrict__ seq_mean,
                                                            float *__restrict__ seq_max,
                                                            int32_t *__restrict__ seq_mismatch,
                                                            uint8_t *__restrict__ seq_flag)
{
    __shared__ double lds_sum[kBlock];
    __shared__ float lds_max[kBlock];
    __shared__ int32_t lds_mis[kBlock];
    __shared__ int32_t lds_nan[kBlock];

    const int64_t s = blockIdx.x;
    const int tid = threadIdx.x;
    int64_t lo = seq_offsets[s], hi = seq_offsets[s + 1];
    if (lo < 0) lo = 0;
    if (hi > N) hi = N;

    double sum = 0.0;
    float mx = -__builtin_inff();
    int32_t mis = 0, any_nan = 0;
    for (int64_t n = lo + tid; n < hi; n += kBlock) {
        const float v = scores[n];
        sum += (double)v;
        any_nan |= (int32_t)(v != v);
        mx = fmaxf(mx, v);
        if (row_flags) mis += (int32_t)((row_flags[n] & kFlagMatch) == 0u);
    }
    lds_sum[tid] = sum;
    lds_max[tid] = mx;
    lds_mis[tid] = mis;
    lds_nan[tid] = any_nan;
    __syncthreads();
#pragma unroll
    for (int half = kBlock / 2; half >= 1; half >>= 1) {
        if (tid < half) {
            lds_sum[tid] += lds_sum[tid + half];
            lds_max[tid] = fmaxf(lds_max[tid], lds_max[tid + half]);
            lds_mis[tid] += lds_mis[tid + half];
            lds_nan[tid] |= lds_nan[tid + half];
        }
        __syncthreads();
    }
    if (tid == 0) {
        const int64_t len = hi - lo;
        float mean = 0.0f, mxo = 0.0f;
        int32_t mo = 0;
        uint8_t fl = 0;
        if (len > 0) {
            mean = (float)(lds_sum[0] / (double)len);
            mxo = lds_nan[0] ? __builtin_nanf("") : lds_max[0];
            mo = lds_mis[0];
            fl = (mean <= threshold) ? 0 : 1;
        }
        if (seq_mean) seq_mean[s] = mean;
        if (seq_max) seq_max[s] = mxo;
        if (seq_mismatch) seq_mismatch[s] = mo;
        if (seq_flag) seq_flag[s] = fl;
    }
}

// Three-class token classification and per-token exfiltratable information (Sec. 7.1 and the
// appendix algorithm "risk classification via score and rank").  Scores are suspiciousness:
//   SAFE (0)        score <= tau                        bits = log2|A_t| if supplied, else 0
//   SUSPICIOUS (1)  score >  tau and 0 <= rank < R      bits = log2 R
//   DANGEROUS (2)   otherwise (NaN score, rank -1)      bits = log2 V
__global__ __launch_bounds__(kBlock) void classify_kernel(const float *__restrict__ scores,
                                                          const int32_t *__restrict__ ranks, int64_t N, float tau,
                                                          int64_t R, float log2_R, float log2_V,
                                                          const float *__restrict__ log2_admissible,
                                                          uint8_t *__restrict__ cls, float *__restrict__ bits)
{
    for (int64_t n = (int64_t)blockIdx.x * kBlock + threadIdx.x; n < N; n += (int64_t)gridDim.x * kBlock) {
        const float s = scores[n];
        const int32_t r = ranks[n];
        uint8_t c;
        float b;
        if (s <= tau) {
            c = 0;
            b = log2_admissible ? log2_admissible[n] : 0.0f;
        } else if (s > tau && R > 0 && r >= 0 && (int64_t)r < R) {
            c = 1;
            b = log2_R;
        } else {
            c = 2;
            b = log2_V;
        }
        cls[n] = c;
        if (bits) bits[n] = b;
    }
}

int launch_classify(const float *scores, const int32_t *ranks, int64_t N, float tau, int64_t R, int64_t V,
                    const float *log2_admissible, uint8_t *cls, float *bits, hipStream_t stream)
{
    int64_t blocks = (N + kBlock - 1) / kBlock;
    if (blocks > 65536) blocks = 65536;
    const float log2_R = R > 0 ? (float)log2((double)R) : 0.0f;
    const float log2_V = (float)log2((double)V);
    classify_kernel<<<dim3((unsigned)blocks), dim3(kBlock), 0, stream>>>(scores, ranks, N, tau, R, log2_R, log2_V,
                                                                         log2_admissible, cls, bits);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

int launch_seq_reduce(const float *scores, const uint8_t *row_flags, const int64_t *seq_offsets, int64_t N,
                      int64_t S, float threshold, float *seq_mean, float *seq_max, int32_t *seq_mismatch,
                      uint8_t *seq_flag, hipStream_t stream)
{
    seq_reduce_kernel<<<dim3((unsigned)S), dim3(kBlock), 0, stream>>>(scores, row_flags, seq_offsets, N, threshold,
                                                                      seq_mean, seq_max, seq_mismatch, seq_flag);
    return hipGetLastError() == hipSuccess ? 0 : 1;
}

}  // namespace difr
