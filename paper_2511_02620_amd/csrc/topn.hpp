// Exact streaming selection of the n largest (key, index) pairs of a row by one workgroup.
//
// Candidates are pushed into an LDS buffer as 64-bit composites (order-preserving image of the float
// key in the high word, complemented index in the low word: a larger composite is a larger key or,
// for equal keys, a smaller index, so all composites of a row are distinct).  Only composites above the
// current threshold are pushed.  When the buffer is half full the workgroup finds the n-th largest
// composite with a radix select (8 passes of 8 bits over the buffer), makes it the new threshold and
// keeps exactly the n entries at or above it.  A round of the row stream pushes at most 2048 entries
// (256 lanes x 8), so with 4096 slots and a check after every round the buffer never overflows, whatever
// the order of the data; nothing that belongs to the final top n is ever dropped, because the threshold
// is always the n-th largest of what has been seen and only grows.
#pragma once

#include "difr_device.hpp"

namespace difr {

constexpr int kTopCap = 4096;      // slots per buffer
constexpr int kTopTrigger = 2048;  // compact when this many slots are used
constexpr int kTopMaxN = 256;      // largest n supported

// float -> uint32 such that a < b  <=>  image(a) < image(b)  (-0 < +0; NaNs must be kept out by the caller)
__device__ __forceinline__ uint32_t float_order_bits(float f)
{
    const uint32_t b = __float_as_uint(f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float float_from_order_bits(uint32_t o)
{
    return __uint_as_float((o & 0x80000000u) ? (o & 0x7FFFFFFFu) : ~o);
}
__device__ __forceinline__ uint64_t top_composite(float key, int32_t index)
{
    return ((uint64_t)float_order_bits(key) << 32) | (uint64_t)(0xFFFFFFFFu - (uint32_t)index);
}
__device__ __forceinline__ float top_key(uint64_t c) { return float_from_order_bits((uint32_t)(c >> 32)); }
__device__ __forceinline__ int32_t top_index(uint64_t c) { return (int32_t)(0xFFFFFFFFu - (uint32_t)c); }

// LDS scratch shared by the selections of one workgroup (they never run at the same time).
struct TopScratch {
    int32_t hist[256];
    int32_t wave_sum[kWaves];
    int32_t sel_bin, sel_need, kept;
    uint64_t tmp[kTopMaxN];
};

struct TopN {
    uint64_t *buf;   // kTopCap slots in LDS
    int32_t *count;  // in LDS
    int n;
    uint64_t theta;  // wave-uniform copy of the threshold: only composites above it are pushed
    bool full;       // this thread's push took the buffer to the compaction trigger (combine over the workgroup
                     // with __syncthreads_or: reading the counter instead would race with the next round's pushes)

    __device__ __forceinline__ void init(uint64_t *buf_, int32_t *count_, int n_)
    {
        buf = buf_;
        count = count_;
        n = n_;
        theta = n_ > 0 ? 0ull : ~0ull;  // nothing wanted: nothing is ever pushed
        full = false;
        if (threadIdx.x == 0) *count = 0;
    }

    __device__ __forceinline__ void push(uint64_t c)
    {
        if (c > theta) {
            const int32_t i = atomicAdd(count, 1);
            if (i < kTopCap) buf[i] = c;  // always true by construction (see the header comment)
            if (i >= kTopTrigger - 1) full = true;
        }
    }

    // All 256 threads, after a __syncthreads() that follows the pushes.  If the buffer holds more than n
    // entries, reduce it to the n largest and raise the threshold to the smallest of them.  Returns true if
    // the threshold moved.  Ends with a __syncthreads().
    __device__ bool compact(TopScratch &s)
    {
        const int tid = threadIdx.x;
        const int cnt = min(*count, kTopCap);
        full = false;
        if (n <= 0) {  // nothing wanted: an impossible threshold
            __syncthreads();
            if (tid == 0) *count = 0;
            theta = ~0ull;
            __syncthreads();
            return true;
        }
        if (cnt <= n) {
            __syncthreads();
            return false;
        }
        uint64_t prefix = 0ull, mask = 0ull;
        int need = n;
        for (int pass = 7; pass >= 0; --pass) {
            const int shift = 8 * pass;
            s.hist[tid] = 0;
            __syncthreads();
            for (int i = tid; i < cnt; i += kBlock) {
                const uint64_t c = buf[i];
                if ((c & mask) == prefix) atomicAdd(&s.hist[(int)((c >> shift) & 255ull)], 1);
            }
            __syncthreads();
            // suffix sums over the 256 bins: thread b gets the number of entries in bins >= b
            int v = s.hist[tid];
            const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const int o = __shfl_down(v, off, 64);
                if (lane + off < 64) v += o;
            }
            if (lane == 0) s.wave_sum[wave] = v;
            __syncthreads();
            for (int w = wave + 1; w < kWaves; ++w) v += s.wave_sum[w];
            const int above = v - s.hist[tid];  // entries in bins > tid
            if (above < need && v >= need) {    // exactly one thread
                s.sel_bin = tid;
                s.sel_need = need - above;
            }
            __syncthreads();
            prefix |= (uint64_t)s.sel_bin << shift;
            mask |= 255ull << shift;
            need = s.sel_need;
            __syncthreads();
        }
        // prefix is now the n-th largest composite; keep the n entries at or above it
        if (tid == 0) s.kept = 0;
        __syncthreads();
        for (int i = tid; i < cnt; i += kBlock) {
            const uint64_t c = buf[i];
            if (c >= prefix) {
                const int j = atomicAdd(&s.kept, 1);
                if (j < kTopMaxN) s.tmp[j] = c;
            }
        }
        __syncthreads();
        if (tid < n) buf[tid] = s.tmp[tid];
        if (tid == 0) *count = n;
        theta = prefix;
        __syncthreads();
        return true;
    }

    // All 256 threads: final compaction, then sort the survivors in descending order into buf[0 .. m),
    // m = min(n, entries seen); returns m.  Bitonic network over 256 slots (empty slots hold 0, which sorts last).
    __device__ int finish_sorted(TopScratch &s)
    {
        const int tid = threadIdx.x;
        __syncthreads();
        compact(s);
        const int m = min(min(*count, kTopCap), n);
        uint64_t mine = tid < m ? buf[tid] : 0ull;
        __syncthreads();
        s.tmp[tid] = mine;
        __syncthreads();
        for (int k = 2; k <= kTopMaxN; k <<= 1) {
            for (int j = k >> 1; j > 0; j >>= 1) {
                const int partner = tid ^ j;
                const uint64_t a = s.tmp[tid], b = s.tmp[partner];
                const bool descending = (tid & k) == 0;
                const bool keep_larger = (tid < partner) == descending;
                const uint64_t mine2 = keep_larger ? (a > b ? a : b) : (a > b ? b : a);
                __syncthreads();
                s.tmp[tid] = mine2;
                __syncthreads();
            }
        }
        buf[tid] = s.tmp[tid];
        __syncthreads();
        return m;
    }
};

}  // namespace difr
