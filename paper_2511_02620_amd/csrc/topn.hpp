// Exact streaming selection of the n largest (key, index) pairs of a row by one workgroup.
//
// Candidates are pushed into an LDS buffer as 64-bit composites (order-preserving image of the float
// key in the high word, complemented index in the low word: a larger composite is a larger key or,
// for equal keys - -0 and +0 are equal -, a smaller index, so all composites of a row are distinct).  Only composites above the
// current threshold are pushed.  A compaction finds a lower bound of the n-th largest composite with a
// radix select over the buffer, makes it the new threshold and keeps the entries at or above it.  In the
// stream the select stops after the top 16 bits of the key (2 passes of 8 bits: the n-th largest key at
// bf16 resolution, a handful of entries too many survive) unless more than kTopKeep entries share them;
// all 8 passes, down to the exact n-th composite, run at the end of the row.  Nothing that belongs to the
// final top n is ever dropped: the threshold is a lower bound of the n-th largest of what has been seen.
//
// Capacity.  The caller works in epochs of a few stream rounds without any barrier.  A push that finds the
// buffer full raises `over` instead of storing its entry, and the caller then starts the row again in a careful
// mode: one wave and one round at a time, with a compaction check after each such step.  A step starts with
// fewer than kTopTrigger entries and adds at most 8 per thread of one wave, so in that mode kTopCapSmall =
// kTopTrigger + 64 * 8 slots always suffice, whatever the order of the data.  Small buffers are what lets five
// workgroups share a compute unit; selections of more than kTopSmallN entries push so much in an ordinary epoch
// that they get kTopCapBig slots instead (the kernels are instantiated for both).
#pragma once

#include "difr_device.hpp"

namespace difr {

constexpr int kTopEpoch = 8;       // stream rounds per epoch (measured: 4 and 16 are both slower)
constexpr int kTopFresh = 16;      // a compaction is due after max(n, kTopFresh) pushes (measured: 8 to 64 within 1%)
constexpr int kTopTrigger = 512;   // a compaction is due at the latest when this many slots are used
constexpr int kTopCapSmall = kTopTrigger + 64 * 8;   // slots per buffer: the trigger plus one round of one wave
constexpr int kTopCapBig = kTopTrigger + 256 * 8;    // ... of the whole workgroup
constexpr int kTopSmallN = 64;     // largest n served with the small buffer
constexpr int kTopMaxN = 256;      // largest n supported
constexpr int kTopKeep = 256;      // a coarse compaction may leave up to this many entries
constexpr int kTopRankMax = 96;    // a coarse compaction of more entries than this goes by radix passes: counting ranks
                                   // costs every thread two instructions per entry, two 8-bit passes about 150 in all

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
// (-0 and +0 are the same key - between them the index decides -, so -0 is read as +0: x + 0 does that)
__device__ __forceinline__ uint64_t top_composite(float key, int32_t index)
{
    return ((uint64_t)float_order_bits(key + 0.0f) << 32) | (uint64_t)(0xFFFFFFFFu - (uint32_t)index);
}
__device__ __forceinline__ float top_key(uint64_t c) { return float_from_order_bits((uint32_t)(c >> 32)); }
__device__ __forceinline__ int32_t top_index(uint64_t c) { return (int32_t)(0xFFFFFFFFu - (uint32_t)c); }

// LDS scratch shared by the selections of one workgroup (they never run at the same time).
struct TopScratch {
    int32_t hist[256];
    int32_t wave_sum[kWaves];
    int32_t sel_bin, sel_need, kept;
    uint64_t sel64;
    uint64_t tmp[kTopKeep];
};

struct TopN {
    uint64_t *buf;   // `cap` slots in LDS
    int cap;
    int32_t *count;  // in LDS
    int n;
    uint64_t theta;  // wave-uniform copy of the threshold: only composites above it are pushed
    int trigger;     // fill level at which the next compaction is due: max(n, kTopFresh) pushes after the last one, so
                     // that the threshold, which is also the bound of the stream's gates, stays fresh
    bool full;       // this thread's push took the buffer to the compaction trigger (combine over the workgroup
                     // with __syncthreads_or: reading the counter instead would race with the next round's pushes)
    bool over;       // a push of this thread found the buffer full: the row must be started again, carefully
    bool priming;    // see begin_prime()
    uint64_t prime_best;

    __device__ __forceinline__ void init(uint64_t *buf_, int32_t *count_, int n_, int cap_)
    {
        buf = buf_;
        cap = cap_;
        count = count_;
        n = n_;
        theta = n_ > 0 ? 0ull : ~0ull;  // nothing wanted: nothing is ever pushed
        trigger = n_ > kTopFresh ? n_ : kTopFresh;
        full = false;
        over = false;
        priming = false;
        prime_best = 0ull;
        if (threadIdx.x == 0) *count = 0;
    }

    __device__ __forceinline__ void new_epoch() { over = false; }

    // Priming.  While there is no threshold every entry of the first round is a candidate: 2048 pushes through
    // one counter and a compaction over all of them.  Instead the first round is run twice: the first time each
    // thread only remembers its best candidate; the n-th largest of those 256 is a valid lower bound of the
    // n-th largest overall (they are real entries), it becomes the threshold, and the second, ordinary run of
    // the round pushes only what lies above it.
    __device__ __forceinline__ void begin_prime()
    {
        priming = true;
        prime_best = 0ull;
    }
    // All 256 threads, after the priming run of the round; ends with a __syncthreads().  Returns true if a
    // threshold was found (the caller re-targets its gates either way and runs the round again).
    __device__ __forceinline__ bool end_prime(TopScratch &s)
    {
        priming = false;
        // (a small selection does not need all 256 candidates: the best of every 4 or 2 neighbouring lanes are real
        // entries too, and the n-th largest of 64 or 128 of them costs a fraction of the rank count over 256 to find -
        // it lies a few ranks lower, which lets a few more entries of the first round through)
        const int group = n <= 32 ? 4 : (n <= 100 ? 2 : 1);
        if (group >= 2) {
            const uint64_t o = __shfl_xor(prime_best, 1, 64);
            if (o > prime_best) prime_best = o;
        }
        if (group >= 4) {
            const uint64_t o = __shfl_xor(prime_best, 2, 64);
            if (o > prime_best) prime_best = o;
        }
        if (prime_best != 0ull && ((int)threadIdx.x & (group - 1)) == 0) {
            const int32_t i = atomicAdd(count, 1);
            buf[i] = prime_best;  // at most one per thread
        }
        __syncthreads();
        const bool moved = compact(s, false);
        // the primed entries are dropped (they come again with the round itself); the n-th largest of them must
        // pass the push test then, so the threshold is put just below it
        if (threadIdx.x == 0) *count = 0;
        if (moved) theta -= 1ull;
        trigger = min(kTopTrigger, n > kTopFresh ? n : kTopFresh);
        full = false;
        __syncthreads();
        return moved;
    }

    __device__ __forceinline__ void push(uint64_t c)
    {
        if (priming) {
            if (c > theta && c > prime_best) prime_best = c;
            return;
        }
        if (c > theta) {
            const int32_t i = atomicAdd(count, 1);
            if (i < cap)
                buf[i] = c;
            else
                over = true;  // no room: the entry is dropped and the row has to be started again
            if (i >= trigger - 1) full = true;
        }
    }

    // All 256 threads, after a barrier that follows the pushes.  If the buffer holds more than n entries,
    // raise the threshold to a lower bound of the n-th largest composite and keep only the entries at or
    // above it: exactly the n largest (coarse = false), or at most kTopKeep of them chosen at the
    // resolution of the top 16 key bits (coarse = true).  Returns true if the threshold moved.  Ends with
    // a __syncthreads().
    __device__ __forceinline__ bool compact(TopScratch &s, bool coarse = false)
    {
        const int tid = threadIdx.x;
        const int cnt = min(*count, cap);
        full = false;
        if (n <= 0) {  // nothing wanted: an impossible threshold
            __syncthreads();
            if (tid == 0) *count = 0;
            theta = ~0ull;
            __syncthreads();
            return true;
        }
        if (cnt <= n) {
            trigger = min(kTopTrigger, cnt + (n > kTopFresh ? n : kTopFresh));
            __syncthreads();
            return false;
        }
        const bool by_rank = !coarse || cnt <= kTopRankMax;
        if (by_rank && cnt <= kBlock) {
            // Few entries: every entry finds its rank by counting the entries above it (broadcast reads), the n
            // best move to the front in rank order and the n-th of them is the new, exact threshold.  Three
            // barriers instead of the dozen of the radix select below.
            const uint64_t mine = tid < cnt ? buf[tid] : 0ull;
            int r = 0;
            for (int i = 0; i < cnt; ++i) r += (int)(buf[i] > mine);
            if (tid < cnt && r == n - 1) s.sel64 = mine;
            __syncthreads();
            if (tid < cnt && r < n) buf[r] = mine;
            if (tid == 0) *count = n;
            theta = s.sel64;
            trigger = min(kTopTrigger, n + (n > kTopFresh ? n : kTopFresh));
            __syncthreads();
            return true;
        }
        if (by_rank && cnt <= 2 * kBlock) {
            // the same with two entries per thread: one broadcast read serves both
            uint64_t mine0 = buf[tid], mine1 = tid + kBlock < cnt ? buf[tid + kBlock] : 0ull;
            int r0 = 0, r1 = 0;
            for (int i = 0; i < cnt; ++i) {
                const uint64_t c = buf[i];
                r0 += (int)(c > mine0);
                r1 += (int)(c > mine1);
            }
            if (r0 == n - 1) s.sel64 = mine0;
            if (tid + kBlock < cnt && r1 == n - 1) s.sel64 = mine1;
            __syncthreads();
            if (r0 < n) buf[r0] = mine0;
            if (tid + kBlock < cnt && r1 < n) buf[r1] = mine1;
            if (tid == 0) *count = n;
            theta = s.sel64;
            trigger = min(kTopTrigger, n + (n > kTopFresh ? n : kTopFresh));
            __syncthreads();
            return true;
        }
        uint64_t prefix = 0ull, mask = 0ull;
        int need = n;        // rank of the wanted composite among the entries that match the prefix
        int at_or_above = cnt;  // entries at or above the prefix found so far (unset low bits zero)
        for (int pass = 7; pass >= 0; --pass) {
            if (coarse && pass < 6 && at_or_above <= kTopKeep) break;
            if (at_or_above == n) break;  // the prefix already separates exactly n entries from the rest
            const int shift = 8 * pass;
            s.hist[tid] = 0;
            __syncthreads();
            for (int i = tid; i < cnt; i += kBlock) {
                const uint64_t c = buf[i];
                if ((c & mask) == prefix) atomicAdd(&s.hist[(int)((c >> shift) & 255ull)], 1);
            }
            __syncthreads();
            // suffix sums over the 256 bins: thread b gets the number of matching entries in bins >= b
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
            const int above = v - s.hist[tid];  // matching entries in bins > tid
            if (above < need && v >= need) {    // exactly one thread
                s.sel_bin = tid;
                s.sel_need = need - above;
                s.kept = (n - need) + v;
            }
            __syncthreads();
            prefix |= (uint64_t)s.sel_bin << shift;
            mask |= 255ull << shift;
            need = s.sel_need;
            at_or_above = s.kept;
            __syncthreads();
        }
        // gather the survivors (at_or_above <= kTopKeep of them) and move them to the front
        if (tid == 0) s.kept = 0;
        __syncthreads();
        for (int i = tid; i < cnt; i += kBlock) {
            const uint64_t c = buf[i];
            if (c >= prefix) {
                const int j = atomicAdd(&s.kept, 1);
                if (j < kTopKeep) s.tmp[j] = c;
            }
        }
        __syncthreads();
        for (int i = tid; i < at_or_above; i += kBlock) buf[i] = s.tmp[i];
        if (tid == 0) *count = at_or_above;
        theta = prefix;
        trigger = min(kTopTrigger, at_or_above + (n > kTopFresh ? n : kTopFresh));
        __syncthreads();
        return true;
    }

    // All 256 threads: reduce to exactly the n largest, then order them.  Afterwards buf[0 .. m) holds them in
    // descending order, m = min(n, entries seen); returns m.  Each survivor finds its rank by counting the
    // survivors above it (m <= 256 broadcast reads, no barriers).
    __device__ __forceinline__ int finish_sorted(TopScratch &s)
    {
        const int tid = threadIdx.x;
        __syncthreads();
        compact(s, false);
        const int m = min(min(*count, cap), n);
        if (tid < m) {
            const uint64_t mine = buf[tid];
            int rank = 0;
            for (int i = 0; i < m; ++i) rank += (int)(buf[i] > mine);
            s.tmp[rank] = mine;
        }
        __syncthreads();
        if (tid < m) buf[tid] = s.tmp[tid];
        __syncthreads();
        return m;
    }
};

}  // namespace difr
