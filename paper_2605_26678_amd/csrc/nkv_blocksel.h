// Workgroup-wide exact selection on values held in registers (gfx950, 1024 threads = 16 wavefronts).
//
// A unit's N <= 1024 * EPT fp32 values live in registers, EPT per thread (element i = tid + j * 1024 sits
// in slot j of thread tid), as their order-preserving integer images (ord_key).  The k-th largest / smallest
// is found by narrowing a key interval [lo, hi]: the interval starts as [min, max] of the unit's keys and is
// cut into at most 2048 equal bins of 2^shift keys; a 2048-bin LDS histogram of the keys inside the interval
// and a workgroup-wide scan give the bin that holds the wanted rank, which becomes the next interval.  The
// bin width shrinks by a factor 2^11 per pass, so at most three passes end at single keys, and after the
// first pass only the few keys inside the chosen bin touch the histogram at all.  Starting from the data's
// own range spreads the first histogram over many bins, whatever the exponents of the values are.
#pragma once

#include "nkv_device.h"

namespace nkv {

constexpr int kSelThreads = 1024;
constexpr int kSelBins = 2048;

struct SelectScratch {
    uint32_t hist[kSelBins];
    uint32_t wsum[kSelThreads / 64];
    uint32_t red[kSelThreads / 64];
    uint32_t bin, rank, count;
};

// Finds the bin that holds rank `want` (1-based) counted from the top (TOP) or the bottom of s.hist.
// Writes s.bin, s.rank (rank inside that bin, in the same direction) and s.count (population of the bin).
// All threads call it; contains barriers; the histogram must be complete (barrier) before the call.
template <bool TOP> __device__ __forceinline__ void block_pick(SelectScratch &s, uint32_t want)
{
    constexpr int PER = kSelBins / kSelThreads;                       // 2 bins per thread
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    uint32_t c[PER], group = 0u;
#pragma unroll
    for (int q = 0; q < PER; ++q) { c[q] = s.hist[tid * PER + q]; group += c[q]; }
    uint32_t incl = group;                                           // inclusive sum towards the scan direction
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t t = TOP ? __shfl_down(incl, o, 64) : __shfl_up(incl, o, 64);
        if (TOP ? lane + o < 64 : lane >= o) incl += t;
    }
    if (lane == (TOP ? 0 : 63)) s.wsum[w] = incl;
    __syncthreads();
    if (TOP) { for (int ww = w + 1; ww < kSelThreads / 64; ++ww) incl += s.wsum[ww]; }
    else     { for (int ww = 0; ww < w; ++ww) incl += s.wsum[ww]; }
    uint32_t cum = incl - group;                                     // entries ranked before this thread's bins
    if (cum < want && want <= incl) {
#pragma unroll
        for (int qq = 0; qq < PER; ++qq) {
            const int q = TOP ? PER - 1 - qq : qq;
            if (cum < want && want <= cum + c[q]) {
                s.bin = (uint32_t)(tid * PER + q);
                s.rank = want - cum;
                s.count = c[q];
            }
            cum += c[q];
        }
    }
    __syncthreads();
}

__device__ __forceinline__ uint32_t block_min_key(uint32_t v, uint32_t *scratch)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = min(v, (uint32_t)__shfl_xor((int)v, o, 64));
    __syncthreads();
    if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = v;
    __syncthreads();
    uint32_t r = scratch[0];
    for (int i = 1; i < kSelThreads / 64; ++i) r = min(r, scratch[i]);
    return r;
}
__device__ __forceinline__ uint32_t block_max_key(uint32_t v, uint32_t *scratch)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = max(v, (uint32_t)__shfl_xor((int)v, o, 64));
    __syncthreads();
    if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = v;
    __syncthreads();
    uint32_t r = scratch[0];
    for (int i = 1; i < kSelThreads / 64; ++i) r = max(r, scratch[i]);
    return r;
}

// Smallest and largest key of the unit (elements with index >= n do not count).
template <int EPT>
__device__ __forceinline__ void block_key_range(const uint32_t (&key)[EPT], int n, SelectScratch &s, uint32_t &kmin,
                                                uint32_t &kmax)
{
    uint32_t lo = 0xffffffffu, hi = 0u;
#pragma unroll
    for (int j = 0; j < EPT; ++j)
        if ((int)threadIdx.x + j * kSelThreads < n) { lo = min(lo, key[j]); hi = max(hi, key[j]); }
    kmin = block_min_key(lo, s.red);
    kmax = block_max_key(hi, s.red);
}

// Bits to drop so that the interval [lo, hi] fits into kSelBins bins.
__device__ __forceinline__ int select_shift(uint32_t lo, uint32_t hi)
{
    const uint32_t width = hi - lo;                                  // >= 0
    const int bits = width == 0u ? 0 : 32 - __clz((int)width);
    return bits > 11 ? bits - 11 : 0;
}

// One narrowing pass: histogram of the keys inside [lo, hi], pick, new interval.  Returns true when the
// interval has become a single key.  All threads call it with the same lo / hi / want.
template <int EPT, bool TOP>
__device__ __forceinline__ bool select_pass(const uint32_t (&key)[EPT], int n, SelectScratch &s, uint32_t &lo,
                                            uint32_t &hi, uint32_t &want, uint32_t &ties)
{
    const int shift = select_shift(lo, hi);
    for (int j = threadIdx.x; j < kSelBins; j += kSelThreads) s.hist[j] = 0u;
    __syncthreads();
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const uint32_t rel = key[j] - lo;                            // wraps for keys below lo: then > hi - lo
        if ((int)threadIdx.x + j * kSelThreads < n && rel <= hi - lo) atomicAdd(&s.hist[rel >> shift], 1u);
    }
    __syncthreads();
    block_pick<TOP>(s, want);
    const uint32_t nlo = lo + (s.bin << shift);
    const uint32_t nhi = shift == 0 ? nlo : min(hi, nlo + ((1u << shift) - 1u));
    want = s.rank;
    ties = s.count;
    lo = nlo;
    hi = nhi;
    return shift == 0;
}

// k-th largest (TOP) or k-th smallest key of the unit, 1 <= k <= n, inside the key range [kmin, kmax] of the
// unit (from block_key_range).  Returns the key T; `rem` = how many of the elements equal to T belong to the
// k selected ones (>= 1); `ties` = how many elements equal T.  All threads of the workgroup must call it;
// contains barriers.
template <int EPT, bool TOP>
__device__ __forceinline__ uint32_t block_select(const uint32_t (&key)[EPT], int n, uint32_t k, SelectScratch &s,
                                                 uint32_t kmin, uint32_t kmax, uint32_t &rem, uint32_t &ties)
{
    uint32_t lo = kmin, hi = kmax, want = k;
    while (!select_pass<EPT, TOP>(key, n, s, lo, hi, want, ties)) {}
    rem = want;
    __syncthreads();                                                 // scratch may be reused right away
    return lo;
}

// The k-th largest and the k-th smallest at once: the first histogram over [kmin, kmax] serves both.
template <int EPT>
__device__ __forceinline__ void block_select_both(const uint32_t (&key)[EPT], int n, uint32_t k, SelectScratch &s,
                                                  uint32_t kmin, uint32_t kmax, uint32_t &t_top, uint32_t &rem_top,
                                                  uint32_t &t_bot, uint32_t &rem_bot)
{
    const int shift = select_shift(kmin, kmax);
    for (int j = threadIdx.x; j < kSelBins; j += kSelThreads) s.hist[j] = 0u;
    __syncthreads();
#pragma unroll
    for (int j = 0; j < EPT; ++j)
        if ((int)threadIdx.x + j * kSelThreads < n) atomicAdd(&s.hist[(key[j] - kmin) >> shift], 1u);
    __syncthreads();
    uint32_t lo[2], hi[2], want[2], ties[2];
    block_pick<true>(s, k);
    lo[0] = kmin + (s.bin << shift);
    hi[0] = shift == 0 ? lo[0] : min(kmax, lo[0] + ((1u << shift) - 1u));
    want[0] = s.rank;
    ties[0] = s.count;
    __syncthreads();
    block_pick<false>(s, k);
    lo[1] = kmin + (s.bin << shift);
    hi[1] = shift == 0 ? lo[1] : min(kmax, lo[1] + ((1u << shift) - 1u));
    want[1] = s.rank;
    ties[1] = s.count;
    __syncthreads();
    if (shift != 0) {
        while (!select_pass<EPT, true>(key, n, s, lo[0], hi[0], want[0], ties[0])) {}
        __syncthreads();
        while (!select_pass<EPT, false>(key, n, s, lo[1], hi[1], want[1], ties[1])) {}
        __syncthreads();
    }
    t_top = lo[0]; rem_top = want[0];
    t_bot = lo[1]; rem_bot = want[1];
}

}  // namespace nkv
