// Workgroup-wide exact selection on values held in registers (gfx950, 1024 threads = 16 wavefronts).
//
// A unit's N <= 1024 * EPT fp32 values live in registers, EPT per thread (element i = tid + j * 1024 sits
// in slot j of thread tid), as their order-preserving integer images (ord_key).  The k-th largest / smallest
// is found by narrowing a key interval [lo, hi]:
//   1. the interval starts as [min, max] of the unit's keys and is cut into at most 2048 equal bins of
//      2^shift keys; a 2048-bin LDS histogram of all keys and a workgroup-wide scan give the bin that holds
//      the wanted rank.  Starting from the data's own range spreads the histogram over many bins, whatever
//      the exponents of the values are;
//   2. the keys inside that bin (a few dozen out of tens of thousands) are copied to a list in LDS, and the
//      narrowing goes on over the list, one key per thread, until the bins are single keys (two more passes
//      at most).  Only if the bin holds more keys than the list does the narrowing continue over the
//      registers.
// The instruction count per element is what bounds these kernels (sixteen wavefronts share four SIMDs), so
// step 1 is three instructions per element when the unit fills its registers exactly, and the copy loop
// keeps branches out of the per-element path: a thread notes its first hit and counts them; threads with
// more than one hit (rare) go over their registers once more.
#pragma once

#include "nkv_device.h"

namespace nkv {

constexpr int kSelThreads = 1024;
constexpr int kSelBins = 2048;
constexpr int kSelList = 1024;       // candidates the LDS list holds: one per thread

struct SelectScratch {
    uint32_t hist[kSelBins];
    uint32_t list[2][kSelList];
    uint32_t nlist[2];
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

// Smallest and largest key of the unit (elements with index >= n do not count).  One reduction for both:
// max over (~min, max).
template <int EPT>
__device__ __forceinline__ void block_key_range(const uint32_t (&key)[EPT], int n, SelectScratch &s, uint32_t &kmin,
                                                uint32_t &kmax)
{
    uint32_t lo = 0xffffffffu, hi = 0u;
    if (n == EPT * kSelThreads) {
#pragma unroll
        for (int j = 0; j < EPT; ++j) { lo = min(lo, key[j]); hi = max(hi, key[j]); }
    } else {
#pragma unroll
        for (int j = 0; j < EPT; ++j)
            if ((int)threadIdx.x + j * kSelThreads < n) { lo = min(lo, key[j]); hi = max(hi, key[j]); }
    }
    uint32_t nlo = ~lo;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        nlo = max(nlo, (uint32_t)__shfl_xor((int)nlo, o, 64));
        hi = max(hi, (uint32_t)__shfl_xor((int)hi, o, 64));
    }
    if ((threadIdx.x & 63) == 0) { s.red[threadIdx.x >> 6] = nlo; s.wsum[threadIdx.x >> 6] = hi; }
    __syncthreads();
    uint32_t a = s.red[0], b = s.wsum[0];
#pragma unroll
    for (int i = 1; i < kSelThreads / 64; ++i) { a = max(a, s.red[i]); b = max(b, s.wsum[i]); }
    kmin = ~a;
    kmax = b;
    __syncthreads();                                                 // red / wsum are free again
}

// Bits to drop so that the interval [lo, hi] fits into kSelBins bins.
__device__ __forceinline__ int select_shift(uint32_t lo, uint32_t hi)
{
    const uint32_t width = hi - lo;                                  // >= 0
    const int bits = width == 0u ? 0 : 32 - __clz((int)width);
    return bits > 11 ? bits - 11 : 0;
}

// Histogram of all keys of the unit over [kmin, kmax] (every key lies inside).  Contains barriers.
template <int EPT>
__device__ __forceinline__ void hist_all(const uint32_t (&key)[EPT], int n, SelectScratch &s, uint32_t kmin, int shift)
{
    for (int j = threadIdx.x; j < kSelBins; j += kSelThreads) s.hist[j] = 0u;
    __syncthreads();
    if (n == EPT * kSelThreads) {
#pragma unroll
        for (int j = 0; j < EPT; ++j) atomicAdd(&s.hist[(key[j] - kmin) >> shift], 1u);
    } else {
#pragma unroll
        for (int j = 0; j < EPT; ++j)
            if ((int)threadIdx.x + j * kSelThreads < n) atomicAdd(&s.hist[(key[j] - kmin) >> shift], 1u);
    }
    __syncthreads();
}

// Copies the keys inside [lo, lo + span] to s.list[which]; s.nlist[which] must be zero (barrier) before, and
// a barrier must follow before the list is read.  The per-element part is branch-free: a thread notes its
// first hit and counts its hits; only wavefronts in which some thread has several hits go over the
// registers again.
template <int EPT>
__device__ __forceinline__ void collect(const uint32_t (&key)[EPT], int n, SelectScratch &s, int which, uint32_t lo,
                                        uint32_t span)
{
    const bool full = n == EPT * kSelThreads;
    uint32_t hits = 0u, first = 0u;
#pragma unroll
    for (int j = EPT - 1; j >= 0; --j) {                             // descending, so `first` ends as the lowest slot's hit
        const bool in = key[j] - lo <= span && (full || (int)threadIdx.x + j * kSelThreads < n);
        first = in ? key[j] : first;
        hits += in ? 1u : 0u;
    }
    uint32_t at = 0u;
    if (hits != 0u) {
        at = atomicAdd(&s.nlist[which], hits);
        if (at < (uint32_t)kSelList) s.list[which][at] = first;
    }
    if (__any(hits > 1u)) {                                          // rare
        uint32_t k = 0u;
#pragma unroll
        for (int j = 0; j < EPT; ++j) {
            const bool in = key[j] - lo <= span && (full || (int)threadIdx.x + j * kSelThreads < n);
            if (in && k != 0u && at + k < (uint32_t)kSelList) s.list[which][at + k] = key[j];
            k += in ? 1u : 0u;
        }
    }
}

// One narrowing pass over the registers: histogram of the keys inside [lo, hi], pick, new interval.  Returns
// true when the interval has become a single key.  All threads call it with the same lo / hi / want.
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

// The same over the first `cnt` entries of s.list[which], one entry per thread.
template <bool TOP>
__device__ __forceinline__ bool list_pass(SelectScratch &s, uint32_t cand, bool have, uint32_t &lo, uint32_t &hi,
                                          uint32_t &want, uint32_t &ties)
{
    const int shift = select_shift(lo, hi);
    for (int j = threadIdx.x; j < kSelBins; j += kSelThreads) s.hist[j] = 0u;
    __syncthreads();
    const uint32_t rel = cand - lo;
    if (have && rel <= hi - lo) atomicAdd(&s.hist[rel >> shift], 1u);
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

// Narrows [lo, hi] (a bin of the first histogram holding `count` keys, already copied to s.list[which] if
// they fit) down to a single key.
template <int EPT, bool TOP>
__device__ __forceinline__ void finish_select(const uint32_t (&key)[EPT], int n, SelectScratch &s, int which,
                                              uint32_t count, uint32_t &lo, uint32_t &hi, uint32_t &want,
                                              uint32_t &ties)
{
    if (count <= 64u) {
        // one wavefront: lane i ranks its candidate against all others; the candidate whose rank interval
        // [greater + 1, greater + equal] holds `want` is the answer
        if (threadIdx.x < 64) {
            const bool have = threadIdx.x < count;
            const uint32_t cand = have ? s.list[which][threadIdx.x] : 0u;
            uint32_t beyond = 0u, equal = 0u;
            for (uint32_t i = 0; i < count; ++i) {
                const uint32_t other = (uint32_t)__builtin_amdgcn_readlane((int)cand, (int)i);
                beyond += (TOP ? other > cand : other < cand) ? 1u : 0u;
                equal += other == cand ? 1u : 0u;
            }
            if (have && beyond < want && want <= beyond + equal) {    // same values write the same results
                s.bin = cand;
                s.rank = want - beyond;
                s.count = equal;
            }
        }
        __syncthreads();
        lo = hi = s.bin;
        want = s.rank;
        ties = s.count;
    } else if (count <= (uint32_t)kSelList) {
        const bool have = threadIdx.x < count;
        const uint32_t cand = have ? s.list[which][threadIdx.x] : 0u;
        while (!list_pass<TOP>(s, cand, have, lo, hi, want, ties)) {}
    } else {
        while (!select_pass<EPT, TOP>(key, n, s, lo, hi, want, ties)) {}
    }
}

// k-th largest (TOP) or k-th smallest key of the unit, 1 <= k <= n, inside the key range [kmin, kmax] of the
// unit (from block_key_range).  Returns the key T; `rem` = how many of the elements equal to T belong to the
// k selected ones (>= 1); `ties` = how many elements equal T.  All threads of the workgroup must call it;
// contains barriers.
template <int EPT, bool TOP>
__device__ __forceinline__ uint32_t block_select(const uint32_t (&key)[EPT], int n, uint32_t k, SelectScratch &s,
                                                 uint32_t kmin, uint32_t kmax, uint32_t &rem, uint32_t &ties)
{
    const int shift = select_shift(kmin, kmax);
    if (threadIdx.x == 0) s.nlist[0] = 0u;
    hist_all<EPT>(key, n, s, kmin, shift);
    block_pick<TOP>(s, k);
    uint32_t lo = kmin + (s.bin << shift), hi = shift == 0 ? lo : min(kmax, lo + ((1u << shift) - 1u));
    uint32_t want = s.rank;
    const uint32_t count = s.count;
    ties = count;
    if (shift != 0) {
        if (count <= (uint32_t)kSelList) collect<EPT>(key, n, s, 0, lo, hi - lo);
        __syncthreads();
        finish_select<EPT, TOP>(key, n, s, 0, count, lo, hi, want, ties);
    }
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
    if (threadIdx.x < 2) s.nlist[threadIdx.x] = 0u;
    hist_all<EPT>(key, n, s, kmin, shift);
    uint32_t lo[2], hi[2], want[2], count[2], ties[2];
    block_pick<true>(s, k);
    lo[0] = kmin + (s.bin << shift);
    hi[0] = shift == 0 ? lo[0] : min(kmax, lo[0] + ((1u << shift) - 1u));
    want[0] = s.rank;
    count[0] = s.count;
    __syncthreads();
    block_pick<false>(s, k);
    lo[1] = kmin + (s.bin << shift);
    hi[1] = shift == 0 ? lo[1] : min(kmax, lo[1] + ((1u << shift) - 1u));
    want[1] = s.rank;
    count[1] = s.count;
    if (shift != 0) {
        if (count[0] <= (uint32_t)kSelList) collect<EPT>(key, n, s, 0, lo[0], hi[0] - lo[0]);
        if (count[1] <= (uint32_t)kSelList) collect<EPT>(key, n, s, 1, lo[1], hi[1] - lo[1]);
        __syncthreads();
        finish_select<EPT, true>(key, n, s, 0, count[0], lo[0], hi[0], want[0], ties[0]);
        __syncthreads();
        finish_select<EPT, false>(key, n, s, 1, count[1], lo[1], hi[1], want[1], ties[1]);
    }
    __syncthreads();
    t_top = lo[0]; rem_top = want[0];
    t_bot = lo[1]; rem_bot = want[1];
}

}  // namespace nkv
