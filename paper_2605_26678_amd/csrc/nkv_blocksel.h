// Workgroup-wide exact selection on values held in registers (gfx950, 1024 threads = 16 wavefronts).
//
// A unit's N <= 1024 * EPT fp32 values live in registers, EPT per thread (element i = tid + j * 1024 sits
// in slot j of thread tid).  The k-th largest / smallest is found by a byte-wise radix select, most
// significant digit first, on the order-preserving integer image of the floats (ord_key): four passes,
// each a 256-bin LDS histogram of the current digit among the still-matching candidates, followed by a
// 64-lane scan that picks the digit holding the wanted rank.  Equal consecutive digits are counted in the
// thread before they are added to LDS, so a degenerate digit (all scores share their exponent) costs one
// atomic per thread instead of one per element.
#pragma once

#include "nkv_device.h"

namespace nkv {

constexpr int kSelThreads = 1024;

struct SelectScratch {
    uint32_t hist[256];
    uint32_t digit, want, ties;
};

// One lane per 4 bins; finds the bin that holds rank `want` counting from the top (TOP) or the bottom.
// Writes s.digit, s.want (rank inside that bin) and s.ties (population of that bin).  Called by one full wave.
template <bool TOP> __device__ __forceinline__ void pick_digit(SelectScratch &s, uint32_t want)
{
    const int lane = threadIdx.x & 63;
    const uint4 h = reinterpret_cast<const uint4 *>(s.hist)[lane];
    const uint32_t c[4] = {h.x, h.y, h.z, h.w};
    const uint32_t group = h.x + h.y + h.z + h.w;
    uint32_t incl = group;                                   // inclusive sum towards the scan direction
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t t = TOP ? __shfl_down(incl, o, 64) : __shfl_up(incl, o, 64);
        if (TOP ? lane + o < 64 : lane >= o) incl += t;
    }
    uint32_t cum = incl - group;                             // candidates ranked before this lane's bins
    if (cum < want && want <= incl) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int b = TOP ? 3 - q : q;
            if (cum < want && want <= cum + c[b]) {
                s.digit = (uint32_t)(4 * lane + b);
                s.want = want - cum;
                s.ties = c[b];
            }
            cum += c[b];
        }
    }
}

// Adds the digit of every matching candidate of this thread to the histogram, run-length compressed.
template <int EPT>
__device__ __forceinline__ void count_digits(const uint32_t (&key)[EPT], int n, uint32_t prefix, int pass,
                                             uint32_t *hist)
{
    const int shift = 24 - 8 * pass;
    uint32_t cur = 0u, cnt = 0u;
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const bool in = (int)threadIdx.x + j * kSelThreads < n &&
                        (pass == 0 || ((key[j] ^ prefix) >> (shift + 8)) == 0u);
        const uint32_t d = (key[j] >> shift) & 255u;
        if (in) {
            if (cnt != 0u && d != cur) { atomicAdd(&hist[cur], cnt); cnt = 0u; }
            cur = d;
            ++cnt;
        }
    }
    if (cnt != 0u) atomicAdd(&hist[cur], cnt);
}

// k-th largest (TOP) or k-th smallest key of the unit, 1 <= k <= n.  Returns the key T; `rem` = how many
// of the elements equal to T belong to the k selected ones (>= 1); `ties` = how many elements equal T.
// All threads of the workgroup must call it; contains barriers.
template <int EPT, bool TOP>
__device__ __forceinline__ uint32_t block_select(const uint32_t (&key)[EPT], int n, uint32_t k, SelectScratch &s,
                                                 uint32_t &rem, uint32_t &ties)
{
    uint32_t prefix = 0u, want = k;
    for (int pass = 0; pass < 4; ++pass) {
        if (threadIdx.x < 256) s.hist[threadIdx.x] = 0u;
        __syncthreads();
        count_digits<EPT>(key, n, prefix, pass, s.hist);
        __syncthreads();
        if (threadIdx.x < 64) pick_digit<TOP>(s, want);
        __syncthreads();
        prefix |= s.digit << (24 - 8 * pass);
        want = s.want;
    }
    rem = want;
    ties = s.ties;
    __syncthreads();                                         // scratch may be reused right away
    return prefix;
}

}  // namespace nkv
