// Exact selection among a few hundred keys by a single wavefront (gfx950, 64 lanes).
#pragma once

#include "nkv_device.h"

namespace nkv {

// `want`-th largest (1-based) of the n keys key_at(0..n-1): byte-wise radix select by one wavefront; hist: 256
// words of LDS owned by the wave.  Returns the key; gt = how many keys are larger, eq = how many are equal.
template <typename F>
__device__ __forceinline__ uint32_t wave_select_fn(int n, uint32_t want, uint32_t *hist, uint32_t &gt, uint32_t &eq,
                                                   F key_at)
{
    const int lane = threadIdx.x & 63;
    uint32_t prefix = 0u;
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        for (int j = lane; j < 256; j += 64) hist[j] = 0u;
        __builtin_amdgcn_wave_barrier();
        for (int i = lane; i < n; i += 64) {
            const uint32_t k = key_at(i);
            if (pass == 0 || (k >> (shift + 8)) == (prefix >> (shift + 8))) atomicAdd(&hist[(k >> shift) & 255u], 1u);
        }
        __builtin_amdgcn_wave_barrier();
        // lane owns digits 4 lane .. 4 lane + 3; running count from the top
        const uint32_t c0 = hist[lane * 4], c1 = hist[lane * 4 + 1], c2 = hist[lane * 4 + 2], c3 = hist[lane * 4 + 3];
        const uint32_t group = c0 + c1 + c2 + c3;
        uint32_t incl = group;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t t = __shfl_down(incl, o, 64);
            if (lane + o < 64) incl += t;
        }
        const uint32_t cum = incl - group;
        uint32_t dig = 0u, below = 0u;
        const bool mine = cum < want && want <= incl;
        if (mine) {
            if (want <= cum + c3) { dig = lane * 4 + 3; below = cum; }
            else if (want <= cum + c3 + c2) { dig = lane * 4 + 2; below = cum + c3; }
            else if (want <= cum + c3 + c2 + c1) { dig = lane * 4 + 1; below = cum + c3 + c2; }
            else { dig = lane * 4; below = cum + c3 + c2 + c1; }
        }
        const unsigned long long who = __ballot(mine);
        const int src = __ffsll((long long)who) - 1;
        dig = (uint32_t)__shfl((int)dig, src, 64);
        below = (uint32_t)__shfl((int)below, src, 64);
        want -= below;
        prefix |= dig << shift;
        __builtin_amdgcn_wave_barrier();
    }
    uint32_t g = 0u, e = 0u;
    for (int i = lane; i < n; i += 64) {
        const uint32_t k = key_at(i);
        g += k > prefix ? 1u : 0u;
        e += k == prefix ? 1u : 0u;
    }
    gt = wave_sum(g);
    eq = wave_sum(e);
    return prefix;
}

// The same over an array (LDS or memory).
__device__ __forceinline__ uint32_t wave_select(const uint32_t *key, int n, uint32_t want, uint32_t *hist,
                                                uint32_t &gt, uint32_t &eq)
{
    return wave_select_fn(n, want, hist, gt, eq, [key](int i) { return key[i]; });
}

}  // namespace nkv
