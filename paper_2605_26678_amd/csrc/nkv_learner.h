// The outer learner's per-token arithmetic (paper Section 2.3 min-max, Section 2.4 blend / surprise / gate),
// shared by the per-head and the slice-wise kernels so that both produce the same bits.
#pragma once

#include <math.h>

#include "nkv_device.h"

namespace nkv {

struct HeadStats {
    float lo[3], inv_range[3];     // inv_range = 0 when the scale is flat
    float w[3];
    float s_lo, s_inv_range, s_mean;
};

__device__ __forceinline__ void normalised(const float a[3], const HeadStats &hs, float at[3])
{
#pragma unroll
    for (int k = 0; k < 3; ++k) at[k] = (a[k] - hs.lo[k]) * hs.inv_range[k];
}

// population standard deviation of three numbers
__device__ __forceinline__ float std3(const float at[3])
{
    const float m = (at[0] + at[1] + at[2]) * (1.0f / 3.0f);
    const float x = at[0] - m, y = at[1] - m, z = at[2] - m;
    return __builtin_amdgcn_sqrtf((x * x + y * y + z * z) * (1.0f / 3.0f));      // hardware square root, 1 ulp
}

// Population standard deviation over the readings of the scales that take part (Section 2.4; Appendix,
// component ablation: a scale that is switched off is left out of blend, winner and deviation alike).
// mask: bit k set = scale k takes part; uniform across a launch.
template <bool ALL = false> __device__ __forceinline__ float surprise_std(const float at[3], int mask)
{
    if (ALL || mask == 7) return std3(at);
    if (mask == 1 || mask == 2 || mask == 4) return 0.f;
    const float x = at[mask & 1 ? 0 : 1], y = at[mask & 4 ? 2 : 1];
    const float m = (x + y) * 0.5f, dx = x - m, dy = y - m;
    return __builtin_amdgcn_sqrtf((dx * dx + dy * dy) * 0.5f);
}

// blend, surprise, gate and route of one token from its three normalised readings (Section 2.4)
// ALL: every scale takes part (known at compile time: the slice-wise kernels are instantiated for that case).
template <bool ALL = false>
__device__ __forceinline__ float routed_score(const float at[3], const HeadStats &st, const LearnerConsts &lc)
{
    const float blend = st.w[0] * at[0] + st.w[1] * at[1] + st.w[2] * at[2];   // a scale that is off has weight 0
    const int mask = ALL ? 7 : lc.scale_mask;
    const float win = fmaxf(mask & 1 ? at[0] : -INFINITY, fmaxf(mask & 2 ? at[1] : -INFINITY, mask & 4 ? at[2] : -INFINITY));
    float s = surprise_std<ALL>(at, mask);
    if (lc.surprise_mode == NKV_SURPRISE_NORMALISED) s = fmaxf((s - st.s_lo) * st.s_inv_range - st.s_mean, 0.f);
    // logistic gate with the hardware's base-2 exponential and reciprocal (1 ulp each; the argument is at
    // most a few tens, so alpha is good to ~1e-6)
    const float alpha = __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.44269504f * lc.kappa * (s - lc.tau)));
    if (lc.gate_mode == NKV_GATE_ONLY_AVERAGE) return blend;
    if (lc.gate_mode == NKV_GATE_ONLY_MAX) return win;
    return (1.0f - alpha) * blend + alpha * win;
}

// Blend weights of a head from the three reliability gaps (Section 2.4): softmax of log prior + beta * gap,
// in double precision.  stats3: {min, 1 / range, gap} of the three scales, 4 floats apart.
__device__ __forceinline__ void head_weights(const float *stats3, const LearnerConsts &lc, HeadStats &hs)
{
    double z[3], zmax = -INFINITY, zsum = 0.0;
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        const float *st = stats3 + k * 4;
        hs.lo[k] = st[0];
        hs.inv_range[k] = st[1];
        z[k] = lc.log_prior[k] + lc.beta * (double)st[2];
        zmax = fmax(zmax, z[k]);
    }
#pragma unroll
    for (int k = 0; k < 3; ++k) { z[k] = exp(z[k] - zmax); zsum += z[k]; }
#pragma unroll
    for (int k = 0; k < 3; ++k) hs.w[k] = (float)(z[k] / zsum);
}

}  // namespace nkv
