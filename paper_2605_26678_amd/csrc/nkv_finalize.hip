// Outer learner: from the three raw anomalies of a head to its final scores
// (paper Section 2.3 min-max, Section 2.4 reliability gaps / blend / surprise / gate, sink pinning).
//
// One workgroup of 1024 threads per unit (prompt, layer, head).  The head's 3*N floats (384 KB at
// N = 32768) stay resident in L2 while the workgroup walks them seven times:
//   pass 1      min / max of each scale
//   pass 2..5   byte-wise radix select (most significant digit first) of the m_p-th largest and the
//               m_p-th smallest value of each scale, six selects at once in LDS histograms
//   pass 6      sums above / below those thresholds (fp64), and min / max / sum of the surprise
//   pass 7      blend, gate, route, pin, write
// The sum of the m largest values is  sum(a > T) + (m - count(a > T)) * T  with T the m-th largest,
// which does not depend on how ties at T are broken.  Min-max is affine and increasing, so the
// selects run on the raw anomalies and the gap is rescaled afterwards.
#include "nkv_blocksel.h"
#include "nkv_learner.h"

namespace nkv {
namespace {

constexpr int kThreads = 1024;

__global__ __launch_bounds__(kThreads) void finalize_kernel(const float *__restrict__ a_raw, int L, int H,
                                                            PromptTab tab, LearnerConsts lc,
                                                            float *__restrict__ scores)
{
    __shared__ uint32_t hist[6][256];
    __shared__ uint32_t sel_prefix[6], sel_want[6];
    __shared__ float fscratch[16];
    __shared__ double dscratch[16];
    __shared__ HeadStats hs;

    const int u = blockIdx.x;                    // (p * L + l) * H + h
    const int h = u % H, l = (u / H) % L, p = u / (H * L);
    const int N = tab.tok_off[p + 1] - tab.tok_off[p];
    const int64_t rows = (int64_t)L * H * tab.T;
    const int64_t base = ((int64_t)l * H + h) * tab.T + tab.tok_off[p];
    const float *a[3] = {a_raw + base, a_raw + rows + base, a_raw + 2 * rows + base};
    const int tid = threadIdx.x;

    // ---- pass 1: min / max per scale ----
    float lo[3], hi[3];
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        float mn = INFINITY, mx = -INFINITY;
        for (int i = tid; i < N; i += kThreads) {
            const float v = a[k][i];
            mn = fminf(mn, v);
            mx = fmaxf(mx, v);
        }
        lo[k] = block_min(mn, fscratch);
        hi[k] = block_max(mx, fscratch);
    }
    if (tid == 0) {
#pragma unroll
        for (int k = 0; k < 3; ++k) {
            const float range = hi[k] - lo[k];
            hs.lo[k] = lo[k];
            hs.inv_range[k] = range < kFlat ? 0.f : 1.0f / range;
        }
    }
    if (tid < 6) { sel_prefix[tid] = 0u; sel_want[tid] = (uint32_t)min(tab.m_p[p], N); }
    __syncthreads();

    // ---- passes 2..5: six radix selects; select s = 2*k + e, e = 0 top (m-th largest), 1 bottom ----
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        for (int j = tid; j < 6 * 256; j += kThreads) (&hist[0][0])[j] = 0u;
        __syncthreads();
        uint32_t pre[6];
#pragma unroll
        for (int s = 0; s < 6; ++s) pre[s] = sel_prefix[s];
        for (int i = tid; i < N; i += kThreads) {
#pragma unroll
            for (int k = 0; k < 3; ++k) {
                const uint32_t key = ord_key(a[k][i]);
                const uint32_t hi_bits = pass == 0 ? 0u : key >> (shift + 8);
                const uint32_t dig = (key >> shift) & 255u;
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    const uint32_t want_hi = pass == 0 ? 0u : pre[2 * k + e] >> (shift + 8);
                    if (hi_bits == want_hi) atomicAdd(&hist[2 * k + e][dig], 1u);
                }
            }
        }
        __syncthreads();
        if (tid < 6) {
            uint32_t want = sel_want[tid];
            const uint32_t dig = radix_pick(hist[tid], want, (tid & 1) == 0);
            sel_want[tid] = want;
            sel_prefix[tid] |= dig << shift;
        }
        __syncthreads();
    }

    // ---- pass 6: sums beyond the thresholds; surprise statistics ----
    const int m = min(tab.m_p[p], N);
    HeadStats st = hs;
    double sums[6];
    {
        uint32_t thr[6];
#pragma unroll
        for (int s = 0; s < 6; ++s) { thr[s] = sel_prefix[s]; sums[s] = 0.0; }
        float smin = INFINITY, smax = -INFINITY;
        double ssum = 0.0;
        for (int i = tid; i < N; i += kThreads) {
            float av[3], at[3];
#pragma unroll
            for (int k = 0; k < 3; ++k) {
                av[k] = a[k][i];
                const uint32_t key = ord_key(av[k]);
                if (key > thr[2 * k]) sums[2 * k] += (double)av[k];
                if (key < thr[2 * k + 1]) sums[2 * k + 1] += (double)av[k];
            }
            normalised(av, st, at);
            const float s = surprise_std(at, lc.scale_mask);
            smin = fminf(smin, s);
            smax = fmaxf(smax, s);
            ssum += (double)s;
        }
#pragma unroll
        for (int s = 0; s < 6; ++s) sums[s] = block_sum(sums[s], dscratch);
        smin = block_min(smin, fscratch);
        smax = block_max(smax, fscratch);
        ssum = block_sum(ssum, dscratch);
        if (tid == 0) {
            double z[3], zmax = -INFINITY, zsum = 0.0;
#pragma unroll
            for (int k = 0; k < 3; ++k) {
                // ties at the threshold: sel_want of them belong to the set
                const double top = sums[2 * k] + (double)sel_want[2 * k] * (double)key_value(thr[2 * k]);
                const double bot = sums[2 * k + 1] + (double)sel_want[2 * k + 1] * (double)key_value(thr[2 * k + 1]);
                const double delta = (top - bot) / (double)m * (double)st.inv_range[k];
                z[k] = lc.log_prior[k] + lc.beta * delta;
                zmax = fmax(zmax, z[k]);
            }
#pragma unroll
            for (int k = 0; k < 3; ++k) { z[k] = exp(z[k] - zmax); zsum += z[k]; }
#pragma unroll
            for (int k = 0; k < 3; ++k) hs.w[k] = (float)(z[k] / zsum);
            const float srange = smax - smin;
            hs.s_lo = smin;
            hs.s_inv_range = srange < kFlat ? 0.f : 1.0f / srange;
            hs.s_mean = (float)((ssum / (double)N - (double)smin) * (double)hs.s_inv_range);
        }
        __syncthreads();
    }

    // ---- pass 7: blend, gate, route, pin ----
    st = hs;
    float *out = scores + base;
    for (int i = tid; i < N; i += kThreads) {
        float av[3], at[3];
#pragma unroll
        for (int k = 0; k < 3; ++k) av[k] = a[k][i];
        normalised(av, st, at);
        const float star = routed_score(at, st, lc);
        out[i] = i < lc.n_sink ? NKV_PIN : star;
    }
}


// ------------------------------------------------------------------------------------------------------
// Units of up to 1024 * EPT tokens: two kernels with the values held in registers.
//   scale_stats_kernel : one workgroup per (unit, scale): min, max and the reliability gap of that scale
//   route_kernel       : one workgroup per unit: weights, surprise statistics, routed score, pinning
// ------------------------------------------------------------------------------------------------------
// stats[(u * 3 + k) * 4 + {0, 1, 2}] = min, 1 / range (0 if flat), reliability gap of scale k of unit u
template <int EPT>
__global__ __launch_bounds__(kSelThreads, EPT <= 16 ? 8 : 4) void scale_stats_kernel(const float *__restrict__ a_raw, int L, int H,
                                                                   PromptTab tab, int u0,
                                                                   float *__restrict__ stats)
{
    __shared__ SelectScratch sel;
    __shared__ double dscratch[32];
    const int k = blockIdx.x, u = u0 + blockIdx.y;
    const int h = u % H, l = (u / H) % L, p = u / (H * L);
    const int N = tab.tok_off[p + 1] - tab.tok_off[p];
    const int64_t rows = (int64_t)L * H * tab.T;
    const float *a = a_raw + (int64_t)k * rows + ((int64_t)l * H + h) * tab.T + tab.tok_off[p];
    const int tid = threadIdx.x;

    uint32_t key[EPT];
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const int i = tid + j * kSelThreads;
        const float v = a[min(i, N - 1)];                      // unconditional: the loads of a thread pipeline
        key[j] = i < N ? ord_key(v) : 0u;
    }
    // Warm the L2 of this die for the workgroup that will follow on this compute unit: only one workgroup of
    // this size fits a compute unit, so nothing else overlaps its load phase with this one's arithmetic.
    // Workgroups go to the dies round-robin, so the one 256 places further on lands on this die again.
    {
        const int id = blockIdx.y * 3 + blockIdx.x + 256, kn = id % 3, un = u0 + id / 3;
        if (un < u0 + (int)gridDim.y) {
            const int hn = un % H, ln = (un / H) % L, pn = un / (H * L);
            const int Nn = tab.tok_off[pn + 1] - tab.tok_off[pn];
            const float *an = a_raw + (int64_t)kn * rows + ((int64_t)ln * H + hn) * tab.T + tab.tok_off[pn];
            if (tid * 32 < Nn) (void)*(const volatile float *)(an + tid * 32);   // one word per 128-byte line
        }
    }
    uint32_t kmin, kmax;
    block_key_range<EPT>(key, N, sel, kmin, kmax);
    const uint32_t m = (uint32_t)min(tab.m_p[p], N);
    uint32_t rem_top, rem_bot, t_top, t_bot;
    block_select_both<EPT>(key, N, m, sel, kmin, kmax, t_top, rem_top, t_bot, rem_bot);
    // sums beyond the thresholds: per thread in fp32 (a handful of terms of magnitude <= 1), across the
    // workgroup in fp64
    float p_top = 0.f, p_bot = 0.f;
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const bool in = N == EPT * kSelThreads || tid + j * kSelThreads < N;
        const float v = key_value(key[j]);
        p_top += in && key[j] > t_top ? v : 0.f;
        p_bot += in && key[j] < t_bot ? v : 0.f;
    }
    double s_top = wave_sum((double)p_top), s_bot = wave_sum((double)p_bot);
    if ((tid & 63) == 0) { dscratch[tid >> 6] = s_top; dscratch[16 + (tid >> 6)] = s_bot; }
    __syncthreads();
    if (tid == 0) {
        s_top = 0.0;
        s_bot = 0.0;
        for (int i = 0; i < kSelThreads / 64; ++i) { s_top += dscratch[i]; s_bot += dscratch[16 + i]; }
        const float lo = key_value(kmin), range = key_value(kmax) - lo;
        const float inv = range < kFlat ? 0.f : 1.0f / range;
        // ties at the threshold: rem of them belong to the set
        const double top = s_top + (double)rem_top * (double)key_value(t_top);
        const double bot = s_bot + (double)rem_bot * (double)key_value(t_bot);
        float *o = stats + ((int64_t)u * 3 + k) * 4;
        o[0] = lo;
        o[1] = inv;
        o[2] = (float)((top - bot) / (double)m * (double)inv);
    }
}

__global__ __launch_bounds__(kSelThreads) void route_kernel(const float *__restrict__ a_raw, int L, int H,
                                                            PromptTab tab, LearnerConsts lc,
                                                            const float *__restrict__ stats,
                                                            float *__restrict__ scores)
{
    __shared__ float fscratch[16];
    __shared__ double dscratch[16];
    __shared__ HeadStats hs;
    const int u = blockIdx.x;
    const int h = u % H, l = (u / H) % L, p = u / (H * L);
    const int N = tab.tok_off[p + 1] - tab.tok_off[p];
    const int64_t rows = (int64_t)L * H * tab.T;
    const int64_t base = ((int64_t)l * H + h) * tab.T + tab.tok_off[p];
    const float *a0 = a_raw + base, *a1 = a_raw + rows + base, *a2 = a_raw + 2 * rows + base;
    const int tid = threadIdx.x;

    if (tid == 0) head_weights(stats + (int64_t)u * 12, lc, hs);
    __syncthreads();
    HeadStats st = hs;
    float smin = INFINITY, smax = -INFINITY;
    double ssum = 0.0;
    constexpr int U = 4;                                  // independent loads in flight per thread and scale
    for (int i0 = tid; i0 < N; i0 += U * kSelThreads) {
        float av[U][3];
#pragma unroll
        for (int q = 0; q < U; ++q) {
            const int i = min(i0 + q * kSelThreads, N - 1);
            av[q][0] = a0[i]; av[q][1] = a1[i]; av[q][2] = a2[i];
        }
#pragma unroll
        for (int q = 0; q < U; ++q) {
            if (i0 + q * kSelThreads < N) {
                float at[3];
                normalised(av[q], st, at);
                const float s = surprise_std(at, lc.scale_mask);
                smin = fminf(smin, s);
                smax = fmaxf(smax, s);
                ssum += (double)s;
            }
        }
    }
    smin = block_min(smin, fscratch);
    smax = block_max(smax, fscratch);
    ssum = block_sum(ssum, dscratch);
    const float srange = smax - smin;
    st.s_lo = smin;
    st.s_inv_range = srange < kFlat ? 0.f : 1.0f / srange;
    st.s_mean = (float)((ssum / (double)N - (double)smin) * (double)st.s_inv_range);

    float *out = scores + base;
    for (int i0 = tid; i0 < N; i0 += U * kSelThreads) {
        float av[U][3];
#pragma unroll
        for (int q = 0; q < U; ++q) {
            const int i = min(i0 + q * kSelThreads, N - 1);
            av[q][0] = a0[i]; av[q][1] = a1[i]; av[q][2] = a2[i];
        }
#pragma unroll
        for (int q = 0; q < U; ++q) {
            const int i = i0 + q * kSelThreads;
            if (i < N) {
                float at[3];
                normalised(av[q], st, at);
                out[i] = i < lc.n_sink ? NKV_PIN : routed_score(at, st, lc);
            }
        }
    }
}

}  // namespace

hipError_t launch_finalize(const float *a_raw, int L, int H, const PromptTab &tab, const LearnerConsts &lc,
                           float *scores, float *stats, void *wide_ws, bool per_head_route, const Prof &prof,
                           hipStream_t st)
{
    int nmax = 0;
    for (int p = 0; p < tab.n; ++p) nmax = max(nmax, tab.tok_off[p + 1] - tab.tok_off[p]);
    const unsigned units = (unsigned)(tab.n * L * H);
    prof.begin(NKV_KERNEL_FINALIZE, st);
    if (wide_ws != nullptr && (nmax > 8192 || units >= 256) && !per_head_route) {
        // Slice-wise kernels where a head has more than one slice (any length) or there are many units (their
        // 256-thread workgroups pack the chip four times as densely); for a few short units the per-head
        // kernels are quicker.
        hipError_t e = launch_stats_wide(a_raw, L, H, tab, lc.scale_mask, stats, wide_ws, st);
        if (e != hipSuccess) return e;
        e = launch_route_wide(a_raw, L, H, tab, lc, stats, wide_ws, scores, st);
        if (e != hipSuccess) return e;
    } else if (nmax <= 32 * kSelThreads) {
        for_each_length_class(tab, L * H, [&](int ept, int u0, int n) {
            const dim3 grid(3, (unsigned)n);
            if (ept == 4) scale_stats_kernel<4><<<grid, kSelThreads, 0, st>>>(a_raw, L, H, tab, u0, stats);
            else if (ept == 8) scale_stats_kernel<8><<<grid, kSelThreads, 0, st>>>(a_raw, L, H, tab, u0, stats);
            else if (ept == 16) scale_stats_kernel<16><<<grid, kSelThreads, 0, st>>>(a_raw, L, H, tab, u0, stats);
            else scale_stats_kernel<32><<<grid, kSelThreads, 0, st>>>(a_raw, L, H, tab, u0, stats);
        });
        route_kernel<<<units, kSelThreads, 0, st>>>(a_raw, L, H, tab, lc, stats, scores);
    } else {
        finalize_kernel<<<units, kThreads, 0, st>>>(a_raw, L, H, tab, lc, scores);
    }
    prof.end(NKV_KERNEL_FINALIZE, st);
    return hipGetLastError();
}

}  // namespace nkv
