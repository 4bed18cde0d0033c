// Per-head statistics of the three anomaly scales (paper Sections 2.3-2.4: min-max range, reliability gap =
// mean of the m_p largest minus mean of the m_p smallest normalised anomalies) spread over the whole chip.
//
// Same numbers as scale_stats_kernel in nkv_finalize.hip (up to the order of floating-point additions), but a
// head's anomalies are not held by one workgroup: they are cut into slices of 8192 tokens and every step
// that touches them runs on one small workgroup per (slice, scale).
//
// Anomalies are -cos, so they lie in [-1, 1]; they are binned by value, bin(a) = floor(1023.5 (a + 1)), a
// monotone map.  "The m largest" is then: all bins above a boundary bin plus the largest few of the boundary
// bin's entries, and only those entries are looked at exactly; likewise from below.
//   stats_hist_kernel    (slice, scale)  2048-bin histogram as 16-bit counts; min and max of the slice
//   stats_pick_kernel    (unit, scale)   the bins that hold the m-th largest and the m-th smallest value
//   stats_collect_kernel (slice)         all three scales: sums of the values above the upper / below the lower
//                                        boundary bin; the boundary bins' entries (as order-preserving keys)
//                                        into two short lists per slice and scale; and, the ranges being known,
//                                        min / max / sum of the slice's surprise statistic
//   stats_finish_kernel  (unit, scale)   one wavefront: exact thresholds inside the boundary bins, the two
//                                        means, min, 1/range, gap
//   route_slice_kernel   (slice)         weights, surprise statistics of the head, routed scores, pinning
// A list that overflows (hundreds of values of one slice in one bin) marks the (unit, scale) and the per-head
// kernel, launched behind and idle otherwise, computes it.
#include "nkv_learner.h"
#include "nkv_slices.h"

namespace nkv {
namespace {

constexpr int kList = 1024;              // keys the finishing wavefront takes per list

struct StatPick {
    int32_t bTop, bBot;                  // boundary bins
    uint32_t needTop, needBot;           // how many of their entries belong to the m largest / smallest
    float lo, inv;                       // min of the (unit, scale) and 1 / range (0 if flat)
};

struct SliceSurprise {                   // the surprise statistic (Section 2.4) over one slice
    float lo, hi;
    double sum;
};

struct SlicePart {                       // what one slice contributes besides its histogram and lists
    float lo, hi;                        // min, max of the slice
    uint32_t nTop, nBot;                 // entries in the two lists
    double sTop, sBot;                   // sums above the upper / below the lower boundary bin
};

// grid (slices, 3)
__global__ __launch_bounds__(kWideThreads) void stats_hist_kernel(const float *__restrict__ a_raw, int64_t rows,
                                                                  PromptTab tab, SliceTab st, int n_slices,
                                                                  uint16_t *__restrict__ part,
                                                                  SlicePart *__restrict__ sp)
{
    __shared__ uint32_t hist[kBins];
    __shared__ float red[2][kWideThreads / 64];
    int p, lh, s, S;
    locate(st, tab, blockIdx.x, p, lh, s, S);
    const int k = blockIdx.y;
    const int N = tab.tok_off[p + 1] - tab.tok_off[p];
    const float *a = a_raw + (int64_t)k * rows + (int64_t)lh * tab.T + tab.tok_off[p];
    const int tid = threadIdx.x;
    for (int j = tid; j < kBins; j += kWideThreads) hist[j] = 0u;
    float v[kPerThread / 4][4];
    const __amdgpu_buffer_rsrc_t vals = slice_values(a, s, N);
#pragma unroll
    for (int j = 0; j < kPerThread / 4; ++j) slice_values4(vals, tid, j, v[j]);
    __syncthreads();
    float lo = INFINITY, hi = -INFINITY;
#pragma unroll
    for (int j = 0; j < kPerThread / 4; ++j) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (s * kSlice + 4 * (j * kWideThreads + tid) + e < N) {
                lo = fminf(lo, v[j][e]);
                hi = fmaxf(hi, v[j][e]);
                atomicAdd(&hist[anomaly_bin(v[j][e])], 1u);
            }
        }
    }
    lo = wave_min(lo);
    hi = wave_max(hi);
    if ((tid & 63) == 0) { red[0][tid >> 6] = lo; red[1][tid >> 6] = hi; }
    __syncthreads();
    const int64_t job_slice = (int64_t)k * n_slices + blockIdx.x;
    if (tid == 0) {
        for (int i = 1; i < kWideThreads / 64; ++i) { lo = fminf(lo, red[0][i]); hi = fmaxf(hi, red[1][i]); }
        sp[job_slice].lo = lo;
        sp[job_slice].hi = hi;
    }
    store_hist16(hist, part + job_slice * kBins);
}

// grid (units, 3); 256 threads, 8 bins each
__global__ __launch_bounds__(kWideThreads) void stats_pick_kernel(int L, int H, PromptTab tab, SliceTab st,
                                                                  int n_slices, const uint16_t *__restrict__ part,
                                                                  const SlicePart *__restrict__ sp,
                                                                  StatPick *__restrict__ picks,
                                                                  uint32_t *__restrict__ failed)
{
    __shared__ uint32_t wtot[kWideThreads / 64];
    const int u = blockIdx.x, k = blockIdx.y;
    const int lh = u % (L * H), p = u / (L * H);
    const int N = tab.tok_off[p + 1] - tab.tok_off[p];
    const int S = (N + kSlice - 1) / kSlice;
    const uint32_t m = (uint32_t)min(tab.m_p[p], N);
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const uint4 *rows = reinterpret_cast<const uint4 *>(part + ((int64_t)k * n_slices + st.off[p] + (int64_t)lh * S) * kBins);
    uint32_t c[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) c[i] = 0u;
    for (int s0 = 0; s0 < S; s0 += 4) {
        uint4 r[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = rows[(int64_t)min(s0 + i, S - 1) * (kBins / 8) + tid];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (s0 + i < S) {
                c[0] += r[i].x & 0xffffu; c[1] += r[i].x >> 16; c[2] += r[i].y & 0xffffu; c[3] += r[i].y >> 16;
                c[4] += r[i].z & 0xffffu; c[5] += r[i].z >> 16; c[6] += r[i].w & 0xffffu; c[7] += r[i].w >> 16;
            }
        }
    }
    uint32_t group = 0u;
#pragma unroll
    for (int i = 0; i < 8; ++i) group += c[i];
    uint32_t incl = group;                                           // inclusive prefix from bin 0 upwards
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t t = __shfl_up(incl, o, 64);
        if (lane >= o) incl += t;
    }
    if (lane == 63) wtot[w] = incl;
    __syncthreads();
    for (int ww = 0; ww < w; ++ww) incl += wtot[ww];
    const uint32_t below = incl - group;                             // entries in bins below this thread's eight
    const uint32_t above = (uint32_t)N - incl;                       // entries in bins above them
    StatPick *out = picks + (int64_t)u * 3 + k;
    if (below < m && m <= incl) {                                    // the m-th smallest lies in one of my bins
        uint32_t cum = below;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (cum < m && m <= cum + c[i]) { out->bBot = tid * 8 + i; out->needBot = m - cum; }
            cum += c[i];
        }
    }
    if (above < m && m <= above + group) {                           // the m-th largest lies in one of my bins
        uint32_t cum = above;
#pragma unroll
        for (int i = 7; i >= 0; --i) {
            if (cum < m && m <= cum + c[i]) { out->bTop = tid * 8 + i; out->needTop = m - cum; }
            cum += c[i];
        }
    }
    if (w == 0) {                                                    // min, max over the unit's slices
        float lo = INFINITY, hi = -INFINITY;
        for (int s = lane; s < S; s += 64) {
            const SlicePart q = sp[(int64_t)k * n_slices + st.off[p] + (int64_t)lh * S + s];
            lo = fminf(lo, q.lo);
            hi = fmaxf(hi, q.hi);
        }
        lo = wave_min(lo);
        hi = wave_max(hi);
        if (lane == 0) {
            const float range = hi - lo;
            out->lo = lo;
            out->inv = range < kFlat ? 0.f : 1.0f / range;
            failed[(int64_t)u * 3 + k] = 0u;
        }
    }
}

// grid: slices.  All three scales of the slice in one pass: what stats_finish_kernel needs of each scale, and --
// the ranges being known -- min, max and sum of the surprise statistic of the slice's tokens.
template <bool ALL>
__global__ __launch_bounds__(kWideThreads, 5) void stats_collect_kernel(const float *__restrict__ a_raw, int64_t rows,
                                                                     int L, int H, PromptTab tab, SliceTab st,
                                                                     int n_slices, int scale_mask,
                                                                     const StatPick *__restrict__ picks,
                                                                     uint32_t *__restrict__ segTop,
                                                                     uint32_t *__restrict__ segBot,
                                                                     SlicePart *__restrict__ sp,
                                                                     SliceSurprise *__restrict__ sur,
                                                                     uint32_t *__restrict__ failed)
{
    constexpr int HALF = kPerThread / 2;
    __shared__ uint32_t nTop[3], nBot[3];
    __shared__ double red[8][kWideThreads / 64];
    __shared__ float fred[2][kWideThreads / 64];
    int p, lh, s, S;
    locate(st, tab, blockIdx.x, p, lh, s, S);
    const int N = tab.tok_off[p + 1] - tab.tok_off[p];
    const float *a = a_raw + (int64_t)lh * tab.T + tab.tok_off[p];
    const int tid = threadIdx.x;
    const int64_t job0 = ((int64_t)p * L * H + lh) * 3;
    StatPick pk[3];
    HeadStats hs;
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        pk[k] = picks[job0 + k];
        hs.lo[k] = pk[k].lo;
        hs.inv_range[k] = pk[k].inv;
    }
    if (tid < 3) { nTop[tid] = 0u; nBot[tid] = 0u; }
    __syncthreads();
    const __amdgpu_buffer_rsrc_t vals[3] = {slice_values(a, s, N), slice_values(a + rows, s, N), slice_values(a + 2 * rows, s, N)};
    float pt[3] = {0.f, 0.f, 0.f}, pb[3] = {0.f, 0.f, 0.f};          // a few dozen terms of magnitude <= 1 each
    float smin = INFINITY, smax = -INFINITY;
    float ssum32 = 0.f;                                              // 32 terms of magnitude <= 0.5
#pragma unroll 1
    for (int half = 0; half < 2; ++half) {
        float v[3][HALF];
#pragma unroll
        for (int k = 0; k < 3; ++k)
#pragma unroll
            for (int j = 0; j < HALF; ++j) v[k][j] = slice_value(vals[k], tid, half * HALF + j);
#pragma unroll
        for (int j = 0; j < HALF; ++j) {
            if (s * kSlice + (half * HALF + j) * kWideThreads + tid < N) {
#pragma unroll
                for (int k = 0; k < 3; ++k) {
                    const float x = v[k][j];
                    const int b = anomaly_bin(x);
                    pt[k] += b > pk[k].bTop ? x : 0.f;
                    pb[k] += b < pk[k].bBot ? x : 0.f;
                    if (b == pk[k].bTop) {
                        const uint32_t at = atomicAdd(&nTop[k], 1u);
                        if (at < (uint32_t)kSeg) segTop[((int64_t)k * n_slices + blockIdx.x) * kSeg + at] = ord_key(x);
                    }
                    if (b == pk[k].bBot) {                           // inverted: the smallest value has the largest key
                        const uint32_t at = atomicAdd(&nBot[k], 1u);
                        if (at < (uint32_t)kSeg) segBot[((int64_t)k * n_slices + blockIdx.x) * kSeg + at] = ~ord_key(x);
                    }
                }
                const float raw[3] = {v[0][j], v[1][j], v[2][j]};
                float at[3];
                normalised(raw, hs, at);
                const float sv = surprise_std<ALL>(at, scale_mask);
                smin = fminf(smin, sv);
                smax = fmaxf(smax, sv);
                ssum32 += sv;
            }
        }
    }
    double ssum = (double)ssum32;
    const int w = tid >> 6;
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        const double t = wave_sum((double)pt[k]), b = wave_sum((double)pb[k]);
        if ((tid & 63) == 0) { red[2 * k][w] = t; red[2 * k + 1][w] = b; }
    }
    ssum = wave_sum(ssum);
    smin = wave_min(smin);
    smax = wave_max(smax);
    if ((tid & 63) == 0) { red[6][w] = ssum; fred[0][w] = smin; fred[1][w] = smax; }
    __syncthreads();
    if (tid < 3) {
        const int k = tid;
        double t = 0.0, b = 0.0;
        for (int i = 0; i < kWideThreads / 64; ++i) { t += red[2 * k][i]; b += red[2 * k + 1][i]; }
        SlicePart *q = sp + (int64_t)k * n_slices + blockIdx.x;
        q->sTop = t;
        q->sBot = b;
        q->nTop = nTop[k];
        q->nBot = nBot[k];
        if (nTop[k] > (uint32_t)kSeg || nBot[k] > (uint32_t)kSeg) failed[job0 + k] = 1u;
    }
    if (tid == 64) {
        double t = 0.0;
        float lo = INFINITY, hi = -INFINITY;
        for (int i = 0; i < kWideThreads / 64; ++i) { t += red[6][i]; lo = fminf(lo, fred[0][i]); hi = fmaxf(hi, fred[1][i]); }
        sur[blockIdx.x] = SliceSurprise{lo, hi, t};
    }
}

// grid: slices.  Blend, gate, route and pinning of the slice's tokens (Section 2.4); every workgroup forms its
// head's weights and surprise statistics itself from the few numbers they depend on.
template <bool ALL>
__global__ __launch_bounds__(kWideThreads, 5) void route_slice_kernel(const float *__restrict__ a_raw, int64_t rows,
                                                                   int L, int H, PromptTab tab, SliceTab st,
                                                                   LearnerConsts lc, const float *__restrict__ stats,
                                                                   const SliceSurprise *__restrict__ sur,
                                                                   float *__restrict__ scores)
{
    __shared__ HeadStats hs;
    int p, lh, s, S;
    locate(st, tab, blockIdx.x, p, lh, s, S);
    const int N = tab.tok_off[p + 1] - tab.tok_off[p];
    const int64_t base = (int64_t)lh * tab.T + tab.tok_off[p];
    const float *a = a_raw + base;
    const int tid = threadIdx.x;
    constexpr int HALF = kPerThread / 2;
    float v[3][HALF];
    const __amdgpu_buffer_rsrc_t vals[3] = {slice_values(a, s, N), slice_values(a + rows, s, N), slice_values(a + 2 * rows, s, N)};
#pragma unroll
    for (int k = 0; k < 3; ++k)
#pragma unroll
        for (int j = 0; j < HALF; ++j) v[k][j] = slice_value(vals[k], tid, j);
    if (tid == 0) {
        head_weights(stats + ((int64_t)p * L * H + lh) * 12, lc, hs);
        float smin = INFINITY, smax = -INFINITY;
        double ssum = 0.0;
        const SliceSurprise *q = sur + (blockIdx.x - s);
        for (int i = 0; i < S; ++i) {                                // the head's slices in order
            smin = fminf(smin, q[i].lo);
            smax = fmaxf(smax, q[i].hi);
            ssum += q[i].sum;
        }
        const float srange = smax - smin;
        hs.s_lo = smin;
        hs.s_inv_range = srange < kFlat ? 0.f : 1.0f / srange;
        hs.s_mean = (float)((ssum / (double)N - (double)smin) * (double)hs.s_inv_range);
    }
    __syncthreads();
    const HeadStats h = hs;
    float *out = scores + base;
#pragma unroll 1
    for (int half = 0; half < 2; ++half) {
        if (half == 1) {
#pragma unroll
            for (int k = 0; k < 3; ++k)
#pragma unroll
                for (int j = 0; j < HALF; ++j) v[k][j] = slice_value(vals[k], tid, HALF + j);
        }
#pragma unroll
        for (int j = 0; j < HALF; ++j) {
            const int i = s * kSlice + (half * HALF + j) * kWideThreads + tid;
            if (i < N) {
                const float raw[3] = {v[0][j], v[1][j], v[2][j]};
                float at[3];
                normalised(raw, h, at);
                out[i] = i < lc.n_sink ? NKV_PIN : routed_score<ALL>(at, h, lc);
            }
        }
    }
}

// grid (units, 3); one wavefront.  stats[(u * 3 + k) * 4 + {0, 1, 2}] = min, 1 / range (0 if flat), gap
__global__ __launch_bounds__(64) void stats_finish_kernel(const float *__restrict__ a_raw, int64_t rows, int L, int H,
                                                          PromptTab tab, SliceTab st, int n_slices,
                                                          const StatPick *__restrict__ picks,
                                                          const uint32_t *__restrict__ segTop,
                                                          const uint32_t *__restrict__ segBot,
                                                          const SlicePart *__restrict__ sp,
                                                          uint32_t *__restrict__ failed, float *__restrict__ stats)
{
    __shared__ uint32_t keys[2][kList];
    __shared__ uint32_t hist[256];
    const int u = blockIdx.x, k = blockIdx.y;
    const int64_t job = (int64_t)u * 3 + k;
    bool bad = failed[job] != 0u;
    const int lh = u % (L * H), p = u / (L * H);
    const int N = tab.tok_off[p + 1] - tab.tok_off[p];
    const int S = (N + kSlice - 1) / kSlice;
    const uint32_t m = (uint32_t)min(tab.m_p[p], N);
    const int lane = threadIdx.x;
    const int64_t slice0 = (int64_t)k * n_slices + st.off[p] + (int64_t)lh * S;
    const StatPick pk = picks[job];
    // slices in order: lists, sums, min, max
    uint32_t nT = 0u, nB = 0u;
    double sTop = 0.0, sBot = 0.0;
    float lo = INFINITY, hi = -INFINITY;
    for (int s = 0; s < S && !bad; ++s) {
        const SlicePart q = sp[slice0 + s];
        if (q.nTop > (uint32_t)kSeg || q.nBot > (uint32_t)kSeg || nT + q.nTop > (uint32_t)kList ||
            nB + q.nBot > (uint32_t)kList) {
            bad = true;
            break;
        }
        for (uint32_t i = lane; i < q.nTop; i += 64) keys[0][nT + i] = segTop[(slice0 + s) * kSeg + i];
        for (uint32_t i = lane; i < q.nBot; i += 64) keys[1][nB + i] = segBot[(slice0 + s) * kSeg + i];
        nT += q.nTop;
        nB += q.nBot;
        sTop += q.sTop;
        sBot += q.sBot;
        lo = fminf(lo, q.lo);
        hi = fmaxf(hi, q.hi);
    }
    // The lists' order depends on the timing of the collecting workgroups, so their entries are added up in
    // fixed point (2^-40 units, exact for fp32 values of magnitude <= 1 down to that resolution): the sum does
    // not depend on the order, and the statistics are reproducible bit for bit.
    constexpr double kFix = 1099511627776.0;                         // 2^40
    if (bad) {
        // More values in one bin than the lists hold (thousands of equal anomalies): this wavefront walks the
        // head's values itself -- slow, exact, and rare.
        const float *a = a_raw + (int64_t)k * rows + (int64_t)lh * tab.T + tab.tok_off[p];
        lo = INFINITY;
        hi = -INFINITY;
        for (int i = lane; i < N; i += 64) {
            lo = fminf(lo, a[i]);
            hi = fmaxf(hi, a[i]);
        }
        lo = wave_min(lo);
        hi = wave_max(hi);
        uint32_t gt, eq;
        const uint32_t Tt = wave_select_fn(N, m, hist, gt, eq, [a](int i) { return ord_key(a[i]); });
        long long part = 0;
        for (int i = lane; i < N; i += 64)
            part += ord_key(a[i]) > Tt ? __double2ll_rn((double)a[i] * kFix) : 0ll;
        const double top = (double)wave_sum(part) / kFix + (double)(m - gt) * (double)key_value(Tt);
        const uint32_t Tb = wave_select_fn(N, m, hist, gt, eq, [a](int i) { return ~ord_key(a[i]); });
        part = 0;
        for (int i = lane; i < N; i += 64)
            part += ~ord_key(a[i]) > Tb ? __double2ll_rn((double)a[i] * kFix) : 0ll;
        const double bot = (double)wave_sum(part) / kFix + (double)(m - gt) * (double)key_value(~Tb);
        if (lane == 0) {
            const float range = hi - lo;
            const float inv = range < kFlat ? 0.f : 1.0f / range;
            float *o = stats + job * 4;
            o[0] = lo;
            o[1] = inv;
            o[2] = (float)((top - bot) / (double)m * (double)inv);
        }
        return;
    }
    __builtin_amdgcn_wave_barrier();
    // upper boundary bin: the needTop largest of its entries belong to the m largest
    uint32_t gt, eq;
    const uint32_t Tt = wave_select(keys[0], (int)nT, pk.needTop, hist, gt, eq);
    long long part = 0;
    for (uint32_t i = lane; i < nT; i += 64)
        part += keys[0][i] > Tt ? __double2ll_rn((double)key_value(keys[0][i]) * kFix) : 0ll;
    double top = sTop + (double)wave_sum(part) / kFix + (double)(pk.needTop - gt) * (double)key_value(Tt);
    // lower boundary bin, on inverted keys
    const uint32_t Tb = wave_select(keys[1], (int)nB, pk.needBot, hist, gt, eq);
    part = 0;
    for (uint32_t i = lane; i < nB; i += 64)
        part += keys[1][i] > Tb ? __double2ll_rn((double)key_value(~keys[1][i]) * kFix) : 0ll;
    double bot = sBot + (double)wave_sum(part) / kFix + (double)(pk.needBot - gt) * (double)key_value(~Tb);
    if (lane == 0) {
        const float range = hi - lo;
        const float inv = range < kFlat ? 0.f : 1.0f / range;
        float *o = stats + job * 4;
        o[0] = lo;
        o[1] = inv;
        o[2] = (float)((top - bot) / (double)m * (double)inv);
    }
}

struct WideWs {
    size_t part, sp, sur, picks, segTop, segBot, failed, total;
};

WideWs wide_ws(int L, int H, const PromptTab &tab)
{
    SliceTab st;
    const size_t slices = 3 * (size_t)fill_slices(L, H, tab, &st), jobs = 3 * (size_t)tab.n * L * H;
    WideWs w;
    size_t off = 0;
    w.part = off;    off += align256(slices * kBins * sizeof(uint16_t));
    w.sp = off;      off += align256(slices * sizeof(SlicePart));
    w.sur = off;     off += align256(slices / 3 * sizeof(SliceSurprise));
    w.picks = off;   off += align256(jobs * sizeof(StatPick));
    w.segTop = off;  off += align256(slices * kSeg * sizeof(uint32_t));
    w.segBot = off;  off += align256(slices * kSeg * sizeof(uint32_t));
    w.failed = off;  off += align256(jobs * sizeof(uint32_t));
    w.total = off;
    return w;
}

}  // namespace

size_t stats_wide_ws_bytes(int L, int H, const PromptTab &tab) { return wide_ws(L, H, tab).total; }

// Enqueues the four kernels that fill `stats`.
hipError_t launch_stats_wide(const float *a_raw, int L, int H, const PromptTab &tab, int scale_mask, float *stats, void *ws,
                             hipStream_t st)
{
    SliceTab stab;
    const int slices = fill_slices(L, H, tab, &stab);
    const WideWs lay = wide_ws(L, H, tab);
    char *base = (char *)ws;
    uint16_t *part = (uint16_t *)(base + lay.part);
    SlicePart *sp = (SlicePart *)(base + lay.sp);
    StatPick *picks = (StatPick *)(base + lay.picks);
    uint32_t *segTop = (uint32_t *)(base + lay.segTop), *segBot = (uint32_t *)(base + lay.segBot);
    uint32_t *failed = (uint32_t *)(base + lay.failed);
    const int64_t rows = (int64_t)L * H * tab.T;
    const unsigned units = (unsigned)(tab.n * L * H);
    stats_hist_kernel<<<dim3((unsigned)slices, 3), kWideThreads, 0, st>>>(a_raw, rows, tab, stab, slices, part, sp);
    SliceSurprise *sur = (SliceSurprise *)(base + lay.sur);
    stats_pick_kernel<<<dim3(units, 3), kWideThreads, 0, st>>>(L, H, tab, stab, slices, part, sp, picks, failed);
    if (scale_mask == 7)
        stats_collect_kernel<true><<<(unsigned)slices, kWideThreads, 0, st>>>(a_raw, rows, L, H, tab, stab, slices, scale_mask,
                                                                             picks, segTop, segBot, sp, sur, failed);
    else
        stats_collect_kernel<false><<<(unsigned)slices, kWideThreads, 0, st>>>(a_raw, rows, L, H, tab, stab, slices, scale_mask,
                                                                              picks, segTop, segBot, sp, sur, failed);
    stats_finish_kernel<<<dim3(units, 3), 64, 0, st>>>(a_raw, rows, L, H, tab, stab, slices, picks, segTop, segBot,
                                                       sp, failed, stats);
    return hipGetLastError();
}

// Final scores from the statistics (complete, including what the per-head kernel redid) and the slices'
// surprise sums left by launch_stats_wide in the same scratch.
hipError_t launch_route_wide(const float *a_raw, int L, int H, const PromptTab &tab, const LearnerConsts &lc,
                             const float *stats, void *ws, float *scores, hipStream_t st)
{
    SliceTab stab;
    const int slices = fill_slices(L, H, tab, &stab);
    const WideWs lay = wide_ws(L, H, tab);
    const SliceSurprise *sur = (const SliceSurprise *)((char *)ws + lay.sur);
    if (lc.scale_mask == 7)
        route_slice_kernel<true><<<(unsigned)slices, kWideThreads, 0, st>>>(a_raw, (int64_t)L * H * tab.T, L, H, tab, stab,
                                                                           lc, stats, sur, scores);
    else
        route_slice_kernel<false><<<(unsigned)slices, kWideThreads, 0, st>>>(a_raw, (int64_t)L * H * tab.T, L, H, tab, stab,
                                                                            lc, stats, sur, scores);
    return hipGetLastError();
}

}  // namespace nkv
