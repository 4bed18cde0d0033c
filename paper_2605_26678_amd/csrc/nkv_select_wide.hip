// Top-B_h selection with ordered compaction (paper Section 2.5) spread over the whole chip: same kept_idx as
// select_fast_kernel / select_kernel of nkv_select.hip, but a head's scores are cut into slices of 8192 tokens
// and every step that touches them runs on one small workgroup per slice (see nkv_slices.h).
//   slice_hist_kernel   (per slice)  2048-bin value histogram of the slice
//   sel_collect_kernel  (per slice)  the bin that holds the unit's B_h-th best score (found by every slice's workgroup
//                                    from the unit's histograms); how many of the slice's scores lie in bins above
//                                    it; the keys of that bin -> the slice's segment
//   sel_finish_kernel   (per unit)   one wavefront: exact threshold T inside the bin, how many of the scores
//                                    tied at T are kept, and per slice how many kept / tied scores precede it
//   sel_compact_kernel  (per slice)  ballots over 64 consecutive tokens + a scan over the slice's groups give
//                                    every kept token its output row; optional count of near-threshold scores
// If a segment overflows (thousands of equal scores in one bin), the unit's finishing wavefront walks the head's
// scores itself.
#include "nkv_slices.h"

namespace nkv {
namespace {

constexpr int kList = 2048;              // keys the finishing wavefront takes

struct SelPick {
    int32_t bT;                          // boundary bin; -1: everything is kept; kBins: nothing is kept
    uint32_t needT;                      // how many entries of the boundary bin are kept
};

struct SelUnit {
    uint32_t T, rem;                     // threshold key, how many of the scores tied at T are kept
    uint32_t mode;                       // 0: threshold; 1: keep all; 2: keep none
    uint32_t pad;
};

struct SelSlice {
    uint32_t above;                      // scores of the slice in bins above the boundary bin
    uint32_t n;                          // keys in the slice's segment
    uint32_t gt_before, eq_before;       // kept-for-sure / tied scores of the unit in the slices before this one
};

// The boundary bin of unit u: the bin that holds its B-th best score, and how many of that bin's entries are kept
// (B = 0: {kBins, 0}, nothing is kept; B = N: {-1, 0}, everything is).  Called by all 256 threads of a workgroup,
// 8 bins each; c_own[i] receives the count of bin 8 tid + i in slice `own` of the unit (own < 0: not asked for).
// wtot: 4 words, s_pick: 2 words of LDS; the result is valid for every thread after the call.
__device__ __forceinline__ SelPick pick_boundary_bin(const uint16_t *__restrict__ part, int64_t slice0, int S, int B, int N, int own,
                                                     uint32_t (&c_own)[8], uint32_t *wtot, int32_t *s_pick)
{
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const uint4 *rows = reinterpret_cast<const uint4 *>(part + slice0 * kBins);
    uint32_t c[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) { c[i] = 0u; c_own[i] = 0u; }
    for (int s0 = 0; s0 < S; s0 += 4) {
        uint4 r[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = rows[(int64_t)min(s0 + i, S - 1) * (kBins / 8) + tid];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (s0 + i < S) {
                const uint32_t t[8] = {r[i].x & 0xffffu, r[i].x >> 16, r[i].y & 0xffffu, r[i].y >> 16,
                                       r[i].z & 0xffffu, r[i].z >> 16, r[i].w & 0xffffu, r[i].w >> 16};
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    c[e] += t[e];
                    if (s0 + i == own) c_own[e] = t[e];
                }
            }
        }
    }
    if (B == 0 || B == N) return SelPick{B == 0 ? kBins : -1, 0u};  // no threshold to find (uniform in the workgroup)
    uint32_t group = 0u;
#pragma unroll
    for (int i = 0; i < 8; ++i) group += c[i];
    uint32_t incl = group;                                           // inclusive sum from the top bin downwards
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t t = __shfl_down(incl, o, 64);
        if (lane + o < 64) incl += t;
    }
    if (lane == 0) wtot[w] = incl;
    __syncthreads();
    for (int ww = w + 1; ww < kWideThreads / 64; ++ww) incl += wtot[ww];
    const uint32_t want = (uint32_t)B;
    uint32_t cum = incl - group;                                     // scores in bins above this thread's eight
    if (cum < want && want <= incl) {
#pragma unroll
        for (int i = 7; i >= 0; --i) {
            if (cum < want && want <= cum + c[i]) { s_pick[0] = tid * 8 + i; s_pick[1] = (int32_t)(want - cum); }
            cum += c[i];
        }
    }
    __syncthreads();
    return SelPick{s_pick[0], (uint32_t)s_pick[1]};
}

// grid: slices.  Every slice's workgroup finds the boundary bin of its unit itself from the unit's slice histograms
// (a few 4 KB rows that the histogram kernel has just written: cheaper than a kernel of its own in between), counts
// its own slice's scores above that bin, and copies its scores of that bin into its segment.  The first slice's
// workgroup records the unit's pick.
__global__ __launch_bounds__(kWideThreads) void sel_collect_kernel(const float *__restrict__ scores,
                                                                   const int32_t *__restrict__ k_per_head, int L, int H,
                                                                   PromptTab tab, SliceTab st,
                                                                   const uint16_t *__restrict__ part,
                                                                   SelPick *__restrict__ picks,
                                                                   uint32_t *__restrict__ seg,
                                                                   SelSlice *__restrict__ ss)
{
    __shared__ uint32_t n_hit;
    __shared__ uint32_t wtot[kWideThreads / 64];
    __shared__ int32_t s_pick[2];
    int p, lh, s, S;
    locate(st, tab, blockIdx.x, p, lh, s, S);
    const int u = p * L * H + lh;
    const int N = tab.tok_off[p + 1] - tab.tok_off[p];
    const float *sc = scores + (int64_t)lh * tab.T + tab.tok_off[p];
    const int tid = threadIdx.x;
    float v[kPerThread];
    const __amdgpu_buffer_rsrc_t vals = slice_values(sc, s, N);
#pragma unroll
    for (int j = 0; j < kPerThread; ++j) v[j] = slice_value(vals, tid, j);
    uint32_t c_own[8];
    const SelPick pk = pick_boundary_bin(part, blockIdx.x - s, S, min(max(k_per_head[u], 0), N), N, s, c_own, wtot, s_pick);
    const int bT = pk.bT;
    {                                                                // this slice's scores in bins above bT
        uint32_t a = 0u;
#pragma unroll
        for (int i = 0; i < 8; ++i) a += tid * 8 + i > bT ? c_own[i] : 0u;
        a = wave_sum(a);
        __syncthreads();                                             // (wtot is free again)
        if ((tid & 63) == 0) wtot[tid >> 6] = a;
    }
    if (tid == 0) n_hit = 0u;
    __syncthreads();
    if (tid == 0) {
        ss[blockIdx.x].above = (wtot[0] + wtot[1]) + (wtot[2] + wtot[3]);
        if (s == 0) picks[u] = pk;
    }
    uint32_t *out = seg + (int64_t)blockIdx.x * kSeg;
    if (bT >= 0 && bT < kBins) {
#pragma unroll
        for (int j = 0; j < kPerThread; ++j) {
            if (s * kSlice + j * kWideThreads + tid < N && score_bin(v[j]) == bT) {
                const uint32_t at = atomicAdd(&n_hit, 1u);
                if (at < (uint32_t)kSeg) out[at] = ord_key(v[j]);
            }
        }
    }
    __syncthreads();
    if (tid == 0) ss[blockIdx.x].n = n_hit;                          // more than kSeg: the finishing kernel sees it and walks the scores
}

// grid: units; one wavefront
__global__ __launch_bounds__(64) void sel_finish_kernel(const float *__restrict__ scores,
                                                        const int32_t *__restrict__ k_per_head, int L, int H,
                                                        PromptTab tab, SliceTab st,
                                                        const SelPick *__restrict__ picks,
                                                        const uint32_t *__restrict__ seg, SelSlice *__restrict__ ss,
                                                        SelUnit *__restrict__ sel, int64_t *__restrict__ head_off,
                                                        int64_t *__restrict__ near_count)
{
    __shared__ uint32_t keys[kList];
    __shared__ uint32_t hist[256];
    const int u = blockIdx.x, lane = threadIdx.x;
    const int lh = u % (L * H), p = u / (L * H);
    const int N = tab.tok_off[p + 1] - tab.tok_off[p];
    if (head_off) {
        // With a few thousand units at most, this wavefront also places its unit in the output -- the rows the
        // units in front of it keep -- which saves the scan kernel that otherwise runs first.
        const int n_units = tab.n * L * H;
        unsigned long long run = 0ull;
        for (int v = lane; v < u; v += 64) {
            const int pv = v / (L * H);
            run += (unsigned long long)min(max(k_per_head[v], 0), tab.tok_off[pv + 1] - tab.tok_off[pv]);
        }
        run = wave_sum(run);
        if (lane == 0) {
            head_off[u] = (int64_t)run;
            if (u == n_units - 1) head_off[n_units] = (int64_t)run + min(max(k_per_head[u], 0), N);
            if (u == 0 && near_count) *near_count = 0;               // the compaction kernel, next on the stream, adds to it
        }
    }
    const int S = (N + kSlice - 1) / kSlice;
    const int64_t slice0 = (int64_t)st.off[p] + (int64_t)lh * S;
    const SelPick pk = picks[u];
    if (pk.bT < 0 || pk.bT >= kBins) {                               // keep all / keep none
        uint32_t run = 0u;
        for (int s = 0; s < S; ++s) {                                // (a few slices; every lane walks them)
            const uint32_t a = ss[slice0 + s].above;
            if (lane == 0) { ss[slice0 + s].gt_before = run; ss[slice0 + s].eq_before = 0u; }
            run += a;
        }
        if (lane == 0) sel[u] = SelUnit{0u, 0u, pk.bT < 0 ? 1u : 2u, 0u};
        return;
    }
    bool bad = false;
    uint32_t n = 0u;
    for (int s = 0; s < S && !bad; ++s) {
        const uint32_t c = ss[slice0 + s].n;
        if (c > (uint32_t)kSeg || n + c > (uint32_t)kList) { bad = true; break; }
        for (uint32_t i = lane; i < c; i += 64) keys[n + i] = seg[(slice0 + s) * kSeg + i];
        n += c;
    }
    if (bad) {
        // More scores in one bin than the lists hold (thousands of equal scores): this wavefront walks the
        // head's scores itself -- slow, exact, and rare.
        const float *sc = scores + (int64_t)lh * tab.T + tab.tok_off[p];
        const uint32_t B = (uint32_t)min(max(k_per_head[u], 0), N);
        uint32_t gt, eq;
        const uint32_t T = wave_select_fn(N, B, hist, gt, eq, [sc](int i) { return ord_key(sc[i]); });
        if (lane == 0) sel[u] = SelUnit{T, B - gt, 0u, 0u};
        uint32_t run_gt = 0u, run_eq = 0u;
        for (int s = 0; s < S; ++s) {
            uint32_t g = 0u, e = 0u;
            for (int i = s * kSlice + lane; i < min((s + 1) * kSlice, N); i += 64) {
                const uint32_t k = ord_key(sc[i]);
                g += k > T ? 1u : 0u;
                e += k == T ? 1u : 0u;
            }
            g = wave_sum(g);
            e = wave_sum(e);
            if (lane == 0) { ss[slice0 + s].gt_before = run_gt; ss[slice0 + s].eq_before = run_eq; }
            run_gt += g;
            run_eq += e;
        }
        return;
    }
    __builtin_amdgcn_wave_barrier();
    uint32_t gt, eq;
    const uint32_t T = wave_select(keys, (int)n, pk.needT, hist, gt, eq);
    if (lane == 0) sel[u] = SelUnit{T, pk.needT - gt, 0u, 0u};
    // per slice: kept-for-sure and tied scores before it
    uint32_t run_gt = 0u, run_eq = 0u, off = 0u;
    for (int s = 0; s < S; ++s) {
        const uint32_t c = ss[slice0 + s].n, above = ss[slice0 + s].above;
        uint32_t g = 0u, e = 0u;
        for (uint32_t i = lane; i < c; i += 64) {
            const uint32_t k = keys[off + i];
            g += k > T ? 1u : 0u;
            e += k == T ? 1u : 0u;
        }
        g = wave_sum(g);
        e = wave_sum(e);
        if (lane == 0) { ss[slice0 + s].gt_before = run_gt; ss[slice0 + s].eq_before = run_eq; }
        run_gt += above + g;
        run_eq += e;
        off += c;
    }
}

// set bits of m in the lanes below this one
__device__ __forceinline__ uint32_t lanes_below(unsigned long long m)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}

// grid: slices
__global__ __launch_bounds__(kWideThreads) void sel_compact_kernel(const float *__restrict__ scores, int L, int H,
                                                                   PromptTab tab, SliceTab st,
                                                                   const SelUnit *__restrict__ sel,
                                                                   const SelSlice *__restrict__ ss,
                                                                   const int64_t *__restrict__ head_off,
                                                                   int64_t row_capacity, float near_tol,
                                                                   int32_t *__restrict__ kept_idx,
                                                                   int64_t *__restrict__ near_count)
{
    constexpr int kGroups = kPerThread * (kWideThreads / 64);        // 64-token groups of a slice, in token order
    __shared__ uint32_t cnt_gt[kGroups], cnt_eq[kGroups];
    __shared__ unsigned long long near_acc[kWideThreads / 64];
    int p, lh, s, S;
    locate(st, tab, blockIdx.x, p, lh, s, S);
    const int u = p * L * H + lh;
    const int N = tab.tok_off[p + 1] - tab.tok_off[p];
    const float *sc = scores + (int64_t)lh * tab.T + tab.tok_off[p];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    float v[kPerThread];
    const __amdgpu_buffer_rsrc_t vals = slice_values(sc, s, N);
#pragma unroll
    for (int j = 0; j < kPerThread; ++j) v[j] = slice_value(vals, tid, j);
    const SelUnit su = sel[u];
    const SelSlice sl = ss[blockIdx.x];
    if (su.mode >= 2u) return;                                       // nothing kept
    const bool all = su.mode == 1u;
    const uint32_t T = su.T, rem = su.rem;
    // population of every 64-token group (chunk j, wave w) = tokens s*kSlice + j*256 + w*64 ...
    uint32_t near = 0u;
    const float tv = key_value(T);
    uint32_t gmask = 0u, emask = 0u;                                 // bit j: slot j is kept for sure / is tied at T
#pragma unroll
    for (int j = 0; j < kPerThread; ++j) {
        const bool in = s * kSlice + j * kWideThreads + tid < N;
        const uint32_t key = ord_key(v[j]);
        const bool gt = in && (all || key > T);
        const bool eq = in && !all && key == T;
        gmask |= (gt ? 1u : 0u) << j;
        emask |= (eq ? 1u : 0u) << j;
        const unsigned long long mg = __ballot(gt), me = __ballot(eq);
        if (lane == 0) {
            cnt_gt[j * (kWideThreads / 64) + w] = (uint32_t)__popcll(mg);
            cnt_eq[j * (kWideThreads / 64) + w] = (uint32_t)__popcll(me);
        }
        if (near_count && in && !all && fabsf(v[j] - tv) <= near_tol) ++near;
        // one group at a time, its flags folded into the words right away: a condition kept for later is two scalar
        // registers, and 128 of them do not fit
        asm volatile("" : "+v"(gmask), "+v"(emask), "+v"(near));
    }
    __syncthreads();
    if (w == 0) {                                                    // exclusive scan over the groups: 2 per lane
        constexpr int PER = kGroups / 64;
        uint32_t g[PER], e[PER], tg = 0u, te = 0u;
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            g[q] = cnt_gt[lane * PER + q];
            e[q] = cnt_eq[lane * PER + q];
            tg += g[q];
            te += e[q];
        }
        uint32_t ig = tg, ie = te;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t a = __shfl_up(ig, o, 64), b = __shfl_up(ie, o, 64);
            if (lane >= o) { ig += a; ie += b; }
        }
        uint32_t rg = ig - tg, re = ie - te;
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            cnt_gt[lane * PER + q] = rg;
            cnt_eq[lane * PER + q] = re;
            rg += g[q];
            re += e[q];
        }
    }
    __syncthreads();
    // The two flag words are all the second pass needs of the values (and the compiler is kept from carrying the
    // first pass's 64 ballots over instead, which costs it more registers than it has).
    asm volatile("" : "+v"(gmask), "+v"(emask));
    const int64_t out0 = head_off[u];
#pragma unroll
    for (int j = 0; j < kPerThread; ++j) {
        const int i = s * kSlice + j * kWideThreads + tid;
        const bool gt = (gmask >> j) & 1u, eq = (emask >> j) & 1u;
        const unsigned long long mg = __ballot(gt), me = __ballot(eq);
        const int grp = j * (kWideThreads / 64) + w;
        const uint32_t gt_before = sl.gt_before + cnt_gt[grp] + lanes_below(mg);
        const uint32_t eq_before = sl.eq_before + cnt_eq[grp] + lanes_below(me);
        if (gt || (eq && eq_before < rem)) {
            const int64_t row = out0 + gt_before + min(eq_before, rem);
            if (row < row_capacity) kept_idx[row] = i;
        }
    }
    if (near_count) {
        const unsigned long long near_w = wave_sum((unsigned long long)near);
        if (lane == 0) near_acc[w] = near_w;
        __syncthreads();
        if (tid == 0) {
            unsigned long long t = 0;
            for (int i = 0; i < kWideThreads / 64; ++i) t += near_acc[i];
            if (t) atomicAdd((unsigned long long *)near_count, t);
        }
    }
}

struct WideWs {
    size_t part, picks, ss, seg, sel, total;
};

WideWs wide_ws(int L, int H, const PromptTab &tab)
{
    SliceTab st;
    const size_t slices = (size_t)fill_slices(L, H, tab, &st), units = (size_t)tab.n * L * H;
    WideWs w;
    size_t off = 0;
    w.part = off;    off += align256(slices * kBins * sizeof(uint16_t));
    w.picks = off;   off += align256(units * sizeof(SelPick));
    w.ss = off;      off += align256(slices * sizeof(SelSlice));
    w.seg = off;     off += align256(slices * kSeg * sizeof(uint32_t));
    w.sel = off;     off += align256(units * sizeof(SelUnit));
    w.total = off;
    return w;
}

}  // namespace

size_t select_wide_ws_bytes(int L, int H, const PromptTab &tab) { return wide_ws(L, H, tab).total; }

// Enqueues the four kernels.  with_head_off: head_off and the zeroing of near_count are not on the stream yet and
// the finishing kernel does them (select_wide_places_units() says when it can).
bool select_wide_places_units(int n_units) { return n_units <= 4096; }

hipError_t launch_select_wide(const float *scores, const int32_t *k_per_head, int L, int H, const PromptTab &tab,
                              float near_tol, int64_t *head_off, int64_t row_capacity, int32_t *kept_idx,
                              int64_t *near_count, bool with_head_off, void *ws, hipStream_t st)
{
    SliceTab stab;
    const int slices = fill_slices(L, H, tab, &stab);
    const WideWs lay = wide_ws(L, H, tab);
    char *base = (char *)ws;
    uint16_t *part = (uint16_t *)(base + lay.part);
    SelPick *picks = (SelPick *)(base + lay.picks);
    SelSlice *ss = (SelSlice *)(base + lay.ss);
    uint32_t *seg = (uint32_t *)(base + lay.seg);
    SelUnit *sel = (SelUnit *)(base + lay.sel);
    const unsigned units = (unsigned)(tab.n * L * H);
    slice_hist_kernel<<<(unsigned)slices, kWideThreads, 0, st>>>(scores, tab, stab, part);
    sel_collect_kernel<<<(unsigned)slices, kWideThreads, 0, st>>>(scores, k_per_head, L, H, tab, stab, part, picks, seg, ss);
    sel_finish_kernel<<<units, 64, 0, st>>>(scores, k_per_head, L, H, tab, stab, picks, seg, ss, sel,
                                            with_head_off ? head_off : nullptr, near_count);
    sel_compact_kernel<<<(unsigned)slices, kWideThreads, 0, st>>>(scores, L, H, tab, stab, sel, ss, head_off, row_capacity,
                                                                 near_tol, kept_idx, near_count);
    return hipGetLastError();
}

}  // namespace nkv
