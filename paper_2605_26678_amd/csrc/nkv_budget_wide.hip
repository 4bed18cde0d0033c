// Head-wise memory competition (paper Section 2.6, Appendix A "Hyperparameters") spread over the whole chip.
//
// Same result as the kernels in nkv_budget.hip (the B_h follow from thresholds, see there), but a head's
// scores are not held by one workgroup: they are cut into slices of 8192 tokens and every step that touches
// scores runs on one small workgroup per slice, so a call with few (layer, head) units still fills the
// chip and nothing waits for a 1024-thread workgroup's serial phases.
//
// Scores are binned by value: bin(v) = floor(2046 v) for 0 <= v <= 1, 0 below, 2047 above 1 (the pinned
// positions).  The map is monotone, so "the k best" is: all bins above a boundary bin, plus the best few of
// the boundary bin's entries -- and only those entries (a few dozen per head) are ever looked at exactly,
// as order-preserving integer keys.
//   slice_hist_kernel   (per slice)          2048-bin histogram of the slice, stored as 16-bit counts
//   layer_pick_kernel   (per prompt, layer)  per head: boundary bin of its m_safe best; pool histogram of the
//                                            layer (bins below a head's boundary bin, and the part of the
//                                            boundary bin that is not protected); boundary bin of the R best
//                                            pool entries; per head the pool entries in bins above it
//   slice_collect_kernel (per slice)         keys of the slice that fall into the head's boundary bin and
//                                            into the layer's boundary bin -> two short lists per slice
//   layer_finish_kernel (per prompt, layer)  exact thresholds inside the two boundary bins (radix selects
//                                            over the lists), ties by head order, B_h
// A list that does not fit (thousands of equal scores in one bin) marks the layer, and the shape-generic
// kernel of nkv_budget.hip computes that layer instead.
#include "nkv_slices.h"

namespace nkv {
namespace {

constexpr int kListT = 512;              // keys a head's boundary-bin list holds
constexpr int kListL = 4096;             // entries a layer's boundary-bin list holds
constexpr int kMaxH = 8;
constexpr int kMaxSeg = 1024;            // segments of a layer the finishing kernel takes (H * slices per head)

struct LayerPick {
    int32_t bT[kMaxH];                   // boundary bin of the head's protected set (kBins: nothing protected)
    uint32_t needT[kMaxH];               // how many entries of that bin are protected
    uint32_t gt[kMaxH];                  // pool entries of the head in bins above bL
    int32_t bL;                          // boundary bin of the layer's R best pool entries
    uint32_t needL;                      // how many pool entries of that bin are admitted
    uint32_t done;                       // budgets already final (R == 0)
    uint32_t pad;
};

// Finds the bin holding rank `want` (1-based) from the top of a kBins-bin histogram of which this thread
// holds bins 2 tid (c0) and 2 tid + 1 (c1); 1024 threads.  out[0] = bin, out[1] = rank inside the bin.
// wsum: 16 words.  The caller puts a barrier between the call and reading `out`.
__device__ __forceinline__ uint32_t scan_from_top(uint32_t group, uint32_t *wsum)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    uint32_t incl = group;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t t = __shfl_down(incl, o, 64);
        if (lane + o < 64) incl += t;
    }
    if (lane == 0) wsum[w] = incl;
    return incl;                                                     // inclusive within the wave; add the waves above
}

__global__ __launch_bounds__(1024) void layer_pick_kernel(int L, int H, PromptTab tab, SliceTab st,
                                                          const uint16_t *__restrict__ part,
                                                          LayerPick *__restrict__ picks, uint32_t *__restrict__ failed,
                                                          int32_t *__restrict__ k_per_head)
{
    __shared__ uint32_t wsum[kMaxH + 1][16];
    __shared__ int32_t s_bT[kMaxH];
    __shared__ uint32_t s_needT[kMaxH], s_gt[kMaxH];
    __shared__ uint32_t s_bL, s_needL;
    const int pl = blockIdx.x, l = pl % L, p = pl / L;
    const int N = tab.tok_off[p + 1] - tab.tok_off[p];
    const int S = (N + kSlice - 1) / kSlice;
    const int k0 = tab.k0[p], m_safe = tab.m_safe[p];
    const uint32_t R = (uint32_t)H * (uint32_t)(k0 - m_safe);
    const int tid = threadIdx.x, w = tid >> 6;
    if (tid < kMaxH) {
        s_gt[tid] = 0u;
        s_bT[tid] = kBins;                                           // nothing protected unless a pick says so
        s_needT[tid] = 0u;
    }
    if (tid == 0) failed[pl] = 0u;
    LayerPick *out = picks + pl;
    if (R == 0u) {                                                   // nothing to compete for
        if (tid < H) k_per_head[(int64_t)pl * H + tid] = m_safe;
        if (tid == 0) out->done = 1u;
        return;
    }
    // Every head's histogram = the sum of its slices' 16-bit counts; thread owns bins 2 tid and 2 tid + 1 of
    // all heads.  All loads are independent.
    uint32_t a[kMaxH], b[kMaxH];
#pragma unroll
    for (int h = 0; h < kMaxH; ++h) {
        a[h] = 0u;
        b[h] = 0u;
    }
    const uint32_t *rows0 = reinterpret_cast<const uint32_t *>(part + ((int64_t)st.off[p] + (int64_t)l * H * S) * kBins);
    for (int s0 = 0; s0 < S; s0 += 4) {                              // four rows of every head in flight
        uint32_t two[kMaxH][4];
#pragma unroll
        for (int h = 0; h < kMaxH; ++h)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                two[h][i] = h < H ? rows0[((int64_t)h * S + min(s0 + i, S - 1)) * (kBins / 2) + tid] : 0u;
#pragma unroll
        for (int h = 0; h < kMaxH; ++h)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (s0 + i < S) {
                    a[h] += two[h][i] & 0xffffu;
                    b[h] += two[h][i] >> 16;
                }
    }
    // per head: boundary bin of its m_safe best (all heads' scans together)
    uint32_t incl[kMaxH];
#pragma unroll
    for (int h = 0; h < kMaxH; ++h) incl[h] = scan_from_top(a[h] + b[h], wsum[h]);
    __syncthreads();
    if (m_safe > 0) {
#pragma unroll
        for (int h = 0; h < kMaxH; ++h) {
            if (h < H) {
                uint32_t up = incl[h];
                for (int ww = w + 1; ww < 16; ++ww) up += wsum[h][ww];
                const uint32_t cum = up - (a[h] + b[h]), want = (uint32_t)m_safe;
                if (cum < want && want <= up) {
                    if (want <= cum + b[h]) { s_bT[h] = tid * 2 + 1; s_needT[h] = want - cum; }
                    else { s_bT[h] = tid * 2; s_needT[h] = want - cum - b[h]; }
                }
            }
        }
    }
    __syncthreads();
    // pool of the layer: what the heads do not protect
    auto pooled = [](int bin, uint32_t count, int bT, uint32_t needT) {
        return bin < bT ? count : (bin == bT ? count - needT : 0u);
    };
    uint32_t pa = 0u, pb = 0u, qa[kMaxH], qb[kMaxH];
#pragma unroll
    for (int h = 0; h < kMaxH; ++h) {
        qa[h] = h < H ? pooled(tid * 2, a[h], s_bT[h], s_needT[h]) : 0u;
        qb[h] = h < H ? pooled(tid * 2 + 1, b[h], s_bT[h], s_needT[h]) : 0u;
        pa += qa[h];
        pb += qb[h];
    }
    {
        uint32_t up = scan_from_top(pa + pb, wsum[kMaxH]);
        __syncthreads();
        for (int ww = w + 1; ww < 16; ++ww) up += wsum[kMaxH][ww];
        const uint32_t cum = up - (pa + pb);
        if (cum < R && R <= up) {
            if (R <= cum + pb) { s_bL = (uint32_t)(tid * 2 + 1); s_needL = R - cum; }
            else { s_bL = (uint32_t)(tid * 2); s_needL = R - cum - pb; }
        }
    }
    __syncthreads();
    const int bL = (int)s_bL;
    // pool entries of every head in bins above bL
#pragma unroll
    for (int h = 0; h < kMaxH; ++h) {
        if (h < H) {
            uint32_t c = (tid * 2 > bL ? qa[h] : 0u) + (tid * 2 + 1 > bL ? qb[h] : 0u);
            c = wave_sum(c);
            if ((tid & 63) == 0 && c != 0u) atomicAdd(&s_gt[h], c);
        }
    }
    __syncthreads();
    if (tid < kMaxH) {
        out->bT[tid] = s_bT[tid];
        out->needT[tid] = s_needT[tid];
        out->gt[tid] = s_gt[tid];
    }
    if (tid == 0) {
        out->bL = bL;
        out->needL = s_needL;
        out->done = 0u;
    }
}

// Every slice has its own segment of kSeg keys in each of the two lists and a count: no atomics on memory,
// nobody waits for a returned value.
__global__ __launch_bounds__(kWideThreads) void slice_collect_kernel(const float *__restrict__ scores, int L, int H,
                                                                     PromptTab tab, SliceTab st,
                                                                     const LayerPick *__restrict__ picks,
                                                                     uint32_t *__restrict__ segT,
                                                                     uint32_t *__restrict__ nSegT,
                                                                     uint32_t *__restrict__ segL,
                                                                     uint32_t *__restrict__ nSegL,
                                                                     uint32_t *__restrict__ failed)
{
    __shared__ uint32_t nT, nL;
    int p, lh, s, S;
    locate(st, tab, blockIdx.x, p, lh, s, S);
    const int l = lh / H, h = lh - l * H, pl = p * L + l;
    const int N = tab.tok_off[p + 1] - tab.tok_off[p];
    const float *sc = scores + (int64_t)lh * tab.T + tab.tok_off[p];
    const int tid = threadIdx.x;
    float v[kPerThread];
    const __amdgpu_buffer_rsrc_t vals = slice_values(sc, s, N);
#pragma unroll
    for (int j = 0; j < kPerThread; ++j) v[j] = slice_value(vals, tid, j);
    const LayerPick *pk = picks + pl;
    const int bT = pk->bT[h], bL = pk->bL;
    const uint32_t done = pk->done;
    if (tid == 0) { nT = 0u; nL = 0u; }
    __syncthreads();
    if (done) return;
    uint32_t *outT = segT + (int64_t)blockIdx.x * kSeg, *outL = segL + (int64_t)blockIdx.x * kSeg;
#pragma unroll
    for (int j = 0; j < kPerThread; ++j) {
        if (s * kSlice + j * kWideThreads + tid < N) {
            const int b = score_bin(v[j]);
            if (b == bT) {
                const uint32_t at = atomicAdd(&nT, 1u);
                if (at < (uint32_t)kSeg) outT[at] = ord_key(v[j]);
            }
            if (b == bL && b <= bT) {                                // bins above bT are protected as a whole
                const uint32_t at = atomicAdd(&nL, 1u);
                if (at < (uint32_t)kSeg) outL[at] = ord_key(v[j]);
            }
        }
    }
    __syncthreads();
    if (tid == 0) {
        nSegT[blockIdx.x] = nT;
        nSegL[blockIdx.x] = nL;
        if (nT > (uint32_t)kSeg || nL > (uint32_t)kSeg) failed[pl] = 1u;
    }
}

__global__ __launch_bounds__(1024) void layer_finish_kernel(int L, int H, PromptTab tab, SliceTab st,
                                                            const LayerPick *__restrict__ picks,
                                                            const uint32_t *__restrict__ segT,
                                                            const uint32_t *__restrict__ nSegT,
                                                            const uint32_t *__restrict__ segL,
                                                            const uint32_t *__restrict__ nSegL,
                                                            uint32_t *__restrict__ failed,
                                                            int32_t *__restrict__ k_per_head)
{
    __shared__ uint32_t keysT[kMaxH][kListT];                        // 16 KB
    __shared__ uint32_t keysL[kListL];                               // 16 KB: pool candidates of the layer's boundary bin
    __shared__ uint8_t headL[kListL];
    __shared__ uint32_t whist[kMaxH][256];
    __shared__ uint32_t Th[kMaxH], remT[kMaxH], totT[kMaxH], dropped[kMaxH], gtL[kMaxH], eqL[kMaxH];
    __shared__ uint32_t cT[kMaxSeg], cL[kMaxSeg], oT[kMaxSeg];       // segment counts and offsets
    __shared__ uint32_t nPool, s_TL, s_gtAll, s_bad;
    const int pl = blockIdx.x, l = pl % L, p = pl / L;
    const LayerPick &pk = picks[pl];                                 // read in place: a private copy would sit in scratch
    if (pk.done) return;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int N = tab.tok_off[p + 1] - tab.tok_off[p];
    const int S = (N + kSlice - 1) / kSlice;
    const int m_safe = tab.m_safe[p];
    const int64_t slice0 = (int64_t)st.off[p] + (int64_t)l * H * S;  // first slice of the layer's first head
    const int nseg = H * S;
    if (tid < kMaxH) { dropped[tid] = 0u; gtL[tid] = 0u; eqL[tid] = 0u; totT[tid] = 0u; }
    if (tid == 0) { nPool = 0u; s_bad = failed[pl] | (nseg > kMaxSeg ? 1u : 0u); }
    // counts of all segments of the layer, then where every segment starts in its head's list
    if (tid < nseg && nseg <= kMaxSeg) {
        cT[tid] = nSegT[slice0 + tid];
        cL[tid] = nSegL[slice0 + tid];
    }
    __syncthreads();
    if (s_bad) {
        if (tid == 0) failed[pl] = 1u;
        return;
    }
    if (tid < nseg) {
        const int h = tid / S;
        uint32_t off = 0u;
        for (int q = h * S; q < tid; ++q) off += cT[q];
        oT[tid] = off;
        if (cT[tid] > (uint32_t)kSeg || cL[tid] > (uint32_t)kSeg || off + cT[tid] > (uint32_t)kListT) s_bad = 1u;
        if (tid == h * S + S - 1) totT[h] = off + cT[tid];
    }
    __syncthreads();
    if (s_bad) {
        if (tid == 0) failed[pl] = 1u;
        return;
    }
    // the keys of every head's boundary bin: wave w copies the segments w, w + 16, ...
    for (int q = w; q < nseg; q += 16) {
        const uint32_t n = cT[q], off = oT[q];
        const int h = q / S;
        for (uint32_t j = lane; j < n; j += 64) keysT[h][off + j] = segT[(slice0 + q) * kSeg + j];
    }
    __syncthreads();
    // exact protection threshold of every head: wave h selects in head h's list
    if (w < H) {
        if (m_safe > 0) {
            uint32_t gt, eq;
            const uint32_t T = wave_select(keysT[w], (int)totT[w], pk.needT[w], whist[w], gt, eq);
            if (lane == 0) { Th[w] = T; remT[w] = pk.needT[w] - gt; }     // remT of the eq keys tied at T are protected
        } else if (lane == 0) {
            Th[w] = 0xFFFFFFFFu;
            remT[w] = 0u;
        }
    }
    __syncthreads();
    // pool candidates of the layer's boundary bin: below the head's threshold, or tied with it and not protected
    // (which of the tied ones does not matter: equal keys)
    for (int q = w; q < nseg; q += 16) {
        const uint32_t n = cL[q];
        const int h = q / S;
        const uint32_t T = Th[h];
        for (uint32_t j = lane; j < n; j += 64) {
            const uint32_t k = segL[(slice0 + q) * kSeg + j];
            bool in = k < T;
            if (k == T) in = atomicAdd(&dropped[h], 1u) >= remT[h];
            if (in) {
                const uint32_t at = atomicAdd(&nPool, 1u);
                if (at < (uint32_t)kListL) {
                    keysL[at] = k;
                    headL[at] = (uint8_t)h;
                }
            }
        }
    }
    __syncthreads();
    if (s_bad || nPool > (uint32_t)kListL) {
        if (tid == 0) failed[pl] = 1u;
        return;
    }
    const int n = (int)nPool;
    if (w == 0) {
        uint32_t gt, eq;
        const uint32_t TL = wave_select(keysL, n, pk.needL, whist[0], gt, eq);
        if (lane == 0) { s_TL = TL; s_gtAll = gt; }
    }
    __syncthreads();
    const uint32_t TL = s_TL;
    for (int i = tid; i < n; i += 1024) {
        if (keysL[i] > TL) atomicAdd(&gtL[headL[i]], 1u);
        else if (keysL[i] == TL) atomicAdd(&eqL[headL[i]], 1u);
    }
    __syncthreads();
    if (tid == 0) {
        uint32_t remaining = pk.needL - s_gtAll;                     // ties at the layer threshold still to admit
        for (int h = 0; h < H; ++h) {
            const uint32_t take = min(remaining, eqL[h]);
            remaining -= take;
            k_per_head[(int64_t)pl * H + h] = (int32_t)((uint32_t)m_safe + pk.gt[h] + gtL[h] + take);
        }
    }
}

struct WideWs {
    size_t part, picks, segT, nSegT, segL, nSegL, failed, total;
};

WideWs wide_ws(int L, int H, const PromptTab &tab)
{
    SliceTab st;
    const size_t slices = (size_t)fill_slices(L, H, tab, &st), layers = (size_t)tab.n * L;
    WideWs w;
    size_t off = 0;
    w.part = off;   off += align256(slices * kBins * sizeof(uint16_t));
    w.picks = off;  off += align256(layers * sizeof(LayerPick));
    w.segT = off;   off += align256(slices * kSeg * sizeof(uint32_t));
    w.nSegT = off;  off += align256(slices * sizeof(uint32_t));
    w.segL = off;   off += align256(slices * kSeg * sizeof(uint32_t));
    w.nSegL = off;  off += align256(slices * sizeof(uint32_t));
    w.failed = off; off += align256(layers * sizeof(uint32_t));
    w.total = off;
    return w;
}

}  // namespace

bool budget_wide_supported(int H) { return H <= kMaxH; }

size_t budget_wide_ws_bytes(int L, int H, const PromptTab &tab) { return wide_ws(L, H, tab).total; }

// Enqueues the four kernels; *failed_flags receives the device address of the per-(prompt, layer) words that
// are non-zero for layers whose budgets have not been written.
hipError_t launch_budget_wide(const float *scores, int L, int H, const PromptTab &tab, int32_t *k_per_head, void *ws,
                              const uint32_t **failed_flags, hipStream_t st)
{
    SliceTab stab;
    const int slices = fill_slices(L, H, tab, &stab);
    const WideWs lay = wide_ws(L, H, tab);
    char *base = (char *)ws;
    uint16_t *part = (uint16_t *)(base + lay.part);
    LayerPick *picks = (LayerPick *)(base + lay.picks);
    uint32_t *segT = (uint32_t *)(base + lay.segT), *nSegT = (uint32_t *)(base + lay.nSegT);
    uint32_t *segL = (uint32_t *)(base + lay.segL), *nSegL = (uint32_t *)(base + lay.nSegL);
    uint32_t *failed = (uint32_t *)(base + lay.failed);
    const unsigned layers = (unsigned)(tab.n * L);
    slice_hist_kernel<<<(unsigned)slices, kWideThreads, 0, st>>>(scores, tab, stab, part);
    layer_pick_kernel<<<layers, 1024, 0, st>>>(L, H, tab, stab, part, picks, failed, k_per_head);
    slice_collect_kernel<<<(unsigned)slices, kWideThreads, 0, st>>>(scores, L, H, tab, stab, picks, segT, nSegT, segL,
                                                                   nSegL, failed);
    layer_finish_kernel<<<layers, 1024, 0, st>>>(L, H, tab, stab, picks, segT, nSegT, segL, nSegL, failed, k_per_head);
    *failed_flags = failed;
    return hipGetLastError();
}

}  // namespace nkv
