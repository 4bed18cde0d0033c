// Head-wise memory competition (paper Section 2.6, Appendix A "Hyperparameters") for layers of more than 8
// heads: the steps of budget_kernel (nkv_budget.hip: A per-head safeguard threshold, B layer threshold over the
// pool, C per-head counts; byte-wise radix selects on the order-preserving image of the scores) with one
// workgroup per (prompt, layer, head) instead of one per (prompt, layer), so that a layer of 32 heads keeps 32
// compute units busy instead of one.  What is a barrier between passes there is a kernel boundary here:
//   head_threshold_kernel  (per unit)           step A: T_h, how many of the ties at T_h are protected, #ties
//   pool_pass_kernel x 4   (per unit)           step B, one byte of TL per launch: the head's share of the
//                                               layer's 256-bin histogram -> atomic adds on memory
//   head_count_kernel      (per unit)           step C: pool entries of the head above TL / tied at TL
//   layer_assign_kernel    (per prompt, layer)  ties at TL in head order, B_h
// Every workgroup of a pass derives the digits picked so far from the histograms of the passes before it, so no
// kernel is needed between two passes.  Exact integer work throughout: the same B_h as budget_kernel.
#include "nkv_internal.h"
#include "nkv_device.h"

namespace nkv {
namespace {

constexpr int kThreads = 1024;

struct HeadT {                   // step A for one head
    uint32_t T, prot, ties, pad; // threshold key; protected among the ties at T; ties at T
};
struct HeadCount {
    uint32_t gt, eq;             // pool entries of the head above TL / tied at TL (without the ties at T_h)
};
struct LayerT {
    uint32_t TL, rem;            // layer threshold; how many of the entries tied at TL are admitted
};

// The bin that holds the want-th entry counted from bin 255 downwards, over a 256-bin histogram held one bin per
// thread by threads 0..255 (`mine`; the other threads pass 0), and the rank left inside that bin (want on
// return).  Every thread receives both.  The same result as a serial walk from bin 255 that ends at bin 0.
// Contains three barriers; scratch: 8 words of LDS.
__device__ __forceinline__ uint32_t pick_from_top(uint32_t mine, uint32_t &want, uint32_t *scratch)
{
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    uint32_t incl = tid < 256 ? mine : 0u;                           // this bin and the wave's higher ones
    if (tid < 256) {
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t t = __shfl_down(incl, o, 64);
            if (lane + o < 64) incl += t;
        }
        if (lane == 0) scratch[w] = incl;
    }
    if (tid == 0) scratch[4] = 0u;                                   // bin 0 unless a higher bin claims the rank
    __syncthreads();
    if (tid < 256) {
        uint32_t above = incl - mine;                                // entries in the bins above this one
        for (int ww = w + 1; ww < 4; ++ww) above += scratch[ww];
        if (tid > 0 && above < want && want <= above + mine) {
            scratch[4] = (uint32_t)tid;
            scratch[5] = want - above;
        }
        if (tid == 0) scratch[6] = want - above;
    }
    __syncthreads();
    const uint32_t dig = scratch[4];
    want = dig ? scratch[5] : scratch[6];
    __syncthreads();
    return dig;
}

// TL's leading bytes and the rank still to be found, from the histograms of the passes already made.
__device__ __forceinline__ void layer_prefix(const uint32_t *__restrict__ lh, int npass, uint32_t R, uint32_t *scratch,
                                             uint32_t &TL, uint32_t &want)
{
    TL = 0u;
    want = R;
    for (int pass = 0; pass < npass; ++pass) {
        const uint32_t mine = threadIdx.x < 256 ? lh[pass * 256 + threadIdx.x] : 0u;
        TL |= pick_from_top(mine, want, scratch) << (24 - 8 * pass);
    }
}

struct UnitRef {
    int h, l, p, pl, N, m_safe;
    int64_t R;
    const float *sc;
};

__device__ __forceinline__ UnitRef unit_ref(const float *scores, int L, int H, const PromptTab &tab)
{
    UnitRef r;
    const int u = blockIdx.x;
    r.h = u % H;
    r.l = (u / H) % L;
    r.p = u / (H * L);
    r.pl = r.p * L + r.l;
    r.N = tab.tok_off[r.p + 1] - tab.tok_off[r.p];
    r.m_safe = tab.m_safe[r.p];
    r.R = (int64_t)H * (tab.k0[r.p] - r.m_safe);
    r.sc = scores + ((int64_t)r.l * H + r.h) * tab.T + tab.tok_off[r.p];
    return r;
}

// grid: units.  Also clears the layer's four histograms (the workgroup of head 0).
__global__ __launch_bounds__(kThreads) void head_threshold_kernel(const float *__restrict__ scores, int L, int H,
                                                                  PromptTab tab, HeadT *__restrict__ ht,
                                                                  uint32_t *__restrict__ lhist)
{
    __shared__ uint32_t hist[256];
    __shared__ uint32_t scratch[8];
    const UnitRef r = unit_ref(scores, L, H, tab);
    const int tid = threadIdx.x;
    if (r.h == 0) lhist[(int64_t)r.pl * 1024 + tid] = 0u;
    uint32_t T = 0xFFFFFFFFu, want = (uint32_t)r.m_safe, ties = 0u;
    if (r.m_safe > 0) {
        T = 0u;
        for (int pass = 0; pass < 4; ++pass) {
            const int shift = 24 - 8 * pass;
            if (tid < 256) hist[tid] = 0u;
            __syncthreads();
            for (int i = tid; i < r.N; i += kThreads) {
                const uint32_t key = ord_key(r.sc[i]);
                if (pass == 0 || (key >> (shift + 8)) == (T >> (shift + 8))) atomicAdd(&hist[(key >> shift) & 255u], 1u);
            }
            __syncthreads();
            const uint32_t dig = pick_from_top(tid < 256 ? hist[tid] : 0u, want, scratch);
            T |= dig << shift;
            if (pass == 3) ties = hist[dig];
            __syncthreads();
        }
    }
    if (tid == 0) ht[blockIdx.x] = HeadT{T, r.m_safe > 0 ? want : 0u, ties, 0u};
}

// grid: units; pass = 0..3
__global__ __launch_bounds__(kThreads) void pool_pass_kernel(const float *__restrict__ scores, int L, int H, PromptTab tab,
                                                             int pass, const HeadT *__restrict__ ht,
                                                             uint32_t *__restrict__ lhist)
{
    __shared__ uint32_t hist[256];
    __shared__ uint32_t scratch[8];
    const UnitRef r = unit_ref(scores, L, H, tab);
    if (r.R <= 0) return;
    const int tid = threadIdx.x;
    uint32_t *lh = lhist + (int64_t)r.pl * 1024;
    uint32_t pre, left;
    layer_prefix(lh, pass, (uint32_t)r.R, scratch, pre, left);
    const HeadT t = ht[blockIdx.x];
    const int shift = 24 - 8 * pass;
    if (tid < 256) hist[tid] = 0u;
    __syncthreads();
    for (int i = tid; i < r.N; i += kThreads) {
        const uint32_t key = ord_key(r.sc[i]);
        if (key < t.T && (pass == 0 || (key >> (shift + 8)) == (pre >> (shift + 8))))
            atomicAdd(&hist[(key >> shift) & 255u], 1u);
    }
    if (tid == 0 && r.m_safe > 0) {                                  // unprotected ties at the head's own threshold
        const uint32_t ex = t.ties - t.prot;
        if (ex > 0u && (pass == 0 || (t.T >> (shift + 8)) == (pre >> (shift + 8))))
            atomicAdd(&hist[(t.T >> shift) & 255u], ex);
    }
    __syncthreads();
    if (tid < 256 && hist[tid] != 0u) atomicAdd(&lh[pass * 256 + tid], hist[tid]);
}

// grid: units
__global__ __launch_bounds__(kThreads) void head_count_kernel(const float *__restrict__ scores, int L, int H, PromptTab tab,
                                                              const HeadT *__restrict__ ht,
                                                              const uint32_t *__restrict__ lhist,
                                                              HeadCount *__restrict__ cnt, LayerT *__restrict__ lt)
{
    __shared__ uint32_t scratch[8];
    __shared__ uint32_t acc[2];
    const UnitRef r = unit_ref(scores, L, H, tab);
    const int tid = threadIdx.x;
    uint32_t TL = 0u, left = 0u;
    if (tid < 2) acc[tid] = 0u;
    if (r.R > 0) {
        layer_prefix(lhist + (int64_t)r.pl * 1024, 4, (uint32_t)r.R, scratch, TL, left);
        const uint32_t th = ht[blockIdx.x].T;
        uint32_t gt = 0u, eq = 0u;
        for (int i = tid; i < r.N; i += kThreads) {
            const uint32_t key = ord_key(r.sc[i]);
            if (key < th) {
                gt += key > TL ? 1u : 0u;
                eq += key == TL ? 1u : 0u;
            }
        }
        gt = wave_sum(gt);
        eq = wave_sum(eq);
        if ((tid & 63) == 0) {
            atomicAdd(&acc[0], gt);
            atomicAdd(&acc[1], eq);
        }
    }
    __syncthreads();
    if (tid == 0) {
        cnt[blockIdx.x] = HeadCount{acc[0], acc[1]};
        if (r.h == 0) lt[r.pl] = LayerT{TL, r.R > 0 ? left : 0u};
    }
}

// grid: prompts * layers; one wavefront, lane 0 walks the heads in order
__global__ __launch_bounds__(64) void layer_assign_kernel(int L, int H, PromptTab tab, const HeadT *__restrict__ ht,
                                                          const HeadCount *__restrict__ cnt,
                                                          const LayerT *__restrict__ lt,
                                                          int32_t *__restrict__ k_per_head)
{
    if (threadIdx.x != 0) return;
    const int pl = blockIdx.x, p = pl / L;
    const int m_safe = tab.m_safe[p];
    const int64_t R = (int64_t)H * (tab.k0[p] - m_safe);
    const LayerT t = lt[pl];
    uint32_t remaining = R > 0 ? t.rem : 0u;
    for (int h = 0; h < H; ++h) {
        const int64_t u = (int64_t)pl * H + h;
        uint32_t b = (uint32_t)m_safe;
        if (R > 0) {
            const HeadT a = ht[u];
            const uint32_t ex = m_safe > 0 ? a.ties - a.prot : 0u;
            uint32_t gt = cnt[u].gt, eq = cnt[u].eq;
            if (a.T > t.TL) gt += ex;
            else if (a.T == t.TL) eq += ex;
            const uint32_t take = min(remaining, eq);
            remaining -= take;
            b += gt + take;
        }
        k_per_head[u] = (int32_t)b;
    }
}

struct HeadsWs {
    size_t ht, lhist, cnt, lt, total;
};

size_t up256(size_t n) { return (n + 255) / 256 * 256; }

HeadsWs heads_ws(int L, int H, const PromptTab &tab)
{
    const size_t layers = (size_t)tab.n * L, units = layers * H;
    HeadsWs w;
    size_t off = 0;
    w.ht = off;     off += up256(units * sizeof(HeadT));
    w.lhist = off;  off += up256(layers * 1024 * sizeof(uint32_t));
    w.cnt = off;    off += up256(units * sizeof(HeadCount));
    w.lt = off;     off += up256(layers * sizeof(LayerT));
    w.total = off;
    return w;
}

}  // namespace

size_t budget_heads_ws_bytes(int L, int H, const PromptTab &tab) { return heads_ws(L, H, tab).total; }

hipError_t launch_budget_heads(const float *scores, int L, int H, const PromptTab &tab, int32_t *k_per_head, void *ws,
                               hipStream_t st)
{
    const HeadsWs lay = heads_ws(L, H, tab);
    char *base = (char *)ws;
    HeadT *ht = (HeadT *)(base + lay.ht);
    uint32_t *lhist = (uint32_t *)(base + lay.lhist);
    HeadCount *cnt = (HeadCount *)(base + lay.cnt);
    LayerT *lt = (LayerT *)(base + lay.lt);
    const unsigned layers = (unsigned)(tab.n * L), units = layers * (unsigned)H;
    head_threshold_kernel<<<units, kThreads, 0, st>>>(scores, L, H, tab, ht, lhist);
    for (int pass = 0; pass < 4; ++pass) pool_pass_kernel<<<units, kThreads, 0, st>>>(scores, L, H, tab, pass, ht, lhist);
    head_count_kernel<<<units, kThreads, 0, st>>>(scores, L, H, tab, ht, lhist, cnt, lt);
    layer_assign_kernel<<<layers, 64, 0, st>>>(L, H, tab, ht, cnt, lt, k_per_head);
    return hipGetLastError();
}

}  // namespace nkv
