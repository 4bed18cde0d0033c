// Head-wise memory competition (paper Section 2.6, Appendix A "Hyperparameters").
//
// Every head of a layer first protects its own m_safe best tokens; the other R = H*(k0 - m_safe) slots
// go to the best unprotected (head, token) pairs of the layer.  Order everywhere: higher score, then
// lower head, then lower token index.  Only the per-head counts B_h are needed, and those follow from
// thresholds, so nothing is sorted:
//   A. per head, the key T_h of its m_safe-th best score and how many of the tokens tied at T_h are
//      protected (the lowest-indexed ones); the e_h = ties - protected others stay in the pool at key T_h;
//   B. over the pool {x < T_h} + {T_h repeated e_h times}, the key TL of the R-th best entry and how many
//      entries tied at TL are admitted (in head-then-index order, so heads are served in ascending order);
//   C. B_h = m_safe + #{pool entries of head h above TL} + its share of the ties at TL.
// All selects are radix selects on an order-preserving integer image of the fp32 scores: exact integer work.
//
// Three implementations:
//   * layers of up to 8 heads, any prompt length: the slice-wise kernels of nkv_budget_wide.hip (the default
//     for prompts of more than 8192 tokens);
//   * prompts of up to 32768 tokens and layers of up to 8 heads: head_safe_kernel (one workgroup per
//     (prompt, layer, head), scores in registers, step A plus a 2048-bin histogram of the head's pool on
//     the top 11 key bits) and layer_budget_kernel (one workgroup per (prompt, layer): the top digit from
//     the heads' histograms, then two passes over the layer's scores for the 11 middle and 10 low bits,
//     the last one with one histogram per head, which also yields step C);
//   * layers of more than 8 heads: the kernels of nkv_budget_heads.hip, budget_kernel's passes with one
//     workgroup per head;
//   * anything else (no scratch given): budget_kernel, one workgroup per (prompt, layer), nine byte-wise passes.
#include "nkv_blocksel.h"

namespace nkv {
namespace {

constexpr int kThreads = 1024;
constexpr int kFastHeads = 8;

struct HeadSafe {                // result of step A for one head
    uint32_t T, rem, ties, pad;
};

// ---------------------------------------------------------------------------------------------------
template <int EPT>
__global__ __launch_bounds__(kSelThreads, 8) void head_safe_kernel(const float *__restrict__ scores, int L, int H,
                                                                 PromptTab tab, int u0, HeadSafe *__restrict__ safe,
                                                                 uint32_t *__restrict__ pool_hist)
{
    __shared__ SelectScratch sel;
    __shared__ uint32_t hist0[2048];
    const int u = u0 + blockIdx.x;
    const int h = u % H, l = (u / H) % L, p = u / (H * L);
    const int N = tab.tok_off[p + 1] - tab.tok_off[p];
    const float *sc = scores + ((int64_t)l * H + h) * tab.T + tab.tok_off[p];
    const int tid = threadIdx.x;
    const int m_safe = tab.m_safe[p];

    uint32_t key[EPT];
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const int i = tid + j * kSelThreads;
        const float v = sc[min(i, N - 1)];                      // unconditional: the loads of a thread pipeline
        key[j] = i < N ? ord_key(v) : 0u;
    }
    uint32_t T = 0xFFFFFFFFu, rem = 0u, ties = 0u;
    if (m_safe > 0) {
        uint32_t kmin, kmax;
        block_key_range<EPT>(key, N, sel, kmin, kmax);
        T = block_select<EPT, true>(key, N, (uint32_t)m_safe, sel, kmin, kmax, rem, ties);
    }
    for (int j = tid; j < 2048; j += kSelThreads) hist0[j] = 0u;
    __syncthreads();
    {
        uint32_t cur = 0u, cnt = 0u;                         // run-length compressed LDS atomics
#pragma unroll
        for (int j = 0; j < EPT; ++j) {
            if (tid + j * kSelThreads < N && key[j] < T) {
                const uint32_t d = key[j] >> 21;
                if (cnt != 0u && d != cur) { atomicAdd(&hist0[cur], cnt); cnt = 0u; }
                cur = d;
                ++cnt;
            }
        }
        if (cnt != 0u) atomicAdd(&hist0[cur], cnt);
        if (tid == 0 && ties > rem) atomicAdd(&hist0[T >> 21], ties - rem);   // unprotected ties at T
    }
    __syncthreads();
    for (int j = tid; j < 2048; j += kSelThreads) pool_hist[(int64_t)u * 2048 + j] = hist0[j];
    if (tid == 0) safe[u] = HeadSafe{T, rem, ties, 0u};
}

// Calls f(h, key) for every score of the H <= kFastHeads heads of a layer (head h at s + h * stride, N scores
// each), the workgroup striding over the rows with U loads per head in flight per thread (the scores sit in
// L2 / memory; few loads at a time would be latency-bound).
template <typename F>
__device__ __forceinline__ void for_each_key(const float *__restrict__ s, int64_t stride, int H, int N, F f)
{
    constexpr int U = 4;
    for (int i0 = threadIdx.x; i0 < N; i0 += U * kThreads) {
        float v[kFastHeads][U];
#pragma unroll
        for (int h = 0; h < kFastHeads; ++h)
#pragma unroll
            for (int q = 0; q < U; ++q)
                v[h][q] = h < H ? s[h * stride + min(i0 + q * kThreads, N - 1)] : 0.f;
#pragma unroll
        for (int h = 0; h < kFastHeads; ++h)
#pragma unroll
            for (int q = 0; q < U; ++q)
                if (h < H && i0 + q * kThreads < N) f(h, ord_key(v[h][q]));
    }
}

// Finds the bin holding rank `want` from the top of an NB-bin histogram (NB = 1024 or 2048); 1024 threads.
// out[0] = bin, out[1] = rank inside the bin.  Contains barriers.
template <int NB>
__device__ __forceinline__ void block_pick_top(const uint32_t *hist, uint32_t want, uint32_t *wsum, uint32_t *out)
{
    constexpr int PER = NB / kThreads;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    uint32_t c[PER], group = 0u;
#pragma unroll
    for (int q = 0; q < PER; ++q) { c[q] = hist[tid * PER + q]; group += c[q]; }
    uint32_t incl = group;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t t = __shfl_down(incl, o, 64);
        if (lane + o < 64) incl += t;
    }
    if (lane == 0) wsum[w] = incl;
    __syncthreads();
    for (int ww = w + 1; ww < kThreads / 64; ++ww) incl += wsum[ww];
    uint32_t cum = incl - group;
    if (cum < want && want <= incl) {
#pragma unroll
        for (int q = PER - 1; q >= 0; --q) {
            if (cum < want && want <= cum + c[q]) { out[0] = (uint32_t)(tid * PER + q); out[1] = want - cum; }
            cum += c[q];
        }
    }
    __syncthreads();
}

__global__ __launch_bounds__(kThreads) void layer_budget_kernel(const float *__restrict__ scores, int L, int H,
                                                                PromptTab tab, const HeadSafe *__restrict__ safe,
                                                                const uint32_t *__restrict__ pool_hist,
                                                                int32_t *__restrict__ k_per_head)
{
    __shared__ uint32_t hist[2048];
    __shared__ uint32_t hist2[kFastHeads][1024];
    __shared__ uint32_t cnt_gt[kFastHeads];
    __shared__ uint32_t Th[kFastHeads], extra[kFastHeads];
    __shared__ uint32_t wsum[16], pick[2];

    const int pl = blockIdx.x, l = pl % L, p = pl / L;
    const int N = tab.tok_off[p + 1] - tab.tok_off[p];
    const int k0 = tab.k0[p], m_safe = tab.m_safe[p];
    const int tid = threadIdx.x;
    const uint32_t R = (uint32_t)H * (uint32_t)(k0 - m_safe);
    int32_t *out = k_per_head + (int64_t)pl * H;
    if (R == 0u) {
        if (tid < H) out[tid] = m_safe;
        return;
    }
    const HeadSafe *hsafe = safe + (int64_t)pl * H;
    const float *sc = scores + (int64_t)l * H * tab.T + tab.tok_off[p];          // head h at sc + h*T
    if (tid < H) {
        Th[tid] = hsafe[tid].T;
        extra[tid] = hsafe[tid].ties - hsafe[tid].rem;
        cnt_gt[tid] = 0u;
    }
    // top 11 bits: add up the heads' pool histograms
    for (int j = tid; j < 2048; j += kThreads) {
        uint32_t s = 0u;
        for (int h = 0; h < H; ++h) s += pool_hist[((int64_t)pl * H + h) * 2048 + j];
        hist[j] = s;
    }
    __syncthreads();
    block_pick_top<2048>(hist, R, wsum, pick);
    const uint32_t d0 = pick[0];
    uint32_t want = pick[1];
    __syncthreads();

    // middle 11 bits among pool entries whose top digit is d0
    for (int j = tid; j < 2048; j += kThreads) hist[j] = 0u;
    __syncthreads();
    uint32_t th[kFastHeads];
#pragma unroll
    for (int h = 0; h < kFastHeads; ++h) th[h] = h < H ? Th[h] : 0u;
    for_each_key(sc, tab.T, H, N, [&](int h, uint32_t key) {
        if (key < th[h] && (key >> 21) == d0) atomicAdd(&hist[(key >> 10) & 2047u], 1u);
    });
    if (tid < H && extra[tid] > 0u && (Th[tid] >> 21) == d0) atomicAdd(&hist[(Th[tid] >> 10) & 2047u], extra[tid]);
    __syncthreads();
    block_pick_top<2048>(hist, want, wsum, pick);
    const uint32_t pre22 = (d0 << 11) | pick[0];
    want = pick[1];
    __syncthreads();

    // low 10 bits, one histogram per head; entries above the 22-bit prefix are counted per head
    for (int j = tid; j < H * 1024; j += kThreads) (&hist2[0][0])[j] = 0u;
    __syncthreads();
    uint32_t gt[kFastHeads];
#pragma unroll
    for (int h = 0; h < kFastHeads; ++h) gt[h] = 0u;
    for_each_key(sc, tab.T, H, N, [&](int h, uint32_t key) {
        if (key < th[h]) {
            const uint32_t hi = key >> 10;
            if (hi > pre22) ++gt[h];
            else if (hi == pre22) atomicAdd(&hist2[h][key & 1023u], 1u);
        }
    });
#pragma unroll
    for (int h = 0; h < kFastHeads; ++h) {
        if (h < H) {
            const uint32_t g = wave_sum(gt[h]);
            if ((tid & 63) == 0 && g != 0u) atomicAdd(&cnt_gt[h], g);
        }
    }
    if (tid < H && extra[tid] > 0u) {
        if ((Th[tid] >> 10) > pre22) atomicAdd(&cnt_gt[tid], extra[tid]);
        else if ((Th[tid] >> 10) == pre22) atomicAdd(&hist2[tid][Th[tid] & 1023u], extra[tid]);
    }
    __syncthreads();
    hist[tid] = 0u;                                           // kThreads == 1024 bins
    {
        uint32_t s = 0u;
        for (int h = 0; h < H; ++h) s += hist2[h][tid];
        hist[tid] = s;
    }
    __syncthreads();
    block_pick_top<1024>(hist, want, wsum, pick);
    const uint32_t d2 = pick[0];
    // entries of each head above the layer threshold inside the last digit's range
    for (int h = 0; h < H; ++h) {
        uint32_t above = tid > (int)d2 ? hist2[h][tid] : 0u;
        above = wave_sum(above);
        if ((tid & 63) == 0 && above != 0u) atomicAdd(&cnt_gt[h], above);
    }
    __syncthreads();
    if (tid == 0) {
        uint32_t remaining = pick[1];                         // ties at the layer threshold still to admit
        for (int h = 0; h < H; ++h) {
            const uint32_t eq = hist2[h][d2];
            const uint32_t take = min(remaining, eq);
            remaining -= take;
            out[h] = (int32_t)((uint32_t)m_safe + cnt_gt[h] + take);
        }
    }
}

// ---------------------------------------------------------------------------------------------------
// Shape-generic version: any prompt length, up to NKV_MAX_HEADS heads.
// only_if (may be NULL): one word per (prompt, layer); layers whose word is zero are left alone.
__global__ __launch_bounds__(kThreads) void budget_kernel(const float *__restrict__ scores, int L, int H,
                                                          PromptTab tab, const uint32_t *__restrict__ only_if,
                                                          int32_t *__restrict__ k_per_head)
{
    __shared__ uint32_t hist[NKV_MAX_HEADS][256];      // 32 KB
    __shared__ uint32_t Th[NKV_MAX_HEADS];             // key of the m_safe-th best score of the head
    __shared__ uint32_t want_h[NKV_MAX_HEADS];         // running rank, ends as #protected among ties at Th
    __shared__ uint32_t ties_h[NKV_MAX_HEADS];         // #scores of the head equal to Th
    __shared__ uint32_t cnt_gt[NKV_MAX_HEADS], cnt_eq[NKV_MAX_HEADS];
    __shared__ uint32_t lhist[256];
    __shared__ uint32_t TL, want_l;

    const int pl = blockIdx.x;                          // p * L + l
    if (only_if && only_if[pl] == 0u) return;
    const int l = pl % L, p = pl / L;
    const int N = tab.tok_off[p + 1] - tab.tok_off[p];
    const int k0 = tab.k0[p], m_safe = tab.m_safe[p];
    const int64_t R = (int64_t)H * (k0 - m_safe);
    const float *sc = scores + (int64_t)l * H * tab.T + tab.tok_off[p];   // head h at sc + h*T
    const int tid = threadIdx.x;

    // ---- A: per-head safeguard thresholds ----
    if (tid < H) { Th[tid] = 0xFFFFFFFFu; want_h[tid] = (uint32_t)m_safe; ties_h[tid] = 0u; }
    __syncthreads();
    if (m_safe > 0) {
        if (tid < H) Th[tid] = 0u;
        for (int pass = 0; pass < 4; ++pass) {
            const int shift = 24 - 8 * pass;
            for (int j = tid; j < H * 256; j += kThreads) (&hist[0][0])[j] = 0u;
            __syncthreads();
            for (int h = 0; h < H; ++h) {
                const uint32_t th = Th[h];
                for (int i = tid; i < N; i += kThreads) {
                    const uint32_t key = ord_key(sc[(int64_t)h * tab.T + i]);
                    if (pass == 0 || (key >> (shift + 8)) == (th >> (shift + 8)))
                        atomicAdd(&hist[h][(key >> shift) & 255u], 1u);
                }
            }
            __syncthreads();
            if (tid < H) {
                uint32_t want = want_h[tid];
                const uint32_t dig = radix_pick(hist[tid], want, 1);
                want_h[tid] = want;
                Th[tid] |= dig << shift;
                if (pass == 3) ties_h[tid] = hist[tid][dig];
            }
            __syncthreads();
        }
    }

    // ---- B: layer threshold over the unprotected pool ----
    if (tid == 0) { TL = 0u; want_l = (uint32_t)R; }
    __syncthreads();
    if (R > 0) {
        for (int pass = 0; pass < 4; ++pass) {
            const int shift = 24 - 8 * pass;
            if (tid < 256) lhist[tid] = 0u;
            __syncthreads();
            const uint32_t pre = TL;
            for (int h = 0; h < H; ++h) {
                const uint32_t th = Th[h];
                for (int i = tid; i < N; i += kThreads) {
                    const uint32_t key = ord_key(sc[(int64_t)h * tab.T + i]);
                    if (key < th && (pass == 0 || (key >> (shift + 8)) == (pre >> (shift + 8))))
                        atomicAdd(&lhist[(key >> shift) & 255u], 1u);
                }
            }
            if (tid < H) {                               // unprotected ties at the head's own threshold
                const uint32_t ex = ties_h[tid] - (m_safe > 0 ? want_h[tid] : 0u);
                const uint32_t key = Th[tid];
                if (m_safe > 0 && ex > 0u && (pass == 0 || (key >> (shift + 8)) == (pre >> (shift + 8))))
                    atomicAdd(&lhist[(key >> shift) & 255u], ex);
            }
            __syncthreads();
            if (tid == 0) {
                uint32_t want = want_l;
                const uint32_t dig = radix_pick(lhist, want, 1);
                want_l = want;
                TL |= dig << shift;
            }
            __syncthreads();
        }
    }

    // ---- C: per-head counts ----
    if (tid < H) { cnt_gt[tid] = 0u; cnt_eq[tid] = 0u; }
    __syncthreads();
    if (R > 0) {
        const uint32_t tl = TL;
        for (int h = 0; h < H; ++h) {
            const uint32_t th = Th[h];
            for (int i = tid; i < N; i += kThreads) {
                const uint32_t key = ord_key(sc[(int64_t)h * tab.T + i]);
                if (key < th) {
                    if (key > tl) atomicAdd(&cnt_gt[h], 1u);
                    else if (key == tl) atomicAdd(&cnt_eq[h], 1u);
                }
            }
        }
    }
    __syncthreads();
    if (tid == 0) {
        uint32_t remaining = R > 0 ? want_l : 0u;
        for (int h = 0; h < H; ++h) {
            uint32_t b = (uint32_t)m_safe;
            if (R > 0) {
                const uint32_t ex = m_safe > 0 ? ties_h[h] - want_h[h] : 0u;
                uint32_t gt = cnt_gt[h], eq = cnt_eq[h];
                if (Th[h] > TL) gt += ex;
                else if (Th[h] == TL) eq += ex;
                const uint32_t take = min(remaining, eq);
                remaining -= take;
                b += gt + take;
            }
            k_per_head[(int64_t)pl * H + h] = (int32_t)b;
        }
    }
}

}  // namespace

size_t budget_ws_bytes(int L, int H, const PromptTab &tab)
{
    const size_t units = (size_t)tab.n * L * H;
    const size_t per_head = units * sizeof(HeadSafe) + units * 2048 * sizeof(uint32_t);
    const size_t wide = budget_wide_supported(H) ? budget_wide_ws_bytes(L, H, tab) : budget_heads_ws_bytes(L, H, tab);
    return per_head > wide ? per_head : wide;
}

hipError_t launch_budget(const float *scores, int L, int H, const PromptTab &tab, int32_t *k_per_head, void *ws,
                         bool per_head_route, const Prof &prof, hipStream_t st)
{
    int nmax = 0;
    for (int p = 0; p < tab.n; ++p) nmax = max(nmax, tab.tok_off[p + 1] - tab.tok_off[p]);
    const unsigned units = (unsigned)(tab.n * L * H);
    prof.begin(NKV_KERNEL_BUDGET, st);
    // Slice-wise kernels where a head has more than one slice or there are many units (five small launches);
    // for a few short units the two per-head launches are quicker.
    const bool per_head_ok = ws != nullptr && H <= kFastHeads && nmax <= 32 * kSelThreads;
    if (ws != nullptr && budget_wide_supported(H) && !(per_head_ok && (per_head_route || (nmax <= 8192 && units < 256)))) {
        const uint32_t *failed = nullptr;
        hipError_t e = launch_budget_wide(scores, L, H, tab, k_per_head, ws, &failed, st);
        if (e != hipSuccess) return e;
        budget_kernel<<<(unsigned)(tab.n * L), kThreads, 0, st>>>(scores, L, H, tab, failed, k_per_head);
    } else if (per_head_ok) {
        HeadSafe *safe = (HeadSafe *)ws;
        uint32_t *pool_hist = (uint32_t *)(safe + units);
        for_each_length_class(tab, L * H, [&](int ept, int u0, int n) {
            if (ept == 4) head_safe_kernel<4><<<n, kSelThreads, 0, st>>>(scores, L, H, tab, u0, safe, pool_hist);
            else if (ept == 8) head_safe_kernel<8><<<n, kSelThreads, 0, st>>>(scores, L, H, tab, u0, safe, pool_hist);
            else if (ept == 16) head_safe_kernel<16><<<n, kSelThreads, 0, st>>>(scores, L, H, tab, u0, safe, pool_hist);
            else head_safe_kernel<32><<<n, kSelThreads, 0, st>>>(scores, L, H, tab, u0, safe, pool_hist);
        });
        layer_budget_kernel<<<(unsigned)(tab.n * L), kThreads, 0, st>>>(scores, L, H, tab, safe, pool_hist, k_per_head);
    } else if (ws != nullptr && H > kFastHeads && !per_head_route) {
        const hipError_t e = launch_budget_heads(scores, L, H, tab, k_per_head, ws, st);
        if (e != hipSuccess) return e;
    } else {
        budget_kernel<<<(unsigned)(tab.n * L), kThreads, 0, st>>>(scores, L, H, tab, nullptr, k_per_head);
    }
    prof.end(NKV_KERNEL_BUDGET, st);
    return hipGetLastError();
}

}  // namespace nkv
