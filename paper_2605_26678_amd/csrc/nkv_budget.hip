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
// Selects are byte-wise radix selects, most significant digit first, on an order-preserving integer image
// of the fp32 scores: exact integer work.  One workgroup of 1024 threads per (prompt, layer); the layer's
// H*N scores (1 MiB at H = 8, N = 32768) are read from L2 nine times.
#include "nkv_device.h"

namespace nkv {
namespace {

constexpr int kThreads = 1024;

__global__ __launch_bounds__(kThreads) void budget_kernel(const float *__restrict__ scores, int L, int H,
                                                          PromptTab tab, int32_t *__restrict__ k_per_head)
{
    __shared__ uint32_t hist[NKV_MAX_HEADS][256];      // 64 KB
    __shared__ uint32_t Th[NKV_MAX_HEADS];             // key of the m_safe-th best score of the head
    __shared__ uint32_t want_h[NKV_MAX_HEADS];         // running rank, ends as #protected among ties at Th
    __shared__ uint32_t ties_h[NKV_MAX_HEADS];         // #scores of the head equal to Th
    __shared__ uint32_t cnt_gt[NKV_MAX_HEADS], cnt_eq[NKV_MAX_HEADS];
    __shared__ uint32_t lhist[256];
    __shared__ uint32_t TL, want_l;

    const int pl = blockIdx.x;                          // p * L + l
    const int l = pl % L, p = pl / L;
    const int N = tab.tok_off[p + 1] - tab.tok_off[p];
    const int k0 = tab.k0[p], m_safe = tab.m_safe[p];
    const int64_t R = (int64_t)H * (k0 - m_safe);
    const float *sc = scores + (int64_t)l * H * tab.T + tab.tok_off[p];   // head h at sc + h*T
    const int tid = threadIdx.x;
    const int64_t total = (int64_t)H * N;

    // ---- A: per-head safeguard thresholds ----
    if (tid < H) { Th[tid] = 0xFFFFFFFFu; want_h[tid] = (uint32_t)m_safe; ties_h[tid] = 0u; }
    __syncthreads();
    if (m_safe > 0) {
        if (tid < H) Th[tid] = 0u;
        for (int pass = 0; pass < 4; ++pass) {
            const int shift = 24 - 8 * pass;
            for (int j = tid; j < H * 256; j += kThreads) (&hist[0][0])[j] = 0u;
            __syncthreads();
            for (int64_t e = tid; e < total; e += kThreads) {
                const int h = (int)(e / N), i = (int)(e - (int64_t)h * N);
                const uint32_t key = ord_key(sc[(int64_t)h * tab.T + i]);
                if (pass == 0 || (key >> (shift + 8)) == (Th[h] >> (shift + 8)))
                    atomicAdd(&hist[h][(key >> shift) & 255u], 1u);
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
            for (int64_t e = tid; e < total; e += kThreads) {
                const int h = (int)(e / N), i = (int)(e - (int64_t)h * N);
                const uint32_t key = ord_key(sc[(int64_t)h * tab.T + i]);
                if (key < Th[h] && (pass == 0 || (key >> (shift + 8)) == (pre >> (shift + 8))))
                    atomicAdd(&lhist[(key >> shift) & 255u], 1u);
            }
            if (tid < H) {                               // unprotected ties at the head's own threshold
                const uint32_t extra = ties_h[tid] - (m_safe > 0 ? want_h[tid] : 0u);
                const uint32_t key = Th[tid];
                if (m_safe > 0 && extra > 0u && (pass == 0 || (key >> (shift + 8)) == (pre >> (shift + 8))))
                    atomicAdd(&lhist[(key >> shift) & 255u], extra);
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
        for (int64_t e = tid; e < total; e += kThreads) {
            const int h = (int)(e / N), i = (int)(e - (int64_t)h * N);
            const uint32_t key = ord_key(sc[(int64_t)h * tab.T + i]);
            if (key < Th[h]) {
                if (key > tl) atomicAdd(&cnt_gt[h], 1u);
                else if (key == tl) atomicAdd(&cnt_eq[h], 1u);
            }
        }
    }
    __syncthreads();
    if (tid == 0) {
        uint32_t remaining = R > 0 ? want_l : 0u;
        for (int h = 0; h < H; ++h) {
            uint32_t b = (uint32_t)m_safe;
            if (R > 0) {
                const uint32_t extra = m_safe > 0 ? ties_h[h] - want_h[h] : 0u;
                uint32_t gt = cnt_gt[h], eq = cnt_eq[h];
                if (Th[h] > TL) gt += extra;
                else if (Th[h] == TL) eq += extra;
                const uint32_t take = min(remaining, eq);
                remaining -= take;
                b += gt + take;
            }
            k_per_head[(int64_t)pl * H + h] = (int32_t)b;
        }
    }
}

}  // namespace

hipError_t launch_budget(const float *scores, int L, int H, const PromptTab &tab, int32_t *k_per_head,
                         const Prof &prof, hipStream_t st)
{
    prof.begin(NKV_KERNEL_BUDGET, st);
    budget_kernel<<<(unsigned)(tab.n * L), kThreads, 0, st>>>(scores, L, H, tab, k_per_head);
    prof.end(NKV_KERNEL_BUDGET, st);
    return hipGetLastError();
}

}  // namespace nkv
