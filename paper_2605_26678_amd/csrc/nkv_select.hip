// Compression operator (paper Section 2.5): per unit keep the B_h best positions (ties: lower index),
// in ascending token order, and copy their K / V rows unchanged into a dense ragged cache.
//
//   head_off_kernel : exclusive scan of the clamped budgets -> first output row of every unit
//   select_kernel   : one workgroup per unit.  Byte-wise radix select of the B_h-th highest score
//                     (threshold key T, and how many of the tokens tied at T are kept), then an ordered
//                     stream compaction: a block-wide scan of (score > T, score == T) flags gives each
//                     kept token its output slot; kept_idx is written in ascending order.
//   gather_kernel   : flat over output rows; each row is a straight 16-byte-vector copy of one K row
//                     and one V row.
#include "nkv_blocksel.h"

namespace nkv {
namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / kWave;

__device__ __forceinline__ int unit_len(const PromptTab &tab, int L, int H, int u)
{
    const int p = u / (H * L);
    return tab.tok_off[p + 1] - tab.tok_off[p];
}

// Inclusive scan across the workgroup of a 64-bit value holding two 32-bit counters.
// Returns the inclusive prefix; *total receives the workgroup sum.  `scratch` holds kWaves + 1 entries.
__device__ __forceinline__ unsigned long long block_scan_incl(unsigned long long v, unsigned long long *scratch,
                                                              unsigned long long *total)
{
    const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        const unsigned long long t = __shfl_up(v, o, kWave);
        if (lane >= o) v += t;
    }
    __syncthreads();
    if (lane == kWave - 1) scratch[w] = v;
    __syncthreads();
    unsigned long long before = 0, all = 0;
    for (int i = 0; i < kWaves; ++i) {
        const unsigned long long s = scratch[i];
        if (i < w) before += s;
        all += s;
    }
    *total = all;
    return v + before;
}

__global__ __launch_bounds__(kThreads) void head_off_kernel(const int32_t *__restrict__ k_per_head, int L, int H,
                                                            PromptTab tab, int64_t *__restrict__ head_off,
                                                            int64_t *__restrict__ near_count)
{
    __shared__ unsigned long long scratch[kWaves + 1];
    const int n_units = tab.n * L * H;
    unsigned long long carry = 0;
    if (threadIdx.x == 0 && near_count) *near_count = 0;
    for (int u0 = 0; u0 < n_units; u0 += kThreads) {
        const int u = u0 + threadIdx.x;
        unsigned long long v = 0;
        if (u < n_units) v = (unsigned long long)min(max(k_per_head[u], 0), unit_len(tab, L, H, u));
        unsigned long long total;
        const unsigned long long incl = block_scan_incl(v, scratch, &total);
        if (u < n_units) head_off[u] = (int64_t)(carry + incl - v);
        carry += total;
    }
    if (threadIdx.x == 0) head_off[n_units] = (int64_t)carry;
}

__global__ __launch_bounds__(kThreads) void select_kernel(const float *__restrict__ scores,
                                                          const int32_t *__restrict__ k_per_head, int L, int H,
                                                          PromptTab tab, float near_tol,
                                                          const int64_t *__restrict__ head_off,
                                                          int64_t row_capacity, int32_t *__restrict__ kept_idx,
                                                          int64_t *__restrict__ near_count)
{
    __shared__ uint32_t hist[256];
    __shared__ uint32_t s_prefix, s_want;
    __shared__ unsigned long long scratch[kWaves + 1];
    __shared__ unsigned long long near_acc[16];

    const int u = blockIdx.x;
    const int h = u % H, l = (u / H) % L, p = u / (H * L);
    const int N = tab.tok_off[p + 1] - tab.tok_off[p];
    const int B = min(max(k_per_head[u], 0), N);
    if (B == 0) return;
    const float *sc = scores + ((int64_t)l * H + h) * tab.T + tab.tok_off[p];
    const int tid = threadIdx.x;
    const int64_t out0 = head_off[u];

    uint32_t T = 0u, rem = 0u;                       // B == N: every key >= 0 is kept
    if (B < N) {
        if (tid == 0) { s_prefix = 0u; s_want = (uint32_t)B; }
        __syncthreads();
        for (int pass = 0; pass < 4; ++pass) {
            const int shift = 24 - 8 * pass;
            if (tid < 256) hist[tid] = 0u;
            __syncthreads();
            const uint32_t pre = s_prefix;
            for (int i = tid; i < N; i += kThreads) {
                const uint32_t key = ord_key(sc[i]);
                if (pass == 0 || (key >> (shift + 8)) == (pre >> (shift + 8)))
                    atomicAdd(&hist[(key >> shift) & 255u], 1u);
            }
            __syncthreads();
            if (tid == 0) {
                uint32_t want = s_want;
                const uint32_t dig = radix_pick(hist, want, 1);
                s_want = want;
                s_prefix |= dig << shift;
            }
            __syncthreads();
        }
        T = s_prefix;
        rem = s_want;
        if (near_count) {                            // tokens within near_tol of the threshold score
            const float tv = key_value(T);
            unsigned long long c = 0;
            for (int i = tid; i < N; i += kThreads) c += fabsf(sc[i] - tv) <= near_tol ? 1ull : 0ull;
            c = block_sum(c, near_acc);
            if (tid == 0) atomicAdd((unsigned long long *)near_count, c);
        }
    }

    // ordered compaction
    uint32_t carry_gt = 0u, carry_eq = 0u;
    for (int i0 = 0; i0 < N; i0 += kThreads) {
        const int i = i0 + tid;
        uint32_t gt = 0u, eq = 0u;
        if (i < N) {
            const uint32_t key = ord_key(sc[i]);
            if (B == N) gt = 1u;
            else { gt = key > T ? 1u : 0u; eq = key == T ? 1u : 0u; }
        }
        const unsigned long long v = ((unsigned long long)gt << 32) | eq;
        unsigned long long total;
        const unsigned long long incl = block_scan_incl(v, scratch, &total);
        const uint32_t gt_before = carry_gt + (uint32_t)(incl >> 32) - gt;
        const uint32_t eq_before = carry_eq + (uint32_t)(incl & 0xffffffffu) - eq;
        if (gt || (eq && eq_before < rem)) {
            const int64_t row = out0 + gt_before + min(eq_before, rem);
            if (row < row_capacity) kept_idx[row] = i;
        }
        carry_gt += (uint32_t)(total >> 32);
        carry_eq += (uint32_t)(total & 0xffffffffu);
    }
}


// Units of up to 1024 * EPT tokens: scores in registers (element tid + j*1024 in slot j).  One radix select,
// then an ordered compaction without per-chunk barriers: every wavefront ballots its 64 consecutive tokens
// of chunk j, the (chunk, wave) population counts are scanned once in token order, and each kept token's
// output slot is its group's offset plus the number of kept lanes below it.
template <int EPT>
__global__ __launch_bounds__(kSelThreads, 8) void select_fast_kernel(const float *__restrict__ scores,
                                                                  const int32_t *__restrict__ k_per_head, int L,
                                                                  int H, PromptTab tab, int u0, float near_tol,
                                                                  const int64_t *__restrict__ head_off,
                                                                  int64_t row_capacity,
                                                                  int32_t *__restrict__ kept_idx,
                                                                  int64_t *__restrict__ near_count)
{
    __shared__ SelectScratch sel;
    __shared__ unsigned long long group_cnt[EPT * kWaves];           // (gt << 32 | eq) per (chunk, wave)
    __shared__ unsigned long long near_acc[16];

    const int u = u0 + blockIdx.x;
    const int h = u % H, l = (u / H) % L, p = u / (H * L);
    const int N = tab.tok_off[p + 1] - tab.tok_off[p];
    const int B = min(max(k_per_head[u], 0), N);
    if (B == 0) return;
    const float *sc = scores + ((int64_t)l * H + h) * tab.T + tab.tok_off[p];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int64_t out0 = head_off[u];

    uint32_t key[EPT];
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const int i = tid + j * kSelThreads;
        const float v = sc[min(i, N - 1)];                      // unconditional: the loads of a thread pipeline
        key[j] = i < N ? ord_key(v) : 0u;
    }
    uint32_t T = 0u, rem = 0u, ties = 0u;                             // B == N: every token is kept
    if (B < N) {
        uint32_t kmin, kmax;
        block_key_range<EPT>(key, N, sel, kmin, kmax);
        T = block_select<EPT, true>(key, N, (uint32_t)B, sel, kmin, kmax, rem, ties);
        if (near_count) {                                             // tokens within near_tol of the threshold score
            const float tv = key_value(T);
            unsigned long long c = 0;
#pragma unroll
            for (int j = 0; j < EPT; ++j)
                if (tid + j * kSelThreads < N && fabsf(key_value(key[j]) - tv) <= near_tol) ++c;
            c = block_sum(c, near_acc);
            if (tid == 0) atomicAdd((unsigned long long *)near_count, c);
        }
    }
    // population of every (chunk, wave) group
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const bool in = tid + j * kSelThreads < N;
        const bool gt = in && (B == N || key[j] > T);
        const bool eq = in && B < N && key[j] == T;
        const unsigned long long mg = __ballot(gt), me = __ballot(eq);
        if (lane == 0) group_cnt[j * kWaves + w] = ((unsigned long long)__popcll(mg) << 32) | (unsigned long long)__popcll(me);
    }
    __syncthreads();
    if (w == 0) {                                                     // exclusive scan over the groups in token order
        constexpr int PER = EPT * kWaves / 64;
        unsigned long long v[PER], tot = 0;
#pragma unroll
        for (int q = 0; q < PER; ++q) { v[q] = group_cnt[lane * PER + q]; tot += v[q]; }
        unsigned long long incl = tot;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const unsigned long long t = __shfl_up(incl, o, 64);
            if (lane >= o) incl += t;
        }
        unsigned long long run = incl - tot;
#pragma unroll
        for (int q = 0; q < PER; ++q) { group_cnt[lane * PER + q] = run; run += v[q]; }
    }
    __syncthreads();
    const unsigned long long below = (1ull << lane) - 1ull;
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        const int i = tid + j * kSelThreads;
        const bool in = i < N;
        const bool gt = in && (B == N || key[j] > T);
        const bool eq = in && B < N && key[j] == T;
        const unsigned long long mg = __ballot(gt), me = __ballot(eq);
        const unsigned long long base = group_cnt[j * kWaves + w];
        const uint32_t gt_before = (uint32_t)(base >> 32) + (uint32_t)__popcll(mg & below);
        const uint32_t eq_before = (uint32_t)(base & 0xffffffffu) + (uint32_t)__popcll(me & below);
        if (gt || (eq && eq_before < rem)) {
            const int64_t row = out0 + gt_before + min(eq_before, rem);
            if (row < row_capacity) kept_idx[row] = i;
        }
    }
}

constexpr int kRowsPerGroup = 64;

// 16-byte vectors; krow16 / vrow16 = vectors per K / V row, epv = elements per vector.
__global__ __launch_bounds__(256) void gather_kernel(const uint4 *__restrict__ keys, const uint4 *__restrict__ values,
                                                     RowMap km, RowMap vm, int epv,
                                                     int L, int H, int krow16, int vrow16, PromptTab tab,
                                                     const int64_t *__restrict__ head_off,
                                                     const int32_t *__restrict__ kept_idx, int64_t row_capacity,
                                                     uint4 *__restrict__ packed_k, uint4 *__restrict__ packed_v)
{
    __shared__ int64_t srck[kRowsPerGroup], srcv[kRowsPerGroup];       // first vector of the source rows
    const int n_units = tab.n * L * H;
    const int64_t rows = min(head_off[n_units], row_capacity);
    const int64_t r0 = (int64_t)blockIdx.x * kRowsPerGroup;
    if (r0 >= rows) return;
    const int nr = (int)min((int64_t)kRowsPerGroup, rows - r0);
    if ((int)threadIdx.x < nr) {
        const int64_t r = r0 + threadIdx.x;
        int lo = 0, hi = n_units;                   // largest u with head_off[u] <= r
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (head_off[mid] <= r) lo = mid; else hi = mid;
        }
        const int u = lo;
        const int h = u % H, l = (u / H) % L, p = u / (H * L);
        const int64_t i = kept_idx[r];
        srck[threadIdx.x] = km.unit(l * H + h, p, tab) / epv + i * krow16;
        srcv[threadIdx.x] = vm.unit(l * H + h, p, tab) / epv + i * vrow16;
    }
    __syncthreads();
    using v4 = unsigned int __attribute__((ext_vector_type(4)));
    // four vectors of a tensor per thread in flight at a time: the loads are unconditional (a slot past the end
    // repeats the last vector), so that they go out together, and only the stores are guarded
    auto move = [&](const uint4 *src, uint4 *dst, const int64_t *first, int row16) {
        const int total = nr * row16;
        for (int j0 = threadIdx.x; j0 < total; j0 += 4 * 256) {
            v4 v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int j = min(j0 + i * 256, total - 1), r = j / row16, c = j - r * row16;
                v[i] = __builtin_nontemporal_load(reinterpret_cast<const v4 *>(src) + first[r] + c);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int j = j0 + i * 256, r = j / row16, c = j - r * row16;
                if (j < total) __builtin_nontemporal_store(v[i], reinterpret_cast<v4 *>(dst) + (r0 + r) * row16 + c);
            }
        }
    };
    move(keys, packed_k, srck, krow16);
    move(values, packed_v, srcv, vrow16);
}

// In-place compaction: grid (units, 2); workgroup (u, 0) moves the kept K rows of unit u to the front of the unit's
// own rows, workgroup (u, 1) the V rows.  The j-th kept row comes from row kept_idx[j] >= j, so rows only move
// forwards; a workgroup takes its unit's rows in pieces of 128, front to back, and loads a whole piece into
// registers before it stores any of it: a piece's sources lie at or behind its own destinations (so no earlier
// piece's store has touched them), and what it overwrites are rows that this and earlier pieces have already read.
constexpr int kInPlaceRows = 128, kInPlaceThreads = 256;
template <int VPT>                       // 16-byte vectors per thread and piece: 128 rows x row16 / 256 threads
__global__ __launch_bounds__(kInPlaceThreads) void compact_inplace_kernel(uint4 *__restrict__ keys, uint4 *__restrict__ values,
                                                                          RowMap km, RowMap vm, int epv, int L, int H,
                                                                          int krow16, int vrow16, PromptTab tab,
                                                                          const int64_t *__restrict__ head_off,
                                                                          const int32_t *__restrict__ kept_idx,
                                                                          int64_t row_capacity)
{
    using v4 = unsigned int __attribute__((ext_vector_type(4)));
    const int u = blockIdx.x, which = blockIdx.y;
    const int h = u % H, l = (u / H) % L, p = u / (H * L);
    const int row16 = which == 0 ? krow16 : vrow16;
    if (VPT * kInPlaceThreads != kInPlaceRows * row16) return;        // (the host launches the matching instance)
    v4 *base = reinterpret_cast<v4 *>(which == 0 ? keys : values) +
               (which == 0 ? km.unit(l * H + h, p, tab) : vm.unit(l * H + h, p, tab)) / epv;
    const int64_t r0 = head_off[u];
    const int64_t B = min(head_off[u + 1], row_capacity) - r0;        // rows whose index the caller's kept_idx holds
    // Loads are unconditional (rows past the piece's end repeat its last row), so that a thread's index loads, and
    // then its row loads, are all in flight together instead of one after the other.
    for (int64_t j0 = 0; j0 < B; j0 += kInPlaceRows) {
        const int nr = (int)min((int64_t)kInPlaceRows, B - j0);
        int src[VPT];
        v4 v[VPT];
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
            const int j = i * kInPlaceThreads + threadIdx.x, r = min(j / row16, nr - 1);
            src[i] = kept_idx[r0 + j0 + r];
        }
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
            const int j = i * kInPlaceThreads + threadIdx.x, c = j % row16;
            v[i] = __builtin_nontemporal_load(base + (int64_t)src[i] * row16 + c);
        }
        // every thread's loads of the piece have returned before any thread stores into the piece's range
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
            const int j = i * kInPlaceThreads + threadIdx.x, r = j / row16, c = j - r * row16;
            if (r < nr) __builtin_nontemporal_store(v[i], base + (j0 + r) * row16 + c);
        }
    }
}

// The yardstick: every workgroup moves contiguous 16 KB pieces with non-temporal 16-byte loads and stores, four
// loads in flight per thread -- the access pattern of the gather above without its indirection.  dst == nullptr:
// loads only (what a pure reader such as the decode consumer can reach); an empty assembly statement that takes
// the loaded registers keeps the compiler from dropping the loads.
__global__ __launch_bounds__(256) void copy_kernel(uint4 *__restrict__ dst, const uint4 *__restrict__ src, size_t n)
{
    using v4 = unsigned int __attribute__((ext_vector_type(4)));
    constexpr size_t kPiece = 1024;                                   // 16-byte vectors per piece
    const v4 *s = reinterpret_cast<const v4 *>(src);
    v4 *d = reinterpret_cast<v4 *>(dst);
    for (size_t p0 = (size_t)blockIdx.x * kPiece; p0 < n; p0 += (size_t)gridDim.x * kPiece) {
        v4 v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const size_t i = p0 + j * 256 + threadIdx.x;
            v[j] = i < n ? __builtin_nontemporal_load(s + i) : v4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const size_t i = p0 + j * 256 + threadIdx.x;
            if (d) {
                if (i < n) __builtin_nontemporal_store(v[j], d + i);
            } else {
                asm volatile("" ::"v"(v[j].x), "v"(v[j].y), "v"(v[j].z), "v"(v[j].w));
            }
        }
    }
}

}  // namespace

hipError_t launch_copy_probe(void *dst, const void *src, size_t bytes, hipStream_t st)
{
    const size_t n = bytes / 16;
    if (n == 0) return hipSuccess;
    const size_t want = (n + 1023) / 1024;
    const unsigned groups = (unsigned)(want < 256 * 64 ? want : 256 * 64);     // up to 64 workgroups per CU
    copy_kernel<<<groups, 256, 0, st>>>((uint4 *)dst, (const uint4 *)src, n);
    return hipGetLastError();
}

hipError_t launch_select_compact(const void *keys, const void *values, const RowMap &km, const RowMap &vm,
                                 void *wide_ws, const float *scores,
                                 const int32_t *k_per_head, int L, int H, int d, int dv, int esize,
                                 const PromptTab &tab, float near_tol, void *packed_k, void *packed_v,
                                 int32_t *kept_idx, int64_t *head_off, int64_t row_capacity,
                                 int64_t *near_count, bool in_place, const Prof &prof, hipStream_t st)
{
    const int n_units = tab.n * L * H;
    int nmax = 0;
    for (int p = 0; p < tab.n; ++p) nmax = max(nmax, tab.tok_off[p + 1] - tab.tok_off[p]);
    const bool wide = wide_ws != nullptr && (nmax > 16384 || n_units >= 2048);
    const bool wide_places = wide && select_wide_places_units(n_units);
    if (!wide_places) head_off_kernel<<<1, kThreads, 0, st>>>(k_per_head, L, H, tab, head_off, near_count);
    prof.begin(NKV_KERNEL_SELECT, st);
#define NKV_SELECT_FAST(EPT)                                                                              \
    select_fast_kernel<EPT><<<(unsigned)n, kSelThreads, 0, st>>>(scores, k_per_head, L, H, tab, u0, near_tol, \
                                                                 head_off, row_capacity, kept_idx, near_count)
    // Slice-wise kernels where a head has more than two slices or there are thousands of units, and the caller
    // gave scratch (for a few hundred units of up to two slices the six launches cost what they save).
    if (wide) {
        const hipError_t e = launch_select_wide(scores, k_per_head, L, H, tab, near_tol, head_off, row_capacity,
                                                kept_idx, near_count, wide_places, wide_ws, st);
        if (e != hipSuccess) return e;
    } else if (nmax <= 32 * kSelThreads)
        for_each_length_class(tab, L * H, [&](int ept, int u0, int n) {
            if (ept == 4) NKV_SELECT_FAST(4);
            else if (ept == 8) NKV_SELECT_FAST(8);
            else if (ept == 16) NKV_SELECT_FAST(16);
            else NKV_SELECT_FAST(32);
        });
    else
        select_kernel<<<(unsigned)n_units, kThreads, 0, st>>>(scores, k_per_head, L, H, tab, near_tol, head_off,
                                                              row_capacity, kept_idx, near_count);
#undef NKV_SELECT_FAST
    prof.end(NKV_KERNEL_SELECT, st);
    // no unit keeps more than its prompt length, so the row count is bounded by L*H*T as well
    const int64_t max_rows = row_capacity < (int64_t)L * H * tab.T ? row_capacity : (int64_t)L * H * tab.T;
    if (max_rows > 0 && in_place) {
        const int krow16 = d * esize / 16, vrow16 = dv * esize / 16;
        prof.begin(NKV_KERNEL_GATHER, st);
        // one instance per row width; K and V rows of different widths take a launch each
        for (int which = 0; which < 2; ++which) {
            const int row16 = which == 0 ? krow16 : vrow16;
            if (which == 1 && vrow16 == krow16) break;                // both were moved by the first launch
            const dim3 grid((unsigned)n_units, vrow16 == krow16 ? 2u : 1u);
            uint4 *k4 = (uint4 *)const_cast<void *>(keys), *v4p = (uint4 *)const_cast<void *>(values);
            uint4 *a = which == 0 ? k4 : v4p, *b = which == 0 ? v4p : k4;          // blockIdx.y == 0 moves `a`
            const RowMap &am = which == 0 ? km : vm, &bm = which == 0 ? vm : km;
#define NKV_INPLACE(VPT)                                                                                             \
    compact_inplace_kernel<VPT><<<grid, kInPlaceThreads, 0, st>>>(a, b, am, bm, 16 / esize, L, H, row16, row16, tab, \
                                                                  head_off, kept_idx, row_capacity)
            switch (row16 * kInPlaceRows / kInPlaceThreads) {
            case 1: NKV_INPLACE(1); break;
            case 2: NKV_INPLACE(2); break;
            case 4: NKV_INPLACE(4); break;
            case 8: NKV_INPLACE(8); break;
            case 16: NKV_INPLACE(16); break;
            case 32: NKV_INPLACE(32); break;
            default: return hipErrorInvalidValue;                     // (refused by the caller: see in_place_supported)
            }
#undef NKV_INPLACE
        }
        prof.end(NKV_KERNEL_GATHER, st);
    } else if (max_rows > 0) {
        const unsigned groups = (unsigned)((max_rows + kRowsPerGroup - 1) / kRowsPerGroup);
        prof.begin(NKV_KERNEL_GATHER, st);
        gather_kernel<<<groups, 256, 0, st>>>((const uint4 *)keys, (const uint4 *)values, km, vm, 16 / esize, L, H,
                                              d * esize / 16,
                                              dv * esize / 16, tab, head_off, kept_idx, row_capacity,
                                              (uint4 *)packed_k, (uint4 *)packed_v);
        prof.end(NKV_KERNEL_GATHER, st);
    }
    return hipGetLastError();
}

}  // namespace nkv
