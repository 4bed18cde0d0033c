// Slices: the unit of work of the kernels that spread a head's per-token values over the whole chip.
//
// A head's N values are cut into slices of 8192 tokens; a kernel that touches the values runs one 256-thread
// workgroup per slice (32 values per thread, element i of the slice in slot i / 256 of thread i % 256, so
// every load instruction of a wavefront is one contiguous 256-byte piece).  Slices are numbered prompt by
// prompt; inside a prompt (layer * H + head)-major, so the slices of a head -- and of a layer -- are contiguous.
//
// Values are binned by a monotone map of the value into 2048 bins; a per-slice histogram is stored as 2048
// 16-bit counts.  Exact work happens only on the entries of one boundary bin, which every slice copies into
// its own segment of kSeg keys.
#pragma once

#include "nkv_wavesel.h"

namespace nkv {
namespace {

constexpr int kSlice = 8192;             // tokens per slice (the counts of a slice fit 16 bits)
constexpr int kBins = 2048;
constexpr int kWideThreads = 256;
constexpr int kPerThread = kSlice / kWideThreads;
constexpr int kSeg = 256;                // keys one slice may contribute to a list

struct SliceTab {                        // first slice of every prompt; a prompt has L*H*S_p slices
    int32_t off[NKV_MAX_PROMPTS + 1];
};

inline size_t align256(size_t x) { return (x + 255) / 256 * 256; }

inline int fill_slices(int L, int H, const PromptTab &tab, SliceTab *st)
{
    int n = 0;
    for (int p = 0; p < tab.n; ++p) {
        st->off[p] = n;
        const int N = tab.tok_off[p + 1] - tab.tok_off[p];
        n += L * H * ((N + kSlice - 1) / kSlice);
    }
    st->off[tab.n] = n;
    return n;
}

// slice id -> prompt, (layer*H + head), slice within the unit, slices per unit
__device__ __forceinline__ void locate(const SliceTab &st, const PromptTab &tab, int id, int &p, int &lh, int &s,
                                       int &S)
{
    p = 0;
    while (p + 1 < tab.n && id >= st.off[p + 1]) ++p;
    const int N = tab.tok_off[p + 1] - tab.tok_off[p];
    S = (N + kSlice - 1) / kSlice;
    const int local = id - st.off[p];
    lh = local / S;
    s = local - lh * S;
}

// The values of slice s of a head of N tokens, as the hardware's bounds-checked buffer: slot j of thread tid is
// element j * 256 + tid of the slice (one instruction of a wavefront reads one contiguous 256-byte piece, the
// address is a 32-bit register and a constant), and elements past the head's last token read as 0.  The whole
// offset goes into the per-lane offset, which the range check is sure to cover.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t slice_values(const float *head, int s, int N)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(head + (int64_t)s * kSlice), 0,
                                             min(N - s * kSlice, kSlice) * 4, 0x00020000);
}

__device__ __forceinline__ float slice_value(__amdgpu_buffer_rsrc_t r, int tid, int j)
{
    return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, tid * 4 + j * (kWideThreads * 4), 0, 0));
}

// Four consecutive values per thread and load, for kernels that do not care which thread holds which value
// (histograms, minima): slot j of thread tid holds elements 4 (j * 256 + tid) .. + 3 of the slice.  The range check
// is per 32-bit word, so a head's last values are delivered and the words behind them read as 0.
__device__ __forceinline__ void slice_values4(__amdgpu_buffer_rsrc_t r, int tid, int j, float (&v)[4])
{
    const auto q = __builtin_amdgcn_raw_buffer_load_b128(r, (j * kWideThreads + tid) * 16, 0, 0);
    v[0] = __uint_as_float(q[0]); v[1] = __uint_as_float(q[1]); v[2] = __uint_as_float(q[2]); v[3] = __uint_as_float(q[3]);
}

// Scores: floor(2046 v) for 0 <= v <= 1, 0 below, 2047 above 1 (the pinned positions).  Monotone in v.
__device__ __forceinline__ int score_bin(float v)
{
    const float x = v * 2046.0f;
    return x >= 2046.0f ? (v > 1.0f ? 2047 : 2046) : (x > 0.f ? (int)x : 0);
}

// Anomalies (-cos, so in [-1, 1]): floor(1023.5 (a + 1)), clamped.  Monotone in a.
__device__ __forceinline__ int anomaly_bin(float a)
{
    const float x = (a + 1.0f) * 1023.5f;
    return x >= 2047.0f ? 2047 : (x > 0.f ? (int)x : 0);
}

// The 2048 counts of a workgroup's LDS histogram as 16-bit values: 8 bins per thread, one 16-byte store.
__device__ __forceinline__ void store_hist16(const uint32_t *hist, uint16_t *row)
{
    const uint32_t *h8 = hist + threadIdx.x * 8;
    reinterpret_cast<uint4 *>(row)[threadIdx.x] = make_uint4(h8[0] | (h8[1] << 16), h8[2] | (h8[3] << 16),
                                                             h8[4] | (h8[5] << 16), h8[6] | (h8[7] << 16));
}

// Histogram of the scores of one slice.  grid: slices; part: [slices][kBins] 16-bit counts.
__global__ __launch_bounds__(kWideThreads) void slice_hist_kernel(const float *__restrict__ scores, PromptTab tab,
                                                                  SliceTab st, uint16_t *__restrict__ part)
{
    __shared__ uint32_t hist[kBins];
    int p, lh, s, S;
    locate(st, tab, blockIdx.x, p, lh, s, S);
    const int N = tab.tok_off[p + 1] - tab.tok_off[p];
    const float *sc = scores + (int64_t)lh * tab.T + tab.tok_off[p];
    const int tid = threadIdx.x;
    for (int j = tid; j < kBins; j += kWideThreads) hist[j] = 0u;
    float v[kPerThread / 4][4];
    const __amdgpu_buffer_rsrc_t vals = slice_values(sc, s, N);
#pragma unroll
    for (int j = 0; j < kPerThread / 4; ++j) slice_values4(vals, tid, j, v[j]);
    __syncthreads();
#pragma unroll
    for (int j = 0; j < kPerThread / 4; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (s * kSlice + 4 * (j * kWideThreads + tid) + e < N) atomicAdd(&hist[score_bin(v[j][e])], 1u);
    __syncthreads();
    store_hist16(hist, part + (int64_t)blockIdx.x * kBins);
}

}  // namespace
}  // namespace nkv
