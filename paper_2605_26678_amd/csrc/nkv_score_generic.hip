// Shape-generic scoring kernels: per-scale cosine anomalies a_s, a_e, a_c (paper Sections 2.1-2.3)
// for any head dim (multiple of 8, <= 1024), any window and block size, fp32, bf16, fp16 or 8-bit (E4M3) keys.
//
// Four small kernels, none of them tuned -- they cover what the streaming kernels do not:
//   1. rnorm   : 1 / max(||k_i||, eps) per token                       (Section 2.1)
//   2. bsum    : sum of k_hat over every episodic block                (Section 2.2, episodic memory)
//   3. ssum    : sum of k_hat over the prompt = sum of its block sums  (Section 2.2, stable memory)
//   4. anomaly : a_s, a_e from the two sums; a_c from the window summed directly for every token
//                (Section 2.2 current memory; Section 2.3)
// Cosines do not depend on the length of the anchor, so sums stand in for the means.
#include "nkv_device.h"

namespace nkv {
namespace {

template <typename T>
__global__ __launch_bounds__(256) void rnorm_kernel(const T *__restrict__ keys, RowMap km, PromptTab tab,
                                                    int64_t rows, int d, float *__restrict__ rnorm)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t row = (int64_t)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (row >= rows) return;
    const int lh = (int)(row / tab.T), tg = (int)(row - (int64_t)lh * tab.T);
    const int p = prompt_of_token(tab, tg);
    const T *k = keys + km.unit(lh, p, tab) + (int64_t)(tg - tab.tok_off[p]) * d;
    float ss = 0.f;
    for (int c = lane; c < d; c += kWave) {
        float x = load_elem<T>(k + c);
        ss = fmaf(x, x, ss);
    }
    ss = wave_sum(ss);
    if (lane == 0) rnorm[row] = 1.0f / fmaxf(sqrtf(ss), kEps);
}

// grid (blocks per head, L*H); thread c owns dims c, c+256, ...
template <typename T>
__global__ __launch_bounds__(256) void bsum_kernel(const T *__restrict__ keys, RowMap km,
                                                   const float *__restrict__ rnorm, int d, PromptTab tab,
                                                   float *__restrict__ bsum)
{
    const int blk = blockIdx.x, lh = blockIdx.y;
    const int p = prompt_of_block(tab, blk);
    const int b = tab.b[p];
    const int n = tab.tok_off[p + 1] - tab.tok_off[p];
    const int lo = (blk - tab.blk_off[p]) * b;
    const int hi = min(lo + b, n);
    const int64_t row0 = (int64_t)lh * tab.T + tab.tok_off[p];
    const T *unit = keys + km.unit(lh, p, tab);
    for (int c = threadIdx.x; c < d; c += blockDim.x) {
        float s = 0.f;
        for (int t = lo; t < hi; ++t) s = fmaf(rnorm[row0 + t], load_elem<T>(unit + (int64_t)t * d + c), s);
        bsum[((int64_t)lh * tab.blk_off[tab.n] + blk) * d + c] = s;
    }
}

// grid (prompts, L*H)
__global__ __launch_bounds__(256) void ssum_kernel(const float *__restrict__ bsum, int d, PromptTab tab,
                                                   float *__restrict__ ssum)
{
    const int p = blockIdx.x, lh = blockIdx.y;
    const int nblk = tab.blk_off[tab.n];
    for (int c = threadIdx.x; c < d; c += blockDim.x) {
        float s = 0.f;
        for (int blk = tab.blk_off[p]; blk < tab.blk_off[p + 1]; ++blk)
            s += bsum[((int64_t)lh * nblk + blk) * d + c];
        ssum[((int64_t)lh * tab.n + p) * d + c] = s;
    }
}

// One wavefront per token; lane owns dims lane, lane+64, ... (NQ of them).
template <typename T, int NQ>
__global__ __launch_bounds__(256) void anomaly_kernel(const T *__restrict__ keys, RowMap km,
                                                      const float *__restrict__ rnorm,
                                                      const float *__restrict__ bsum,
                                                      const float *__restrict__ ssum, int LH, int d, int window,
                                                      PromptTab tab, float *__restrict__ a_raw)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t rows = (int64_t)LH * tab.T;
    const int64_t row = (int64_t)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (row >= rows) return;
    const int lh = (int)(row / tab.T);
    const int tg = (int)(row - (int64_t)lh * tab.T);
    const int p = prompt_of_token(tab, tg);
    const int i = tg - tab.tok_off[p];
    const int blk = tab.blk_off[p] + i / tab.b[p];
    const int64_t row0 = (int64_t)lh * tab.T + tab.tok_off[p];
    const T *unit = keys + km.unit(lh, p, tab);
    const float *S = ssum + ((int64_t)lh * tab.n + p) * d;
    const float *Bs = bsum + ((int64_t)lh * tab.blk_off[tab.n] + blk) * d;

    float kh[NQ], acc[NQ];
    const float rn = rnorm[row];
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        const int c = lane + q * kWave;
        kh[q] = c < d ? rn * load_elem<T>(unit + (int64_t)i * d + c) : 0.f;
        acc[q] = 0.f;
    }
    const int lo = max(0, i - window + 1);
    for (int j = lo; j <= i; ++j) {
        const float rj = rnorm[row0 + j];
        const T *kj = unit + (int64_t)j * d;
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const int c = lane + q * kWave;
            if (c < d) acc[q] = fmaf(rj, load_elem<T>(kj + c), acc[q]);
        }
    }
    float kk = 0.f, ds = 0.f, ns = 0.f, de = 0.f, ne = 0.f, dc = 0.f, nc = 0.f;
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        const int c = lane + q * kWave;
        const float s = c < d ? S[c] : 0.f, e = c < d ? Bs[c] : 0.f;
        kk = fmaf(kh[q], kh[q], kk);
        ds = fmaf(kh[q], s, ds);
        ns = fmaf(s, s, ns);
        de = fmaf(kh[q], e, de);
        ne = fmaf(e, e, ne);
        dc = fmaf(kh[q], acc[q], dc);
        nc = fmaf(acc[q], acc[q], nc);
    }
    kk = wave_sum(kk); ds = wave_sum(ds); ns = wave_sum(ns); de = wave_sum(de);
    ne = wave_sum(ne); dc = wave_sum(dc); nc = wave_sum(nc);
    if (lane == 0) {
        const float nk = fmaxf(sqrtf(kk), kEps);
        a_raw[row] = -ds / (nk * fmaxf(sqrtf(ns), kEps));
        a_raw[rows + row] = -de / (nk * fmaxf(sqrtf(ne), kEps));
        a_raw[2 * rows + row] = -dc / (nk * fmaxf(sqrtf(nc), kEps));
    }
}

template <typename T>
hipError_t run(const T *keys, const RowMap &km, int LH, int d, int window, const PromptTab &tab, float *a_raw, float *rnorm,
               float *bsum, float *ssum, const Prof &prof, hipStream_t st)
{
    const int64_t rows = (int64_t)LH * tab.T;
    const unsigned row_grid = (unsigned)((rows + 3) / 4);
    rnorm_kernel<T><<<row_grid, 256, 0, st>>>(keys, km, tab, rows, d, rnorm);
    bsum_kernel<T><<<dim3(tab.blk_off[tab.n], LH), 256, 0, st>>>(keys, km, rnorm, d, tab, bsum);
    ssum_kernel<<<dim3(tab.n, LH), 256, 0, st>>>(bsum, d, tab, ssum);
    const int nq = (d + kWave - 1) / kWave;
    prof.begin(NKV_KERNEL_SCAN, st);
#define NKV_ANOM(NQ) anomaly_kernel<T, NQ><<<row_grid, 256, 0, st>>>(keys, km, rnorm, bsum, ssum, LH, d, window, tab, a_raw)
    if (nq <= 1) NKV_ANOM(1);
    else if (nq <= 2) NKV_ANOM(2);
    else if (nq <= 4) NKV_ANOM(4);
    else if (nq <= 8) NKV_ANOM(8);
    else NKV_ANOM(16);
#undef NKV_ANOM
    prof.end(NKV_KERNEL_SCAN, st);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_score_generic(const void *keys, const RowMap &km, int dtype, int LH, int d, int window, const PromptTab &tab,
                                float *a_raw, float *rnorm, float *bsum, float *ssum, const Prof &prof,
                                hipStream_t st)
{
    if (dtype == NKV_DTYPE_F32)
        return run<float>((const float *)keys, km, LH, d, window, tab, a_raw, rnorm, bsum, ssum, prof, st);
    if (dtype == NKV_DTYPE_F16)
        return run<f16_t>((const f16_t *)keys, km, LH, d, window, tab, a_raw, rnorm, bsum, ssum, prof, st);
    if (dtype == NKV_DTYPE_F8_E4M3)
        return run<f8e4m3_t>((const f8e4m3_t *)keys, km, LH, d, window, tab, a_raw, rnorm, bsum, ssum, prof, st);
    return run<uint16_t>((const uint16_t *)keys, km, LH, d, window, tab, a_raw, rnorm, bsum, ssum, prof, st);
}

}  // namespace nkv
