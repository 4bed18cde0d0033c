// Device-side helpers shared by the libnkv kernels (gfx950, 64-wide wavefronts).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nkv_internal.h"

namespace nkv {

constexpr int kWave = 64;

// Order-preserving map float -> uint32 (larger float <=> larger key); -0 and +0 share a key.
__device__ __forceinline__ uint32_t ord_key(float x)
{
    uint32_t u = __float_as_uint(x);
    if (u == 0x80000000u) u = 0u;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ float key_value(uint32_t k)
{
    uint32_t u = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
    return __uint_as_float(u);
}

__device__ __forceinline__ float bf16_to_f32(uint16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// Element types that share a storage width are told apart by these wrappers.
struct f16_t { uint16_t bits; };
struct f8e4m3_t { uint8_t bits; };

// OCP 8-bit float, 4 exponent bits (bias 7), 3 mantissa bits, no infinities, S.1111.111 = NaN.
__device__ __forceinline__ float f8e4m3_to_f32(uint8_t v)
{
    const uint32_t e = (v >> 3) & 15u, m = v & 7u;
    uint32_t mag;
    if (e == 0u) mag = __float_as_uint((float)m * 0.001953125f);            // subnormal: m * 2^-9
    else if (e == 15u && m == 7u) mag = 0x7fc00000u;
    else mag = ((e + 120u) << 23) | (m << 20);
    return __uint_as_float(mag | ((uint32_t)(v & 0x80u) << 24));
}

template <typename T> __device__ __forceinline__ float load_elem(const T *p);
template <> __device__ __forceinline__ float load_elem<float>(const float *p) { return *p; }
template <> __device__ __forceinline__ float load_elem<uint16_t>(const uint16_t *p) { return bf16_to_f32(*p); }
template <> __device__ __forceinline__ float load_elem<f16_t>(const f16_t *p)
{
    return (float)*reinterpret_cast<const _Float16 *>(p);
}
template <> __device__ __forceinline__ float load_elem<f8e4m3_t>(const f8e4m3_t *p) { return f8e4m3_to_f32(p->bits); }

// Prompt that owns global token row t (0 <= t < tab.T).
__device__ __forceinline__ int prompt_of_token(const PromptTab &tab, int t)
{
    int p = 0;
    while (p + 1 < tab.n && t >= tab.tok_off[p + 1]) ++p;
    return p;
}

// Prompt that owns per-head block index blk (0 <= blk < tab.blk_off[tab.n]).
__device__ __forceinline__ int prompt_of_block(const PromptTab &tab, int blk)
{
    int p = 0;
    while (p + 1 < tab.n && blk >= tab.blk_off[p + 1]) ++p;
    return p;
}

template <typename T> __device__ __forceinline__ T wave_sum(T v)
{
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}
__device__ __forceinline__ float wave_min(float v)
{
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) v = fminf(v, __shfl_xor(v, o, kWave));
    return v;
}
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}

// Block-wide reductions for blockDim.x a multiple of 64 and <= 1024.  `scratch` holds >= 16 elements.
// Every thread receives the result; contains two barriers.
template <typename T> __device__ __forceinline__ T block_sum(T v, T *scratch)
{
    v = wave_sum(v);
    const int w = threadIdx.x / kWave, nw = blockDim.x / kWave;
    __syncthreads();
    if ((threadIdx.x & (kWave - 1)) == 0) scratch[w] = v;
    __syncthreads();
    T r = scratch[0];
    for (int i = 1; i < nw; ++i) r += scratch[i];
    return r;
}
__device__ __forceinline__ float block_min(float v, float *scratch)
{
    v = wave_min(v);
    const int w = threadIdx.x / kWave, nw = blockDim.x / kWave;
    __syncthreads();
    if ((threadIdx.x & (kWave - 1)) == 0) scratch[w] = v;
    __syncthreads();
    float r = scratch[0];
    for (int i = 1; i < nw; ++i) r = fminf(r, scratch[i]);
    return r;
}
__device__ __forceinline__ float block_max(float v, float *scratch)
{
    v = wave_max(v);
    const int w = threadIdx.x / kWave, nw = blockDim.x / kWave;
    __syncthreads();
    if ((threadIdx.x & (kWave - 1)) == 0) scratch[w] = v;
    __syncthreads();
    float r = scratch[0];
    for (int i = 1; i < nw; ++i) r = fmaxf(r, scratch[i]);
    return r;
}

// One digit step of a most-significant-digit-first radix select over 256-bin histograms.
// hist: counts of the current digit among candidates.  top != 0: walk from bin 255 down, else from 0 up,
// until the running count reaches `want` (1-based rank among the candidates).  Returns the digit and
// reduces `want` by the candidates passed over.  Serial; called by one thread per select.
__device__ __forceinline__ uint32_t radix_pick(const uint32_t *hist, uint32_t &want, int top)
{
    uint32_t cum = 0;
    if (top) {
        for (int b = 255; b > 0; --b) {
            uint32_t c = hist[b];
            if (cum + c >= want) { want -= cum; return (uint32_t)b; }
            cum += c;
        }
        want -= cum;
        return 0u;
    }
    for (int b = 0; b < 255; ++b) {
        uint32_t c = hist[b];
        if (cum + c >= want) { want -= cum; return (uint32_t)b; }
        cum += c;
    }
    want -= cum;
    return 255u;
}

}  // namespace nkv
