// Decode-side consumer of the compressed cache: one new token's attention over the rows the compression
// operator kept (paper Section 2.5 for the layout of the cache, Appendix A "Complexity": retained keys and
// values are unchanged, so ordinary attention applies; Section 3.5 reports the per-token decode latency).
//
// For unit u = (prompt, layer, KV head) and the G query heads that read it (grouped-query attention, query
// head j reads KV head j / G):   out_j = sum_i softmax_i(scale <q_j, k_i>) v_i   over the unit's rows.
//
// The work is one read of every retained K and V row, so it is bound by HBM.  Units have different lengths
// (head-wise budgets), so they are cut into chunks of 256 rows and one workgroup handles one chunk for all G
// query heads at once (K and V are read once, not G times):
//   decode_plan_kernel    : chunk_off[u] = chunks before unit u (exclusive scan of ceil(len_u / 256))
//   decode_chunk_kernel   : per chunk, running-maximum softmax in base 2: (m, l, o[0..D)) per query head
//   decode_combine_kernel : per (unit, query head) merges the chunks' partial results
// Lane layout in decode_chunk_kernel as in the scoring kernel: a row is spread over D/8 lanes (16 bytes each),
// one wave load fetches 64/(D/8) rows; <q, k> uses the packed 16-bit dot instruction on the stored bits (exact
// products, fp32 accumulation) and a DPP sum over the lanes of a row; every group of D/8 lanes keeps its own
// running (m, l, o) for the rows it sees, rescaled once per batch of four rows, and the groups and waves are
// merged through LDS at the end of the chunk.
// Anything outside bf16 / fp16 with d = dv in {64, 128} and G <= 8 goes to decode_generic_kernel (one workgroup per
// unit and query head, no scratch).
#include "nkv_device.h"

namespace nkv {
namespace {

constexpr int kChunk = 256;              // rows per workgroup
constexpr int kDecThreads = 256;
constexpr float kNone = -1.0e30f;        // running maximum before any row was seen
constexpr float kLn2 = 0.6931471805599453f;

using u32x4 = unsigned int __attribute__((ext_vector_type(4)));

template <int CTRL> __device__ __forceinline__ float dpp_add(float v)
{
    return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
template <int LPR> __device__ __forceinline__ float group_sum(float v)
{
    v = dpp_add<0xB1>(v);                        // quad_perm [1,0,3,2]
    v = dpp_add<0x4E>(v);                        // quad_perm [2,3,0,1]
    v = dpp_add<0x141>(v);                       // row_half_mirror
    if (LPR == 16) v = dpp_add<0x140>(v);        // row_mirror
    return v;
}

// <a, b> over the eight bf16 pairs of two packed 16-byte pieces.  The compiler does not see the register
// write inside the assembly, so the wait states a DPP read of the result needs are spent here.
// F16: the sixteen-bit values are fp16 instead of bf16 (the only two places that know).
template <bool F16> __device__ __forceinline__ float dot8_for_dpp(const u32x4 &a, const u32x4 &b)
{
    float acc = 0.f;
    if constexpr (F16)
        asm("v_dot2c_f32_f16 %0, %1, %5\n\t"
            "v_dot2c_f32_f16 %0, %2, %6\n\t"
            "v_dot2c_f32_f16 %0, %3, %7\n\t"
            "v_dot2c_f32_f16 %0, %4, %8\n\t"
            "s_nop 1"
            : "+v"(acc)
            : "v"(a.x), "v"(a.y), "v"(a.z), "v"(a.w), "v"(b.x), "v"(b.y), "v"(b.z), "v"(b.w));
    else
        asm("v_dot2c_f32_bf16 %0, %1, %5\n\t"
            "v_dot2c_f32_bf16 %0, %2, %6\n\t"
            "v_dot2c_f32_bf16 %0, %3, %7\n\t"
            "v_dot2c_f32_bf16 %0, %4, %8\n\t"
            "s_nop 1"
            : "+v"(acc)
            : "v"(a.x), "v"(a.y), "v"(a.z), "v"(a.w), "v"(b.x), "v"(b.y), "v"(b.z), "v"(b.w));
    return acc;
}

template <bool F16> __device__ __forceinline__ void unpack8(const u32x4 &r, float k[8])
{
    if constexpr (F16) {
        using f16x2 = _Float16 __attribute__((ext_vector_type(2)));
        const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const f16x2 v = __builtin_bit_cast(f16x2, w[i]);
            k[2 * i] = (float)v.x;
            k[2 * i + 1] = (float)v.y;
        }
    } else {
        k[0] = __uint_as_float(r.x << 16); k[1] = __uint_as_float(r.x & 0xffff0000u);
        k[2] = __uint_as_float(r.y << 16); k[3] = __uint_as_float(r.y & 0xffff0000u);
        k[4] = __uint_as_float(r.z << 16); k[5] = __uint_as_float(r.z & 0xffff0000u);
        k[6] = __uint_as_float(r.w << 16); k[7] = __uint_as_float(r.w & 0xffff0000u);
    }
}

__device__ __forceinline__ int64_t clamp_row(int64_t r, int64_t rows) { return r < 0 ? 0 : (r > rows ? rows : r); }

// One workgroup of 1024 threads.  chunk_off has n_units + 1 entries.
__global__ __launch_bounds__(1024) void decode_plan_kernel(const int64_t *__restrict__ head_off, int n_units,
                                                           int64_t rows, int32_t *__restrict__ chunk_off)
{
    __shared__ int32_t sums[16];                                      // per-wave totals
    const int per = (n_units + 1023) / 1024;
    const int u0 = min(threadIdx.x * per, n_units), u1 = min(u0 + per, n_units);
    int32_t mine = 0;
    for (int u = u0; u < u1; ++u) {
        const int64_t len = clamp_row(head_off[u + 1], rows) - clamp_row(head_off[u], rows);
        mine += (int32_t)((max(len, (int64_t)0) + kChunk - 1) / kChunk);
    }
    // exclusive scan of the 1024 per-thread counts: inside every wave by shuffles, then over the 16 wave totals
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    int32_t incl = mine;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int32_t t = __shfl_up(incl, o, 64);
        if (lane >= o) incl += t;
    }
    if (lane == 63) sums[wv] = incl;
    __syncthreads();
    int32_t before = 0, total = 0;
    for (int i = 0; i < 16; ++i) {
        const int32_t t = sums[i];
        if (i < wv) before += t;
        total += t;
    }
    if (threadIdx.x == 0) chunk_off[n_units] = total;
    int32_t run = before + incl - mine;
    for (int u = u0; u < u1; ++u) {
        chunk_off[u] = run;
        const int64_t len = clamp_row(head_off[u + 1], rows) - clamp_row(head_off[u], rows);
        run += (int32_t)((max(len, (int64_t)0) + kChunk - 1) / kChunk);
    }
}

// part: per chunk and query head D + 2 floats: running maximum (base-2 logits), sum of weights, weighted values.
template <int D, int G, bool F16>
__global__ __launch_bounds__(kDecThreads) void decode_chunk_kernel(const uint16_t *__restrict__ q,
                                                                   const uint16_t *__restrict__ pk,
                                                                   const uint16_t *__restrict__ pv,
                                                                   const int64_t *__restrict__ head_off,
                                                                   const int32_t *__restrict__ chunk_off, int n_units,
                                                                   int64_t rows, float scale_log2,
                                                                   float *__restrict__ part)
{
    constexpr int LPR = D / 8, RPW = 64 / LPR, NLD = 64 / RPW, U = 4, NW = kDecThreads / 64;
    constexpr int kRowBytes = D * 2;
    __shared__ float lds_m[NW * RPW][G], lds_l[NW * RPW][G];
    __shared__ float lds_o[NW * RPW][G][D];
    const int chunk = blockIdx.x;
    if (chunk >= chunk_off[n_units]) return;
    int lo = 0, hi = n_units;                                        // largest u with chunk_off[u] <= chunk
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (chunk_off[mid] <= chunk) lo = mid; else hi = mid;
    }
    const int u = lo, ci = chunk - chunk_off[u];
    const int64_t first = clamp_row(head_off[u], rows), len = clamp_row(head_off[u + 1], rows) - first;
    const int n = (int)min((int64_t)kChunk, len - (int64_t)ci * kChunk);     // rows of this chunk, >= 1
    const int64_t r0 = first + (int64_t)ci * kChunk;

    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63, gi = lane / LPR, c = lane % LPR;
    u32x4 qv[G];
#pragma unroll
    for (int g = 0; g < G; ++g)
        qv[g] = *reinterpret_cast<const u32x4 *>(q + ((int64_t)u * G + g) * D + c * 8);

    float m[G], l[G], o[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        m[g] = kNone;
        l[g] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[g][e] = 0.f;
    }
    // rows past the end of the chunk read as zeros and get weight 0
    const __amdgpu_buffer_rsrc_t krs = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(pk) + r0 * D, 0,
                                                                         n * kRowBytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t vrs = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(pv) + r0 * D, 0,
                                                                         n * kRowBytes, 0x00020000);
    if (w * 64 < n) {
#pragma unroll 1
        for (int b0 = 0; b0 < NLD; b0 += U) {
            const int row0 = w * 64 + b0 * RPW + gi;                 // this lane group's row in load b0
            if (w * 64 + b0 * RPW >= n) break;                       // uniform in the wave
            u32x4 kr[U], vr[U];
#pragma unroll
            for (int i = 0; i < U; ++i)
                kr[i] = __builtin_amdgcn_raw_buffer_load_b128(krs, (row0 + i * RPW) * kRowBytes + c * 16, 0, 2);   // aux 2: non-temporal
#pragma unroll
            for (int i = 0; i < U; ++i)
                vr[i] = __builtin_amdgcn_raw_buffer_load_b128(vrs, (row0 + i * RPW) * kRowBytes + c * 16, 0, 2);
            float s[U][G];
#pragma unroll
            for (int i = 0; i < U; ++i) {
                const bool valid = row0 + i * RPW < n;
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    const float d = group_sum<LPR>(dot8_for_dpp<F16>(kr[i], qv[g]));
                    s[i][g] = valid ? d * scale_log2 : kNone;
                }
            }
            float p[U][G];
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float mb = m[g];
#pragma unroll
                for (int i = 0; i < U; ++i) mb = fmaxf(mb, s[i][g]);
                const float corr = __builtin_amdgcn_exp2f(m[g] - mb);    // 1 if nothing changed, 0 from kNone
                m[g] = mb;
                l[g] *= corr;
#pragma unroll
                for (int e = 0; e < 8; ++e) o[g][e] *= corr;
#pragma unroll
                for (int i = 0; i < U; ++i) {
                    p[i][g] = row0 + i * RPW < n ? __builtin_amdgcn_exp2f(s[i][g] - mb) : 0.f;
                    l[g] += p[i][g];
                }
            }
#pragma unroll
            for (int i = 0; i < U; ++i) {
                float v[8];
                unpack8<F16>(vr[i], v);
#pragma unroll
                for (int g = 0; g < G; ++g)
#pragma unroll
                    for (int e = 0; e < 8; ++e) o[g][e] = fmaf(p[i][g], v[e], o[g][e]);
            }
        }
    }
    // ---- merge the lane groups and waves of the workgroup ----
    const int slot = w * RPW + gi;
#pragma unroll
    for (int g = 0; g < G; ++g) {
        if (c == 0) {
            lds_m[slot][g] = m[g];
            lds_l[slot][g] = l[g];
        }
        *reinterpret_cast<float4 *>(&lds_o[slot][g][c * 8]) = make_float4(o[g][0], o[g][1], o[g][2], o[g][3]);
        *reinterpret_cast<float4 *>(&lds_o[slot][g][c * 8 + 4]) = make_float4(o[g][4], o[g][5], o[g][6], o[g][7]);
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < G * D; idx += kDecThreads) {
        const int g = idx / D, e = idx - g * D;
        float mm = kNone;
#pragma unroll
        for (int sl = 0; sl < NW * RPW; ++sl) mm = fmaxf(mm, lds_m[sl][g]);
        float ll = 0.f, oo = 0.f;
#pragma unroll
        for (int sl = 0; sl < NW * RPW; ++sl) {
            const float f = __builtin_amdgcn_exp2f(lds_m[sl][g] - mm);
            ll = fmaf(f, lds_l[sl][g], ll);
            oo = fmaf(f, lds_o[sl][g][e], oo);
        }
        float *dst = part + ((int64_t)chunk * G + g) * (D + 2);
        if (e == 0) {
            dst[0] = mm;
            dst[1] = ll;
        }
        dst[2 + e] = oo;
    }
}

// grid: n_units * G workgroups of D threads (D = 64 or 128: one or two waves)
template <int D>
__global__ __launch_bounds__(D) void decode_combine_kernel(const float *__restrict__ part,
                                                           const int32_t *__restrict__ chunk_off, int G,
                                                           float *__restrict__ out, float *__restrict__ lse)
{
    __shared__ float red[D / 64];
    const int u = blockIdx.x / G, g = blockIdx.x - u * G, e = threadIdx.x;
    const int c0 = chunk_off[u], c1 = chunk_off[u + 1];
    // the largest running maximum: chunks spread over the threads, then one reduction
    float mm = kNone;
    for (int ch = c0 + e; ch < c1; ch += D) mm = fmaxf(mm, part[((int64_t)ch * G + g) * (D + 2)]);
    mm = wave_max(mm);
    if ((e & 63) == 0) red[e >> 6] = mm;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < D / 64; ++i) mm = fmaxf(mm, red[i]);
    // weighted sums, four chunks' loads in flight at a time; the order of the additions is fixed
    float ll = 0.f, oo = 0.f;
    int ch = c0;
    for (; ch + 4 <= c1; ch += 4) {
        float pm[4], pl[4], po[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float *src = part + ((int64_t)(ch + i) * G + g) * (D + 2);
            pm[i] = src[0];
            pl[i] = src[1];
            po[i] = src[2 + e];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float f = __builtin_amdgcn_exp2f(pm[i] - mm);
            ll = fmaf(f, pl[i], ll);
            oo = fmaf(f, po[i], oo);
        }
    }
    for (; ch < c1; ++ch) {
        const float *src = part + ((int64_t)ch * G + g) * (D + 2);
        const float f = __builtin_amdgcn_exp2f(src[0] - mm);
        ll = fmaf(f, src[1], ll);
        oo = fmaf(f, src[2 + e], oo);
    }
    out[((int64_t)u * G + g) * D + e] = ll > 0.f ? oo / ll : 0.f;
    if (lse && e == 0) lse[(int64_t)u * G + g] = ll > 0.f ? (mm + log2f(ll)) * kLn2 : -INFINITY;
}

// Any dtype, d, dv and group size.  grid: n_units * G workgroups of 256 threads; wave w takes rows w, w+4, ...;
// lane owns dims lane, lane + 64, ... of the key (dot) and of the value (accumulation).
template <typename T, int NQ>
__global__ __launch_bounds__(kDecThreads) void decode_generic_kernel(const T *__restrict__ q, const T *__restrict__ pk,
                                                                     const T *__restrict__ pv,
                                                                     const int64_t *__restrict__ head_off, int G,
                                                                     int d, int dv, int64_t rows, float scale_log2,
                                                                     float *__restrict__ out, float *__restrict__ lse)
{
    constexpr int NW = kDecThreads / 64;
    __shared__ float lds_m[NW], lds_l[NW];
    __shared__ float lds_o[NW][NQ * 64];
    const int u = blockIdx.x / G, g = blockIdx.x - u * G;
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t first = clamp_row(head_off[u], rows), len = max(clamp_row(head_off[u + 1], rows) - first, (int64_t)0);
    const T *qj = q + ((int64_t)u * G + g) * d;
    float m = kNone, l = 0.f, acc[NQ];
#pragma unroll
    for (int k = 0; k < NQ; ++k) acc[k] = 0.f;
    for (int64_t i = w; i < len; i += NW) {
        const T *kr = pk + (first + i) * d;
        float dot = 0.f;
        for (int cc = lane; cc < d; cc += 64) dot = fmaf(load_elem<T>(qj + cc), load_elem<T>(kr + cc), dot);
        const float s = wave_sum(dot) * scale_log2;
        const float mb = fmaxf(m, s), corr = __builtin_amdgcn_exp2f(m - mb), p = __builtin_amdgcn_exp2f(s - mb);
        m = mb;
        l = fmaf(l, corr, p);
        const T *vr = pv + (first + i) * dv;
#pragma unroll
        for (int k = 0; k < NQ; ++k) {
            const int cc = lane + 64 * k;
            acc[k] = fmaf(acc[k], corr, cc < dv ? p * load_elem<T>(vr + cc) : 0.f);
        }
    }
    if (lane == 0) {
        lds_m[w] = m;
        lds_l[w] = l;
    }
#pragma unroll
    for (int k = 0; k < NQ; ++k) lds_o[w][lane + 64 * k] = acc[k];
    __syncthreads();
    float mm = kNone;
    for (int i = 0; i < NW; ++i) mm = fmaxf(mm, lds_m[i]);
    float ll = 0.f;
    for (int i = 0; i < NW; ++i) ll = fmaf(__builtin_amdgcn_exp2f(lds_m[i] - mm), lds_l[i], ll);
    for (int e = threadIdx.x; e < dv; e += kDecThreads) {
        float oo = 0.f;
        for (int i = 0; i < NW; ++i) oo = fmaf(__builtin_amdgcn_exp2f(lds_m[i] - mm), lds_o[i][e], oo);
        out[((int64_t)u * G + g) * dv + e] = ll > 0.f ? oo / ll : 0.f;
    }
    if (lse && threadIdx.x == 0) lse[(int64_t)u * G + g] = ll > 0.f ? (mm + log2f(ll)) * kLn2 : -INFINITY;
}

int64_t max_chunks(int64_t n_units, int64_t rows) { return rows / kChunk + n_units; }

template <int D, bool F16>
hipError_t run_fast(const uint16_t *q, const uint16_t *pk, const uint16_t *pv, const int64_t *head_off, int n_units,
                    int G, int64_t rows, float scale_log2, float *out, float *lse, void *ws, const Prof &prof,
                    hipStream_t st)
{
    int32_t *chunk_off = (int32_t *)ws;
    float *part = (float *)((char *)ws + ((size_t)(n_units + 1) * 4 + 255) / 256 * 256);
    decode_plan_kernel<<<1, 1024, 0, st>>>(head_off, n_units, rows, chunk_off);
    const unsigned groups = (unsigned)max_chunks(n_units, rows);
    prof.begin(NKV_KERNEL_DECODE, st);
#define NKV_DEC(GG)                                                                                             \
    case GG:                                                                                                   \
        decode_chunk_kernel<D, GG, F16><<<groups, kDecThreads, 0, st>>>(q, pk, pv, head_off, chunk_off, n_units, rows, \
                                                                   scale_log2, part);                         \
        break
    switch (G) {
        NKV_DEC(1); NKV_DEC(2); NKV_DEC(3); NKV_DEC(4); NKV_DEC(5); NKV_DEC(6); NKV_DEC(7); NKV_DEC(8);
    default: return hipErrorInvalidValue;
    }
#undef NKV_DEC
    prof.end(NKV_KERNEL_DECODE, st);
    decode_combine_kernel<D><<<(unsigned)(n_units * G), D, 0, st>>>(part, chunk_off, G, out, lse);
    return hipGetLastError();
}

template <typename T>
hipError_t run_generic(const T *q, const T *pk, const T *pv, const int64_t *head_off, int n_units, int G, int d,
                       int dv, int64_t rows, float scale_log2, float *out, float *lse, const Prof &prof,
                       hipStream_t st)
{
    const unsigned groups = (unsigned)(n_units * G);
    const int nq = (dv + 63) / 64;
    prof.begin(NKV_KERNEL_DECODE, st);
#define NKV_DECG(NQ) \
    decode_generic_kernel<T, NQ><<<groups, kDecThreads, 0, st>>>(q, pk, pv, head_off, G, d, dv, rows, scale_log2, out, lse)
    if (nq <= 1) NKV_DECG(1);
    else if (nq <= 2) NKV_DECG(2);
    else if (nq <= 4) NKV_DECG(4);
    else if (nq <= 8) NKV_DECG(8);
    else NKV_DECG(16);
#undef NKV_DECG
    prof.end(NKV_KERNEL_DECODE, st);
    return hipGetLastError();
}

}  // namespace

bool decode_fast_supported(int dtype, int d, int dv, int G)
{
    return (dtype == NKV_DTYPE_BF16 || dtype == NKV_DTYPE_F16) && d == dv && (d == 64 || d == 128) && G >= 1 && G <= 8;
}

size_t decode_ws_bytes(int dtype, int d, int dv, int G, int64_t n_units, int64_t rows)
{
    if (!decode_fast_supported(dtype, d, dv, G)) return 0;
    return ((size_t)(n_units + 1) * 4 + 255) / 256 * 256 + (size_t)max_chunks(n_units, rows) * G * (d + 2) * 4;
}

hipError_t launch_decode(const void *q, const void *pk, const void *pv, const int64_t *head_off, int dtype,
                         int n_units, int G, int d, int dv, int64_t rows, double scale, float *out, float *lse,
                         void *ws, const Prof &prof, hipStream_t st)
{
    const float scale_log2 = (float)(scale * 1.4426950408889634);
    if (decode_fast_supported(dtype, d, dv, G)) {
        const uint16_t *q16 = (const uint16_t *)q, *k16 = (const uint16_t *)pk, *v16 = (const uint16_t *)pv;
        if (dtype == NKV_DTYPE_F16) {
            if (d == 128) return run_fast<128, true>(q16, k16, v16, head_off, n_units, G, rows, scale_log2, out, lse, ws, prof, st);
            return run_fast<64, true>(q16, k16, v16, head_off, n_units, G, rows, scale_log2, out, lse, ws, prof, st);
        }
        if (d == 128) return run_fast<128, false>(q16, k16, v16, head_off, n_units, G, rows, scale_log2, out, lse, ws, prof, st);
        return run_fast<64, false>(q16, k16, v16, head_off, n_units, G, rows, scale_log2, out, lse, ws, prof, st);
    }
    if (dtype == NKV_DTYPE_F32)
        return run_generic<float>((const float *)q, (const float *)pk, (const float *)pv, head_off, n_units, G, d, dv,
                                  rows, scale_log2, out, lse, prof, st);
    if (dtype == NKV_DTYPE_F16)
        return run_generic<f16_t>((const f16_t *)q, (const f16_t *)pk, (const f16_t *)pv, head_off, n_units, G, d, dv,
                                  rows, scale_log2, out, lse, prof, st);
    return run_generic<uint16_t>((const uint16_t *)q, (const uint16_t *)pk, (const uint16_t *)pv, head_off, n_units, G,
                                 d, dv, rows, scale_log2, out, lse, prof, st);
}

}  // namespace nkv
