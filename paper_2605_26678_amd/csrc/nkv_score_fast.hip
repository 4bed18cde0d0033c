// Streaming scoring kernels for bf16 keys, head dim 64 or 128, window 64, episodic block size <= 256
// (paper Sections 2.1-2.3: normalised keys, stable / episodic / current anchors, cosine anomalies).
//
// Work decomposition.  One workgroup per (layer, head, episodic block).  The block (<= 256 tokens) is cut
// into 64-token chunks, one wavefront per chunk, plus one "halo" wavefront for the 64 tokens in front of the
// block (the current-memory window of the block's first tokens reaches back that far).  Inside a wavefront
// a key row is spread over LPR = D/8 lanes (16 bytes = 8 bf16 each), so a 64-lane load instruction fetches
// 64/LPR whole rows; lane (g, c) owns dims 8c..8c+7 of the TPT = LPR consecutive tokens g*TPT .. g*TPT+TPT-1
// of the chunk.  The chunk stays in registers as packed bf16 from the first touch to the last.
//
// Per chunk:  1/||k|| per token (sum of squares reduced over the LPR lanes with DPP);  the partial sums
// T[g] = sum of k_hat over the sub-group's tokens.  Partial sums go through LDS: they give the chunk and
// block totals (episodic anchor; the block totals are also the partial sums of the stable anchor) and the
// window sum in front of every sub-group.  The window sum then slides token by token,
//     W_i = W_{i-1} - k_hat_{i-64} + k_hat_i,
// re-seeded exactly at every sub-group boundary (every TPT tokens) from the partial sums, so no long
// running sum and no cancellation beyond TPT steps.  k_hat_{i-64} sits at the same lane position of the
// previous chunk, which the wavefront re-loads (an L1/L2 hit: the neighbouring wavefront has just read it).
// Cosines do not depend on the anchor's length, so sums stand in for means everywhere.
//
// The stable anchor needs every key of the prompt before the first a_s can be computed.  Here that is a
// second kernel (a_s only) that re-reads the keys.
#include "nkv_device.h"

namespace nkv {
namespace {

template <int CTRL> __device__ __forceinline__ float dpp_mov(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}

// Sum over the LPR lanes that share a key row; every lane of the group receives the total.
template <int LPR> __device__ __forceinline__ float row_sum(float v)
{
    v += dpp_mov<0xB1>(v);                       // quad_perm [1,0,3,2]
    v += dpp_mov<0x4E>(v);                       // quad_perm [2,3,0,1]
    v += dpp_mov<0x141>(v);                      // row_half_mirror: the other quad of the 8-lane half
    if (LPR == 16) v += dpp_mov<0x140>(v);       // row_mirror: the other half of the 16-lane row
    return v;
}

__device__ __forceinline__ void unpack8(const uint4 &r, float k[8])
{
    k[0] = __uint_as_float(r.x << 16); k[1] = __uint_as_float(r.x & 0xffff0000u);
    k[2] = __uint_as_float(r.y << 16); k[3] = __uint_as_float(r.y & 0xffff0000u);
    k[4] = __uint_as_float(r.z << 16); k[5] = __uint_as_float(r.z & 0xffff0000u);
    k[6] = __uint_as_float(r.w << 16); k[7] = __uint_as_float(r.w & 0xffff0000u);
}

// 1 / max(||k||, 1e-12) from the sum of squares.
__device__ __forceinline__ float inv_norm(float ss) { return ss < 1e-24f ? 1e12f : __builtin_amdgcn_rsqf(ss); }

__device__ __forceinline__ float neg_cos(float dot_scaled, float knorm, float anchor_sq)
{
    return -dot_scaled / (fmaxf(knorm, kEps) * fmaxf(sqrtf(anchor_sq), kEps));
}

constexpr int kMaxChunks = 4;                    // data chunks per block: block size <= 256

// grid (blocks per head, L*H); blockDim = 64 * (chunks + 1)
template <int D>
__global__ __launch_bounds__(64 * (kMaxChunks + 1)) void scan_kernel(const uint16_t *__restrict__ keys,
                                                                     PromptTab tab, float *__restrict__ a_raw,
                                                                     float *__restrict__ bsum, int64_t rows)
{
    constexpr int LPR = D / 8, SG = 64 / LPR, TPT = LPR;
    __shared__ float lds_rn[kMaxChunks + 1][64];
    __shared__ float lds_T[kMaxChunks + 1][SG][D];
    __shared__ float lds_C[kMaxChunks + 1][D];

    const int blk = blockIdx.x, lh = blockIdx.y;
    const int p = prompt_of_block(tab, blk);
    const int b = tab.b[p];
    const int N = tab.tok_off[p + 1] - tab.tok_off[p];
    const int blk_lo = (blk - tab.blk_off[p]) * b;
    const int blk_hi = min(blk_lo + b, N);
    const int64_t row0 = (int64_t)lh * tab.T + tab.tok_off[p];        // row of the prompt's token 0
    const uint4 *kbase = reinterpret_cast<const uint4 *>(keys) + row0 * LPR;

    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int g = lane / LPR, c = lane % LPR;
    // wave 0: halo chunk [blk_lo-64, blk_lo); wave w >= 1: data chunk [blk_lo + 64(w-1), ...) cut at blk_hi
    const int t0 = blk_lo + 64 * (w - 1) + g * TPT;                   // first token of this lane
    const int lim = w == 0 ? blk_lo : blk_hi;                         // tokens below lim (and >= 0) exist
    const bool active = w >= 1 && blk_lo + 64 * (w - 1) < blk_hi;     // data wave with at least one token

    // ---- first touch: load the chunk, 1/||k||, partial sums ----
    uint4 raw[TPT];
    float rn[TPT], T[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) T[e] = 0.f;
#pragma unroll
    for (int j = 0; j < TPT; ++j) {
        const int t = t0 + j;
        raw[j] = (t >= 0 && t < lim) ? kbase[(int64_t)t * LPR + c] : make_uint4(0u, 0u, 0u, 0u);
    }
#pragma unroll
    for (int j = 0; j < TPT; ++j) {
        float k[8];
        unpack8(raw[j], k);
        float ss = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) ss = fmaf(k[e], k[e], ss);
        ss = row_sum<LPR>(ss);
        const int t = t0 + j;
        rn[j] = (t >= 0 && t < lim) ? inv_norm(ss) : 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) T[e] = fmaf(rn[j], k[e], T[e]);
    }
    {
        float4 *dst = reinterpret_cast<float4 *>(&lds_T[w][g][c * 8]);
        dst[0] = make_float4(T[0], T[1], T[2], T[3]);
        dst[1] = make_float4(T[4], T[5], T[6], T[7]);
        // lane (g, c) publishes the norm of token g*TPT + c of its chunk (TPT == LPR)
        float mine = 0.f;
#pragma unroll
        for (int j = 0; j < TPT; ++j) mine = (j == c) ? rn[j] : mine;
        lds_rn[w][lane] = mine;
    }
    __syncthreads();

    // ---- chunk totals; window sum in front of this lane's first token ----
    float W[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) W[e] = 0.f;
    if (w >= 1) {
        float own[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) own[e] = 0.f;
#pragma unroll
        for (int gg = 0; gg < SG; ++gg) {
            const float4 *cur = reinterpret_cast<const float4 *>(&lds_T[w][gg][c * 8]);
            const float4 *prv = reinterpret_cast<const float4 *>(&lds_T[w - 1][gg][c * 8]);
            const float4 a0 = cur[0], a1 = cur[1], b0 = prv[0], b1 = prv[1];
            const float cv[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
            const float pv[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                own[e] += cv[e];
                // tokens [i-63, i] for i = first token - 1: the previous chunk from sub-group g on,
                // this chunk up to sub-group g-1
                W[e] += gg >= g ? pv[e] : cv[e];
            }
        }
        if (g == 0) {
            float4 *dst = reinterpret_cast<float4 *>(&lds_C[w][c * 8]);
            dst[0] = make_float4(own[0], own[1], own[2], own[3]);
            dst[1] = make_float4(own[4], own[5], own[6], own[7]);
        }
    }
    __syncthreads();
    if (!active) return;

    // ---- block total = episodic anchor (up to length) ----
    float Bs[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) Bs[e] = 0.f;
    const int nch = (blk_hi - blk_lo + 63) >> 6;
    for (int ww = 1; ww <= nch; ++ww) {
        const float4 *src = reinterpret_cast<const float4 *>(&lds_C[ww][c * 8]);
        const float4 a0 = src[0], a1 = src[1];
        Bs[0] += a0.x; Bs[1] += a0.y; Bs[2] += a0.z; Bs[3] += a0.w;
        Bs[4] += a1.x; Bs[5] += a1.y; Bs[6] += a1.z; Bs[7] += a1.w;
    }
    float bsq = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) bsq = fmaf(Bs[e], Bs[e], bsq);
    bsq = row_sum<LPR>(bsq);
    if (w == 1 && g == 0) {
        float4 *dst = reinterpret_cast<float4 *>(bsum + ((int64_t)lh * tab.blk_off[tab.n] + blk) * D + c * 8);
        dst[0] = make_float4(Bs[0], Bs[1], Bs[2], Bs[3]);
        dst[1] = make_float4(Bs[4], Bs[5], Bs[6], Bs[7]);
    }

    // ---- slide the window over this lane's tokens; episodic and current anomalies ----
    float out_e = 0.f, out_c = 0.f;
#pragma unroll
    for (int j = 0; j < TPT; ++j) {
        const int t = t0 + j;
        const int tp = t - 64;                                      // the token that leaves the window
        const uint4 praw = tp >= 0 ? kbase[(int64_t)tp * LPR + c] : make_uint4(0u, 0u, 0u, 0u);
        const float rnp = lds_rn[w - 1][g * TPT + j];               // 0 where the token does not exist
        float kp[8], k[8];
        unpack8(praw, kp);
        unpack8(raw[j], k);
        float wd = 0.f, wn = 0.f, bd = 0.f, ss = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            W[e] = fmaf(-rnp, kp[e], W[e]);
            W[e] = fmaf(rn[j], k[e], W[e]);
            wd = fmaf(k[e], W[e], wd);
            wn = fmaf(W[e], W[e], wn);
            bd = fmaf(k[e], Bs[e], bd);
            ss = fmaf(k[e], k[e], ss);
        }
        wd = row_sum<LPR>(wd);
        wn = row_sum<LPR>(wn);
        bd = row_sum<LPR>(bd);
        ss = row_sum<LPR>(ss);
        const float knorm = sqrtf(ss) * rn[j];                      // ||k_hat||: 1 unless the key is ~0
        const float ae = neg_cos(rn[j] * bd, knorm, bsq);
        const float ac = neg_cos(rn[j] * wd, knorm, wn);
        out_e = (j == c) ? ae : out_e;
        out_c = (j == c) ? ac : out_c;
    }
    const int tok = blk_lo + 64 * (w - 1) + lane;                   // lane (g, c) reports token g*TPT + c
    if (tok < blk_hi) {
        a_raw[rows + row0 + tok] = out_e;
        a_raw[2 * rows + row0 + tok] = out_c;
    }
}

// grid (prompts, L*H): stable anchor (up to length) = sum of the prompt's block totals, in block order
template <int D>
__global__ __launch_bounds__(D) void ssum_kernel(const float *__restrict__ bsum, PromptTab tab, float *__restrict__ ssum)
{
    const int p = blockIdx.x, lh = blockIdx.y, cdim = threadIdx.x;
    const int nblk = tab.blk_off[tab.n];
    float s = 0.f;
    for (int blk = tab.blk_off[p]; blk < tab.blk_off[p + 1]; ++blk) s += bsum[((int64_t)lh * nblk + blk) * D + cdim];
    ssum[((int64_t)lh * tab.n + p) * D + cdim] = s;
}

// Stable anomaly a_s: second touch of the keys.  grid (ceil(T/256), L*H), 256 threads = 4 chunks of 64 tokens.
template <int D>
__global__ __launch_bounds__(256) void stable_kernel(const uint16_t *__restrict__ keys, PromptTab tab,
                                                     const float *__restrict__ ssum, float *__restrict__ a_raw)
{
    constexpr int LPR = D / 8, TPT = LPR;
    const int lh = blockIdx.y;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int g = lane / LPR, c = lane % LPR;
    const int tg0 = blockIdx.x * 256 + wv * 64;                      // first global token of this wave
    if (tg0 >= tab.T) return;
    const uint4 *kbase = reinterpret_cast<const uint4 *>(keys) + (int64_t)lh * tab.T * LPR;
    float out = 0.f;
#pragma unroll
    for (int j = 0; j < TPT; ++j) {
        const int tg = tg0 + g * TPT + j;
        const bool ok = tg < tab.T;
        const uint4 raw = ok ? kbase[(int64_t)tg * LPR + c] : make_uint4(0u, 0u, 0u, 0u);
        const int p = prompt_of_token(tab, ok ? tg : tab.T - 1);
        const float4 *S = reinterpret_cast<const float4 *>(ssum + ((int64_t)lh * tab.n + p) * D + c * 8);
        const float4 s0 = S[0], s1 = S[1];
        const float sv[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
        float k[8];
        unpack8(raw, k);
        float ss = 0.f, sd = 0.f, sq = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            ss = fmaf(k[e], k[e], ss);
            sd = fmaf(k[e], sv[e], sd);
            sq = fmaf(sv[e], sv[e], sq);
        }
        ss = row_sum<LPR>(ss);
        sd = row_sum<LPR>(sd);
        sq = row_sum<LPR>(sq);
        const float rn = inv_norm(ss);
        const float as = neg_cos(rn * sd, sqrtf(ss) * rn, sq);
        out = (j == c) ? as : out;
    }
    const int tok = tg0 + lane;
    if (tok < tab.T) a_raw[(int64_t)lh * tab.T + tok] = out;
}

template <int D>
hipError_t run(const uint16_t *keys, int LH, const PromptTab &tab, float *a_raw, float *bsum, float *ssum,
               const Prof &prof, hipStream_t st)
{
    int bmax = 0;
    for (int p = 0; p < tab.n; ++p) bmax = tab.b[p] > bmax ? tab.b[p] : bmax;
    const int waves = (bmax + 63) / 64 + 1;
    const int64_t rows = (int64_t)LH * tab.T;
    prof.begin(NKV_KERNEL_SCAN, st);
    scan_kernel<D><<<dim3(tab.blk_off[tab.n], LH), 64 * waves, 0, st>>>(keys, tab, a_raw, bsum, rows);
    prof.end(NKV_KERNEL_SCAN, st);
    ssum_kernel<D><<<dim3(tab.n, LH), D, 0, st>>>(bsum, tab, ssum);
    stable_kernel<D><<<dim3((tab.T + 255) / 256, LH), 256, 0, st>>>(keys, tab, ssum, a_raw);
    return hipGetLastError();
}

}  // namespace

bool fast_score_supported(int dtype, int d, int window, const PromptTab &tab)
{
    if (dtype != NKV_DTYPE_BF16 || (d != 64 && d != 128) || window != 64) return false;
    for (int p = 0; p < tab.n; ++p)
        if (tab.b[p] > 64 * kMaxChunks) return false;
    return true;
}

size_t fast_score_ws_floats(int, int, const PromptTab &) { return 0; }

hipError_t launch_score_fast(const void *keys, int LH, int d, const PromptTab &tab, float *a_raw, float *bsum,
                             float *ssum, const Prof &prof, hipStream_t st)
{
    if (d == 128) return run<128>((const uint16_t *)keys, LH, tab, a_raw, bsum, ssum, prof, st);
    return run<64>((const uint16_t *)keys, LH, tab, a_raw, bsum, ssum, prof, st);
}

}  // namespace nkv
