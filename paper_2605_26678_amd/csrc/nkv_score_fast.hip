// Streaming scoring kernel for bf16 keys, head dim 64 or 128, window 64, episodic block size <= 256
// (paper Sections 2.1-2.3: normalised keys, stable / episodic / current anchors, cosine anomalies).
//
// Work decomposition.  One workgroup per (layer, head, episodic block).  The block (<= 256 tokens) is cut
// into 64-token chunks, one wavefront per chunk.  Inside a wavefront a key row is spread over LPR = D/8
// lanes (16 bytes = 8 bf16 each), so one 64-lane load instruction fetches 64/LPR whole rows; lane (g, c)
// owns dims 8c..8c+7 of the TPT = LPR consecutive tokens g*TPT .. g*TPT+TPT-1 of the chunk.  The chunk
// stays in registers as packed bf16 from the first touch to the last.  The 64 "halo" tokens in front of
// the block (the current-memory window of the block's first tokens reaches back that far) are split
// evenly over the wavefronts, which only need their norms and partial sums.
//
// Per chunk: 1/||k|| per token (sum of squares reduced over the LPR lanes with DPP) and the partial sums
// T[g] = sum of k_hat over the sub-group's tokens.  Partial sums go through LDS: they give the chunk and
// block totals (episodic anchor; the block totals are also the partial sums of the stable anchor) and the
// window sum in front of every sub-group.  The window sum then slides token by token,
//     W_i = W_{i-1} - k_hat_{i-64} + k_hat_i,
// re-seeded exactly at every sub-group boundary (every TPT tokens) from the partial sums, so no long
// running sum and no cancellation beyond TPT steps.  k_hat_{i-64} sits at the same lane position of the
// previous chunk, which the wavefront re-loads (an L1/L2 hit: a neighbouring wavefront has just read it).
// Cosines do not depend on the anchor's length, so sums stand in for means everywhere.
//
// The stable anchor needs every key of the prompt before the first a_s can be computed.  Two ways:
//   fused   : workgroups take tickets in start order; all blocks of a (layer, head, prompt) unit have
//             consecutive tickets.  Each workgroup publishes its block total and bumps the unit's arrival
//             counter; the last one to arrive adds the block totals up in block order (deterministic),
//             publishes the sum and raises the unit's flag; the others wait for the flag with their chunk
//             still in registers, then compute a_s.  A waiting workgroup only ever waits for workgroups
//             with tickets of the same unit, all of which have started or can start as long as the chip
//             can hold one unit's workgroups at once -- the host checks that before choosing this path.
//             Waits are bounded; a timeout is recorded in the sync area and the kernel still ends.
//   2-pass  : stable_kernel re-reads the keys after ssum_kernel (any prompt length).
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

using u32x4 = unsigned int __attribute__((ext_vector_type(4)));

// 16-byte load through a buffer descriptor: the address is one 32-bit byte offset per lane plus an
// immediate, and an offset outside [0, num_records) (tokens before the prompt or past its end) reads zeros.
__device__ __forceinline__ u32x4 row_load(__amdgpu_buffer_rsrc_t rsrc, int byte_off)
{
    return __builtin_amdgcn_raw_buffer_load_b128(rsrc, byte_off, 0, 0);
}

__device__ __forceinline__ void unpack8(const u32x4 &r, float k[8])
{
    k[0] = __uint_as_float(r.x << 16); k[1] = __uint_as_float(r.x & 0xffff0000u);
    k[2] = __uint_as_float(r.y << 16); k[3] = __uint_as_float(r.y & 0xffff0000u);
    k[4] = __uint_as_float(r.z << 16); k[5] = __uint_as_float(r.z & 0xffff0000u);
    k[6] = __uint_as_float(r.w << 16); k[7] = __uint_as_float(r.w & 0xffff0000u);
}

// Makes the compiler forget what it knows about a packed row, so that the unpacked floats of one phase
// are not kept alive (8 registers per token) for the next phase; costs no instruction.
__device__ __forceinline__ void forget(u32x4 &r) { asm volatile("" : "+v"(r.x), "+v"(r.y), "+v"(r.z), "+v"(r.w)); }

__device__ __forceinline__ void load8(const float *src, float v[8])
{
    const float4 a = reinterpret_cast<const float4 *>(src)[0], b = reinterpret_cast<const float4 *>(src)[1];
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}

__device__ __forceinline__ void store8(float *dst, const float v[8])
{
    reinterpret_cast<float4 *>(dst)[0] = make_float4(v[0], v[1], v[2], v[3]);
    reinterpret_cast<float4 *>(dst)[1] = make_float4(v[4], v[5], v[6], v[7]);
}

// 1 / max(||k||, 1e-12) from the sum of squares.
__device__ __forceinline__ float inv_norm(float ss) { return ss < 1e-24f ? 1e12f : __builtin_amdgcn_rsqf(ss); }

__device__ __forceinline__ float neg_cos(float dot_scaled, float knorm, float anchor_sq)
{
    return -dot_scaled / (fmaxf(knorm, kEps) * fmaxf(sqrtf(anchor_sq), kEps));
}

// Accesses other workgroups must see / have written: performed at agent (device) scope.
__device__ __forceinline__ void agent_store(float *p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float agent_load(const float *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// 16-byte agent-scope accesses through a buffer descriptor (cache policy bit 4 = sc1 on gfx94x/gfx950).
__device__ __forceinline__ float4 agent_load16(__amdgpu_buffer_rsrc_t rsrc, int byte_off)
{
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, byte_off, 0, 16);
    return make_float4(__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w));
}
__device__ __forceinline__ void agent_store16(__amdgpu_buffer_rsrc_t rsrc, int byte_off, float4 f)
{
    const u32x4 v = {__float_as_uint(f.x), __float_as_uint(f.y), __float_as_uint(f.z), __float_as_uint(f.w)};
    __builtin_amdgcn_raw_buffer_store_b128(v, rsrc, byte_off, 0, 16);
}

// Waits until every memory access this wave has issued so far has completed; also keeps the compiler from
// moving memory accesses across it.  Agent-scope stores are visible to the whole device once complete, so
// "agent_store ...; wait_own_accesses(); agent-scope atomic" publishes data without an L2 write-back.
__device__ __forceinline__ void wait_own_accesses() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

constexpr int kMaxChunks = 4;                    // chunks per block: block size <= 256
constexpr uint32_t kSpinLimit = 1u << 22;        // ~1 s of polling before a wait gives up

constexpr int kUnitStride = 64;                  // words between the counters of two units

// Sync area of the fused path (all zero before the launch).
struct ScanSync {
    uint32_t ticket;
    uint32_t timeouts;
    uint32_t pad[62];
    uint32_t unit[1];                            // [units][kUnitStride]: arrivals, flag, padding to 256 bytes
};

// NW wavefronts = chunks per block.  grid: one workgroup per (layer*head, block); 1-D when FUSED.
template <int D, int NW, bool FUSED>
__global__ __launch_bounds__(64 * NW, NW == 4 ? 3 : 4)
void scan_kernel(const uint16_t *__restrict__ keys, PromptTab tab, float *__restrict__ a_raw,
                 float *__restrict__ bsum, float *__restrict__ ssum, ScanSync *__restrict__ sync, int64_t rows)
{
    constexpr int LPR = D / 8, SG = 64 / LPR, TPT = LPR;
    constexpr int HT = (TPT + NW - 1) / NW;                           // halo tokens per lane
    __shared__ float lds_rn[NW + 1][64];                              // [0]: halo chunk, [1 + w]: chunk w
    __shared__ float lds_T[NW][SG][D];                                // partial sums of the chunks
    __shared__ float lds_Th[NW][SG][D];                               // partial sums of the halo chunk
    __shared__ float lds_C[NW][D];                                    // chunk totals
    __shared__ int s_ticket, s_last;

    const int nblk = tab.blk_off[tab.n];
    int wg = blockIdx.x;
    if (FUSED) {
        if (threadIdx.x == 0) s_ticket = (int)atomicAdd(&sync->ticket, 1u);
        __syncthreads();
        wg = s_ticket;
    }
    const int lh = wg / nblk, blk = wg - lh * nblk;
    const int p = prompt_of_block(tab, blk);
    const int b = tab.b[p];
    const int N = tab.tok_off[p + 1] - tab.tok_off[p];
    const int blk_lo = (blk - tab.blk_off[p]) * b;
    const int blk_hi = min(blk_lo + b, N);
    const int64_t row0 = (int64_t)lh * tab.T + tab.tok_off[p];        // row of the prompt's token 0

    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int g = lane / LPR, c = lane % LPR;
    const int t0 = blk_lo + 64 * w + g * TPT;                         // first token of this lane

    // ---- first touch: the chunk and this wave's share of the halo ----
    // Rows are addressed relative to the prompt's first row; rows outside the prompt read as zeros, rows of
    // the prompt that lie outside this block get weight 0 below.
    constexpr int kRowBytes = D * 2;
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(keys) + row0 * D, 0, N * kRowBytes, 0x00020000);
    const int lane_off = t0 * kRowBytes + c * 16;
    u32x4 raw[TPT], hraw[HT];
#pragma unroll
    for (int j = 0; j < TPT; ++j) raw[j] = row_load(rsrc, lane_off + j * kRowBytes);
    const int halo_off = (blk_lo - 64 + g * TPT + HT * w) * kRowBytes + c * 16;
#pragma unroll
    for (int jj = 0; jj < HT; ++jj) hraw[jj] = row_load(rsrc, halo_off + jj * kRowBytes);
    float rn[TPT], T[8], kn_mine = 1.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) T[e] = 0.f;
#pragma unroll
    for (int j = 0; j < TPT; ++j) {
        float k[8];
        unpack8(raw[j], k);
        float ss = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) ss = fmaf(k[e], k[e], ss);
        ss = row_sum<LPR>(ss);
        rn[j] = (t0 + j < blk_hi) ? inv_norm(ss) : 0.f;
        if (j == c) kn_mine = ss < 1e-24f ? sqrtf(ss) * 1e12f : 1.f;   // ||k_hat|| of this lane's own token
#pragma unroll
        for (int e = 0; e < 8; ++e) T[e] = fmaf(rn[j], k[e], T[e]);
        if ((j & 3) == 3) __builtin_amdgcn_sched_barrier(0);          // bound the unpacked temporaries
    }
    store8(&lds_T[w][g][c * 8], T);
    {
        float mine = 0.f;                                             // lane (g, c) owns token g*TPT + c
#pragma unroll
        for (int j = 0; j < TPT; ++j) mine = (j == c) ? rn[j] : mine;
        lds_rn[1 + w][lane] = mine;
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) T[e] = 0.f;
#pragma unroll
    for (int jj = 0; jj < HT; ++jj) {
        float k[8];
        unpack8(hraw[jj], k);
        float ss = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) ss = fmaf(k[e], k[e], ss);
        ss = row_sum<LPR>(ss);
        const int q = HT * w + jj;
        const bool ok = q < TPT && blk_lo - 64 + g * TPT + q >= 0;
        const float r = ok ? inv_norm(ss) : 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) T[e] = fmaf(r, k[e], T[e]);
        if (c == jj && q < TPT) lds_rn[0][g * TPT + q] = r;
        if ((jj & 3) == 3) __builtin_amdgcn_sched_barrier(0);
    }
    store8(&lds_Th[w][g][c * 8], T);
    __syncthreads();

    // ---- chunk totals; window sum in front of this lane's first token ----
    float W[8];
    {
        float own[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) { W[e] = 0.f; own[e] = 0.f; }
#pragma unroll
        for (int gg = 0; gg < SG; ++gg) {
            float cv[8], pv[8];
            load8(&lds_T[w][gg][c * 8], cv);
            if (w == 0) {
#pragma unroll
                for (int e = 0; e < 8; ++e) pv[e] = 0.f;
                if (gg >= g) {
#pragma unroll
                    for (int ww = 0; ww < NW; ++ww) {
                        float hv[8];
                        load8(&lds_Th[ww][gg][c * 8], hv);
#pragma unroll
                        for (int e = 0; e < 8; ++e) pv[e] += hv[e];
                    }
                }
            } else {
                load8(&lds_T[w - 1][gg][c * 8], pv);
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                own[e] += cv[e];
                // tokens [i-63, i] for i = first token - 1: the previous chunk from sub-group g on,
                // this chunk up to sub-group g-1
                W[e] += gg >= g ? pv[e] : cv[e];
            }
            __builtin_amdgcn_sched_barrier(0);                        // one sub-group's partials at a time
        }
        if (g == 0) store8(&lds_C[w][c * 8], own);
    }
    __syncthreads();
    // A wave whose chunk lies past the end of the block runs along on zero-weight tokens and stores nothing.

    // ---- block total = episodic anchor (up to length) ----
    float Bs[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) Bs[e] = 0.f;
    const int nch = (blk_hi - blk_lo + 63) >> 6;
#pragma unroll
    for (int ww = 0; ww < NW; ++ww) {
        if (ww < nch) {
            float cv[8];
            load8(&lds_C[ww][c * 8], cv);
#pragma unroll
            for (int e = 0; e < 8; ++e) Bs[e] += cv[e];
        }
    }
    float bsq = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) bsq = fmaf(Bs[e], Bs[e], bsq);
    bsq = row_sum<LPR>(bsq);
    float *bsum_unit = bsum + ((int64_t)lh * nblk + tab.blk_off[p]) * D;      // block totals of this unit
    const int ublk = blk - tab.blk_off[p], unblk = tab.blk_off[p + 1] - tab.blk_off[p];
    // Everything other workgroups read (block totals, the unit's sum, counters) is written and read with
    // agent-scope accesses, which go to the level of the memory hierarchy all compute units share; ordering
    // then only needs this wave's own stores to have completed, not a write-back of the whole L2.
    uint32_t *ucnt = FUSED ? &sync->unit[kUnitStride * ((int64_t)lh * tab.n + p)] : nullptr;
    if (w == 0) {
        if (g == 0) {
#pragma unroll
            for (int e = 0; e < 8; ++e) agent_store(bsum_unit + (int64_t)ublk * D + c * 8 + e, Bs[e]);
        }
        if (FUSED) {
            wait_own_accesses();
            if (lane == 0) {
                const uint32_t arrived = __hip_atomic_fetch_add(ucnt, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                s_last = arrived == (uint32_t)unblk - 1u ? 1 : 0;
            }
        }
    }


    // ---- stable anchor: the workgroup that completes the unit adds the block totals up right away ----
    // (before its own window loop, so that the sum is ready long before anybody needs it)
    float *S_unit = ssum + ((int64_t)lh * tab.n + p) * D;
    const __amdgpu_buffer_rsrc_t srs = __builtin_amdgcn_make_buffer_rsrc(S_unit, 0, D * 4, 0x00020000);
    if (FUSED) __syncthreads();                                       // s_last is known; lds_T is free again
    if (FUSED && s_last) {                                            // uniform over the workgroup
        // thread = (slice, 4 dims): slice s adds blocks s, s + NS, s + 2 NS, ... with several loads in
        // flight; the slices are then added in order.  The order depends on the shape only.
        constexpr int VPR = D / 4, NS = 64 * NW / VPR;
        const __amdgpu_buffer_rsrc_t brs = __builtin_amdgcn_make_buffer_rsrc(bsum_unit, 0, unblk * D * 4, 0x00020000);
        const int vec = threadIdx.x % VPR, slice = threadIdx.x / VPR;
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int bb = slice; bb < unblk; bb += 4 * NS) {
            float4 v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)                               // blocks past the end read as zeros
                v[i] = agent_load16(brs, (bb + i * NS) * D * 4 + vec * 16);
#pragma unroll
            for (int i = 0; i < 4; ++i) { acc.x += v[i].x; acc.y += v[i].y; acc.z += v[i].z; acc.w += v[i].w; }
        }
        float *part = &lds_T[0][0][0];                                // NS * D floats fit (see the static_assert)
        static_assert(NS * D <= NW * SG * D, "partial sums of the unit do not fit the LDS scratch");
        reinterpret_cast<float4 *>(part)[slice * VPR + vec] = acc;
        __syncthreads();
        if (threadIdx.x < VPR) {
            float4 tot = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int sl = 0; sl < NS; ++sl) {
                const float4 v = reinterpret_cast<const float4 *>(part)[sl * VPR + vec];
                tot.x += v.x; tot.y += v.y; tot.z += v.z; tot.w += v.w;
            }
            agent_store16(srs, vec * 16, tot);
            wait_own_accesses();
            if (threadIdx.x == 0) __hip_atomic_store(ucnt + 1, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }

    // ---- slide the window over this lane's tokens; episodic and current dots ----
    float wd_m = 0.f, wn_m = 1.f, bd_m = 0.f, rn_m = 0.f;
    constexpr int GR = 4;                                             // tokens per software-pipeline stage
#pragma unroll
    for (int j = 0; j < TPT; ++j) forget(raw[j]);
    u32x4 pnext[GR];
#pragma unroll
    for (int i = 0; i < GR; ++i) pnext[i] = row_load(rsrc, lane_off + (i - 64) * kRowBytes);
#pragma unroll
    for (int j0 = 0; j0 < TPT; j0 += GR) {
        u32x4 pcur[GR];
#pragma unroll
        for (int i = 0; i < GR; ++i) pcur[i] = pnext[i];
        if (j0 + GR < TPT) {                                          // re-load the next stage's leaving tokens
#pragma unroll
            for (int i = 0; i < GR; ++i) pnext[i] = row_load(rsrc, lane_off + (j0 + GR + i - 64) * kRowBytes);
        }
#pragma unroll
        for (int i = 0; i < GR; ++i) {
            const int j = j0 + i;
            const float rnp = lds_rn[w][g * TPT + j];                 // 0 where the leaving token does not exist
            float kp[8], k[8];
            unpack8(pcur[i], kp);
            unpack8(raw[j], k);
            float wd = 0.f, wn = 0.f, bd = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                W[e] = fmaf(-rnp, kp[e], W[e]);
                W[e] = fmaf(rn[j], k[e], W[e]);
                wd = fmaf(k[e], W[e], wd);
                wn = fmaf(W[e], W[e], wn);
                bd = fmaf(k[e], Bs[e], bd);
            }
            wd = row_sum<LPR>(wd);
            wn = row_sum<LPR>(wn);
            bd = row_sum<LPR>(bd);
            if (j == c) { wd_m = wd; wn_m = wn; bd_m = bd; rn_m = rn[j]; }
        }
        __builtin_amdgcn_sched_barrier(0);                            // one stage at a time
    }
    const int tok = blk_lo + 64 * w + lane;                           // lane (g, c) reports token g*TPT + c
    if (tok < blk_hi) {
        a_raw[rows + row0 + tok] = neg_cos(rn_m * bd_m, kn_mine, bsq);
        a_raw[2 * rows + row0 + tok] = neg_cos(rn_m * wd_m, kn_mine, wn_m);
    }
    if (!FUSED) return;

    // ---- stable anomaly: wait for the unit's sum (normally long since there), one more dot per token ----
    if (w == 0) {                                                     // one wave polls, the others sit at the barrier
        uint32_t spins = 0;
        while (__hip_atomic_load(ucnt + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u) {
            if (++spins > kSpinLimit) {
                if (lane == 0) atomicAdd(&sync->timeouts, 1u);
                break;
            }
            __builtin_amdgcn_s_sleep(16);
        }
    }
    __syncthreads();
    float S[8];
    {
        const float4 s0 = agent_load16(srs, c * 32), s1 = agent_load16(srs, c * 32 + 16);
        S[0] = s0.x; S[1] = s0.y; S[2] = s0.z; S[3] = s0.w; S[4] = s1.x; S[5] = s1.y; S[6] = s1.z; S[7] = s1.w;
    }
    float ssq = 0.f, sd_m = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) ssq = fmaf(S[e], S[e], ssq);
    ssq = row_sum<LPR>(ssq);
#pragma unroll
    for (int j = 0; j < TPT; ++j) forget(raw[j]);
#pragma unroll
    for (int j = 0; j < TPT; ++j) {
        float k[8];
        unpack8(raw[j], k);
        float sd = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) sd = fmaf(k[e], S[e], sd);
        sd = row_sum<LPR>(sd);
        if (j == c) sd_m = sd;
        if ((j & 3) == 3) __builtin_amdgcn_sched_barrier(0);
    }
    if (tok < blk_hi) a_raw[row0 + tok] = neg_cos(rn_m * sd_m, kn_mine, ssq);
}

__global__ void zero_kernel(uint32_t *p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
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

// Stable anomaly a_s by a second touch of the keys.  grid (ceil(T/256), L*H), 4 waves of 64 tokens.
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
    float sd_m = 0.f, ss_m = 0.f, sq_m = 1.f;
#pragma unroll
    for (int j = 0; j < TPT; ++j) {
        const int tg = tg0 + g * TPT + j;
        const bool ok = tg < tab.T;
        const uint4 r4 = ok ? kbase[(int64_t)tg * LPR + c] : make_uint4(0u, 0u, 0u, 0u);
        const u32x4 raw = {r4.x, r4.y, r4.z, r4.w};
        const int p = prompt_of_token(tab, ok ? tg : tab.T - 1);
        float sv[8], k[8];
        load8(ssum + ((int64_t)lh * tab.n + p) * D + c * 8, sv);
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
        if (j == c) { sd_m = sd; ss_m = ss; sq_m = sq; }
    }
    const int tok = tg0 + lane;
    if (tok < tab.T) {
        const float rn = inv_norm(ss_m);
        a_raw[(int64_t)lh * tab.T + tok] = neg_cos(rn * sd_m, sqrtf(ss_m) * rn, sq_m);
    }
}

template <int D, int NW, bool FUSED>
void launch_scan(const uint16_t *keys, int LH, const PromptTab &tab, float *a_raw, float *bsum, float *ssum,
                 ScanSync *sync, hipStream_t st)
{
    const int64_t rows = (int64_t)LH * tab.T;
    scan_kernel<D, NW, FUSED><<<(unsigned)(tab.blk_off[tab.n] * LH), 64 * NW, 0, st>>>(keys, tab, a_raw, bsum, ssum,
                                                                                      sync, rows);
}

template <int D, int NW, bool FUSED> int resident_workgroups()
{
    static int cached = -1;                                          // per instantiation; benign if raced
    if (cached < 0) {
        int per_cu = 0, dev = 0;
        hipDeviceProp_t prop;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, scan_kernel<D, NW, FUSED>, 64 * NW, 0) != hipSuccess ||
            hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess)
            return 0;
        cached = per_cu * prop.multiProcessorCount;
    }
    return cached;
}

template <int D, int NW>
hipError_t run_nw(const uint16_t *keys, int LH, const PromptTab &tab, float *a_raw, float *bsum, float *ssum,
                  void *sync_area, bool allow_fused, const Prof &prof, hipStream_t st)
{
    int max_unit_blocks = 0;
    for (int p = 0; p < tab.n; ++p) max_unit_blocks = max(max_unit_blocks, tab.blk_off[p + 1] - tab.blk_off[p]);
    // fused only if the chip can hold two units' worth of workgroups at once (see the header comment)
    const bool fused = allow_fused && 2 * max_unit_blocks <= resident_workgroups<D, NW, true>();
    if (fused) {
        const int words = 64 + kUnitStride * LH * tab.n;
        zero_kernel<<<(words + 255) / 256, 256, 0, st>>>((uint32_t *)sync_area, words);
        prof.begin(NKV_KERNEL_SCAN, st);
        launch_scan<D, NW, true>(keys, LH, tab, a_raw, bsum, ssum, (ScanSync *)sync_area, st);
        prof.end(NKV_KERNEL_SCAN, st);
    } else {
        prof.begin(NKV_KERNEL_SCAN, st);
        launch_scan<D, NW, false>(keys, LH, tab, a_raw, bsum, ssum, nullptr, st);
        prof.end(NKV_KERNEL_SCAN, st);
        ssum_kernel<D><<<dim3(tab.n, LH), D, 0, st>>>(bsum, tab, ssum);
        stable_kernel<D><<<dim3((tab.T + 255) / 256, LH), 256, 0, st>>>(keys, tab, ssum, a_raw);
    }
    return hipGetLastError();
}

template <int D>
hipError_t run(const uint16_t *keys, int LH, const PromptTab &tab, float *a_raw, float *bsum, float *ssum,
               void *sync_area, bool allow_fused, const Prof &prof, hipStream_t st)
{
    int bmax = 0;
    for (int p = 0; p < tab.n; ++p) bmax = max(bmax, tab.b[p]);
    switch ((bmax + 63) / 64) {
    case 1: return run_nw<D, 1>(keys, LH, tab, a_raw, bsum, ssum, sync_area, allow_fused, prof, st);
    case 2: return run_nw<D, 2>(keys, LH, tab, a_raw, bsum, ssum, sync_area, allow_fused, prof, st);
    case 3: return run_nw<D, 3>(keys, LH, tab, a_raw, bsum, ssum, sync_area, allow_fused, prof, st);
    default: return run_nw<D, 4>(keys, LH, tab, a_raw, bsum, ssum, sync_area, allow_fused, prof, st);
    }
}

}  // namespace

bool fast_score_supported(int dtype, int d, int window, const PromptTab &tab)
{
    if (dtype != NKV_DTYPE_BF16 || (d != 64 && d != 128) || window != 64) return false;
    for (int p = 0; p < tab.n; ++p)
        if (tab.b[p] > 64 * kMaxChunks) return false;
    return true;
}

size_t fast_score_sync_bytes(int LH, const PromptTab &tab) { return (size_t)(64 + kUnitStride * LH * tab.n) * 4; }

hipError_t launch_score_fast(const void *keys, int LH, int d, const PromptTab &tab, float *a_raw, float *bsum,
                             float *ssum, void *sync_area, bool allow_fused, const Prof &prof, hipStream_t st)
{
    if (d == 128) return run<128>((const uint16_t *)keys, LH, tab, a_raw, bsum, ssum, sync_area, allow_fused, prof, st);
    return run<64>((const uint16_t *)keys, LH, tab, a_raw, bsum, ssum, sync_area, allow_fused, prof, st);
}

}  // namespace nkv
