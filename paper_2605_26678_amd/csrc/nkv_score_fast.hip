// Streaming scoring kernel for bf16, fp16 or 8-bit (E4M3) keys, head dim 64 or 128, window 64, episodic block size <= 256
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
// Arithmetic.  The kernel is bound by vector-ALU issue, not by memory, so every phase is written for a
// low instruction count:
//   * ||k||^2 comes from the packed bf16 pairs directly (v_dot2c_f32_bf16: two exact products and an fp32
//     accumulation per instruction), without unpacking;
//   * a quantity that every token needs summed over the LPR lanes of its row (norms, dots) is reduced for
//     all TPT rows of a lane at once by a transposing butterfly: each step halves the number of live
//     values, and lane c ends up with the total of row c.  This costs ~2 instructions per row instead of
//     log2(LPR) + 1, and the result lands in the lane that reports the token;
//   * 1/||k|| is computed once per token and handed to the row's lanes through LDS.
//
// Per chunk: 1/||k|| per token and the partial sums T[g] = sum of k_hat over the sub-group's tokens.
// Partial sums go through LDS: they give the chunk and block totals (episodic anchor; the block totals
// are also the partial sums of the stable anchor) and the window sum in front of every sub-group.  The
// window sum then slides token by token,
//     W_i = W_{i-1} - k_hat_{i-64} + k_hat_i,
// re-seeded exactly at every sub-group boundary (every TPT tokens) from the partial sums, so no long
// running sum and no cancellation beyond TPT steps.  k_hat_{i-64} sits at the same lane position of the
// previous chunk, i.e. in the registers of the wavefront in front: it is handed over through LDS, four rows
// per step (the first wavefront slides over the halo rows, which also pass through LDS).
// Cosines do not depend on the anchor's length, so sums stand in for means everywhere.
//
// Placement.  The chip's compute units sit in 8 dies (XCDs) with one L2 each; workgroups are started in
// launch order and consecutive ones go to different dies.  Blocks are therefore not taken in launch order:
// workgroup i is item i / 8 of the queue of die i % 8, and a die's queue walks that die's share of each
// (layer, head)'s blocks -- runs of up to 16 consecutive blocks, dealt to the dies round-robin -- so the halo
// of a block was fetched by the same L2 moments before.  All dies work on the same (layer, head) at the same
// time.  The assignment is pure arithmetic on the launch index (no counter to fetch before the first load
// can be issued); should the hardware place a workgroup on another die, only that locality is lost.
//
// The stable anchor needs every key of the prompt before the first a_s can be computed.  Two ways:
//   fused   : all blocks of a (layer, head, prompt) unit are started close together.  The block totals
//             and the unit sums live in memory that is filled with a NaN bit pattern before the launch, so
//             a 32-bit word that has been written is recognisable by itself and no flags, counters or
//             waits for completed stores are needed.  Each workgroup stores its block total (agent scope)
//             and goes on to its window loop.  Every unit has one more item, queued in front of the
//             unit's blocks on one die: the workgroup that gets it does nothing but poll the unit's block
//             totals, add them up in block order and store the unit sum.  After its window loop every
//             block's workgroup polls the unit sum with its chunk still in registers, then computes a_s.
//             Nobody waits without bound: a block's workgroup that does not find the unit sum within a
//             few dozen polls puts its block on a list and leaves without a_s, and a small kernel
//             afterwards computes a_s of the listed blocks from a second read of their keys with the same
//             arithmetic, so the result does not depend on who computed it.  The summing workgroups wait
//             only for block totals, which are stored before any waiting.  So the path is correct
//             whatever the order and placement in which the hardware starts workgroups; that every die's
//             window of resident workgroups normally covers a unit's blocks (the host checks it) only
//             keeps the list short.
//   2-pass  : block totals go to memory, ssum_kernel adds them up and stable_kernel re-reads the keys
//             (any prompt length).
#include "nkv_scan_common.h"

namespace nkv {
namespace {

// NW wavefronts = chunks per block.  grid: one workgroup per (layer*head, block), 1-D.
template <int D, int NW, bool FUSED, int KF>
__global__ __launch_bounds__(64 * NW, NW == 1 ? 2 : (D == 64 ? 4 : 3)) // one-wave blocks (b <= 64) need more registers
void scan_kernel(const uint8_t *__restrict__ keys, RowMap km, PromptTab tab, ScanPlan plan, float *__restrict__ a_raw,
                 float *__restrict__ bsum, float *__restrict__ ssum, uint32_t *__restrict__ sync, int LH,
                 int64_t rows, int poll_limit, uint32_t spin_limit)
{
    constexpr int LPR = D / 8, SG = 64 / LPR, TPT = LPR;
    constexpr int HT = (TPT + NW - 1) / NW;                           // halo tokens per lane
    constexpr int NST = TPT / 4;                                      // 4-row steps per lane
    __shared__ float lds_rn[NW + 1][64];                              // [0]: halo chunk, [1 + w]: chunk w
    __shared__ float lds_T[NW][SG][D];                                // partial sums of the chunks, later of the halo chunk
    __shared__ Piece<KF> lds_h[TPT][64];                                  // halo rows, by the window row that needs them
    __shared__ float lds_C[NW][D];                                    // chunk totals
    __shared__ float lds_S[D];                                        // the unit's sum, once complete
    // Rows on their way to the next wave: two buffers, or one at head dim 64, where a second barrier per step
    // costs less than the fourth workgroup per compute unit that the smaller LDS footprint admits is worth.
    constexpr int kXBuf = D == 64 ? 1 : 2;
    __shared__ Piece<KF> lds_x[kXBuf][NW > 1 ? NW - 1 : 1][4][64];
    __shared__ int s_have;

    const int nblk = plan.nblk;
    int lh, blk, layer, head;
    if (FUSED) {
        // Static assignment: workgroups are started in launch order and go to the dies round-robin, so
        // workgroup i is item i / 8 of the queue of die i % 8 (if it lands on another die the result is the
        // same, only the halo comes from memory).  Everything here is scalar arithmetic on the launch index.
        const int x = (int)(blockIdx.x & (kDies - 1));
        const uint32_t t = blockIdx.x >> 3;
        const int run = plan.run, len = plan.len[x];
        if (t >= queue_start(LH, len, tab.n, x)) return;              // the dies' queues differ slightly in length
        // lh of item t: a first guess from the average number of items per lh, then exact
        int l = min(LH - 1, (int)((float)t * plan.inv_items[x]));
        while (l > 0 && queue_start(l, len, tab.n, x) > t) --l;
        while (l + 1 < LH && queue_start(l + 1, len, tab.n, x) <= t) ++l;
        const int r = (int)(t - queue_start(l, len, tab.n, x));
        lh = l;
        const int nsum = l % kDies == x ? tab.n : 0;                  // the unit sums of lh come first in the segment
        {
            const int rb = max(r - nsum, 0), cyc = div_by(rb, run, plan.inv_run);          // die_block(run, x, rb)
            blk = (cyc * kDies + x) * run + (rb - cyc * run);
        }
        layer = div_by(lh, km.H, plan.inv_H);
        head = lh - layer * km.H;
        const int sum_of = r < nsum ? r : -1;                         // prompt whose unit sum is to be formed
        if (sum_of >= 0) {                                            // uniform: this workgroup adds a unit up
            const int p = sum_of;
            static_assert(64 * NW / (D / 4) * D <= NW * SG * D, "partial sums of the unit do not fit the LDS scratch");
            if (!add_unit_up<D, NW, true>(bsum + ((int64_t)lh * nblk + tab.blk_off[p]) * D,
                                          tab.blk_off[p + 1] - tab.blk_off[p], ssum + ((int64_t)lh * tab.n + p) * D,
                                          &lds_T[0][0][0], spin_limit) &&
                threadIdx.x == 0)
                atomicAdd(sync + kTimeoutWord, 1u);
            return;
        }
    } else {
        lh = blockIdx.x / nblk;
        blk = blockIdx.x - lh * nblk;
        layer = lh / km.H;
        head = lh - layer * km.H;
    }
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
    constexpr int ES = key_bytes<KF>(), kRowBytes = D * ES;
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t *>(keys) + km.unit(layer, head, p, tab) * ES, 0, N * kRowBytes, 0x00020000);
    const int lane_off = t0 * kRowBytes + c * (8 * ES);
    Piece<KF> raw[TPT], hraw[HT];
    // a full block's last 64 tokens (the last wave's) are read again as the next block's halo: they stay in the L2;
    // the other waves' rows are marked non-temporal
    if (w < NW - 1) {
#pragma unroll
        for (int j = 0; j < TPT; ++j) raw[j] = row_load<KF, 2>(rsrc, lane_off + j * kRowBytes);
    } else {
#pragma unroll
        for (int j = 0; j < TPT; ++j) raw[j] = row_load<KF>(rsrc, lane_off + j * kRowBytes);
    }
    const int halo_off = (blk_lo - 64 + g * TPT + HT * w) * kRowBytes + c * (8 * ES);
#pragma unroll
    for (int jj = 0; jj < HT; ++jj) hraw[jj] = row_load<KF>(rsrc, halo_off + jj * kRowBytes);

    // ---- norms: one token per lane (lane (g, c) reports token g*TPT + c = lane of the chunk) ----
    float rn_m, kn_m;
    {
        float ss[TPT];
#pragma unroll
        for (int j = 0; j < TPT; ++j) ss[j] = sumsq8<KF>(raw[j]);
        if constexpr (KF == kKeyF8) {                                 // or the unpacked rows stay alive for the next phase
#pragma unroll
            for (int j = 0; j < TPT; ++j) forget(raw[j]);
        }
        const float ss_m = transpose_reduce<LPR>(ss);
        rn_m = (blk_lo + 64 * w + lane < blk_hi) ? inv_norm(ss_m) : 0.f;
        kn_m = ss_m < 1e-24f ? sqrtf(ss_m) * 1e12f : 1.f;             // ||k_hat|| of this lane's own token
        lds_rn[1 + w][lane] = rn_m;
    }
    float T[8];
    // ---- partial sums of the chunk: the row's 1/||k|| comes back from LDS (same wave: in order) ----
#pragma unroll
    for (int e = 0; e < 8; ++e) T[e] = 0.f;
#pragma unroll
    for (int s = 0; s < NST; ++s) {
        const float4 r4 = *reinterpret_cast<const float4 *>(&lds_rn[1 + w][g * TPT + 4 * s]);
        const float rr[4] = {r4.x, r4.y, r4.z, r4.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float k[8];
            unpack8<KF>(raw[4 * s + i], k);
#pragma unroll
            for (int e = 0; e < 8; ++e) T[e] = fmaf(rr[i], k[e], T[e]);
        }
        __builtin_amdgcn_sched_barrier(0);                            // bound the unpacked temporaries
    }
    store8(&lds_T[w][g][c * 8], T);
    __syncthreads();

    // ---- chunk totals; window sum in front of this lane's first token ----
    float W[8];
    {
        float own[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) { W[e] = 0.f; own[e] = 0.f; }
#pragma unroll 2
        for (int gg = 0; gg < SG; ++gg) {
            float cv[8], pv[8];
            load8(&lds_T[w][gg][c * 8], cv);
            if (w == 0) {                                             // the halo's share is added further down
#pragma unroll
                for (int e = 0; e < 8; ++e) pv[e] = 0.f;
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
    const int unblk = tab.blk_off[p + 1] - tab.blk_off[p];
    float *bsum_unit = bsum + ((int64_t)lh * nblk + tab.blk_off[p]) * D;      // block totals of this unit
    float *S_unit = ssum + ((int64_t)lh * tab.n + p) * D;
    if (FUSED) {
        // One wave stores the block total: vector memory instructions complete in order as far as the
        // compiler can rely on, so the wave that issues the stores waits for them at its next load; the
        // other waves do not.  The duty rotates with the block index.
        const __amdgpu_buffer_rsrc_t brs = __builtin_amdgcn_make_buffer_rsrc(bsum_unit, 0, unblk * D * 4, 0x00020000);
        if (w == blk % NW && g == 0) {
            const int off = ((blk - tab.blk_off[p]) * D + c * 8) * 4;
            agent_store16(brs, off, Bs[0], Bs[1], Bs[2], Bs[3]);
            agent_store16(brs, off + 16, Bs[4], Bs[5], Bs[6], Bs[7]);
        }
    } else if (w == 0 && g == 0) {
        store8(bsum + ((int64_t)lh * nblk + blk) * D + c * 8, Bs);
    }

    // ---- halo share: norms and partial sums (after the block total is on its way: only the window needs them) ----
#pragma unroll
    for (int e = 0; e < 8; ++e) T[e] = 0.f;
#pragma unroll
    for (int jj = 0; jj < HT; ++jj) {
        const float ssh = row_sum<LPR>(sumsq8_for_dpp<KF>(hraw[jj]));
        const int q = HT * w + jj;
        const bool ok = q < TPT && blk_lo - 64 + g * TPT + q >= 0;
        const float r = ok ? inv_norm(ssh) : 0.f;
        float k[8];
        unpack8<KF>(hraw[jj], k);
#pragma unroll
        for (int e = 0; e < 8; ++e) T[e] = fmaf(r, k[e], T[e]);
        if (c == jj && q < TPT) lds_rn[0][g * TPT + q] = r;
        if (q < TPT) lds_h[q][lane] = hraw[jj];                       // wave 0 slides over these rows
    }
    store8(&lds_T[w][g][c * 8], T);
    if (NW > 1 && w < NW - 1) {                                       // rows 0..3 for the next wave's first window step
#pragma unroll
        for (int i = 0; i < 4; ++i) lds_x[0][w][i][lane] = raw[i];
    }
    __syncthreads();
    if (w == 0) {                                                     // previous chunk of wave 0 = the halo chunk
#pragma unroll 2
        for (int gg = 0; gg < SG; ++gg) {
            if (gg >= g) {
#pragma unroll
                for (int ww = 0; ww < NW; ++ww) {
                    float hv[8];
                    load8(&lds_T[ww][gg][c * 8], hv);
#pragma unroll
                    for (int e = 0; e < 8; ++e) W[e] += hv[e];
                }
            }
        }
    }

    // ---- slide the window over this lane's tokens: current-memory dots ----
    // Four rows per step; the per-lane partial dots of the four rows enter the transposing butterfly.
    float wd_m = 0.f, wn_m = 1.f, bd_m = 0.f;
    const __amdgpu_buffer_rsrc_t srs = __builtin_amdgcn_make_buffer_rsrc(S_unit, 0, D * 4, 0x00020000);
    u32x4 sv0 = {kUnwritten, kUnwritten, kUnwritten, kUnwritten}, sv1 = sv0;
    {
        StreamReduce<LPR> red_wd, red_wn, red_bd;                     // the episodic dot rides along: same unpacked row
#pragma unroll
        for (int j = 0; j < TPT; ++j) forget(raw[j]);
        // Leaving rows come through LDS: wave 0 slides over the halo rows every wave stored while it worked on
        // its share of the halo; the other waves get theirs from the wave in front of them, four rows per
        // step, double-buffered: one barrier per step separates the writes of a buffer from its reads
        // and its reads from the writes two steps later.
#pragma unroll
        for (int s = 0; s < NST; ++s) {
            if (NW > 1 && kXBuf == 2) {
                if (s > 0) __syncthreads();
                if (s + 1 < NST && w < NW - 1) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) lds_x[(s + 1) & 1][w][i][lane] = raw[4 * s + 4 + i];
                }
            }
            if (NW > 1 && kXBuf == 1 && s > 0) {                      // one buffer: reads of step s - 1, then the writes
                __syncthreads();
                if (w < NW - 1) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) lds_x[0][w][i][lane] = raw[4 * s + i];
                }
                __syncthreads();
            }
            const Piece<KF> *leaving = w == 0 ? &lds_h[4 * s][lane] : &lds_x[s & (kXBuf - 1)][NW > 1 ? w - 1 : 0][0][lane];
            const float4 r4 = *reinterpret_cast<const float4 *>(&lds_rn[1 + w][g * TPT + 4 * s]);
            const float4 q4 = *reinterpret_cast<const float4 *>(&lds_rn[w][g * TPT + 4 * s]);
            const float rr[4] = {r4.x, r4.y, r4.z, r4.w};
            const float rp[4] = {q4.x, q4.y, q4.z, q4.w};             // 0 where the leaving token does not exist
            if (FUSED && s == NST - 1 && w == 0 && lane < LPR) {      // first look at the unit sum, a step early
                sv0 = agent_load16(srs, lane * 32);
                sv1 = agent_load16(srs, lane * 32 + 16);
            }
            float pw[4], pn[4], pb[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float kp[8], k[8];
                const Piece<KF> pl = leaving[i * 64];
                unpack8<KF>(pl, kp);
                unpack8<KF>(raw[4 * s + i], k);
                float wd = 0.f, wn = 0.f, bd = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    W[e] = fmaf(-rp[i], kp[e], W[e]);
                    W[e] = fmaf(rr[i], k[e], W[e]);
                    wd = fmaf(k[e], W[e], wd);
                    wn = fmaf(W[e], W[e], wn);
                    bd = fmaf(k[e], Bs[e], bd);
                }
                pw[i] = wd; pn[i] = wn; pb[i] = bd;
                __builtin_amdgcn_sched_barrier(0);                    // one row at a time
            }
            if (s == 0) { red_wd.template push<0>(pw, wd_m); red_wn.template push<0>(pn, wn_m); red_bd.template push<0>(pb, bd_m); }
            if (s == 1) { red_wd.template push<1>(pw, wd_m); red_wn.template push<1>(pn, wn_m); red_bd.template push<1>(pb, bd_m); }
            if constexpr (LPR == 16) {
                if (s == 2) { red_wd.template push<2>(pw, wd_m); red_wn.template push<2>(pn, wn_m); red_bd.template push<2>(pb, bd_m); }
                if (s == 3) { red_wd.template push<3>(pw, wd_m); red_wn.template push<3>(pn, wn_m); red_bd.template push<3>(pb, bd_m); }
            }
            __builtin_amdgcn_sched_barrier(0);                        // one step at a time
        }
    }
    const int tok = blk_lo + 64 * w + lane;                           // lane (g, c) reports token g*TPT + c
    if (tok < blk_hi) {
        a_raw[2 * rows + row0 + tok] = neg_cos(rn_m * wd_m, kn_m, wn_m);
        a_raw[rows + row0 + tok] = neg_cos(rn_m * bd_m, kn_m, bsq);
    }

    // ---- stable dots against the unit's sum ----
    // The sum is normally there when a workgroup gets here.
    float S[8];
    float ssq = 1.f;
    bool have_S = false;
    if (FUSED) {
        if (w == 0) {                                                 // LPR lanes poll, the other waves sit at the barrier
            bool got = false;
            for (int polls = 0; poll_limit >= 0; ++polls) {           // poll_limit < 0: defer without looking
                const bool ok = lane >= LPR || (all_written(sv0) && all_written(sv1));
                got = __all(ok);
                if (got || polls >= poll_limit) break;
                __builtin_amdgcn_s_sleep(8);
                if (lane < LPR) {
                    sv0 = agent_load16(srs, lane * 32);
                    sv1 = agent_load16(srs, lane * 32 + 16);
                }
            }
            if (got && lane < LPR) {
                *reinterpret_cast<u32x4 *>(&lds_S[lane * 8]) = sv0;
                *reinterpret_cast<u32x4 *>(&lds_S[lane * 8 + 4]) = sv1;
            }
            if (lane == 0) {
                s_have = got ? 1 : 0;
                if (!got) sync[kSyncWords + atomicAdd(sync + kDeferCountWord, 1u)] = (uint32_t)(lh * nblk + blk);
            }
        }
        __syncthreads();
        have_S = s_have != 0;
        if (have_S) load8(&lds_S[c * 8], S);
        else {
#pragma unroll
            for (int e = 0; e < 8; ++e) S[e] = 0.f;
        }
        ssq = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) ssq = fmaf(S[e], S[e], ssq);
        ssq = row_sum<LPR>(ssq);
    }
    if (FUSED && have_S) {
#pragma unroll
        for (int j = 0; j < TPT; ++j) forget(raw[j]);
        float sd[TPT];
#pragma unroll
        for (int j = 0; j < TPT; ++j) {
            float k[8];
            unpack8<KF>(raw[j], k);
            float accs = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) accs = fmaf(k[e], S[e], accs);
            sd[j] = accs;
            if ((j & 3) == 3) __builtin_amdgcn_sched_barrier(0);
        }
        const float sd_m = transpose_reduce<LPR>(sd);
        if (tok < blk_hi) a_raw[row0 + tok] = neg_cos(rn_m * sd_m, kn_m, ssq);
    }
}

// a_s of the blocks whose workgroups did not wait for their unit's sum.  One workgroup per listed block at a
// time, one wave per chunk, same lane layout, same instruction sequences for the norm, the dot and the
// cosine as scan_kernel, so the values are the ones scan_kernel would have stored.
template <int D, int NW, int KF>
__global__ __launch_bounds__(64 * NW) void deferred_stable_kernel(const uint8_t *__restrict__ keys, RowMap km,
                                                                  PromptTab tab, const float *__restrict__ bsum,
                                                                  float *__restrict__ ssum,
                                                                  const uint32_t *__restrict__ sync,
                                                                  float *__restrict__ a_raw)
{
    constexpr int LPR = D / 8, TPT = LPR, ES = key_bytes<KF>(), kRowBytes = D * ES;
    __shared__ float part[64 * NW / (D / 4) * D];
    const int nblk = tab.blk_off[tab.n];
    const uint32_t count = sync[kDeferCountWord];
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int g = lane / LPR, c = lane % LPR;
    for (uint32_t i = blockIdx.x; i < count; i += gridDim.x) {
        const int id = (int)sync[kSyncWords + i], lh = id / nblk, blk = id - lh * nblk;
        const int p = prompt_of_block(tab, blk);
        const int b = tab.b[p], N = tab.tok_off[p + 1] - tab.tok_off[p];
        const int blk_lo = (blk - tab.blk_off[p]) * b, blk_hi = min(blk_lo + b, N);
        const int64_t row0 = (int64_t)lh * tab.T + tab.tok_off[p];
        float *S_unit = ssum + ((int64_t)lh * tab.n + p) * D;
        ensure_unit_sum<D, NW>(bsum + ((int64_t)lh * nblk + tab.blk_off[p]) * D, tab.blk_off[p + 1] - tab.blk_off[p], S_unit, part);
        const __amdgpu_buffer_rsrc_t srs = __builtin_amdgcn_make_buffer_rsrc(S_unit, 0, D * 4, 0x00020000);
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint8_t *>(keys) + km.unit(lh, p, tab) * ES, 0, N * kRowBytes, 0x00020000);
        const int lane_off = (blk_lo + 64 * w + g * TPT) * kRowBytes + c * (8 * ES);
        Piece<KF> raw[TPT];
#pragma unroll
        for (int j = 0; j < TPT; ++j) raw[j] = row_load<KF>(rsrc, lane_off + j * kRowBytes);
        float ss[TPT];
#pragma unroll
        for (int j = 0; j < TPT; ++j) ss[j] = sumsq8<KF>(raw[j]);
        const float ss_m = transpose_reduce<LPR>(ss);
        const int tok = blk_lo + 64 * w + lane;
        const float rn_m = tok < blk_hi ? inv_norm(ss_m) : 0.f;
        const float kn_m = ss_m < 1e-24f ? sqrtf(ss_m) * 1e12f : 1.f;
        float S[8];
        {
            const u32x4 s0 = agent_load16(srs, c * 32), s1 = agent_load16(srs, c * 32 + 16);
            S[0] = __uint_as_float(s0.x); S[1] = __uint_as_float(s0.y); S[2] = __uint_as_float(s0.z); S[3] = __uint_as_float(s0.w);
            S[4] = __uint_as_float(s1.x); S[5] = __uint_as_float(s1.y); S[6] = __uint_as_float(s1.z); S[7] = __uint_as_float(s1.w);
        }
        float ssq = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) ssq = fmaf(S[e], S[e], ssq);
        ssq = row_sum<LPR>(ssq);
        float sd[TPT];
#pragma unroll
        for (int j = 0; j < TPT; ++j) {
            float k[8];
            unpack8<KF>(raw[j], k);
            float acc = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc = fmaf(k[e], S[e], acc);
            sd[j] = acc;
        }
        const float sd_m = transpose_reduce<LPR>(sd);
        if (tok < blk_hi) a_raw[row0 + tok] = neg_cos(rn_m * sd_m, kn_m, ssq);
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

// Stable anomaly a_s by a second touch of the keys.  grid (ceil(T/256), L*H), 4 waves of 64 tokens.
template <int D, int KF>
__global__ __launch_bounds__(256) void stable_kernel(const uint8_t *__restrict__ keys, RowMap km, PromptTab tab,
                                                     const float *__restrict__ ssum, float *__restrict__ a_raw)
{
    constexpr int LPR = D / 8, TPT = LPR, ES = key_bytes<KF>();
    const int lh = blockIdx.y;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int g = lane / LPR, c = lane % LPR;
    const int tg0 = blockIdx.x * 256 + wv * 64;                      // first global token of this wave
    if (tg0 >= tab.T) return;
    float sd_m = 0.f, ss_m = 0.f, sq_m = 1.f;
#pragma unroll
    for (int j = 0; j < TPT; ++j) {
        const int tg = tg0 + g * TPT + j;
        const bool ok = tg < tab.T;
        const int p = prompt_of_token(tab, ok ? tg : tab.T - 1);
        const uint8_t *row = keys + (km.unit(lh, p, tab) + (int64_t)(tg - tab.tok_off[p]) * D) * ES;
        Piece<KF> raw = {};
        if (ok) raw = reinterpret_cast<const Piece<KF> *>(row)[c];
        float sv[8], k[8];
        load8(ssum + ((int64_t)lh * tab.n + p) * D + c * 8, sv);
        unpack8<KF>(raw, k);
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

template <int D, int NW, bool FUSED, int KF>
void launch_scan(const uint8_t *keys, const RowMap &km, int LH, const PromptTab &tab, float *a_raw, float *bsum, float *ssum,
                 uint32_t *sync, int poll_limit, uint32_t spin_limit, hipStream_t st)
{
    const int64_t rows = (int64_t)LH * tab.T;
    ScanPlan plan;
    const unsigned queued = fill_scan_plan(LH, tab, km.H, &plan);
    const unsigned groups = FUSED ? queued : (unsigned)(tab.blk_off[tab.n] * LH);
    scan_kernel<D, NW, FUSED, KF><<<groups, 64 * NW, 0, st>>>(keys, km, tab, plan, a_raw, bsum, ssum, sync, LH, rows,
                                                              poll_limit, spin_limit);
}

template <int D, int NW, bool FUSED, int KF> int resident_workgroups()
{
    static int cached = -1;                                          // per instantiation; benign if raced
    if (cached < 0) {
        int per_cu = 0, dev = 0;
        hipDeviceProp_t prop;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, scan_kernel<D, NW, FUSED, KF>, 64 * NW, 0) != hipSuccess ||
            hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess)
            return 0;
        cached = per_cu * prop.multiProcessorCount;
    }
    return cached;
}


template <int D, int NW, int KF>
hipError_t run_nw(const uint8_t *keys, const RowMap &km, int LH, const PromptTab &tab, float *a_raw, float *bsum, float *ssum,
                  void *sync_area, int mode, const Prof &prof, hipStream_t st)
{
    int max_unit_blocks = 0;
    for (int p = 0; p < tab.n; ++p) max_unit_blocks = max(max_unit_blocks, tab.blk_off[p + 1] - tab.blk_off[p]);
    // fused only if the chip can hold a unit's workgroups at once (see the header comment); from half of that
    // on, workgroups that wait for the unit sum hold up some of those behind them, which still costs less than
    // a second read of the keys
    // (queue arithmetic is 32-bit: keep the number of items far below 2^32 / 8)
    const int64_t items = (int64_t)LH * (tab.blk_off[tab.n] + tab.n);
    const bool allow_fused = mode != kScanTwoPass, no_unit_sums = mode == kScanRepairAll;
    const bool defer_all = mode == kScanDeferAll || no_unit_sums;
    const bool fused = allow_fused && items < (1ll << 28) && max_unit_blocks <= resident_workgroups<D, NW, true, KF>();
    if (fused) {
        // the counters start at zero, block totals and unit sums as "unwritten"
        const size_t nb = (size_t)LH * tab.blk_off[tab.n] * D / 4, ns = (size_t)LH * tab.n * D / 4;
        const size_t n16 = kSyncWords / 4 + nb + ns;
        prepare_kernel<<<(unsigned)min((n16 + 255) / 256, (size_t)2048), 256, 0, st>>>(
            (uint4 *)sync_area, kSyncWords / 4, (uint4 *)bsum, nb, (uint4 *)ssum, ns);
        prof.begin(NKV_KERNEL_SCAN, st);
        launch_scan<D, NW, true, KF>(keys, km, LH, tab, a_raw, bsum, ssum, (uint32_t *)sync_area,
                                 defer_all ? -1 : kPollLimit, no_unit_sums ? 0u : kSpinLimit, st);
        prof.end(NKV_KERNEL_SCAN, st);
        deferred_stable_kernel<D, NW, KF><<<defer_all ? 4096 : 256, 64 * NW, 0, st>>>(keys, km, tab, bsum, ssum,
                                                                                  (const uint32_t *)sync_area, a_raw);
    } else {
        // (the counters a caller may ask for read as zero on this route)
        prepare_kernel<<<1, 256, 0, st>>>((uint4 *)sync_area, kSyncWords / 4, nullptr, 0, nullptr, 0);
        prof.begin(NKV_KERNEL_SCAN, st);
        launch_scan<D, NW, false, KF>(keys, km, LH, tab, a_raw, bsum, ssum, nullptr, 0, 0u, st);
        prof.end(NKV_KERNEL_SCAN, st);
        ssum_kernel<D><<<dim3(tab.n, LH), D, 0, st>>>(bsum, tab, ssum);
        stable_kernel<D, KF><<<dim3((tab.T + 255) / 256, LH), 256, 0, st>>>(keys, km, tab, ssum, a_raw);
    }
    return hipGetLastError();
}

template <int D, int KF>
hipError_t run(const uint8_t *keys, const RowMap &km, int LH, const PromptTab &tab, float *a_raw, float *bsum, float *ssum,
               void *sync_area, int mode, const Prof &prof, hipStream_t st)
{
    int bmax = 0;
    for (int p = 0; p < tab.n; ++p) bmax = max(bmax, tab.b[p]);
    switch ((bmax + 63) / 64) {
    case 1: return run_nw<D, 1, KF>(keys, km, LH, tab, a_raw, bsum, ssum, sync_area, mode, prof, st);
    case 2: return run_nw<D, 2, KF>(keys, km, LH, tab, a_raw, bsum, ssum, sync_area, mode, prof, st);
    case 3: return run_nw<D, 3, KF>(keys, km, LH, tab, a_raw, bsum, ssum, sync_area, mode, prof, st);
    default: return run_nw<D, 4, KF>(keys, km, LH, tab, a_raw, bsum, ssum, sync_area, mode, prof, st);
    }
}

}  // namespace

bool fast_score_supported(int dtype, int d, int window, const PromptTab &tab)
{
    if ((dtype != NKV_DTYPE_BF16 && dtype != NKV_DTYPE_F8_E4M3 && dtype != NKV_DTYPE_F16) || (d != 64 && d != 128) || window != 64) return false;
    for (int p = 0; p < tab.n; ++p) {
        if (tab.b[p] > 64 * kMaxChunks) return false;
        // a prompt's rows are addressed by 32-bit byte offsets from its first row
        if ((int64_t)(tab.tok_off[p + 1] - tab.tok_off[p] + 256) * d * 2 >= (1ll << 31)) return false;
    }
    return true;
}

size_t fast_score_sync_bytes(int LH, const PromptTab &tab)
{
    return ((size_t)kSyncWords + (size_t)LH * tab.blk_off[tab.n]) * 4;       // counters + the list of deferred blocks
}

hipError_t launch_score_fast(const void *keys, const RowMap &km, int dtype, int LH, int d, const PromptTab &tab, float *a_raw,
                             float *bsum, float *ssum, void *sync_area, int mode, const Prof &prof,
                             hipStream_t st)
{
    const uint8_t *k = (const uint8_t *)keys;
    if (dtype == NKV_DTYPE_F8_E4M3) {
        if (d == 128) return run<128, kKeyF8>(k, km, LH, tab, a_raw, bsum, ssum, sync_area, mode, prof, st);
        return run<64, kKeyF8>(k, km, LH, tab, a_raw, bsum, ssum, sync_area, mode, prof, st);
    }
    if (dtype == NKV_DTYPE_F16) {
        if (d == 128) return run<128, kKeyF16>(k, km, LH, tab, a_raw, bsum, ssum, sync_area, mode, prof, st);
        return run<64, kKeyF16>(k, km, LH, tab, a_raw, bsum, ssum, sync_area, mode, prof, st);
    }
    if (d == 128) return run<128, kKeyBF16>(k, km, LH, tab, a_raw, bsum, ssum, sync_area, mode, prof, st);
    return run<64, kKeyBF16>(k, km, LH, tab, a_raw, bsum, ssum, sync_area, mode, prof, st);
}

}  // namespace nkv
