// Streaming scoring kernel for bf16 or fp16 keys of head dim 128, window 64, episodic block size <= 256 (paper
// Sections 2.1-2.3), with every dot product of the pass formed by the matrix cores.  (Written out below for bf16;
// fp16 differs in the product instruction, in unpacking, and in how an fp32 anchor is cut into three terms.)
//
// The pass is a stream over the keys and nothing else is read from memory, but written for the vector unit it
// needs ~2300 instructions per 64 tokens and is bound by their issue.  Here the vector unit keeps only the work
// that is a sum over tokens (the partial sums of normalised keys that the anchors are made of); everything that
// is a contraction over the head dimension goes through v_mfma_f32_16x16x32_bf16, whose products of bf16 values
// are exact and whose sums are fp32:
//
//   * a block is cut into groups of 16 tokens.  T_q = sum of k_hat over group q (vector unit).  The window sum in
//     front of group q's first token is exact in terms of groups: Seed_q = T_{q-4} + ... + T_{q-1}.
//   * for token i of group G, with P the group 64 tokens earlier (token i' = i - 64 leaves as i enters),
//         W_i = Seed_G + sum_{j in G, j <= i} k_hat_j - sum_{j' in P, j' <= i'} k_hat_j',
//     so <k_i, W_i> = <k_i, Seed_G> + sum_{j <= i} w_j A[i][j] - sum_{j' <= i'} w_j' X[i][j'] with the Gram tiles
//     A = K_G K_G^T and X = K_G K_P^T of the raw keys and w = 1 / ||k||.
//   * ||W_i||^2 follows the window inside the group: it is ||Seed_G||^2 plus the running sum of
//         ||W_i||^2 - ||W_{i-1}||^2 = 2 <W_i, d_i> - ||d_i||^2,   d_i = k_hat_i - k_hat_i',
//     which needs <k_i', W_i> (same tiles, the other triangle) and X[i][i'].  At most 16 terms are added up.
//   * <k, anchor> for the anchors that are vectors (Seed_G, the block total, the unit sum): the fp32 anchor is
//     split into three bf16 terms (8 + 8 + 8 mantissa bits, exact) that form rows of the left operand.
//
// Layouts.  A wave owns the groups q = w, w + 4, w + 8, w + 12 of the block (so the group 64 tokens earlier is
// its own previous group) and the group of the halo in front of them.  A group is loaded row-wise (lane (g, c):
// rows 4g .. 4g+3, dims 8c .. 8c+7; four contiguous 256-byte pieces per load instruction), which is the layout
// the partial sums want, and passes through 4 KB of LDS private to the wave to become a matrix operand (lane
// (q, n): token n, dims 32 kk + 8q .. + 7 in operand register kk).  Operands stay in registers until the unit's
// sum has arrived.  A 16 x 16 result leaves lane (q, n) with column n, rows 4q .. 4q+3: sums over rows are four
// multiply-adds per lane followed by a sum over the four lanes n, n+16, n+32, n+48.
//
// Protocol.  A block's workgroup adds its total to the unit's self-counting accumulators (nkv_scan_common.h) as
// soon as it has it; the add returns the word's previous contents, and whoever finds that it was the last of the
// unit's blocks to add to a word stores the word's final value, as fp32, into the unit's sum -- memory that
// starts out "unwritten" and in which every word is stored exactly once.  After its window phase a workgroup looks
// at the unit's sum: if it is complete it forms a_s from the operands still in its registers; if not after a
// bounded number of looks, it puts its block on a list and leaves, and deferred_stable_tile_kernel computes a_s
// of the listed blocks after the pass, when every sum is complete.  No workgroup ever waits for anything but
// stores that workgroups already running (or finished) issue unconditionally, and every wait is bounded.
// (Looking at the accumulators themselves instead of a copy stored once was tried: loads of words that other
// workgroups are adding to cost the pass a quarter of its time under sustained load.)
#include "nkv_scan_common.h"

namespace nkv {
namespace {

using bf16x8 = __bf16 __attribute__((ext_vector_type(8)));
using f16x8 = _Float16 __attribute__((ext_vector_type(8)));
using f32x4 = float __attribute__((ext_vector_type(4)));

constexpr int kGroup = 16;                       // tokens per group
constexpr int kPitch = 272;                      // bytes between the rows of a staged group: 16 lanes that read the
                                                 // same piece of 16 rows touch every LDS bank once
constexpr int kStageBytes = kGroup * kPitch;
constexpr int kTileWaves = 4;


// KF: the keys' 16-bit format (kKeyBF16 or kKeyF16), which is also the format the anchors' terms are staged in
template <int KF> __device__ __forceinline__ f32x4 mma(const u32x4 &a, const u32x4 &b, f32x4 c)
{
    if constexpr (KF == kKeyF16)
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// D[m][n] = sum over the head dimension of a's row m and b's row n
template <int KF, int KS> __device__ __forceinline__ f32x4 tile(const u32x4 (&a)[KS], const u32x4 (&b)[KS])
{
    f32x4 c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) c = mma<KF>(a[kk], b[kk], c);
    return c;
}

// x summed over the four lanes n, n + 16, n + 32, n + 48; every lane receives the total.
// permlane32_swap(x, x) = (x of the lower half in both halves, x of the upper half in both halves); the 16-lane
// swap does the same with even and odd rows of 16 lanes.
__device__ __forceinline__ float sum_over_rows16(float x)
{
    const uint32_t u = __float_as_uint(x);
    const auto a = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    const float s = __uint_as_float(a[0]) + __uint_as_float(a[1]);
    const uint32_t v = __float_as_uint(s);
    const auto b = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// T[e], e < 8: partial sums of dims 8c + e held by lane (g, c).  Summed over g; lane (g, c) receives the totals
// of dims 8c + 2g and 8c + 2g + 1.  Each step halves the number of live values.
__device__ __forceinline__ float2 sum_over_rows16_transposing(const float (&T)[8])
{
    float U[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {                // lower half: dim e, upper half: dim e + 4
        const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(T[e]), __float_as_uint(T[e + 4]), false, false);
        U[e] = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    }
    float V[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) {                // rows 0..3 of 16 lanes: dims e, e + 2, e + 4, e + 6
        const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(U[e]), __float_as_uint(U[e + 2]), false, false);
        V[e] = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    }
    return make_float2(V[0], V[1]);
}

// inclusive running sum over the 16 lanes of a row (lanes n = 0 .. 15 of every group of 16)
__device__ __forceinline__ float row_prefix_sum(float x)
{
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x111, 0xf, 0xf, true));   // row_shr:1
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x112, 0xf, 0xf, true));   // row_shr:2
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x114, 0xf, 0xf, true));   // row_shr:4
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x118, 0xf, 0xf, true));   // row_shr:8
    return x;
}

// fp32 -> three 16-bit terms whose sum is the value.  bf16: each term takes the next 8 mantissa bits, exact.  fp16:
// each term is the rounded remainder (11 bits each; the remainders are exact, the last term is off by at most 2^-33
// of the value or by fp16's smallest step, 6e-8, whichever is larger); the value must be below fp16's largest, 65504.
template <int KF> __device__ __forceinline__ void split3(float x, uint32_t &hi, uint32_t &mid, uint32_t &lo)
{
    if constexpr (KF == kKeyF16) {
        const _Float16 h = (_Float16)x;
        const float r1 = x - (float)h;
        const _Float16 m = (_Float16)r1;
        const float r2 = r1 - (float)m;
        const _Float16 l = (_Float16)r2;
        hi = __builtin_bit_cast(unsigned short, h);
        mid = __builtin_bit_cast(unsigned short, m);
        lo = __builtin_bit_cast(unsigned short, l);
        return;
    }
    const uint32_t b0 = __float_as_uint(x) & 0xffff0000u;
    const float r1 = x - __uint_as_float(b0);
    const uint32_t b1 = __float_as_uint(r1) & 0xffff0000u;
    const float r2 = r1 - __uint_as_float(b1);
    hi = b0 >> 16;
    mid = b1 >> 16;
    lo = __float_as_uint(r2) >> 16;
}

// A vector of which this lane holds dims 2 lane and 2 lane + 1, as the three terms of rows row0 .. row0 + 2
// of a staged left operand.
template <int KF> __device__ __forceinline__ void stage_anchor(uint8_t *stage, int row0, int lane, float v0, float v1)
{
    uint32_t h0, m0, l0, h1, m1, l1;
    split3<KF>(v0, h0, m0, l0);
    split3<KF>(v1, h1, m1, l1);
    *reinterpret_cast<uint32_t *>(stage + (row0 + 0) * kPitch + 4 * lane) = h0 | (h1 << 16);
    *reinterpret_cast<uint32_t *>(stage + (row0 + 1) * kPitch + 4 * lane) = m0 | (m1 << 16);
    *reinterpret_cast<uint32_t *>(stage + (row0 + 2) * kPitch + 4 * lane) = l0 | (l1 << 16);
}

// The staged 16 rows as a matrix operand: lane (q, n) takes dims 32 kk + 8 q .. + 7 of row n.
__device__ __forceinline__ void read_operand(const uint8_t *stage, int lane, u32x4 (&x)[4])
{
    const uint8_t *mine = stage + (lane & 15) * kPitch + 16 * (lane >> 4);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) x[kk] = *reinterpret_cast<const u32x4 *>(mine + 64 * kk);
}

// Sum of the squares of a lane's eight values of a row, ready to be read by any vector instruction (see above).
template <int KF> __device__ __forceinline__ float piece_sumsq(const u32x4 &r)
{
    float acc = 0.f;
    if constexpr (KF == kKeyF16)
        asm("v_dot2c_f32_f16 %0, %1, %1\n\t"
            "v_dot2c_f32_f16 %0, %2, %2\n\t"
            "v_dot2c_f32_f16 %0, %3, %3\n\t"
            "v_dot2c_f32_f16 %0, %4, %4\n\t"
            "s_nop 3"
            : "+v"(acc)
            : "v"(r.x), "v"(r.y), "v"(r.z), "v"(r.w));
    else
        asm("v_dot2c_f32_bf16 %0, %1, %1\n\t"
            "v_dot2c_f32_bf16 %0, %2, %2\n\t"
            "v_dot2c_f32_bf16 %0, %3, %3\n\t"
            "v_dot2c_f32_bf16 %0, %4, %4\n\t"
            "s_nop 3"
            : "+v"(acc)
            : "v"(r.x), "v"(r.y), "v"(r.z), "v"(r.w));
    return acc;
}

// One group of 16 tokens in row-wise layout (lane (g, c): rows 4g .. 4g+3, dims 8c .. 8c+7; tok0 = the group's
// first token, which may lie in front of the prompt): ||k||^2 and the weight 1/||k|| of every row (0 for tokens
// outside [0, tok_end)) go to ss_out / w_out, and to ww for this lane's own rows.
template <int KF> __device__ __forceinline__ void group_norms(const u32x4 (&raw)[4], int tok0, int tok_end, int g, int c, float *w_out,
                                            float *ss_out, float (&ww)[4])
{
    float ss[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        ss[j] = row_sum<16>(piece_sumsq<KF>(raw[j]));
        const int tok = tok0 + 4 * g + j;
        ww[j] = (tok >= 0 && tok < tok_end) ? inv_norm(ss[j]) : 0.f;
    }
    if (c == 0) {
        *reinterpret_cast<float4 *>(w_out + 4 * g) = make_float4(ww[0], ww[1], ww[2], ww[3]);
        *reinterpret_cast<float4 *>(ss_out + 4 * g) = make_float4(ss[0], ss[1], ss[2], ss[3]);
    }
}

// The same, and the weighted sum of the group's rows to sum_out (D floats).
template <int KF> __device__ __forceinline__ void group_sum(const u32x4 (&raw)[4], int tok0, int tok_end, int g, int c, float *w_out,
                                          float *ss_out, float *sum_out)
{
    float ww[4];
    group_norms<KF>(raw, tok0, tok_end, g, c, w_out, ss_out, ww);
    float T[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) T[e] = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float k[8];
        unpack8<KF>(raw[j], k);
#pragma unroll
        for (int e = 0; e < 8; ++e) T[e] = fmaf(ww[j], k[e], T[e]);
    }
    *reinterpret_cast<float2 *>(sum_out + 8 * c + 2 * g) = sum_over_rows16_transposing(T);
}

__device__ __forceinline__ float sum3(const f32x4 &d) { return (d[0] + d[1]) + d[2]; }

// sum over this lane's four rows of wm[rho] * d[rho]
__device__ __forceinline__ float weighted(const f32x4 &d, const float (&wm)[4])
{
    return fmaf(wm[3], d[3], fmaf(wm[2], d[2], fmaf(wm[1], d[1], wm[0] * d[0])));
}

// One item of the pass: a block of one (layer, head, prompt) unit with everything a workgroup needs to know about
// it, worked out once by plan_kernel so that the pass itself starts an item with one scalar load instead of a
// chain of dependent ones (kernel arguments, per-prompt tables, divisions).
struct TileItem {
    int64_t key_off;                     // element offset of the unit's first row
    int64_t row0;                        // the unit's first row in the planes of a_raw
    int32_t N;                           // tokens of the unit; < 0: this slot of the die's queue is empty
    int32_t blk_lo, blk_hi;              // the block's tokens, unit-local
    int32_t unit;                        // index of the unit's accumulators
    int32_t unblk;                       // blocks of the unit
    int32_t id;                          // (layer, head) * blocks per head + block: what the deferred list holds
    int32_t pad[2];
};
static_assert(sizeof(TileItem) == 48, "items are read as three 16-byte pieces");

// Items in launch order: item i belongs to die i % 8 and is entry i / 8 of that die's queue (the queues of
// scan_kernel in nkv_score_fast.hip without the items that add a unit up: for every (layer, head) in turn the
// die's runs of consecutive blocks).  Also clears the counters and the accumulators and marks the units' sums unwritten.
__global__ __launch_bounds__(256) void plan_kernel(TileItem *__restrict__ items, uint32_t n_items, RowMap km, PromptTab tab,
                                                   ScanPlan plan, int LH, uint4 *sync, size_t n_sync, uint4 *accum, size_t n_accum,
                                                   uint4 *sums, size_t n_sums)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const uint4 zero = make_uint4(0u, 0u, 0u, 0u), none = make_uint4(kUnwritten, kUnwritten, kUnwritten, kUnwritten);
    for (size_t k = i; k < n_sync + n_accum + n_sums; k += (size_t)gridDim.x * blockDim.x) {
        if (k < n_sync) sync[k] = zero;
        else if (k < n_sync + n_accum) accum[k - n_sync] = zero;
        else sums[k - n_sync - n_accum] = none;
    }
    for (size_t k = i; k < n_items; k += (size_t)gridDim.x * blockDim.x) {
        const int x = (int)(k & (kDies - 1));
        const uint32_t t = (uint32_t)(k >> 3);
        const int len = plan.len[x];
        TileItem it;
        it.pad[0] = it.pad[1] = 0;
        const int lh = len > 0 ? (int)(t / (uint32_t)len) : LH;
        if (lh >= LH) {
            it.key_off = it.row0 = 0;
            it.N = -1;
            it.blk_lo = it.blk_hi = it.unit = it.unblk = it.id = 0;
        } else {
            const int r = (int)(t - (uint32_t)lh * (uint32_t)len);
            const int blk = die_block(plan.run, x, r);
            const int p = prompt_of_block(tab, blk);
            const int b = tab.b[p];
            it.N = tab.tok_off[p + 1] - tab.tok_off[p];
            it.blk_lo = (blk - tab.blk_off[p]) * b;
            it.blk_hi = min(it.blk_lo + b, it.N);
            it.key_off = km.unit(lh, p, tab);
            it.row0 = (int64_t)lh * tab.T + tab.tok_off[p];
            it.unit = lh * tab.n + p;
            it.unblk = tab.blk_off[p + 1] - tab.blk_off[p];
            it.id = lh * plan.nblk + blk;
        }
        items[k] = it;
    }
}

// grid: one workgroup of 256 threads per item, in the items' order.  (Resident workgroups that loop over the items
// instead were tried: without the hardware handing out blocks as slots fall free, all workgroups of the chip move
// through their loading and computing phases in step, and the pass takes 0.90 ms instead of 0.77.)
template <int KF> __global__ __launch_bounds__(64 * kTileWaves, 4)
void scan_tile_kernel(const uint8_t *__restrict__ keys, const TileItem *__restrict__ items, float *__restrict__ a_raw,
                      unsigned long long *__restrict__ acc, float *__restrict__ ssum, uint32_t *__restrict__ sync, int64_t rows,
                      int poll_limit)
{
    constexpr int D = 128, NW = kTileWaves, kRowBytes = D * 2;
    __shared__ __attribute__((aligned(16))) uint8_t lds_stage[NW][kStageBytes];   // a wave's group on its way to operand layout, later its anchors
    __shared__ __attribute__((aligned(16))) float lds_T[4 + 16][D];               // group sums: 4 halo groups, then the block's
    __shared__ __attribute__((aligned(16))) float lds_w[NW][5][kGroup];           // 1/||k|| per token of a wave's groups (0: no such token)
    __shared__ __attribute__((aligned(16))) float lds_ss[NW][5][kGroup];          // ||k||^2
    __shared__ __attribute__((aligned(16))) float lds_S[D];                       // the unit's sum, once complete
    __shared__ int s_have;

    const TileItem it = items[blockIdx.x];
    if (it.N < 0) return;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int g = lane >> 4, c = lane & 15;                           // row-wise layout: rows 4g .., dims 8c ..
    const int qq = g, n = c;                                          // operand / result layout: token n, quarter qq
    uint8_t *stage = lds_stage[w];

    const int N = it.N, blk_lo = it.blk_lo, blk_hi = it.blk_hi, unblk = it.unblk;
    const int ng = (blk_hi - blk_lo + kGroup - 1) / kGroup;           // groups of the block, <= 16
    const int64_t row0 = it.row0;                                     // row of the prompt's token 0

    // ---- first touch: this wave's groups, then its group of the halo.  Rows outside the prompt read as zeros. ----
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t *>(keys) + it.key_off * 2, 0, N * kRowBytes, 0x00020000);
    u32x4 raw[5][4];
    bool ex[5];                                                       // group m - 1 of the chain exists (m = 0: halo)
#pragma unroll
    for (int mm = 0; mm < 5; ++mm) {
        const int m = (mm + 1) % 5;                                   // the halo is needed last
        const int q = w + 4 * (m - 1);                                // block-local group index, < 0: halo
        ex[m] = q < ng;
        if (ex[m]) {
            const int off = (blk_lo + kGroup * q + 4 * g) * kRowBytes + 16 * c;
#pragma unroll
            // a full block's last 64 tokens (m = 4) are read again, as the next block's halo, and the halo has just
            // been read by the block in front: those stay in the L2; the other rows are marked non-temporal (aux 2)
            for (int j = 0; j < 4; ++j)
                raw[m][j] = (m >= 1 && m <= 3) ? row_load<KF, 2>(rsrc, off + j * kRowBytes) : row_load<KF>(rsrc, off + j * kRowBytes);
        }
    }

    // ---- the block's own groups: norms and partial sums, nothing else in front of the block total ----
#pragma unroll
    for (int m = 1; m < 5; ++m)
        if (ex[m]) group_sum<KF>(raw[m], blk_lo + kGroup * (w + 4 * (m - 1)), blk_hi, g, c, lds_w[w][m], lds_ss[w][m], lds_T[4 + w + 4 * (m - 1)]);
    __syncthreads();

    // ---- block total = episodic anchor (up to length); lane: dims 2 lane, 2 lane + 1 ----
    unsigned long long *acc_unit = acc + (int64_t)it.unit * D;
    float bsq, b0 = 0.f, b1 = 0.f;
    for (int q = 0; q < ng; ++q) {
        const float2 t2 = *reinterpret_cast<const float2 *>(&lds_T[4 + q][2 * lane]);
        b0 += t2.x;
        b1 += t2.y;
    }
    const bool poster = w == (it.id & (NW - 1));                      // one wave adds the block total to the unit's sum
    unsigned long long after0 = 0ull, after1 = 0ull;                  // the accumulators right after this block's add
    if (poster) {
        const unsigned long long t0 = accum_term(b0), t1 = accum_term(b1);
        after0 = __hip_atomic_fetch_add(acc_unit + 2 * lane, t0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + t0;
        after1 = __hip_atomic_fetch_add(acc_unit + 2 * lane + 1, t1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + t1;
    }
    bsq = sum_over_rows16(row_sum<16>(fmaf(b0, b0, b1 * b1)));

    // ---- the halo group's sum (the window sums in front of the block's first groups need it) ----
    group_sum<KF>(raw[0], blk_lo + kGroup * (w - 4), blk_hi, g, c, lds_w[w][0], lds_ss[w][0], lds_T[w]);

    float *S_unit = ssum + (int64_t)it.unit * D;
    if (poster) {                                                     // (the adds have had the halo group to come back)
        const __amdgpu_buffer_rsrc_t prs = __builtin_amdgcn_make_buffer_rsrc(S_unit, 0, D * 4, 0x00020000);
        constexpr int kNoStore = 0x40000000;
        // the last block to add to a word stores the word's final value; a word's adds take turns, so exactly one does
        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(accum_value(after0)), prs,
                                              accum_complete(after0, unblk) ? 8 * lane : kNoStore, 0, 16);
        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(accum_value(after1)), prs,
                                              accum_complete(after1, unblk) ? 8 * lane + 4 : kNoStore, 0, 16);
    }

    // ---- every group through the staging rows into operand layout ----
    u32x4 X[5][4];
#pragma unroll
    for (int m = 0; m < 5; ++m) {
        if (ex[m]) {
#pragma unroll
            for (int j = 0; j < 4; ++j) *reinterpret_cast<u32x4 *>(stage + (4 * g + j) * kPitch + 16 * c) = raw[m][j];
            __builtin_amdgcn_wave_barrier();
            read_operand(stage, lane, X[m]);
            __builtin_amdgcn_wave_barrier();                          // the next group reuses the staging rows
        }
    }
    stage_anchor<KF>(stage, 4, lane, b0, b1);                             // rows 4 .. 6: the block total's three terms
    __syncthreads();                                                  // the halo groups' sums
    // ---- the chain of this wave's groups ----
    // lane (qq, n) of a result holds rows 4 qq + rho, column n.  Masked weights of the rows: rows j <= n count.
    const __amdgpu_buffer_rsrc_t out_c = __builtin_amdgcn_make_buffer_rsrc(a_raw + 2 * rows + row0, 0, blk_hi * 4, 0x00020000);
    const __amdgpu_buffer_rsrc_t out_e = __builtin_amdgcn_make_buffer_rsrc(a_raw + rows + row0, 0, blk_hi * 4, 0x00020000);
    const __amdgpu_buffer_rsrc_t out_s = __builtin_amdgcn_make_buffer_rsrc(a_raw + row0, 0, blk_hi * 4, 0x00020000);
    constexpr int kNoStore = 0x40000000;                              // an offset past any buffer, also with a block's offset added: the store is dropped
    const int off_q0 = qq == 0 ? 4 * n : kNoStore, off_q1 = qq == 1 ? 4 * n : kNoStore;
    float wm_prev[4], alpha_prev;
    {
        const float4 w4 = *reinterpret_cast<const float4 *>(&lds_w[w][0][4 * qq]);
        const float ww[4] = {w4.x, w4.y, w4.z, w4.w};
#pragma unroll
        for (int rho = 0; rho < 4; ++rho) wm_prev[rho] = 4 * qq + rho <= n ? ww[rho] : 0.f;
        alpha_prev = weighted(tile<KF, 4>(X[0], X[0]), wm_prev);          // halo group: its own triangle only
    }
#pragma unroll
    for (int m = 1; m < 5; ++m) {
        if (ex[m]) {
            const int q = w + 4 * (m - 1);
            // window sum in front of the group = the four groups before it
            float s0, s1;
            {
                const float2 t0 = *reinterpret_cast<const float2 *>(&lds_T[q][2 * lane]);
                const float2 t1 = *reinterpret_cast<const float2 *>(&lds_T[q + 1][2 * lane]);
                const float2 t2 = *reinterpret_cast<const float2 *>(&lds_T[q + 2][2 * lane]);
                const float2 t3 = *reinterpret_cast<const float2 *>(&lds_T[q + 3][2 * lane]);
                s0 = ((t0.x + t1.x) + t2.x) + t3.x;
                s1 = ((t0.y + t1.y) + t2.y) + t3.y;
            }
            const float P0 = sum_over_rows16(row_sum<16>(fmaf(s0, s0, s1 * s1)));
            stage_anchor<KF>(stage, 0, lane, s0, s1);                     // rows 0 .. 2: the seed's three terms
            __builtin_amdgcn_wave_barrier();
            u32x4 An[4];
            read_operand(stage, lane, An);
            __builtin_amdgcn_wave_barrier();                          // the next group rewrites rows 0 .. 2
            const f32x4 AT = tile<KF, 4>(X[m], X[m]);                     // [j in G][i in G]
            const f32x4 XT = tile<KF, 4>(X[m - 1], X[m]);                 // [j' in P][i in G]
            const f32x4 XX = tile<KF, 4>(X[m], X[m - 1]);                 // [j in G][i' in P]
            const f32x4 AG = tile<KF, 4>(An, X[m]);                       // [anchor row][i in G]
            const f32x4 AP = tile<KF, 4>(An, X[m - 1]);                   // [anchor row][i' in P]
            float wm[4];
            {
                const float4 w4 = *reinterpret_cast<const float4 *>(&lds_w[w][m][4 * qq]);
                const float ww[4] = {w4.x, w4.y, w4.z, w4.w};
#pragma unroll
                for (int rho = 0; rho < 4; ++rho) wm[rho] = 4 * qq + rho <= n ? ww[rho] : 0.f;
            }
            const float alpha = weighted(AT, wm);                     // <k_i, entered rows of G>, partial
            const float beta = weighted(XT, wm_prev);                 // <k_i, left rows of P>, partial
            const float gamma = weighted(XX, wm);                     // <k_i', entered rows of G>, partial
            // X[i][i']: row i of this lane's column i' = n sits in lane group n / 4, register n % 4
            float xd = (n & 2) ? ((n & 1) ? XX[3] : XX[2]) : ((n & 1) ? XX[1] : XX[0]);
            xd = (n >> 2) == qq ? xd : 0.f;
            // 1/||k|| (0: no such token) and ||k||^2 of token n of this group and of the one 64 tokens earlier
            const float wn = lds_w[w][m][n], wp = lds_w[w][m - 1][n], ssn = lds_ss[w][m][n], ssp = lds_ss[w][m - 1][n];
            const float c_part = (qq == 0 ? sum3(AG) : 0.f) + (alpha - beta);
            const float e_part = (qq == 0 ? sum3(AP) : 0.f) + (gamma - alpha_prev);
            const float gsum = qq == 0 ? wn * wn * ssn + wp * wp * ssp : 0.f;
            const float d_part = 2.f * (wn * c_part - wp * e_part) + (2.f * wn * wp * xd - gsum);
            const float cdot = sum_over_rows16(c_part);               // <k_i, W_i>
            const float Pn = P0 + row_prefix_sum(sum_over_rows16(d_part));
            const float knn = ssn < 1e-24f ? sqrtf(ssn) * 1e12f : 1.f;
            const float ac = neg_cos(wn * cdot, knn, Pn);
            const float ae = neg_cos(wn * sum3(AG), knn, bsq);        // meaningful in lane group 1 (rows 4 .. 6)
            const int soff = (blk_lo + kGroup * q) * 4;                // (an offset that was past the buffer stays past it)
            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(ac), out_c, off_q0 + soff, 0, 0);
            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(ae), out_e, off_q1 + soff, 0, 0);
#pragma unroll
            for (int rho = 0; rho < 4; ++rho) wm_prev[rho] = wm[rho];
            alpha_prev = alpha;
            __builtin_amdgcn_sched_barrier(0);                        // one group at a time
        }
    }
    // ---- stable dots against the unit's sum ----
    if (w == 0) {                                                     // 32 lanes look, the other waves sit at the barrier
        const __amdgpu_buffer_rsrc_t srs = __builtin_amdgcn_make_buffer_rsrc(S_unit, 0, D * 4, 0x00020000);
        bool got = false;
        for (int polls = 0; poll_limit >= 0; ++polls) {               // poll_limit < 0: defer without looking
            u32x4 sv = {0u, 0u, 0u, 0u};
            if (lane < 32) sv = agent_load16(srs, lane * 16);
            got = __all(all_written(sv));
            if (got) {
                if (lane < 32) *reinterpret_cast<u32x4 *>(&lds_S[4 * lane]) = sv;
                break;
            }
            if (polls >= poll_limit) break;
            __builtin_amdgcn_s_sleep(8);
        }
        if (lane == 0) {
            s_have = got ? 1 : 0;
            if (!got) sync[kSyncWords + atomicAdd(sync + kDeferCountWord, 1u)] = (uint32_t)it.id;
        }
    }
    __syncthreads();
    if (s_have != 0) {
        float2 s2 = *reinterpret_cast<const float2 *>(&lds_S[2 * lane]);
        if constexpr (KF == kKeyF16) { s2.x *= 0.25f; s2.y *= 0.25f; }   // a sum over 65 536 unit vectors stays inside fp16's range; the cosine does not see the factor
        const float ssq = sum_over_rows16(row_sum<16>(fmaf(s2.x, s2.x, s2.y * s2.y)));
        stage_anchor<KF>(stage, 0, lane, s2.x, s2.y);
        __builtin_amdgcn_wave_barrier();
        u32x4 An[4];
        read_operand(stage, lane, An);
#pragma unroll
        for (int m = 1; m < 5; ++m) {
            if (ex[m]) {
                const int q = w + 4 * (m - 1);
                const f32x4 AS = tile<KF, 4>(An, X[m]);
                const float wn = lds_w[w][m][n], ssn = lds_ss[w][m][n];
                const float knn = ssn < 1e-24f ? sqrtf(ssn) * 1e12f : 1.f;
                const float as = neg_cos(wn * sum3(AS), knn, ssq);
                __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(as), out_s, off_q0 + (blk_lo + kGroup * q) * 4, 0, 0);
            }
        }
    }
}

// a_s of the blocks whose workgroups did not wait for their unit's sum: the same operands (loaded in operand
// layout directly), norms, split and product as in scan_tile_kernel, so the values are the ones it would have
// stored.
template <int KF>
__global__ __launch_bounds__(64 * kTileWaves) void deferred_stable_tile_kernel(const uint8_t *__restrict__ keys, RowMap km,
                                                                               PromptTab tab,
                                                                               const float *__restrict__ ssum,
                                                                               const uint32_t *__restrict__ sync,
                                                                               float *__restrict__ a_raw)
{
    constexpr int D = 128, NW = kTileWaves, kRowBytes = D * 2;
    __shared__ __attribute__((aligned(16))) uint8_t lds_stage[NW][kStageBytes];
    __shared__ __attribute__((aligned(16))) float lds_w[NW][kGroup], lds_ss[NW][kGroup];
    const int nblk = tab.blk_off[tab.n];
    const uint32_t count = sync[kDeferCountWord];
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int qq = lane >> 4, n = lane & 15, g = qq, c = n;
    uint8_t *stage = lds_stage[w];
    constexpr int kNoStore = 0x40000000;
    const int off_q0 = qq == 0 ? 4 * n : kNoStore;
    for (uint32_t i = blockIdx.x; i < count; i += gridDim.x) {
        const int id = (int)sync[kSyncWords + i], lh = id / nblk, blk = id - lh * nblk;
        const int p = prompt_of_block(tab, blk);
        const int b = tab.b[p], N = tab.tok_off[p + 1] - tab.tok_off[p];
        const int blk_lo = (blk - tab.blk_off[p]) * b, blk_hi = min(blk_lo + b, N);
        const int ng = (blk_hi - blk_lo + kGroup - 1) / kGroup;
        const int64_t row0 = (int64_t)lh * tab.T + tab.tok_off[p];
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint8_t *>(keys) + km.unit(lh, p, tab) * 2, 0, N * kRowBytes, 0x00020000);
        const __amdgpu_buffer_rsrc_t out_s = __builtin_amdgcn_make_buffer_rsrc(a_raw + row0, 0, blk_hi * 4, 0x00020000);
        // every word of the unit's sum has been stored by now (the pass has ended)
        float2 s2 = *reinterpret_cast<const float2 *>(ssum + ((int64_t)lh * tab.n + p) * D + 2 * lane);
        if constexpr (KF == kKeyF16) { s2.x *= 0.25f; s2.y *= 0.25f; }   // as in scan_tile_kernel
        const float ssq = sum_over_rows16(row_sum<16>(fmaf(s2.x, s2.x, s2.y * s2.y)));
        __builtin_amdgcn_wave_barrier();                              // the previous block's reads of the staged rows
        stage_anchor<KF>(stage, 0, lane, s2.x, s2.y);
        __builtin_amdgcn_wave_barrier();
        u32x4 An[4];
        read_operand(stage, lane, An);
        for (int q = w; q < ng; q += 4) {
            const int tok0 = blk_lo + kGroup * q;
            u32x4 raw[4], X[4];                                       // the group row-wise (norms) and as an operand
            const int roff = (tok0 + 4 * g) * kRowBytes + 16 * c, off = (tok0 + n) * kRowBytes + 16 * qq;
#pragma unroll
            for (int j = 0; j < 4; ++j) raw[j] = row_load<KF>(rsrc, roff + j * kRowBytes);
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) X[kk] = row_load<KF>(rsrc, off + 64 * kk);
            float ww[4];
            group_norms<KF>(raw, tok0, blk_hi, g, c, lds_w[w], lds_ss[w], ww);
            __builtin_amdgcn_wave_barrier();
            const float wn = lds_w[w][n], ss = lds_ss[w][n];
            __builtin_amdgcn_wave_barrier();                          // the next group rewrites them
            const float knn = ss < 1e-24f ? sqrtf(ss) * 1e12f : 1.f;
            const f32x4 AS = tile<KF, 4>(An, X);
            const float as = neg_cos(wn * sum3(AS), knn, ssq);
            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(as), out_s, off_q0 + tok0 * 4, 0, 0);
        }
    }
}

int resident_tile_workgroups()
{
    static int cached = -1;                                          // benign if raced
    if (cached < 0) {
        int per_cu = 0, dev = 0;
        hipDeviceProp_t prop;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, scan_tile_kernel<kKeyBF16>, 64 * kTileWaves, 0) != hipSuccess ||
            hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess)
            return 0;
        cached = per_cu * prop.multiProcessorCount;
    }
    return cached;
}

}  // namespace

bool tile_score_supported(int dtype, int d, int window, const PromptTab &tab, int LH)
{
    if ((dtype != NKV_DTYPE_BF16 && dtype != NKV_DTYPE_F16) || d != 128 || window != 64) return false;
    int max_unit_blocks = 0;
    for (int p = 0; p < tab.n; ++p) {
        if (tab.b[p] > 256) return false;
        if ((int64_t)(tab.tok_off[p + 1] - tab.tok_off[p] + 256) * d * 2 >= (1ll << 31)) return false;
        max_unit_blocks = max(max_unit_blocks, tab.blk_off[p + 1] - tab.blk_off[p]);
    }
    const int64_t items = (int64_t)LH * (tab.blk_off[tab.n] + tab.n);
    // A unit's blocks have to be resident together, and from a quarter of the chip's resident workgroups per unit on
    // (prompts of more than 65 536 tokens) the vector formulation, three workgroups per CU and no returning atomics in
    // front of a barrier, copes better with workgroups that wait for their unit (131 072 tokens: 4.2 against 4.8 ms).
    return items < (1ll << 28) && max_unit_blocks <= min(resident_tile_workgroups() / 4, kMaxUnitBlocks);
}

size_t tile_score_plan_bytes(int LH, const PromptTab &tab)
{
    ScanPlan plan;
    return (size_t)fill_scan_plan(LH, tab, 1, &plan, false) * sizeof(TileItem);
}

hipError_t launch_score_tile(const void *keys, const RowMap &km, int dtype, int LH, const PromptTab &tab, float *a_raw,
                             void *accum, float *ssum, void *sync_area, void *plan_area, int mode, const Prof &prof,
                             hipStream_t st)
{
    constexpr int D = 128;
    const bool defer_all = mode == kScanDeferAll || mode == kScanRepairAll;   // no unit is added up by a workgroup of its own here
    const size_t na = (size_t)LH * tab.n * D * 8 / 16;                        // accumulators, in 16-byte pieces
    ScanPlan plan;
    const unsigned n_items = fill_scan_plan(LH, tab, km.H, &plan, false);
    plan_kernel<<<(unsigned)min(((size_t)n_items + 255) / 256, (size_t)2048), 256, 0, st>>>(
        (TileItem *)plan_area, n_items, km, tab, plan, LH, (uint4 *)sync_area, kSyncWords / 4, (uint4 *)accum, na, (uint4 *)ssum,
        na / 2);
    const unsigned n_deferred = defer_all ? 4096 : 256;
    prof.begin(NKV_KERNEL_SCAN, st);
    if (dtype == NKV_DTYPE_F16)
        scan_tile_kernel<kKeyF16><<<n_items, 64 * kTileWaves, 0, st>>>((const uint8_t *)keys, (const TileItem *)plan_area, a_raw,
                                                                      (unsigned long long *)accum, ssum, (uint32_t *)sync_area,
                                                                      (int64_t)LH * tab.T, defer_all ? -1 : kPollLimit);
    else
        scan_tile_kernel<kKeyBF16><<<n_items, 64 * kTileWaves, 0, st>>>((const uint8_t *)keys, (const TileItem *)plan_area, a_raw,
                                                                       (unsigned long long *)accum, ssum, (uint32_t *)sync_area,
                                                                       (int64_t)LH * tab.T, defer_all ? -1 : kPollLimit);
    prof.end(NKV_KERNEL_SCAN, st);
    if (dtype == NKV_DTYPE_F16)
        deferred_stable_tile_kernel<kKeyF16><<<n_deferred, 64 * kTileWaves, 0, st>>>((const uint8_t *)keys, km, tab, ssum,
                                                                                    (const uint32_t *)sync_area, a_raw);
    else
        deferred_stable_tile_kernel<kKeyBF16><<<n_deferred, 64 * kTileWaves, 0, st>>>((const uint8_t *)keys, km, tab, ssum,
                                                                                     (const uint32_t *)sync_area, a_raw);
    return hipGetLastError();
}

}  // namespace nkv
