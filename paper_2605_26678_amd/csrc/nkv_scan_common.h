// Pieces shared by the streaming scoring kernels (gfx950): packed key rows and their loads, cross-lane
// reductions, and the protocol of the fused pass (self-validating block totals and unit sums, the dies' queues,
// the summing of a unit).  See nkv_score_fast.hip for how the pass uses them.
#pragma once

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

// ---- transposing butterfly ---------------------------------------------------------------------------
// merge_k(x, y): lanes whose bit k of the lane index is 0 receive x + x(partner), the others y + y(partner),
// partner = lane ^ (1 << k).  Two values go in, one comes out, and which of the two a lane keeps is decided
// by one bit of its index; after log2(LPR) merges lane c holds the complete sum of the value with index c.
//
// Bits 2 and 3 use DPP row rotations with a bank mask (a bank is 4 lanes): the first add is written by all
// lanes, the second only by the banks whose lanes keep x.  row_ror:n hands lane i the value of lane
// (i - n) mod 16.  The compiler does not track DPP read-after-write hazards inside inline assembly; the
// leading s_nop covers inputs written by the instruction just before the block, and inside a block no DPP
// source is written by the block itself.
__device__ __forceinline__ void merge_bit2_x4(float (&r)[4], float x0, float x1, float x2, float x3, float y0,
                                              float y1, float y2, float y3)
{
    asm("s_nop 1\n\t"
        "v_add_f32_dpp %0, %8, %8 row_ror:4 row_mask:0xf bank_mask:0xf\n\t"
        "v_add_f32_dpp %1, %9, %9 row_ror:4 row_mask:0xf bank_mask:0xf\n\t"
        "v_add_f32_dpp %2, %10, %10 row_ror:4 row_mask:0xf bank_mask:0xf\n\t"
        "v_add_f32_dpp %3, %11, %11 row_ror:4 row_mask:0xf bank_mask:0xf\n\t"
        "v_add_f32_dpp %0, %4, %4 row_ror:12 row_mask:0xf bank_mask:0x5\n\t"
        "v_add_f32_dpp %1, %5, %5 row_ror:12 row_mask:0xf bank_mask:0x5\n\t"
        "v_add_f32_dpp %2, %6, %6 row_ror:12 row_mask:0xf bank_mask:0x5\n\t"
        "v_add_f32_dpp %3, %7, %7 row_ror:12 row_mask:0xf bank_mask:0x5"
        : "=&v"(r[0]), "=&v"(r[1]), "=&v"(r[2]), "=&v"(r[3])
        : "v"(x0), "v"(x1), "v"(x2), "v"(x3), "v"(y0), "v"(y1), "v"(y2), "v"(y3));
}

__device__ __forceinline__ void merge_bit3_x4(float (&r)[4], float x0, float x1, float x2, float x3, float y0,
                                              float y1, float y2, float y3)
{
    asm("s_nop 1\n\t"
        "v_add_f32_dpp %0, %8, %8 row_ror:8 row_mask:0xf bank_mask:0xf\n\t"
        "v_add_f32_dpp %1, %9, %9 row_ror:8 row_mask:0xf bank_mask:0xf\n\t"
        "v_add_f32_dpp %2, %10, %10 row_ror:8 row_mask:0xf bank_mask:0xf\n\t"
        "v_add_f32_dpp %3, %11, %11 row_ror:8 row_mask:0xf bank_mask:0xf\n\t"
        "v_add_f32_dpp %0, %4, %4 row_ror:8 row_mask:0xf bank_mask:0x3\n\t"
        "v_add_f32_dpp %1, %5, %5 row_ror:8 row_mask:0xf bank_mask:0x3\n\t"
        "v_add_f32_dpp %2, %6, %6 row_ror:8 row_mask:0xf bank_mask:0x3\n\t"
        "v_add_f32_dpp %3, %7, %7 row_ror:8 row_mask:0xf bank_mask:0x3"
        : "=&v"(r[0]), "=&v"(r[1]), "=&v"(r[2]), "=&v"(r[3])
        : "v"(x0), "v"(x1), "v"(x2), "v"(x3), "v"(y0), "v"(y1), "v"(y2), "v"(y3));
}

// Bits 0 and 1 stay inside a quad, below the granularity of a bank mask: select, then one DPP add.
__device__ __forceinline__ float merge_bit0(float x, float y)
{
    const bool hi = (threadIdx.x & 1) != 0;
    const float keep = hi ? y : x, send = hi ? x : y;
    return keep + dpp_mov<0xB1>(send);
}
__device__ __forceinline__ float merge_bit1(float x, float y)
{
    const bool hi = (threadIdx.x & 2) != 0;
    const float keep = hi ? y : x, send = hi ? x : y;
    return keep + dpp_mov<0x4E>(send);
}

// Four values whose indices differ in bits 0 and 1 -> the one value of this lane.
__device__ __forceinline__ float merge_low4(const float (&b)[4])
{
    return merge_bit1(merge_bit0(b[0], b[1]), merge_bit0(b[2], b[3]));
}

// v[j], j < LPR: partial sums of row j held by this lane.  Returns the full sum of row c = lane % LPR.
template <int LPR> __device__ __forceinline__ float transpose_reduce(const float (&v)[LPR])
{
    float a[4];
    merge_bit2_x4(a, v[0], v[1], v[2], v[3], v[4], v[5], v[6], v[7]);
    if constexpr (LPR == 16) {
        float a2[4], b[4];
        merge_bit2_x4(a2, v[8], v[9], v[10], v[11], v[12], v[13], v[14], v[15]);
        merge_bit3_x4(b, a[0], a[1], a[2], a[3], a2[0], a2[1], a2[2], a2[3]);
        return merge_low4(b);
    } else {
        return merge_low4(a);
    }
}

// The same butterfly fed four rows at a time (rows 4s .. 4s+3 in step s), so that a loop that produces
// its rows in order never holds more than eight partial values per quantity.
template <int LPR> struct StreamReduce {
    float hold[4], half[4];
    template <int S> __device__ __forceinline__ void push(const float (&p)[4], float &out)
    {
        if constexpr (S == 0 || S == 2) {
#pragma unroll
            for (int i = 0; i < 4; ++i) hold[i] = p[i];
        } else if constexpr (S == 1) {
            merge_bit2_x4(half, hold[0], hold[1], hold[2], hold[3], p[0], p[1], p[2], p[3]);
            if constexpr (LPR == 8) out = merge_low4(half);
        } else {
            float a2[4], b[4];
            merge_bit2_x4(a2, hold[0], hold[1], hold[2], hold[3], p[0], p[1], p[2], p[3]);
            merge_bit3_x4(b, half[0], half[1], half[2], half[3], a2[0], a2[1], a2[2], a2[3]);
            out = merge_low4(b);
        }
    }
};

using u32x4 = unsigned int __attribute__((ext_vector_type(4)));

using u32x2 = unsigned int __attribute__((ext_vector_type(2)));
using f32x2 = float __attribute__((ext_vector_type(2)));

// Key formats of the streaming kernels (template parameter KF).  A lane's packed row piece holds eight values of
// a row: 16 bytes of bf16 or fp16, or 8 bytes of 8-bit E4M3 (4 exponent bits, bias 7, no infinities).  It stays
// packed in registers and in LDS from the first touch to the last; only the load, unpacking and the sum of
// squares know the format.
constexpr int kKeyF8 = 1, kKeyBF16 = 2, kKeyF16 = 3;
template <int KF> constexpr int key_bytes() { return KF == kKeyF8 ? 1 : 2; }
template <int KF> struct PieceOf { using type = u32x4; };
template <> struct PieceOf<kKeyF8> { using type = u32x2; };
template <int KF> using Piece = typename PieceOf<KF>::type;

// Load of a row piece through a buffer descriptor: the address is one 32-bit byte offset per lane plus an
// immediate, and an offset outside [0, num_records) (tokens before the prompt or past its end) reads zeros.
// AUX: cache policy bits of the instruction (0: default, 2: non-temporal, for rows nobody reads again).
template <int KF, int AUX = 0> __device__ __forceinline__ Piece<KF> row_load(__amdgpu_buffer_rsrc_t rsrc, int byte_off)
{
    if constexpr (KF == kKeyF8) return __builtin_amdgcn_raw_buffer_load_b64(rsrc, byte_off, 0, AUX);
    else return __builtin_amdgcn_raw_buffer_load_b128(rsrc, byte_off, 0, AUX);
}

using f16x2 = _Float16 __attribute__((ext_vector_type(2)));

// 8-bit keys: the hardware's pairwise E4M3 -> fp32 conversion, exact.
__device__ __forceinline__ void unpack8_f8(const u32x2 &r, float k[8])
{
    const f32x2 a = __builtin_amdgcn_cvt_pk_f32_fp8((int)r.x, false), b = __builtin_amdgcn_cvt_pk_f32_fp8((int)r.x, true);
    const f32x2 c = __builtin_amdgcn_cvt_pk_f32_fp8((int)r.y, false), d = __builtin_amdgcn_cvt_pk_f32_fp8((int)r.y, true);
    k[0] = a.x; k[1] = a.y; k[2] = b.x; k[3] = b.y; k[4] = c.x; k[5] = c.y; k[6] = d.x; k[7] = d.y;
}

template <int KF> __device__ __forceinline__ void unpack8(const Piece<KF> &r, float k[8])
{
    if constexpr (KF == kKeyF8) {
        unpack8_f8(r, k);
    } else if constexpr (KF == kKeyF16) {
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

// Sum of the squares of the eight bf16 values of a packed row piece: four dot-product instructions, each
// adding two exact bf16 x bf16 products to an fp32 accumulator.
template <int KF> __device__ __forceinline__ float sumsq8(const Piece<KF> &r)
{
    float acc = 0.f;
    if constexpr (KF == kKeyF8) {
        float k[8];
        unpack8_f8(r, k);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc = fmaf(k[e], k[e], acc);
    } else if constexpr (KF == kKeyF16)
        asm("v_dot2c_f32_f16 %0, %1, %1\n\t"
            "v_dot2c_f32_f16 %0, %2, %2\n\t"
            "v_dot2c_f32_f16 %0, %3, %3\n\t"
            "v_dot2c_f32_f16 %0, %4, %4"
            : "+v"(acc)
            : "v"(r.x), "v"(r.y), "v"(r.z), "v"(r.w));
    else
        asm("v_dot2c_f32_bf16 %0, %1, %1\n\t"
            "v_dot2c_f32_bf16 %0, %2, %2\n\t"
            "v_dot2c_f32_bf16 %0, %3, %3\n\t"
            "v_dot2c_f32_bf16 %0, %4, %4"
            : "+v"(acc)
            : "v"(r.x), "v"(r.y), "v"(r.z), "v"(r.w));
    return acc;
}

// The same for a value that compiler-generated DPP instructions read next: the compiler does not see the
// write inside the assembly, so the two wait states a DPP read needs after it are spent here.
template <int KF> __device__ __forceinline__ float sumsq8_for_dpp(const Piece<KF> &r)
{
    float acc = 0.f;
    if constexpr (KF == kKeyF8) {                                     // plain code: the compiler sees the hazard itself
        float k[8];
        unpack8_f8(r, k);
#pragma unroll
        for (int e = 0; e < 8; ++e) acc = fmaf(k[e], k[e], acc);
    } else if constexpr (KF == kKeyF16)
        asm("v_dot2c_f32_f16 %0, %1, %1\n\t"
            "v_dot2c_f32_f16 %0, %2, %2\n\t"
            "v_dot2c_f32_f16 %0, %3, %3\n\t"
            "v_dot2c_f32_f16 %0, %4, %4\n\t"
            "s_nop 1"
            : "+v"(acc)
            : "v"(r.x), "v"(r.y), "v"(r.z), "v"(r.w));
    else
        asm("v_dot2c_f32_bf16 %0, %1, %1\n\t"
            "v_dot2c_f32_bf16 %0, %2, %2\n\t"
            "v_dot2c_f32_bf16 %0, %3, %3\n\t"
            "v_dot2c_f32_bf16 %0, %4, %4\n\t"
            "s_nop 1"
            : "+v"(acc)
            : "v"(r.x), "v"(r.y), "v"(r.z), "v"(r.w));
    return acc;
}

// Makes the compiler forget what it knows about a packed row, so that the unpacked floats of one phase
// are not kept alive (8 registers per token) for the next phase; costs no instruction.
__device__ __forceinline__ void forget(u32x4 &r) { asm volatile("" : "+v"(r.x), "+v"(r.y), "+v"(r.z), "+v"(r.w)); }
__device__ __forceinline__ void forget(u32x2 &r) { asm volatile("" : "+v"(r.x), "+v"(r.y)); }

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

// -cos from <k_hat, anchor>, ||k_hat|| and ||anchor||^2, norms clamped at 1e-12: the hardware's reciprocal
// and reciprocal square root (1 ulp each) instead of a division and a square root.
__device__ __forceinline__ float neg_cos(float dot_scaled, float knorm, float anchor_sq)
{
    return -dot_scaled * __builtin_amdgcn_rcpf(fmaxf(knorm, kEps)) * __builtin_amdgcn_rsqf(fmaxf(anchor_sq, kEps * kEps));
}

// ---- self-validating words (fused path) ----------------------------------------------------------------
// Block totals and unit sums are finite floats; memory that still holds kUnwritten has not been stored to.
// Validity is judged per 32-bit word, the unit every store writes atomically.
constexpr uint32_t kUnwritten = 0xFFFFFFFFu;

// 16-byte agent-scope accesses through a buffer descriptor (cache policy bit 4 = sc1 on gfx94x/gfx950): they
// go to the level of the memory hierarchy that all compute units of the device share.
// The compiler barrier keeps a polling loop from having its load hoisted: to the compiler the intrinsic is a
// plain read of memory this thread never writes.
__device__ __forceinline__ u32x4 agent_load16(__amdgpu_buffer_rsrc_t rsrc, int byte_off)
{
    asm volatile("" ::: "memory");
    return __builtin_amdgcn_raw_buffer_load_b128(rsrc, byte_off, 0, 16);
}
__device__ __forceinline__ void agent_store16(__amdgpu_buffer_rsrc_t rsrc, int byte_off, float a, float b, float c,
                                              float d)
{
    const u32x4 v = {__float_as_uint(a), __float_as_uint(b), __float_as_uint(c), __float_as_uint(d)};
    __builtin_amdgcn_raw_buffer_store_b128(v, rsrc, byte_off, 0, 16);
}
__device__ __forceinline__ bool all_written(const u32x4 &v)
{
    return v.x != kUnwritten && v.y != kUnwritten && v.z != kUnwritten && v.w != kUnwritten;
}

constexpr int kMaxChunks = 4;                    // chunks per block: block size <= 256
constexpr uint32_t kSpinLimit = 1u << 13;        // polls of a summing workgroup before it gives up (~20 ms); the
                                                 // unit's sum is then formed after the pass
constexpr int kPollLimit = 48;                   // polls of a block's workgroup before it defers its a_s (~0.1 ms)
constexpr int kDies = 8;                         // queues (one per XCD of an MI355X)

// Sync area of the fused path (the first kSyncWords are zero before the launch), in 32-bit words.
constexpr int kTimeoutWord = 0;                  // summing workgroups that gave up (never, in practice)
constexpr int kDeferCountWord = 1;               // blocks on the list
constexpr int kSyncWords = 32;                   // the list (one word per block) follows

// The blocks of a (layer, head) are dealt to the dies in runs of consecutive blocks, round-robin: runs keep a
// block's halo on the die of the block before it, dealing them round-robin gives every die the same mix of
// prompts when a batch holds prompts of different lengths.  A run is at most 16 blocks, and as long as it can
// be for the blocks to go round the dies a whole number of times (160 blocks: twice round in runs of 10, not
// once in runs of 16 with two more runs left over for the first two dies).
__host__ __device__ __forceinline__ int run_length(int nblk)
{
    const int rounds = (nblk + 16 * kDies - 1) / (16 * kDies);
    const int r = (nblk + rounds * kDies - 1) / (rounds * kDies);
    return r < 1 ? 1 : r;
}
// number of blocks of one (layer, head) that belong to die x
__host__ __device__ __forceinline__ int die_blocks(int nblk, int run, int x)
{
    const int cycles = nblk / (run * kDies), rem = nblk - cycles * run * kDies;
    return cycles * run + min(max(rem - x * run, 0), run);
}
// the r-th of them
__device__ __forceinline__ int die_block(int run, int x, int r) { return ((r / run) * kDies + x) * run + r % run; }

// Queue of die x: for lh = 0, 1, ...: if lh % kDies == x one "add the unit up" item per prompt (in front, so
// that the summing workgroups are already polling when the unit's last block totals arrive), then the len
// blocks of its segment.  First item of lh in that queue:
__host__ __device__ __forceinline__ uint32_t queue_start(int lh, int len, int n_prompts, int x)
{
    return (uint32_t)lh * (uint32_t)len + (uint32_t)n_prompts * ((uint32_t)(lh + kDies - 1 - x) / kDies);
}

// Constants of one launch of the fused pass, worked out on the host so that a workgroup finds its item without
// integer divisions (each costs a few hundred cycles in front of the workgroup's first load).
struct ScanPlan {
    int32_t nblk, run;
    int32_t len[kDies];                  // blocks of a (layer, head) that belong to each die
    float inv_items[kDies];              // kDies / (kDies * len + prompts): items of a die's queue per (layer, head), inverted
    float inv_run, inv_H;
};

// a / b for 0 <= a < 2^24, b >= 1, with 1 / b at hand
__device__ __forceinline__ int div_by(int a, int b, float inv_b)
{
    int q = (int)((float)a * inv_b);
    if (q * b > a) --q;
    else if ((q + 1) * b <= a) ++q;
    return q;
}

// Adds the block totals of one (layer, head, prompt) unit up and stores the unit's sum; called by a whole
// workgroup of 64 * NW threads.  thread = (slice, 4 dims): slice s adds blocks s, s + NS, s + 2 NS, ... in that
// order, then the slices are added in order, so the order of the additions depends on the shape only and
// every caller gets the same bits.  WAIT: the block totals may still be on their way; a thread keeps polling
// the words it has not seen written yet, at most spin_limit times (0: do not even look), and if any thread
// gives up nothing is stored and the call returns false.  part: LDS, 64 * NW / (D / 4) * D floats.
template <int D, int NW, bool WAIT>
__device__ __forceinline__ bool add_unit_up(const float *bsum_unit, int unblk, float *ssum_unit, float *part,
                                            uint32_t spin_limit)
{
    const __amdgpu_buffer_rsrc_t brs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(bsum_unit), 0,
                                                                         unblk * D * 4, 0x00020000);
    constexpr int VPR = D / 4, NS = 64 * NW / VPR, KB = 16;
    const int vec = threadIdx.x % VPR, slice = threadIdx.x / VPR;
    float4 tot = make_float4(0.f, 0.f, 0.f, 0.f);
    uint32_t spins = 0;
    bool gave_up = WAIT && spin_limit == 0u;
    for (int b0 = slice; b0 < unblk && !gave_up; b0 += KB * NS) {
        u32x4 v[KB];
#pragma unroll
        for (int i = 0; i < KB; ++i) v[i] = u32x4{kUnwritten, kUnwritten, kUnwritten, kUnwritten};
        for (;;) {
            bool ok = true;
#pragma unroll
            for (int i = 0; i < KB; ++i)                              // blocks past the end read as zeros
                if (!all_written(v[i])) v[i] = agent_load16(brs, ((b0 + i * NS) * D + vec * 4) * 4);
            if (!WAIT) break;
#pragma unroll
            for (int i = 0; i < KB; ++i) ok = ok && all_written(v[i]);
            if (ok) break;
            if (++spins > spin_limit) {
                gave_up = true;
                break;
            }
            __builtin_amdgcn_s_sleep(4);
        }
#pragma unroll
        for (int i = 0; i < KB; ++i) {
            tot.x += __uint_as_float(v[i].x); tot.y += __uint_as_float(v[i].y);
            tot.z += __uint_as_float(v[i].z); tot.w += __uint_as_float(v[i].w);
        }
    }
    if (WAIT && __syncthreads_or(gave_up)) return false;
    reinterpret_cast<float4 *>(part)[slice * VPR + vec] = tot;
    __syncthreads();
    if (threadIdx.x < VPR) {
        float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int sl = 0; sl < NS; ++sl) {
            const float4 q = reinterpret_cast<const float4 *>(part)[sl * VPR + vec];
            t.x += q.x; t.y += q.y; t.z += q.z; t.w += q.w;
        }
        const __amdgpu_buffer_rsrc_t out = __builtin_amdgcn_make_buffer_rsrc(ssum_unit, 0, D * 4, 0x00020000);
        agent_store16(out, vec * 16, t.x, t.y, t.z, t.w);
    }
    return true;
}

// The constants of one launch of the fused pass; returns the number of workgroups to launch (the longest of the
// dies' queues, times the number of dies).
inline unsigned fill_scan_plan(int LH, const PromptTab &tab, int H, ScanPlan *plan, bool sum_items = true)
{
    const int nsum = sum_items ? tab.n : 0;                           // "add the unit up" items per (layer, head)
    plan->nblk = tab.blk_off[tab.n];
    plan->run = run_length(plan->nblk);
    plan->inv_run = 1.0f / (float)plan->run;
    plan->inv_H = 1.0f / (float)H;
    uint32_t longest = 0;
    for (int x = 0; x < kDies; ++x) {                                 // 8 queues of (nearly) equal length, interleaved
        plan->len[x] = die_blocks(plan->nblk, plan->run, x);
        plan->inv_items[x] = (float)kDies / (float)(kDies * plan->len[x] + nsum);
        const uint32_t items = queue_start(LH, plan->len[x], nsum, x);
        longest = items > longest ? items : longest;
    }
    return longest * kDies;
}

// The unit's sum for a kernel that runs after the pass.  If the pass left it unwritten (its summing workgroup gave
// up waiting, which the scheduling of workgroups makes possible in principle) the calling workgroup -- all of its
// 64 * NW threads -- forms it now from the block totals, with the additions in the pass's order; several
// workgroups doing so at once store the same bits.  Afterwards the sum is to be read with agent-scope loads.
// part: LDS as for add_unit_up.
template <int D, int NW>
__device__ __forceinline__ void ensure_unit_sum(const float *bsum_unit, int unblk, float *ssum_unit, float *part)
{
    const __amdgpu_buffer_rsrc_t srs = __builtin_amdgcn_make_buffer_rsrc(ssum_unit, 0, D * 4, 0x00020000);
    bool missing = false;
    if (threadIdx.x < D / 4) missing = !all_written(agent_load16(srs, threadIdx.x * 16));
    if (!__syncthreads_or(missing)) return;
    add_unit_up<D, NW, false>(bsum_unit, unblk, ssum_unit, part, 0u);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
}

// ---- self-counting accumulators (matrix-core pass) -------------------------------------------------------
// The unit's sum as 64-bit integers, one per head dimension: every block adds (its total in 2^-31 fixed point)
// * 2^12 + 1 with one integer atomic per dimension, so the low 12 bits of a word count the blocks that have
// added to it and a word is complete when they equal the unit's number of blocks.  Integer additions commute:
// the sum does not depend on the order the blocks arrive in, and nothing has to be ordered or fenced -- every
// word says by itself whether it is complete.  Range: a component of a normalised key is at most 1, so
// |total| <= 256 per block and |sum| < 2^20 for the at most 4095 blocks of a unit: 20 + 31 bits and the sign
// above the 12 count bits fill the word exactly.
constexpr int kCountBits = 12;
constexpr int kMaxUnitBlocks = (1 << kCountBits) - 1;
constexpr int kAccumFrac = 31;                   // fraction bits of the fixed-point sum

// what a block adds for its total v
__device__ __forceinline__ unsigned long long accum_term(float v)
{
    const float fl = floorf(v);                                      // v - floor(v) is exact in fp32
    const long long hi = (long long)(int)fl;
    const long long lo = (long long)(uint32_t)((v - fl) * (float)(1u << kAccumFrac));   // < 2^31, truncated
    const long long q = hi * (1ll << kAccumFrac) + lo;               // v in units of 2^-31
    return ((unsigned long long)q << kCountBits) + 1ull;
}
__device__ __forceinline__ bool accum_complete(unsigned long long a, int blocks) { return (int)(a & kMaxUnitBlocks) == blocks; }
// the sum, rounded once to fp32
__device__ __forceinline__ float accum_value(unsigned long long a)
{
    const long long q = (long long)a >> kCountBits;                  // arithmetic shift: units of 2^-31
    const double d = (double)(int)(q >> 32) * 4294967296.0 + (double)(uint32_t)q;
    return (float)(d * (1.0 / (double)(1u << kAccumFrac)));
}

// What the fused pass expects to find in memory, in one launch: counters at zero, block totals and unit sums
// "unwritten".  16-byte stores, grid-stride over the three areas one after the other.
__global__ __launch_bounds__(256) void prepare_kernel(uint4 *sync, size_t n_sync, uint4 *bsum, size_t n_bsum,
                                                      uint4 *ssum, size_t n_ssum)
{
    const uint4 zero = make_uint4(0u, 0u, 0u, 0u);
    const uint4 none = make_uint4(kUnwritten, kUnwritten, kUnwritten, kUnwritten);
    const size_t total = n_sync + n_bsum + n_ssum;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        if (i < n_sync) sync[i] = zero;
        else if (i < n_sync + n_bsum) bsum[i - n_sync] = none;
        else ssum[i - n_sync - n_bsum] = none;
    }
}

}  // namespace
}  // namespace nkv
