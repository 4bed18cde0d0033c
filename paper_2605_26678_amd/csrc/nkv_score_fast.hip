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
template <int KF> __device__ __forceinline__ Piece<KF> row_load(__amdgpu_buffer_rsrc_t rsrc, int byte_off)
{
    if constexpr (KF == kKeyF8) return __builtin_amdgcn_raw_buffer_load_b64(rsrc, byte_off, 0, 0);
    else return __builtin_amdgcn_raw_buffer_load_b128(rsrc, byte_off, 0, 0);
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
constexpr uint32_t kSpinLimit = 1u << 22;        // polls of a summing workgroup before it gives up (~seconds)
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
#pragma unroll
    for (int j = 0; j < TPT; ++j) raw[j] = row_load<KF>(rsrc, lane_off + j * kRowBytes);
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

// ---- matrix-core formulation of the same pass ----------------------------------------------------------
// Every dot product of the pass is a row of a matrix product with bf16 inputs, which the matrix cores form
// exactly (bf16 x bf16 products, fp32 sums):
//   current window   <k_t, sum_{s in [t-63, t]} w_s k_s> = sum_s w_s G[t][s] with the Gram matrix G = K K^T of
//                    the raw keys and w_s = 1 / ||k_s||: a weighted sum over a 64-wide band of G.  The square of
//                    the window sum's norm follows the window: P_t = P_{t-1} + 2 c_t - g_t - (2 f_q - g_q),
//                    q = t - 64, with c_t = <k^_t, window sum at t>, f_q = <k^_q, sum of k^_q .. k^_{q+63}> (the
//                    same band, forwards) and g = ||k^||^2; P at the token in front of the chunk is the sum over
//                    a 64 x 64 square of G, which the forward band's pieces add up to.
//   chunk sums       sum_s w_s k_s, needed as a vector: a product with an identity matrix hands every lane 16
//                    tokens of one dimension (a transpose), which it then adds up with the weights.
//   episodic/stable  <k_t, anchor> with the fp32 anchor split into three bf16 terms (8 + 8 + 8 mantissa bits:
//                    the split is exact), as three rows of a product against the keys.
// One wave per 64-token chunk; it holds the chunk and the 64 tokens in front of it (128 rows) as operands of
// v_mfma_f32_32x32x16_bf16: lane (r = lane % 32, h = lane / 32) has dims 16 kk + 8 h .. + 7 of row r of each
// 32-row set, kk = 0 .. D/16 - 1.  A product's 32 x 32 result leaves lane (n, h) with column n, rows
// 8 i + 4 h + j in register 4 i + j.  The vector unit only norms the rows (dot instructions on the packed
// values) and adds weighted result registers; it never unpacks a key.
using bf16x8 = __bf16 __attribute__((ext_vector_type(8)));
using f32x16 = float __attribute__((ext_vector_type(16)));

template <int KS> __device__ __forceinline__ f32x16 mm_tile(const u32x4 (&a)[KS], const u32x4 (&b)[KS])
{
    f32x16 c = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < KS; ++kk)
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[kk]), __builtin_bit_cast(bf16x8, b[kk]),
                                                    c, 0, 0, 0);
    return c;
}

// Sum over this lane's 16 rows of w[row] * c[row][n], rows rho = 8 i + 4 h + j restricted by MASK against the
// lane's column n: 0 all, 1 rho > n, 2 rho <= n, 3 rho >= n, 4 rho < n.  w: the row set's 32 weights in LDS.
template <int MASK> __device__ __forceinline__ float col_sum(const f32x16 &c, const float *w, int n, int h)
{
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float4 w4 = *reinterpret_cast<const float4 *>(w + 8 * i + 4 * h);
        const float ww[4] = {w4.x, w4.y, w4.z, w4.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int rho = 8 * i + 4 * h + j;
            const bool keep = MASK == 0 ? true : MASK == 1 ? rho > n : MASK == 2 ? rho <= n : MASK == 3 ? rho >= n : rho < n;
            s = fmaf(keep ? ww[j] : 0.f, c[4 * i + j], s);
        }
    }
    return s;
}

// Sum of squares of this lane's half row, then of the whole row (the other half sits 32 lanes away).
template <int KS> __device__ __forceinline__ float row_sumsq(const u32x4 (&x)[KS])
{
    float acc = 0.f;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk)
        asm("v_dot2c_f32_bf16 %0, %1, %1\n\t"
            "v_dot2c_f32_bf16 %0, %2, %2\n\t"
            "v_dot2c_f32_bf16 %0, %3, %3\n\t"
            "v_dot2c_f32_bf16 %0, %4, %4"
            : "+v"(acc)
            : "v"(x[kk].x), "v"(x[kk].y), "v"(x[kk].z), "v"(x[kk].w));
    return acc + __shfl_xor(acc, 32, 64);
}

// fp32 -> three bf16 terms whose sum is the value (each takes the next 8 mantissa bits)
__device__ __forceinline__ void split3(float x, uint16_t &hi, uint16_t &mid, uint16_t &lo)
{
    const uint32_t b0 = __float_as_uint(x) & 0xffff0000u;
    const float r1 = x - __uint_as_float(b0);
    const uint32_t b1 = __float_as_uint(r1) & 0xffff0000u;
    const float r2 = r1 - __uint_as_float(b1);
    hi = (uint16_t)(b0 >> 16);
    mid = (uint16_t)(b1 >> 16);
    lo = (uint16_t)(__float_as_uint(r2) >> 16);
}

// <k, anchor> for the 64 tokens of a chunk (token = lane): the anchor's three terms (terms[4][D] bf16 in LDS,
// written by this wave, row 3 zeros) are rows 0-2 and 4-6 of the left operand, so that the result registers 0-2 hold them for
// columns n in lanes h = 0 (rows 0-2) and h = 1 (rows 4-6) alike; the low half takes the chunk's first 32
// tokens, the high half the other 32.
template <int D> __device__ __forceinline__ float anchor_dot(const uint16_t *terms, const u32x4 (&c0)[D / 16],
                                                             const u32x4 (&c1)[D / 16], int r, int h)
{
    constexpr int KS = D / 16;
    const uint16_t *mine = terms + (r < 8 ? (r & 3) : 3) * D + 8 * h;  // row 3 holds zeros
    f32x16 d0 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, d1 = d0;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
        const bf16x8 a = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(mine + 16 * kk));
        d0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, c0[kk]), d0, 0, 0, 0);
        d1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, c1[kk]), d1, 0, 0, 0);
    }
    return h ? (d1[0] + d1[1]) + d1[2] : (d0[0] + d0[1]) + d0[2];
}

template <int D, int NW>
__global__ __launch_bounds__(64 * NW, 3)
void scan_mfma_kernel(const uint8_t *__restrict__ keys, RowMap km, PromptTab tab, ScanPlan plan, float *__restrict__ a_raw,
                      float *__restrict__ bsum, float *__restrict__ ssum, uint32_t *__restrict__ sync, int LH, int64_t rows,
                      int poll_limit, uint32_t spin_limit)
{
    constexpr int KS = D / 16, LPR = D / 8, SG = 64 / LPR;
    __shared__ float lds_rn[NW][128];                                 // 1/||k|| of a wave's 128 rows (0: no such token)
    __shared__ float lds_wb[NW][64];                                  // the same for the chunk, 0 outside the block
    __shared__ float lds_C[NW][D];                                    // chunk totals
    __shared__ __attribute__((aligned(16))) uint16_t lds_terms[NW][4][D];   // an anchor's bf16 terms and a row of zeros, per wave
    __shared__ float lds_S[D];
    __shared__ float lds_T[NW * SG * D];                              // scratch of a summing workgroup
    __shared__ int s_have;

    const int nblk = plan.nblk;
    int lh, blk, layer, head;
    {
        const int x = (int)(blockIdx.x & (kDies - 1));
        const uint32_t t = blockIdx.x >> 3;
        const int run = plan.run, len = plan.len[x];
        if (t >= queue_start(LH, len, tab.n, x)) return;
        int l = min(LH - 1, (int)((float)t * plan.inv_items[x]));
        while (l > 0 && queue_start(l, len, tab.n, x) > t) --l;
        while (l + 1 < LH && queue_start(l + 1, len, tab.n, x) <= t) ++l;
        const int r = (int)(t - queue_start(l, len, tab.n, x));
        lh = l;
        const int nsum = l % kDies == x ? tab.n : 0;
        {
            const int rb = max(r - nsum, 0), cyc = div_by(rb, run, plan.inv_run);
            blk = (cyc * kDies + x) * run + (rb - cyc * run);
        }
        layer = div_by(lh, km.H, plan.inv_H);
        head = lh - layer * km.H;
        const int sum_of = r < nsum ? r : -1;
        if (sum_of >= 0) {
            const int p = sum_of;
            if (!add_unit_up<D, NW, true>(bsum + ((int64_t)lh * nblk + tab.blk_off[p]) * D,
                                          tab.blk_off[p + 1] - tab.blk_off[p], ssum + ((int64_t)lh * tab.n + p) * D,
                                          lds_T, spin_limit) &&
                threadIdx.x == 0)
                atomicAdd(sync + kTimeoutWord, 1u);
            return;
        }
    }
    const int p = prompt_of_block(tab, blk);
    const int b = tab.b[p];
    const int N = tab.tok_off[p + 1] - tab.tok_off[p];
    const int blk_lo = (blk - tab.blk_off[p]) * b;
    const int blk_hi = min(blk_lo + b, N);
    const int64_t row0 = (int64_t)lh * tab.T + tab.tok_off[p];
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r = lane & 31, h = lane >> 5;
    const int t0 = blk_lo + 64 * w;                                   // first token of this wave's chunk

    // ---- first touch: the chunk (two sets of 32 rows) and the 32 rows in front of it; rows outside the prompt
    // read as zeros.  Three sets are held at a time: the columns are taken in two halves, the second half of
    // the chunk makes room for the first half of the halo in between and is read again (from L2) at the end.
    constexpr int kRowBytes = D * 2;
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t *>(keys) + km.unit(layer, head, p, tab) * 2, 0, N * kRowBytes, 0x00020000);
    u32x4 XA[KS], XB[KS], XH[KS];                                     // C0; C1, later H0, later C1 again; H1
    const int lane_off = (t0 + r) * kRowBytes + 16 * h;               // row r of set C0
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) XA[kk] = row_load<kKeyBF16>(rsrc, lane_off + 32 * kk);
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) XB[kk] = row_load<kKeyBF16>(rsrc, lane_off + 32 * kRowBytes + 32 * kk);
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) XH[kk] = row_load<kKeyBF16>(rsrc, lane_off - 32 * kRowBytes + 32 * kk);

    // ---- norms of the chunk ----
    float rn[4], gd[4], ssv[4];                                       // 1/||k||, ||k^||^2, ||k||^2 of row r of H0, H1, C0, C1
#define NKV_NORM_SET(set, x)                                          \
    do {                                                              \
        ssv[set] = row_sumsq<KS>(x);                                  \
        const int tk = t0 - 64 + 32 * (set) + r;                      \
        rn[set] = (tk >= 0 && tk < N) ? inv_norm(ssv[set]) : 0.f;     \
        gd[set] = rn[set] * rn[set] * ssv[set];                       \
        if (h == 0) lds_rn[w][32 * (set) + r] = rn[set];              \
    } while (0)
    NKV_NORM_SET(2, XA);
    NKV_NORM_SET(3, XB);
    if (h == 0) {
        lds_wb[w][r] = t0 + r < blk_hi ? rn[2] : 0.f;
        lds_wb[w][32 + r] = t0 + 32 + r < blk_hi ? rn[3] : 0.f;
    }
    const float rn_m = h ? rn[3] : rn[2];                             // this lane's own token t0 + lane
    const float gd_m = h ? gd[3] : gd[2], ss_m = h ? ssv[3] : ssv[2];
    const float kn_m = ss_m < 1e-24f ? sqrtf(ss_m) * 1e12f : 1.f;     // ||k^|| is 1 unless the norm was clamped
    __builtin_amdgcn_wave_barrier();

    // ---- chunk total: transpose by an identity product, then the weighted sum over the 16 rows a lane holds ----
    {
        u32x4 ident[2];                                               // B[k][n] = (n == k) and (n == 16 + k), k = 8 h + e
#pragma unroll
        for (int o = 0; o < 2; ++o) {
            uint32_t v[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int k0 = 8 * h + 2 * q + 16 * o;
                v[q] = (r == k0 ? 0x3f80u : 0u) | (r == k0 + 1 ? 0x3f800000u : 0u);
            }
            ident[o] = u32x4{v[0], v[1], v[2], v[3]};
        }
#pragma unroll
        for (int q = 0; q < KS / 2; ++q) {                            // dims 32 q + n
            float part = 0.f;
#pragma unroll
            for (int set = 2; set < 4; ++set) {
                f32x16 c = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, set == 2 ? XA[2 * q] : XB[2 * q]),
                                                            __builtin_bit_cast(bf16x8, ident[0]), c, 0, 0, 0);
                c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    __builtin_bit_cast(bf16x8, set == 2 ? XA[2 * q + 1] : XB[2 * q + 1]), __builtin_bit_cast(bf16x8, ident[1]),
                    c, 0, 0, 0);
                part += col_sum<0>(c, &lds_wb[w][32 * (set - 2)], r, h);
            }
            part += __shfl_xor(part, 32, 64);
            if (h == 0) lds_C[w][32 * q + r] = part;
        }
    }
    __syncthreads();

    // ---- block total = episodic anchor (up to length); every wave forms it for itself ----
    const int nch = (blk_hi - blk_lo + 63) >> 6;
    const int unblk = tab.blk_off[p + 1] - tab.blk_off[p];
    float *bsum_unit = bsum + ((int64_t)lh * nblk + tab.blk_off[p]) * D;
    float *S_unit = ssum + ((int64_t)lh * tab.n + p) * D;
    float bsq = 0.f;
    {
        constexpr int DPL = D / 64;                                   // dims per lane: 64 lanes cover the D dims
        float Bv[DPL];
#pragma unroll
        for (int e = 0; e < DPL; ++e) {
            const int dim = DPL * lane + e;
            float s = 0.f;
#pragma unroll
            for (int ww = 0; ww < NW; ++ww)
                if (ww < nch) s += lds_C[ww][dim];
            Bv[e] = s;
            bsq = fmaf(s, s, bsq);
            uint16_t t0b, t1b, t2b;
            split3(s, t0b, t1b, t2b);
            lds_terms[w][0][dim] = t0b;
            lds_terms[w][1][dim] = t1b;
            lds_terms[w][2][dim] = t2b;
            lds_terms[w][3][dim] = 0;                                 // the row the other lanes of the left operand read
        }
        bsq = wave_sum(bsq);
        if (w == blk % NW) {                                          // one wave stores the block total
            const __amdgpu_buffer_rsrc_t brs = __builtin_amdgcn_make_buffer_rsrc(bsum_unit, 0, unblk * D * 4, 0x00020000);
            const int off = ((blk - tab.blk_off[p]) * D + DPL * lane) * 4;
            if constexpr (DPL == 2) {
                const float o0 = __shfl_down(Bv[0], 1, 64), o1 = __shfl_down(Bv[1], 1, 64);
                if ((lane & 1) == 0) agent_store16(brs, off, Bv[0], Bv[1], o0, o1);
            } else {
                const float o1 = __shfl_down(Bv[0], 1, 64), o2 = __shfl_down(Bv[0], 2, 64), o3 = __shfl_down(Bv[0], 3, 64);
                if ((lane & 3) == 0) agent_store16(brs, off, Bv[0], o1, o2, o3);
            }
        }
    }
    __builtin_amdgcn_wave_barrier();
    const int tok = t0 + lane;
    {
        const float bd = anchor_dot<D>(&lds_terms[w][0][0], XA, XB, r, h);
        if (tok < blk_hi) a_raw[rows + row0 + tok] = neg_cos(rn_m * bd, kn_m, bsq);
    }

    // ---- current window: bands of the Gram matrix, the chunk's second half of columns first ----
    {
        const float *wH0 = &lds_rn[w][0], *wH1 = &lds_rn[w][32], *wC0 = &lds_rn[w][64], *wC1 = &lds_rn[w][96];
        NKV_NORM_SET(1, XH);
        __builtin_amdgcn_wave_barrier();
        // One tile at a time (the scheduling barriers): twelve tiles' worth of result registers would not fit.
#define NKV_TILE(acc, MASK, A, B, W)                                  \
    do {                                                              \
        acc += col_sum<MASK>(mm_tile<KS>(A, B), W, r, h);             \
        asm volatile("" : "+v"(acc));                                 \
    } while (0)
        // backward band of tokens t0 + 32 .., forward band of tokens t0 - 32 ..
        float c1 = 0.f, f1 = 0.f, c0 = 0.f, f0 = 0.f;
        NKV_TILE(c1, 1, XH, XB, wH1);
        NKV_TILE(c1, 0, XA, XB, wC0);
        NKV_TILE(c1, 2, XB, XB, wC1);
        NKV_TILE(f1, 3, XH, XH, wH1);
        const float sq1 = f1;                                         // the part inside the 64 x 64 square
        NKV_TILE(f1, 0, XA, XH, wC0);
        NKV_TILE(f1, 4, XB, XH, wC1);
        // the chunk's second half makes room for the first half of the halo
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) XB[kk] = row_load<kKeyBF16>(rsrc, lane_off - 64 * kRowBytes + 32 * kk);
        __builtin_amdgcn_sched_barrier(0);
        NKV_TILE(c0, 0, XH, XA, wH1);
        NKV_TILE(c0, 2, XA, XA, wC0);
        NKV_NORM_SET(0, XB);
        __builtin_amdgcn_wave_barrier();
        NKV_TILE(c0, 1, XB, XA, wH0);
        NKV_TILE(f0, 3, XB, XB, wH0);
        NKV_TILE(f0, 0, XH, XB, wH1);
        const float sq0 = f0;
        NKV_TILE(f0, 4, XA, XB, wC0);
#undef NKV_TILE
#undef NKV_NORM_SET
        // and comes back for the stable dots while this wave waits for the unit sum
#pragma unroll
        for (int kk = 0; kk < KS; ++kk) XB[kk] = row_load<kKeyBF16>(rsrc, lane_off + 32 * kRowBytes + 32 * kk);
        __builtin_amdgcn_sched_barrier(0);
        float v[6] = {c0, c1, f0, f1, sq0, sq1};
#pragma unroll
        for (int i = 0; i < 6; ++i) v[i] += __shfl_xor(v[i], 32, 64);
        const float c_m = rn_m * (h ? v[1] : v[0]);                   // <k^_t, window sum at t>, t = t0 + lane
        const float rq = h ? rn[1] : rn[0], gq = h ? gd[1] : gd[0];   // q = t - 64
        const float f_m = rq * (h ? v[3] : v[2]);
        // square of the window sum's norm at token t0 - 1: the 64 x 64 square, from its lower triangles
        float P0 = h ? 2.f * rq * v[5] - gq : 2.f * rq * v[4] - gq;
        P0 = wave_sum(P0);
        float d = (2.f * c_m - gd_m) - (2.f * f_m - gq);              // P_t - P_{t-1}
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const float up = __shfl_up(d, o, 64);
            if (lane >= o) d += up;
        }
        if (tok < blk_hi) a_raw[2 * rows + row0 + tok] = neg_cos(c_m, kn_m, P0 + d);
    }

    // ---- stable dots against the unit's sum ----
    const __amdgpu_buffer_rsrc_t srs = __builtin_amdgcn_make_buffer_rsrc(S_unit, 0, D * 4, 0x00020000);
    if (w == 0) {
        u32x4 sv0 = {kUnwritten, kUnwritten, kUnwritten, kUnwritten}, sv1 = sv0;
        bool got = false;
        for (int polls = 0; poll_limit >= 0; ++polls) {
            if (lane < LPR) {
                sv0 = agent_load16(srs, lane * 32);
                sv1 = agent_load16(srs, lane * 32 + 16);
            }
            const bool ok = lane >= LPR || (all_written(sv0) && all_written(sv1));
            got = __all(ok);
            if (got || polls >= poll_limit) break;
            __builtin_amdgcn_s_sleep(8);
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
    if (s_have != 0) {
        constexpr int DPL = D / 64;
        float ssq = 0.f;
#pragma unroll
        for (int e = 0; e < DPL; ++e) {
            const int dim = DPL * lane + e;
            const float s = lds_S[dim];
            ssq = fmaf(s, s, ssq);
            uint16_t t0b, t1b, t2b;
            split3(s, t0b, t1b, t2b);
            lds_terms[w][0][dim] = t0b;
            lds_terms[w][1][dim] = t1b;
            lds_terms[w][2][dim] = t2b;
        }
        ssq = wave_sum(ssq);
        __builtin_amdgcn_wave_barrier();
        const float sd = anchor_dot<D>(&lds_terms[w][0][0], XA, XB, r, h);
        if (tok < blk_hi) a_raw[row0 + tok] = neg_cos(rn_m * sd, kn_m, ssq);
    }
}

// a_s of the listed blocks for scan_mfma_kernel: the same loads, norms, split and product as there.
template <int D, int NW>
__global__ __launch_bounds__(64 * NW, 2) void deferred_stable_mfma_kernel(const uint8_t *__restrict__ keys, RowMap km,
                                                                          PromptTab tab, const float *__restrict__ ssum,
                                                                          const uint32_t *__restrict__ sync,
                                                                          float *__restrict__ a_raw)
{
    constexpr int KS = D / 16, kRowBytes = D * 2, DPL = D / 64;
    __shared__ __attribute__((aligned(16))) uint16_t lds_terms[NW][4][D];
    const int nblk = tab.blk_off[tab.n];
    const uint32_t count = sync[kDeferCountWord];
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r = lane & 31, h = lane >> 5;
    for (uint32_t i = blockIdx.x; i < count; i += gridDim.x) {
        const int id = (int)sync[kSyncWords + i], lh = id / nblk, blk = id - lh * nblk;
        const int p = prompt_of_block(tab, blk);
        const int b = tab.b[p], N = tab.tok_off[p + 1] - tab.tok_off[p];
        const int blk_lo = (blk - tab.blk_off[p]) * b, blk_hi = min(blk_lo + b, N);
        const int64_t row0 = (int64_t)lh * tab.T + tab.tok_off[p];
        const int t0 = blk_lo + 64 * w;
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint8_t *>(keys) + km.unit(lh, p, tab) * 2, 0, N * kRowBytes, 0x00020000);
        u32x4 X[2][KS];
        float rn[2], ssv[2];
#pragma unroll
        for (int set = 0; set < 2; ++set) {
            const int off = (t0 + 32 * set + r) * kRowBytes + 16 * h;
#pragma unroll
            for (int kk = 0; kk < KS; ++kk) X[set][kk] = row_load<kKeyBF16>(rsrc, off + 32 * kk);
        }
#pragma unroll
        for (int set = 0; set < 2; ++set) {
            ssv[set] = row_sumsq<KS>(X[set]);
            const int tk = t0 + 32 * set + r;
            rn[set] = (tk >= 0 && tk < N) ? inv_norm(ssv[set]) : 0.f;
        }
        const float rn_m = h ? rn[1] : rn[0], ss_m = h ? ssv[1] : ssv[0];
        const float kn_m = ss_m < 1e-24f ? sqrtf(ss_m) * 1e12f : 1.f;
        const float *S = ssum + ((int64_t)lh * tab.n + p) * D;
        float ssq = 0.f;
        __builtin_amdgcn_wave_barrier();                              // the previous block's reads of the terms
#pragma unroll
        for (int e = 0; e < DPL; ++e) {
            const int dim = DPL * lane + e;
            const float s = S[dim];
            ssq = fmaf(s, s, ssq);
            uint16_t t0b, t1b, t2b;
            split3(s, t0b, t1b, t2b);
            lds_terms[w][0][dim] = t0b;
            lds_terms[w][1][dim] = t1b;
            lds_terms[w][2][dim] = t2b;
            lds_terms[w][3][dim] = 0;
        }
        ssq = wave_sum(ssq);
        __builtin_amdgcn_wave_barrier();
        const float sd = anchor_dot<D>(&lds_terms[w][0][0], X[0], X[1], r, h);
        const int tok = t0 + lane;
        if (tok < blk_hi) a_raw[row0 + tok] = neg_cos(rn_m * sd, kn_m, ssq);
    }
}

// a_s of the blocks whose workgroups did not wait for their unit's sum.  One workgroup per listed block at a
// time, one wave per chunk, same lane layout, same instruction sequences for the norm, the dot and the
// cosine as scan_kernel, so the values are the ones scan_kernel would have stored.
template <int D, int NW, int KF>
__global__ __launch_bounds__(64 * NW) void deferred_stable_kernel(const uint8_t *__restrict__ keys, RowMap km,
                                                                  PromptTab tab,
                                                                  const float *__restrict__ ssum,
                                                                  const uint32_t *__restrict__ sync,
                                                                  float *__restrict__ a_raw)
{
    constexpr int LPR = D / 8, TPT = LPR, ES = key_bytes<KF>(), kRowBytes = D * ES;
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
        load8(ssum + ((int64_t)lh * tab.n + p) * D + c * 8, S);
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

// Unit sums that the scan left unwritten (its summing workgroup gave up waiting, which the scheduling of
// workgroups makes possible in principle): formed here, after the scan, from the block totals, with the
// additions in the same order.  grid: one workgroup of 64 * NW threads per (layer*head, prompt).
template <int D, int NW>
__global__ __launch_bounds__(64 * NW) void unit_sum_repair_kernel(const float *__restrict__ bsum, PromptTab tab,
                                                                  float *__restrict__ ssum)
{
    __shared__ float part[64 * NW / (D / 4) * D];
    const int lh = blockIdx.x / tab.n, p = blockIdx.x - lh * tab.n;
    float *ssum_unit = ssum + ((int64_t)lh * tab.n + p) * D;
    bool missing = false;
    for (int i = threadIdx.x; i < D; i += 64 * NW) missing = missing || __float_as_uint(ssum_unit[i]) == kUnwritten;
    if (!__syncthreads_or(missing)) return;
    const int nblk = tab.blk_off[tab.n];
    add_unit_up<D, NW, false>(bsum + ((int64_t)lh * nblk + tab.blk_off[p]) * D, tab.blk_off[p + 1] - tab.blk_off[p],
                              ssum_unit, part, 0u);
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

template <int D, int NW, bool FUSED, int KF, bool MFMA = false>
void launch_scan(const uint8_t *keys, const RowMap &km, int LH, const PromptTab &tab, float *a_raw, float *bsum, float *ssum,
                 uint32_t *sync, int poll_limit, uint32_t spin_limit, hipStream_t st)
{
    const int64_t rows = (int64_t)LH * tab.T;
    unsigned groups = (unsigned)(tab.blk_off[tab.n] * LH);
    ScanPlan plan;
    plan.nblk = tab.blk_off[tab.n];
    plan.run = run_length(plan.nblk);
    plan.inv_run = 1.0f / (float)plan.run;
    plan.inv_H = 1.0f / (float)km.H;
    uint32_t longest = 0;
    for (int x = 0; x < kDies; ++x) {                                 // 8 queues of (nearly) equal length, interleaved
        plan.len[x] = die_blocks(plan.nblk, plan.run, x);
        plan.inv_items[x] = (float)kDies / (float)(kDies * plan.len[x] + tab.n);
        const uint32_t items = queue_start(LH, plan.len[x], tab.n, x);
        longest = items > longest ? items : longest;
    }
    if (FUSED) groups = longest * kDies;
    if constexpr (MFMA)
        scan_mfma_kernel<D, NW><<<groups, 64 * NW, 0, st>>>(keys, km, tab, plan, a_raw, bsum, ssum, sync, LH, rows,
                                                            poll_limit, spin_limit);
    else
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


template <int D, int NW> int resident_workgroups_mfma()
{
    static int cached = -1;
    if (cached < 0) {
        int per_cu = 0, dev = 0;
        hipDeviceProp_t prop;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, scan_mfma_kernel<D, NW>, 64 * NW, 0) != hipSuccess ||
            hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess)
            return 0;
        cached = per_cu * prop.multiProcessorCount;
    }
    return cached;
}

template <int D, int NW, int KF>
hipError_t run_nw(const uint8_t *keys, const RowMap &km, int LH, const PromptTab &tab, float *a_raw, float *bsum, float *ssum,
                  void *sync_area, int mode, bool mfma, const Prof &prof, hipStream_t st)
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
    if (KF == kKeyBF16 && mfma && fused && max_unit_blocks <= resident_workgroups_mfma<D, NW>()) {
        // the matrix-core formulation of the fused pass (same protocol, its own kernel for the deferred blocks)
        const size_t nb = (size_t)LH * tab.blk_off[tab.n] * D / 4, ns = (size_t)LH * tab.n * D / 4;
        const size_t n16 = kSyncWords / 4 + nb + ns;
        prepare_kernel<<<(unsigned)min((n16 + 255) / 256, (size_t)2048), 256, 0, st>>>(
            (uint4 *)sync_area, kSyncWords / 4, (uint4 *)bsum, nb, (uint4 *)ssum, ns);
        prof.begin(NKV_KERNEL_SCAN, st);
        launch_scan<D, NW, true, kKeyBF16, true>(keys, km, LH, tab, a_raw, bsum, ssum, (uint32_t *)sync_area,
                                          defer_all ? -1 : kPollLimit, no_unit_sums ? 0u : kSpinLimit, st);
        prof.end(NKV_KERNEL_SCAN, st);
        unit_sum_repair_kernel<D, NW><<<LH * tab.n, 64 * NW, 0, st>>>(bsum, tab, ssum);
        deferred_stable_mfma_kernel<D, NW><<<defer_all ? 4096 : 256, 64 * NW, 0, st>>>(keys, km, tab, ssum,
                                                                                       (const uint32_t *)sync_area, a_raw);
    } else if (fused) {
        // the counters start at zero, block totals and unit sums as "unwritten"
        const size_t nb = (size_t)LH * tab.blk_off[tab.n] * D / 4, ns = (size_t)LH * tab.n * D / 4;
        const size_t n16 = kSyncWords / 4 + nb + ns;
        prepare_kernel<<<(unsigned)min((n16 + 255) / 256, (size_t)2048), 256, 0, st>>>(
            (uint4 *)sync_area, kSyncWords / 4, (uint4 *)bsum, nb, (uint4 *)ssum, ns);
        prof.begin(NKV_KERNEL_SCAN, st);
        launch_scan<D, NW, true, KF>(keys, km, LH, tab, a_raw, bsum, ssum, (uint32_t *)sync_area,
                                 defer_all ? -1 : kPollLimit, no_unit_sums ? 0u : kSpinLimit, st);
        prof.end(NKV_KERNEL_SCAN, st);
        unit_sum_repair_kernel<D, NW><<<LH * tab.n, 64 * NW, 0, st>>>(bsum, tab, ssum);
        deferred_stable_kernel<D, NW, KF><<<defer_all ? 4096 : 256, 64 * NW, 0, st>>>(keys, km, tab, ssum,
                                                                                  (const uint32_t *)sync_area, a_raw);
    } else {
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
               void *sync_area, int mode, bool mfma, const Prof &prof, hipStream_t st)
{
    int bmax = 0;
    for (int p = 0; p < tab.n; ++p) bmax = max(bmax, tab.b[p]);
    switch ((bmax + 63) / 64) {
    case 1: return run_nw<D, 1, KF>(keys, km, LH, tab, a_raw, bsum, ssum, sync_area, mode, mfma, prof, st);
    case 2: return run_nw<D, 2, KF>(keys, km, LH, tab, a_raw, bsum, ssum, sync_area, mode, mfma, prof, st);
    case 3: return run_nw<D, 3, KF>(keys, km, LH, tab, a_raw, bsum, ssum, sync_area, mode, mfma, prof, st);
    default: return run_nw<D, 4, KF>(keys, km, LH, tab, a_raw, bsum, ssum, sync_area, mode, mfma, prof, st);
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
                             float *bsum, float *ssum, void *sync_area, int mode, bool mfma, const Prof &prof,
                             hipStream_t st)
{
    const uint8_t *k = (const uint8_t *)keys;
    if (dtype == NKV_DTYPE_F8_E4M3) {
        if (d == 128) return run<128, kKeyF8>(k, km, LH, tab, a_raw, bsum, ssum, sync_area, mode, false, prof, st);
        return run<64, kKeyF8>(k, km, LH, tab, a_raw, bsum, ssum, sync_area, mode, false, prof, st);
    }
    if (dtype == NKV_DTYPE_F16) {
        if (d == 128) return run<128, kKeyF16>(k, km, LH, tab, a_raw, bsum, ssum, sync_area, mode, false, prof, st);
        return run<64, kKeyF16>(k, km, LH, tab, a_raw, bsum, ssum, sync_area, mode, false, prof, st);
    }
    if (d == 128) return run<128, kKeyBF16>(k, km, LH, tab, a_raw, bsum, ssum, sync_area, mode, mfma, prof, st);
    return run<64, kKeyBF16>(k, km, LH, tab, a_raw, bsum, ssum, sync_area, mode, mfma, prof, st);
}

}  // namespace nkv
