/*
 * nkv.h -- C ABI of the MI355X (gfx950) NestedKV prefill compression pass.
 *
 * The pass runs once after a prompt is prefilled (paper Section 2, Appendix A
 * "Inference pipeline").  For every prompt p, layer l and KV head h it
 *   1. scores each cached key by its cosine anomaly against a stable, an
 *      episodic (block) and a current (sliding window) anchor and combines the
 *      three readings with the head-adaptive blend and the surprise gate
 *      (Sections 2.1-2.4)                                   -> nkv_score
 *   2. lets the heads of a layer compete for the layer's budget under a
 *      per-head safeguard (Section 2.6, Appendix A)         -> nkv_budget
 *   3. keeps each head's B_h best positions and packs their K/V rows
 *      (Section 2.5)                                        -> nkv_select_compact
 *
 * General rules
 *   - Every tensor pointer is a DEVICE pointer owned by the caller; structs,
 *     cu_seqlens and r_per_prompt are HOST memory read during the call only.
 *   - Tensors are dense (keys / values unless strides are given), row-major, innermost dimension fastest:
 *       keys   [L][H][T][d]     values [L][H][T][dv]     scores [L][H][T]
 *     T = cu_seqlens[n_prompts] is the total token count; prompt p owns the
 *     token rows [cu_seqlens[p], cu_seqlens[p+1]) of every (layer, head).
 *     A "unit" is one (prompt, layer, head); units are numbered
 *     u = (p * L + l) * H + h.
 *   - Calls only enqueue work on `hip_stream` (a hipStream_t, NULL = default
 *     stream) and never synchronise or allocate.  The only state the library keeps is what it asked the
 *     runtime once per process: the occupancy of its scan kernels (first nkv_score on a device) and, for
 *     nkv_budget_noalloc, the address of its static scratch array.
 *     Scratch memory is the caller's `ws` (device, 256-byte aligned, at least
 *     nkv_workspace_bytes() bytes); its contents are undefined afterwards.
 *     The calls can be recorded into a HIP graph; nkv_score asks the runtime for a
 *     kernel's occupancy the first time it runs on a device, so call it once
 *     outside a capture first.  Keys / values may also be given by strides
 *     (nkv_shape.key_strides).
 *   - Return value: NKV_OK or a negative nkv_status.  Argument errors are
 *     detected on the host before anything is enqueued.  Inputs must be finite;
 *     behaviour on NaN/Inf keys or scores is undefined (but never out of bounds).
 *   - The library is the only implementation: there is no CPU fallback.
 */
#ifndef NKV_H
#define NKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum nkv_status {
    NKV_OK = 0,
    NKV_EINVAL = -1,       /* null pointer, bad parameter value, r outside [0,1]      */
    NKV_ESHAPE = -2,       /* bad L/H/d/dv, non-monotone cu_seqlens, empty prompt     */
    NKV_EWORKSPACE = -3,   /* ws is NULL, misaligned or smaller than required         */
    NKV_EHIP = -4,         /* a HIP call failed (launch error)                        */
    NKV_EUNSUPPORTED = -5, /* valid request outside what the kernels cover            */
    NKV_ESCRATCH = -6      /* nkv_budget_noalloc: the shape needs more scratch than   */
                           /* NKV_STATIC_SCRATCH_BYTES                                */
} nkv_status;

/* Element type of keys and values (and of the packed outputs, whose rows are copies).                  */
/* F8_E4M3: the 8-bit OCP format with 4 exponent bits (bias 7), 3 mantissa bits, no infinities,         */
/* S.1111.111 = NaN, largest finite value 448.  The scores are cosines, so a positive scale factor per   */
/* tensor, per head or per token that a quantised cache carries does not enter and is not asked for     */
/* (Section 2.1 normalises every key); a per-channel scale would, and is not supported.  Rows of 8-bit   */
/* elements need d and dv to be multiples of 16.  (The paper's own experiments use bf16 caches; other    */
/* cache dtypes are its stated future work, Section 5.)                                                  */
enum { NKV_DTYPE_F32 = 0, NKV_DTYPE_BF16 = 1, NKV_DTYPE_F16 = 2, NKV_DTYPE_F8_E4M3 = 3 };
enum { NKV_GATE_SURPRISE = 0, NKV_GATE_ONLY_AVERAGE = 1, NKV_GATE_ONLY_MAX = 2 };
enum { NKV_SURPRISE_NORMALISED = 0, NKV_SURPRISE_RAW = 1 };
enum {
    NKV_FLAG_GENERIC_KERNELS = 1u,    /* force the shape-generic scoring kernels                            */
    NKV_FLAG_TWO_PASS_STABLE = 2u,    /* streaming kernels: compute the stable anomaly in a second pass     */
                                      /* over the keys instead of inside the single fused pass             */
    NKV_FLAG_DEFER_STABLE = 4u,       /* streaming kernels, fused pass: no workgroup waits for its unit's   */
                                      /* sum; every block takes the deferred route (exercises that route)   */
    NKV_FLAG_NO_UNIT_SUMS = 8u,       /* as DEFER_STABLE, and the pass forms no unit sum either: all of     */
                                      /* them come from the kernel that fills in missing ones (exercises it) */
    NKV_FLAG_BUDGET_PER_HEAD = 16u,   /* nkv_budget: the kernels that hold a whole head in one workgroup     */
                                      /* instead of the slice-wise ones                                      */
    NKV_FLAG_STATS_PER_HEAD = 32u,    /* nkv_score: the same choice for the per-head statistics              */
    NKV_FLAG_SELECT_PER_HEAD = 64u,   /* nkv_select_compact: the same choice for the top-B_h selection       */
    NKV_FLAG_VECTOR_SCAN = 128u,      /* streaming kernels: the vector-unit formulation of the fused pass    */
                                      /* also for 16-bit keys of head dim 128, where the matrix-core one is  */
                                      /* the default                                                         */
    NKV_FLAG_COMPACT_IN_PLACE = 256u  /* nkv_select_compact: the kept rows of a unit move to the front of    */
                                      /* the unit's own rows in keys / values (no packed buffers)            */
};
/* Kernels a caller can ask to have timed, see nkv_params.prof_start. */
enum {
    NKV_KERNEL_SCAN = 0,       /* key-streaming anomaly kernel of nkv_score / nkv_score_raw   */
    NKV_KERNEL_FINALIZE = 1,   /* per-head statistics, blend, gate of nkv_score               */
    NKV_KERNEL_BUDGET = 2,     /* nkv_budget                                                  */
    NKV_KERNEL_SELECT = 3,     /* threshold search + ordered compaction of nkv_select_compact */
    NKV_KERNEL_GATHER = 4,     /* K/V row copies of nkv_select_compact                        */
    NKV_KERNEL_DECODE = 5,     /* attention over the retained rows of nkv_decode_attention    */
    NKV_KERNEL_COUNT = 6
};

#define NKV_MAX_PROMPTS 64        /* prompts per call                                   */
#define NKV_MAX_HEAD_DIM 1024     /* d and dv; both must be multiples of 8              */
#define NKV_MAX_HEADS 32          /* KV heads per layer                                 */
#define NKV_MAX_LAYER_TENSORS 128 /* layers when every layer has a tensor of its own    */
#define NKV_PIN 3.0e38f           /* score written to pinned sink positions             */
#define NKV_STATIC_SCRATCH_BYTES (32u << 20) /* scratch array inside the library, see nkv_budget_noalloc */

/*
 * Fixed policy constants (Appendix A "Hyperparameters").  nkv_params_default()
 * fills in the paper's values; struct_size must be sizeof(nkv_params).
 */
typedef struct nkv_params {
    uint32_t struct_size;
    int32_t  window;          /* W = 64, current-memory window (Section 2.2)                       */
    int32_t  block_div;       /* 32  \  episodic block size b = clip(floor(N/div), min, max),      */
    int32_t  block_min;       /* 128  } N = that prompt's length (Section 2.2)                     */
    int32_t  block_max;       /* 256 /                                                             */
    int32_t  n_sink;          /* 4 leading positions pinned to NKV_PIN (Section 2.3)               */
    int32_t  gate_mode;       /* NKV_GATE_*: surprise gate, or the "only average" / "only max"     */
                              /* ablations of Section 3.4                                          */
    int32_t  surprise_mode;   /* NORMALISED: min-max within the head, mean-centre, rectify, then   */
                              /* gate (Appendix A); RAW: gate the std itself (Section 2.4 literal) */
    uint32_t flags;           /* NKV_FLAG_*                                                        */
    int32_t  scale_mask;      /* bit 0 / 1 / 2 set: the stable / episodic / current scale takes part; 0 is  */
                              /* read as 7 (all three).  A scale that is off is left out of the blend, the   */
                              /* winner and the standard deviation alike: 3 is the Appendix's component     */
                              /* ablation "Stable + episodic (no current)", 1 its "Single-scale stable       */
                              /* score".  (A prior weight of 0 only removes a scale from the blend.)  At     */
                              /* least one scale that takes part needs a positive prior weight (NKV_EINVAL). */
    double   top_frac;        /* p = 0.10: top/bottom sets hold max(1, floor(p*N)) tokens          */
    double   prior[3];        /* (0.4, 0.4, 0.2): stable, episodic, current (Section 2.4)          */
    double   beta;            /* 3.0  blend temperature                                            */
    double   tau;             /* 0.60 gate threshold                                               */
    double   kappa;           /* 10.0 gate sharpness                                               */
    double   safeguard;       /* 0.20: each head first keeps floor(safeguard * k0) own tokens      */
    double   near_tol;        /* 1e-5: half-width of the band nkv_select_compact counts around a   */
                              /* head's selection threshold                                        */
    /* Optional timing: if prof_start[k] and prof_stop[k] are both non-NULL hipEvent_t handles, the    */
    /* call that launches kernel k (NKV_KERNEL_*) records them on its stream right before and right    */
    /* after that launch.  The caller owns the events and reads them after synchronising.              */
    void    *prof_start[NKV_KERNEL_COUNT];
    void    *prof_stop[NKV_KERNEL_COUNT];
    /* Optional health counters of the fused streaming scan: NULL, or a DEVICE pointer to two uint32 that        */
    /* nkv_score / nkv_score_raw fill on their stream: [0] workgroups that gave up adding a unit's block totals  */
    /* up inside the pass (the unit's sum was then formed afterwards; 0 in normal operation, and always 0 for    */
    /* 16-bit keys of head dim 128, whose pass adds every block straight into the unit's sum), [1] blocks whose  */
    /* stable anomaly was computed after the pass because the unit's sum did not arrive within the bounded       */
    /* wait.  Neither affects the result.  Both are 0 on the routes that do not use the fused pass.              */
    void    *scan_counters;
} nkv_params;

typedef struct nkv_shape {
    int32_t L;                /* layers                                              */
    int32_t H;                /* KV heads per layer                                  */
    int32_t d;                /* key head dim                                        */
    int32_t dv;               /* value head dim                                      */
    int32_t dtype;            /* NKV_DTYPE_* of keys and values                      */
    int32_t n_prompts;        /* 1..NKV_MAX_PROMPTS                                  */
    const int32_t *cu_seqlens;/* HOST, n_prompts + 1 entries, cu[0] = 0, increasing  */
    /* Where the rows of keys / values lie.  NULL: dense [L][H][T][d] (values [L][H][T][dv]), the prompts */
    /* of a head concatenated along the token axis.  Otherwise HOST, 3 entries {layer, head, prompt} in   */
    /* elements: token n of prompt p, head h, layer l starts at                                            */
    /*     l * layer + h * head + p * prompt + n * d         if prompt != 0 (one slab per prompt),         */
    /*     l * layer + h * head + (cu_seqlens[p] + n) * d    if prompt == 0 (concatenated prompts).        */
    /* A unit's rows are contiguous in either case.  A cache tensor [B][H][N_max][d] of one layer is       */
    /* {0, N_max*d, H*N_max*d} with L = 1.  Entries must be multiples of 16 bytes and units must not       */
    /* overlap (NKV_EINVAL).  scores, a_raw and the packed outputs keep their dense layouts.               */
    const int64_t *key_strides;
    const int64_t *value_strides;
    /* Every layer in a tensor of its own (a framework's list of per-layer caches).  NULL, or HOST, L      */
    /* entries: where layer l's tensor starts, in elements from the keys / values pointer handed to the   */
    /* call, i.e. (address of layer l's tensor - address of layer 0's tensor) / element size, entry 0 = 0; */
    /* negative entries are fine.  The layer entry of the strides is then not used (strides NULL: every    */
    /* layer tensor is a dense [H][T][d]).  Entries must be multiples of 16 bytes, L <=                    */
    /* NKV_MAX_LAYER_TENSORS, and layers must not overlap (NKV_EINVAL).                                    */
    const int64_t *key_layer_offsets;
    const int64_t *value_layer_offsets;
} nkv_shape;

/* Fills *p with the paper's constants.  Returns NKV_EINVAL if p is NULL. */
int nkv_params_default(nkv_params *p);

/* Host-side closed forms, the same ones the kernels are launched with.
 *   nkv_block_size : b = clip(floor(N / block_div), block_min, block_max)      (Section 2.2)
 *   nkv_k0         : floor((1 - r) * N + 1e-9), positions a head keeps before competition (Appendix A)
 *   nkv_m_safe     : floor(safeguard * k0 + 1e-9)                              (Appendix A)
 *   nkv_m_p        : max(1, floor(top_frac * N + 1e-9))                        (Section 2.4)
 * They return -1 on invalid arguments. */
int64_t nkv_block_size(int64_t N, const nkv_params *p);
int64_t nkv_k0(int64_t N, double r);
int64_t nkv_m_safe(int64_t k0, double safeguard);
int64_t nkv_m_p(int64_t N, double top_frac);

/* Rows nkv_select_compact will write: sum over prompts of L * H * k0(N_p, r_p)
 * (the budgets of a layer always add up to H * k0, Section 2.6). */
int nkv_packed_rows(const nkv_shape *shape, const double *r_per_prompt, int64_t *rows);

/* Bytes of scratch that cover any of the three calls below for this shape. */
int nkv_workspace_bytes(const nkv_shape *shape, const nkv_params *params, size_t *bytes);

/*
 * Scores (Sections 2.1-2.4).  keys -> scores[L][H][T] fp32: per prompt and head
 * the routed score a* in [0,1], with the first min(n_sink, N) positions of every
 * prompt set to NKV_PIN.  fp32 arithmetic on the stored key values.
 */
int nkv_score(const void *keys, const nkv_shape *shape, const nkv_params *params,
              float *scores, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * The three per-scale anomalies before any normalisation (Section 2.3):
 * a_raw[3][L][H][T] fp32 = a_s, a_e, a_c = -cos(k_hat, anchor).  This is the
 * first stage of nkv_score made visible for inspection.
 */
int nkv_score_raw(const void *keys, const nkv_shape *shape, const nkv_params *params,
                  float *a_raw, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Head-wise memory competition (Section 2.6, Appendix A).  For prompt p with
 * eviction ratio r_per_prompt[p] in [0,1]: k0 = nkv_k0(N_p, r), every head keeps
 * its own nkv_m_safe(k0) best tokens, the other H*(k0 - m_safe) slots of a layer
 * go to the best remaining (head, token) pairs; k_per_head[u] = B_h, and the B_h
 * of a layer add up to H*k0.  Order: higher score, then lower head, then lower
 * token index.  Exact integer work on the fp32 scores given.  `ws` may be NULL
 * (ws_bytes 0): a slower kernel that needs no scratch is used then.
 */
int nkv_budget(const float *scores, const nkv_shape *shape, const nkv_params *params,
               const double *r_per_prompt, int32_t *k_per_head, void *ws, size_t ws_bytes,
               void *hip_stream);

/*
 * nkv_budget for callers that cannot allocate device memory or hand over scratch: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same inputs, same k_per_head, same kernels;
 * the scratch is an array of NKV_STATIC_SCRATCH_BYTES (32 MiB) that lives inside the library's code object
 * (one copy per GPU the library runs on, held until the process ends), so the call takes no ws argument and
 * calls no allocating routine.  A shape whose budget kernels need more than that (about 4000 (prompt, layer,
 * head) units, or about 44 million (head, token) scores in prompts of more than 8192 tokens) is refused with
 * NKV_ESCRATCH before anything is enqueued.  The first call on a device looks the array's address up (a
 * host-side runtime query): make that call outside a capture.  All calls on one GPU share the array: calls
 * that overlap in time on one GPU (different streams or threads) race and give undefined budgets; calls on
 * one stream, or otherwise ordered, are safe.  Nothing in the array has to survive or be cleared between
 * calls.
 */
int nkv_budget_noalloc(const float *scores, const nkv_shape *shape, const nkv_params *params,
                       const double *r_per_prompt, int32_t *k_per_head, void *hip_stream);

/*
 * Compression operator (Section 2.5).  For every unit u keep the k_per_head[u]
 * positions with the highest score (ties: lower index) and copy their K and V
 * rows unchanged, in ascending token order:
 *   head_off[u]                  first output row of unit u; head_off[P*L*H] = total rows  (int64)
 *   kept_idx [rows]              prompt-local token index of every output row              (int32)
 *   packed_k [rows][d], packed_v [rows][dv]   bitwise copies of the kept rows
 * `row_capacity` is the number of rows the three output buffers can hold; rows
 * beyond it are not written (head_off still reports the true offsets).
 * k_per_head[u] outside [0, N_p] is clamped.  If near_threshold_count is not
 * NULL it receives the number of tokens whose score lies within params->near_tol
 * of their head's selection threshold (the B_h-th highest score), summed over all
 * units with 0 < B_h < N_p; these are the positions whose fate can change under
 * score perturbations of that size.  `ws` may be NULL (ws_bytes 0): the selection then runs one workgroup per
 * unit; with scratch (nkv_workspace_bytes) prompts of more than 16384 tokens, and batches of 2048 units and
 * more, are selected slice-wise (same result, quicker).
 *
 * In place (params->flags & NKV_FLAG_COMPACT_IN_PLACE): the method only removes cached positions and leaves the
 * retained keys and values unchanged (Appendix A, "Scoring cost"), so the cache can shrink where it lies instead
 * of being copied into a second one.  packed_k and packed_v must be NULL, and the kept rows of
 * unit u are moved to rows 0 .. B_u - 1 of the unit's own rows inside `keys` and `values`, which this call
 * therefore WRITES (the rows behind them keep stale contents).  head_off and kept_idx are written as above;
 * row_capacity then only bounds kept_idx.  A kept row never moves backwards (the j-th kept token has index >= j),
 * and a unit is moved by one workgroup front to back, so no row is overwritten before it has been read.
 * K and V rows must be 32, 64, ..., 1024 bytes long (a power of two); other widths are refused with
 * NKV_EUNSUPPORTED, packed buffers given together with the flag with NKV_EINVAL.
 */
int nkv_select_compact(const void *keys, const void *values, const float *scores,
                       const int32_t *k_per_head, const nkv_shape *shape, const nkv_params *params,
                       void *packed_k, void *packed_v, int32_t *kept_idx, int64_t *head_off,
                       int64_t row_capacity, int64_t *near_threshold_count,
                       void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Decode-side consumer of the compressed cache (Appendix A: retained keys and values are
 * unchanged, so ordinary attention runs over them; Section 3.5 measures the per-token decode
 * latency).  One new token's queries against the output of nkv_select_compact, grouped-query
 * attention with G = n_q_heads / H query heads per KV head: for unit u = (p, l, h) and g < G,
 *   s_i = scale * <q[p][l][h*G+g], packed_k[i]>,  i = head_off[u] .. head_off[u+1]-1
 *   out[p][l][h*G+g] = sum_i softmax(s)_i * packed_v[i]                    fp32 [P][L][n_q_heads][dv]
 *   lse[p][l][h*G+g] = log sum_i exp(s_i)   (optional, may be NULL)        fp32 [P][L][n_q_heads]
 * q is [P][L][n_q_heads][d] in the dtype of the cache.  `rows` is the number of rows packed_k /
 * packed_v hold; head_off entries are clamped to it.  A unit without rows gives out = 0,
 * lse = -inf.  shape->key_strides / value_strides are not used (the packed cache is dense).
 * fp32 arithmetic: exact bf16 products accumulated in fp32, base-2 exponentials of the hardware.
 * Scratch: nkv_decode_workspace_bytes (0 for shapes outside bf16 / fp16, d = dv in {64,128}, G <= 8,
 * which take a slower kernel).  NKV_DTYPE_F8_E4M3 caches are refused (NKV_EUNSUPPORTED): attention
 * over them needs the cache's scale factors, which this library never sees.  Asynchronous on hip_stream.
 */
int nkv_decode_workspace_bytes(const nkv_shape *shape, int32_t n_q_heads, int64_t rows, size_t *bytes);
int nkv_decode_attention(const void *q, const void *packed_k, const void *packed_v, const int64_t *head_off,
                         int64_t rows, const nkv_shape *shape, const nkv_params *params, int32_t n_q_heads,
                         double scale, float *out, float *lse, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Plain device-to-device copy of `bytes` bytes (a multiple of 16, both pointers 16-byte aligned): contiguous
 * 16 KB pieces per workgroup, non-temporal 16-byte loads and stores -- the access pattern of the K/V gather
 * without its indirection.  dst == NULL: the loads only (what a pure reader can reach).  Not part of the pass:
 * it is the yardstick the benchmark measures attainable HBM bandwidth with and calibrates hardware byte
 * counters against.
 */
int nkv_copy_probe(void *dst, const void *src, size_t bytes, void *hip_stream);

/* Static, human-readable text for a status code. */
const char *nkv_strerror(int status);

/* Library version, major * 10000 + minor * 100 + patch. */
int nkv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* NKV_H */
