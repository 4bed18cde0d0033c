// Internal declarations shared by the HIP sources of libnkv (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nkv.h"

namespace nkv {

// Per-prompt integers, passed to kernels by value (kernel argument segment).
struct PromptTab {
    int32_t n;                               // prompts
    int32_t T;                               // total tokens
    int32_t tok_off[NKV_MAX_PROMPTS + 1];    // first token row of the prompt (cu_seqlens)
    int32_t b[NKV_MAX_PROMPTS];              // episodic block size of the prompt
    int32_t blk_off[NKV_MAX_PROMPTS + 1];    // blocks before this prompt (per head)
    int32_t m_p[NKV_MAX_PROMPTS];            // size of the top / bottom sets
    int32_t k0[NKV_MAX_PROMPTS];             // filled for nkv_budget only
    int32_t m_safe[NKV_MAX_PROMPTS];         // filled for nkv_budget only
};

// Where the rows of a (layer, head, prompt) unit start inside the keys (or values) tensor, in elements.
// The rows of a unit are always contiguous (row n at +n*d).  prompt == 0: the prompts of a head are
// concatenated along the token axis (unit p starts tok_off[p] rows into the head); otherwise every prompt has
// its own slab and unit p starts p * prompt elements into the head.
struct RowMap {
    int64_t layer, head, prompt;
    int32_t H, d;
    int32_t per_layer;                   // non-zero: layer l starts at layer_off[l] instead of l * layer
    int64_t layer_off[NKV_MAX_LAYER_TENSORS];
    __host__ __device__ int64_t unit(int l, int h, int p, const PromptTab &tab) const
    {
        return (per_layer ? layer_off[l] : l * layer) + h * head +
               (prompt != 0 ? p * prompt : (int64_t)tab.tok_off[p] * d);
    }
    __host__ __device__ int64_t unit(int lh, int p, const PromptTab &tab) const
    {
        const int l = lh / H;
        return unit(l, lh - l * H, p, tab);
    }
};

// Scalars of the outer learner in the precision the kernels use them.
struct LearnerConsts {
    double log_prior[3];
    double beta;
    float tau, kappa;
    int32_t n_sink, gate_mode, surprise_mode;
    int32_t scale_mask;                  // bit k set: scale k (stable, episodic, current) takes part
};

// Optional event pair around one kernel launch (nkv_params.prof_start / prof_stop).
struct Prof {
    void *const *start = nullptr;
    void *const *stop = nullptr;
    void begin(int k, hipStream_t st) const
    {
        if (start && start[k] && stop[k]) (void)hipEventRecord((hipEvent_t)start[k], st);
    }
    void end(int k, hipStream_t st) const
    {
        if (start && start[k] && stop[k]) (void)hipEventRecord((hipEvent_t)stop[k], st);
    }
};

constexpr float kEps = 1e-12f;    // clamp of vector norms
constexpr float kFlat = 1e-6f;    // a min-max range below this carries no ranking

// ---- scoring, shape-generic kernels (any d multiple of 8, any window / block size, fp32 or bf16) ----
hipError_t launch_score_generic(const void *keys, const RowMap &km, int dtype, int LH, int d, int window, const PromptTab &tab,
                                float *a_raw, float *rnorm, float *bsum, float *ssum, const Prof &prof,
                                hipStream_t st);

// ---- scoring, streaming kernels for bf16 keys, d in {64,128}, window 64, block size <= 256 ----
bool fast_score_supported(int dtype, int d, int window, const PromptTab &tab);
size_t fast_score_sync_bytes(int LH, const PromptTab &tab);
// How the stable anomaly is obtained.  kScanDeferAll: fused pass, but every block takes the deferred route;
// kScanRepairAll: in addition no unit sum is formed inside the pass, all come from the repair kernel.
enum { kScanFused = 0, kScanTwoPass = 1, kScanDeferAll = 2, kScanRepairAll = 3 };
hipError_t launch_score_fast(const void *keys, const RowMap &km, int dtype, int LH, int d, const PromptTab &tab, float *a_raw,
                             float *bsum, float *ssum, void *sync_area, int mode, const Prof &prof, hipStream_t st);

// ---- scoring, matrix-core formulation of the fused streaming pass (bf16 or fp16, d = 128, window 64, block size <= 256) ----
bool tile_score_supported(int dtype, int d, int window, const PromptTab &tab, int LH);
size_t tile_score_plan_bytes(int LH, const PromptTab &tab);    // the list of items the pass works through
hipError_t launch_score_tile(const void *keys, const RowMap &km, int dtype, int LH, const PromptTab &tab, float *a_raw,
                             void *accum, float *ssum, void *sync_area, void *plan_area, int mode, const Prof &prof,
                             hipStream_t st);

// Units are numbered prompt by prompt, so the units of consecutive prompts of similar length form one
// range.  Calls f(ept, unit0, units) for every maximal run of prompts whose lengths need the same number
// ept in {4, 8, 16, 32} of values per thread in the 1024-thread per-unit kernels (N <= 1024 * ept).
template <typename F> inline void for_each_length_class(const PromptTab &tab, int LH, F f)
{
    auto cls = [](int N) { return N <= 4096 ? 4 : N <= 8192 ? 8 : N <= 16384 ? 16 : 32; };
    int p = 0;
    while (p < tab.n) {
        const int c = cls(tab.tok_off[p + 1] - tab.tok_off[p]);
        int q = p + 1;
        while (q < tab.n && cls(tab.tok_off[q + 1] - tab.tok_off[q]) == c) ++q;
        f(c, p * LH, (q - p) * LH);
        p = q;
    }
}

// ---- per-head statistics, blend weights, gate and final scores ----
// wide_ws: scratch of stats_wide_ws_bytes() for the slice-wise statistics (NULL: per-head kernels only);
// per_head_route: do not use the slice-wise kernels
hipError_t launch_finalize(const float *a_raw, int L, int H, const PromptTab &tab, const LearnerConsts &lc,
                           float *scores, float *stats, void *wide_ws, bool per_head_route, const Prof &prof,
                           hipStream_t st);
// slice-wise statistics (nkv_finalize_wide.hip)
size_t stats_wide_ws_bytes(int L, int H, const PromptTab &tab);
hipError_t launch_stats_wide(const float *a_raw, int L, int H, const PromptTab &tab, int scale_mask, float *stats, void *ws,
                             hipStream_t st);
hipError_t launch_route_wide(const float *a_raw, int L, int H, const PromptTab &tab, const LearnerConsts &lc,
                             const float *stats, void *ws, float *scores, hipStream_t st);

// ---- head-wise budgets ----
size_t budget_ws_bytes(int L, int H, const PromptTab &tab);
// ws == nullptr selects the shape-generic kernel, which needs no scratch
// per_head_route: use the kernels that hold a head in one workgroup instead of the slice-wise ones
hipError_t launch_budget(const float *scores, int L, int H, const PromptTab &tab, int32_t *k_per_head, void *ws,
                         bool per_head_route, const Prof &prof, hipStream_t st);
// slice-wise kernels (nkv_budget_wide.hip)
// heads-parallel budget kernels for layers of more than 8 heads (nkv_budget_heads.hip)
size_t budget_heads_ws_bytes(int L, int H, const PromptTab &tab);
hipError_t launch_budget_heads(const float *scores, int L, int H, const PromptTab &tab, int32_t *k_per_head, void *ws,
                               hipStream_t st);
bool budget_wide_supported(int H);
size_t budget_wide_ws_bytes(int L, int H, const PromptTab &tab);
hipError_t launch_budget_wide(const float *scores, int L, int H, const PromptTab &tab, int32_t *k_per_head, void *ws,
                              const uint32_t **failed_flags, hipStream_t st);

// ---- selection, ordered compaction, gather ----
// wide_ws: scratch of select_wide_ws_bytes() for the slice-wise selection (NULL: per-unit kernels only)
size_t select_wide_ws_bytes(int L, int H, const PromptTab &tab);
bool select_wide_places_units(int n_units);           // launch_select_wide can fill head_off and zero near_count itself
hipError_t launch_select_wide(const float *scores, const int32_t *k_per_head, int L, int H, const PromptTab &tab,
                              float near_tol, int64_t *head_off, int64_t row_capacity, int32_t *kept_idx,
                              int64_t *near_count, bool with_head_off, void *ws, hipStream_t st);
hipError_t launch_select_compact(const void *keys, const void *values, const RowMap &km, const RowMap &vm,
                                 void *wide_ws, const float *scores,
                                 const int32_t *k_per_head, int L, int H, int d, int dv, int esize,
                                 const PromptTab &tab, float near_tol, void *packed_k, void *packed_v,
                                 int32_t *kept_idx, int64_t *head_off, int64_t row_capacity,
                                 int64_t *near_count, bool in_place, const Prof &prof, hipStream_t st);

// ---- decode-side consumer: attention of one new token over the packed cache ----
bool decode_fast_supported(int dtype, int d, int dv, int G);
size_t decode_ws_bytes(int dtype, int d, int dv, int G, int64_t n_units, int64_t rows);
hipError_t launch_decode(const void *q, const void *pk, const void *pv, const int64_t *head_off, int dtype,
                         int n_units, int G, int d, int dv, int64_t rows, double scale, float *out, float *lse,
                         void *ws, const Prof &prof, hipStream_t st);

// ---- plain copy, the bandwidth yardstick ----
hipError_t launch_copy_probe(void *dst, const void *src, size_t bytes, hipStream_t st);

}  // namespace nkv
