// extern "C" entry points of libnkv: argument checks, workspace layout, launches.  See include/nkv.h.
#include <math.h>
#include <string.h>

#include <mutex>

#include "nkv_internal.h"

// Scratch of nkv_budget_noalloc, the entry point for callers that cannot allocate.  Every device the library
// runs on holds its own copy at its own address until the process ends.  In host code the array's name is
// only a handle for hipGetSymbolAddress; every use of the memory goes through the address that call returns.
static __device__ __align__(256) unsigned char scratch[NKV_STATIC_SCRATCH_BYTES];

namespace nkv {
namespace {

constexpr size_t kAlign = 256;
size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

int check_params(const nkv_params *p)
{
    if (!p || p->struct_size != sizeof(nkv_params)) return NKV_EINVAL;
    if (p->window < 1 || p->block_div < 1 || p->block_min < 1 || p->block_max < p->block_min) return NKV_EINVAL;
    if (p->n_sink < 0) return NKV_EINVAL;
    if (p->gate_mode < 0 || p->gate_mode > 2 || p->surprise_mode < 0 || p->surprise_mode > 1) return NKV_EINVAL;
    if (!(p->top_frac > 0.0 && p->top_frac <= 1.0)) return NKV_EINVAL;
    for (int k = 0; k < 3; ++k)
        if (!(p->prior[k] >= 0.0) || !isfinite(p->prior[k])) return NKV_EINVAL;
    if (p->scale_mask < 0 || p->scale_mask > 7) return NKV_EINVAL;
    {
        const int mask = p->scale_mask ? p->scale_mask : 7;
        double on = 0.0;
        for (int k = 0; k < 3; ++k) on += (mask >> k) & 1 ? p->prior[k] : 0.0;
        if (!(on > 0.0)) return NKV_EINVAL;                           // the scales that take part need prior weight
    }
    if (!isfinite(p->beta) || !isfinite(p->tau) || !isfinite(p->kappa)) return NKV_EINVAL;
    if (!(p->safeguard >= 0.0 && p->safeguard <= 1.0)) return NKV_EINVAL;
    if (!(p->near_tol >= 0.0) || !isfinite(p->near_tol)) return NKV_EINVAL;
    return NKV_OK;
}

int esize_of(int dtype) { return dtype == NKV_DTYPE_F32 ? 4 : dtype == NKV_DTYPE_F8_E4M3 ? 1 : 2; }

// strides: NULL (dense [L][H][T][row]) or {layer, head, prompt} in elements; layer_offsets: NULL or L entries
int fill_map(const nkv_shape *s, const int64_t *strides, const int64_t *layer_offsets, int row, RowMap *m)
{
    const int64_t T = s->cu_seqlens[s->n_prompts];
    m->H = s->H;
    m->d = row;
    m->per_layer = layer_offsets != nullptr;
    const int epv = 16 / esize_of(s->dtype);
    if (layer_offsets) {
        if (s->L > NKV_MAX_LAYER_TENSORS || layer_offsets[0] != 0) return NKV_EINVAL;
        for (int l = 0; l < s->L; ++l) {
            if (layer_offsets[l] % epv) return NKV_EINVAL;
            m->layer_off[l] = layer_offsets[l];
        }
    }
    if (!strides) {
        m->layer = (int64_t)s->H * T * row;
        m->head = T * row;
        m->prompt = 0;
        if (layer_offsets)                                            // dense layer tensors must not overlap
            for (int i = 0; i < s->L; ++i)
                for (int j = i + 1; j < s->L; ++j) {
                    const int64_t gap = layer_offsets[i] > layer_offsets[j] ? layer_offsets[i] - layer_offsets[j]
                                                                          : layer_offsets[j] - layer_offsets[i];
                    if (gap < m->layer) return NKV_EINVAL;
                }
        return NKV_OK;
    }
    for (int i = 0; i < 3; ++i)
        if (strides[i] < 0 || strides[i] % epv) return NKV_EINVAL;
    // a slab must hold its unit: the longest prompt for per-prompt slabs, all prompts for concatenated ones
    int64_t nmax = 0;
    for (int p = 0; p < s->n_prompts; ++p)
        nmax = nmax > s->cu_seqlens[p + 1] - s->cu_seqlens[p] ? nmax : s->cu_seqlens[p + 1] - s->cu_seqlens[p];
    // No two units may overlap: with the axes of extent > 1 ordered by stride, each stride must cover the
    // whole extent of the axis below it (the innermost one a unit's rows).
    int64_t st[3] = {strides[0], strides[1], strides[2]};
    int64_t ext[3] = {layer_offsets ? 1 : s->L, s->H, strides[2] ? s->n_prompts : 1};
    for (int i = 0; i < 3; ++i)
        for (int j = i + 1; j < 3; ++j)
            if (st[j] < st[i]) {
                const int64_t a = st[i], e = ext[i];
                st[i] = st[j]; ext[i] = ext[j];
                st[j] = a; ext[j] = e;
            }
    int64_t cover = (strides[2] ? nmax : T) * row;
    for (int i = 0; i < 3; ++i) {
        if (ext[i] <= 1) continue;
        if (st[i] < cover) return NKV_EINVAL;
        cover = st[i] * ext[i];
    }
    if (layer_offsets)                                                // cover = what one layer's tensor spans
        for (int i = 0; i < s->L; ++i)
            for (int j = i + 1; j < s->L; ++j) {
                const int64_t gap = layer_offsets[i] > layer_offsets[j] ? layer_offsets[i] - layer_offsets[j]
                                                                      : layer_offsets[j] - layer_offsets[i];
                if (gap < cover) return NKV_EINVAL;
            }
    m->layer = strides[0];
    m->head = strides[1];
    m->prompt = strides[2];
    return NKV_OK;
}

int check_shape(const nkv_shape *s)
{
    if (!s || !s->cu_seqlens) return NKV_EINVAL;
    if (s->dtype < NKV_DTYPE_F32 || s->dtype > NKV_DTYPE_F8_E4M3) return NKV_EINVAL;
    if (s->dtype == NKV_DTYPE_F8_E4M3 && (s->d % 16 || s->dv % 16)) return NKV_ESHAPE;     // rows are 16-byte vectors
    if (s->L < 1 || s->H < 1 || s->H > NKV_MAX_HEADS || (int64_t)s->L * s->H > 65535) return NKV_ESHAPE;
    if (s->d < 8 || s->d > NKV_MAX_HEAD_DIM || s->d % 8) return NKV_ESHAPE;
    if (s->dv < 8 || s->dv > NKV_MAX_HEAD_DIM || s->dv % 8) return NKV_ESHAPE;
    if (s->n_prompts < 1 || s->n_prompts > NKV_MAX_PROMPTS) return NKV_ESHAPE;
    if (s->cu_seqlens[0] != 0) return NKV_ESHAPE;
    for (int p = 0; p < s->n_prompts; ++p)
        if (s->cu_seqlens[p + 1] <= s->cu_seqlens[p]) return NKV_ESHAPE;
    const int64_t T = s->cu_seqlens[s->n_prompts];
    if ((int64_t)s->H * T >= (1ll << 31)) return NKV_ESHAPE;          // per-layer counters are 32-bit
    if ((int64_t)s->L * s->H * T >= (1ll << 40)) return NKV_ESHAPE;
    RowMap m;
    int rc = fill_map(s, s->key_strides, s->key_layer_offsets, s->d, &m);
    if (rc) return rc;
    return fill_map(s, s->value_strides, s->value_layer_offsets, s->dv, &m);
}

void fill_tab(const nkv_shape *s, const nkv_params *p, PromptTab *tab)
{
    memset(tab, 0, sizeof(*tab));
    tab->n = s->n_prompts;
    tab->T = s->cu_seqlens[s->n_prompts];
    int blk = 0;
    for (int i = 0; i < s->n_prompts; ++i) {
        const int64_t N = s->cu_seqlens[i + 1] - s->cu_seqlens[i];
        tab->tok_off[i] = s->cu_seqlens[i];
        tab->b[i] = (int32_t)nkv_block_size(N, p);
        tab->blk_off[i] = blk;
        blk += (int)((N + tab->b[i] - 1) / tab->b[i]);
        tab->m_p[i] = (int32_t)nkv_m_p(N, p->top_frac);
    }
    tab->tok_off[s->n_prompts] = tab->T;
    tab->blk_off[s->n_prompts] = blk;
}

// Workspace of the scoring call, in floats from the (aligned) start.
struct ScoreWs {
    size_t sync, plan, a_raw, rnorm, bsum, ssum, stats, wide, total_bytes;
};

ScoreWs score_ws(const nkv_shape *s, const PromptTab &tab, bool with_a_raw)
{
    const size_t rows = (size_t)s->L * s->H * tab.T;
    const size_t LH = (size_t)s->L * s->H;
    ScoreWs w;
    size_t off = 0;
    w.sync = off;   off += align_up(fast_score_sync_bytes((int)LH, tab));
    w.plan = off;   off += align_up(tile_score_plan_bytes((int)LH, tab));
    w.a_raw = off;  off += with_a_raw ? align_up(3 * rows * 4) : 0;
    w.rnorm = off;  off += align_up(rows * 4);
    w.bsum = off;   off += align_up(LH * tab.blk_off[tab.n] * s->d * 4);
    w.ssum = off;   off += align_up(LH * tab.n * s->d * 8);                      // unit sums: fp32, or 64-bit accumulators
    w.stats = off;  off += align_up(LH * tab.n * 3 * 4 * 4);                 // per unit and scale: min, 1/range, gap
    w.wide = off;   off += with_a_raw ? align_up(stats_wide_ws_bytes(s->L, s->H, tab)) : 0;
    w.total_bytes = off;
    return w;
}

int check_ws(const void *ws, size_t have, size_t need)
{
    if (need == 0) return NKV_OK;
    if (!ws || ((uintptr_t)ws % kAlign) != 0 || have < need) return NKV_EWORKSPACE;
    return NKV_OK;
}

// The fused scan's health counters (first words of its sync area), or zeros, to the caller's two words.
__global__ void scan_counters_kernel(const uint32_t *sync, uint32_t *out)
{
    if (threadIdx.x < 2) out[threadIdx.x] = sync ? sync[threadIdx.x] : 0u;
}

int run_raw(const void *keys, const nkv_shape *s, const nkv_params *p, const PromptTab &tab, float *a_raw,
            char *ws, const ScoreWs &lay, hipStream_t st)
{
    const int LH = s->L * s->H;
    const Prof prof{p->prof_start, p->prof_stop};
    RowMap km;
    const int rc = fill_map(s, s->key_strides, s->key_layer_offsets, s->d, &km);
    if (rc) return rc;
    hipError_t e;
    bool streaming = true;                                            // the sync area starts with this call's counters
    const int mode = (p->flags & NKV_FLAG_TWO_PASS_STABLE)  ? kScanTwoPass
                     : (p->flags & NKV_FLAG_NO_UNIT_SUMS)  ? kScanRepairAll
                     : (p->flags & NKV_FLAG_DEFER_STABLE)  ? kScanDeferAll : kScanFused;
    if (!(p->flags & NKV_FLAG_GENERIC_KERNELS) && !(p->flags & NKV_FLAG_VECTOR_SCAN) && mode != kScanTwoPass &&
        tile_score_supported(s->dtype, s->d, p->window, tab, LH))
        e = launch_score_tile(keys, km, s->dtype, LH, tab, a_raw, ws + lay.ssum, (float *)(ws + lay.bsum), ws + lay.sync, ws + lay.plan,
                              mode, prof, st);
    else if (!(p->flags & NKV_FLAG_GENERIC_KERNELS) && fast_score_supported(s->dtype, s->d, p->window, tab))
        e = launch_score_fast(keys, km, s->dtype, LH, s->d, tab, a_raw, (float *)(ws + lay.bsum), (float *)(ws + lay.ssum),
                              ws + lay.sync, mode, prof, st);
    else {
        streaming = false;
        e = launch_score_generic(keys, km, s->dtype, LH, s->d, p->window, tab, a_raw, (float *)(ws + lay.rnorm),
                                 (float *)(ws + lay.bsum), (float *)(ws + lay.ssum), prof, st);
    }
    if (e == hipSuccess && p->scan_counters) {
        scan_counters_kernel<<<1, 64, 0, st>>>(streaming ? (const uint32_t *)(ws + lay.sync) : nullptr,
                                               (uint32_t *)p->scan_counters);
        e = hipGetLastError();
    }
    return e == hipSuccess ? NKV_OK : NKV_EHIP;
}

// The address of the static scratch array on the current device: looked up once per device, with that device
// current, and kept.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_lock;
void *g_scratch_ptr[kMaxDevices];

int static_scratch(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return NKV_EHIP;
    std::lock_guard<std::mutex> guard(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return NKV_EHIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return NKV_OK;
}

// argument checks and per-prompt integers shared by nkv_budget and nkv_budget_noalloc
int prepare_budget(const float *scores, const nkv_shape *shape, const nkv_params *params, const double *r_per_prompt,
                   const int32_t *k_per_head, PromptTab *tab)
{
    if (!scores || !r_per_prompt || !k_per_head) return NKV_EINVAL;
    int rc = check_shape(shape);
    if (rc) return rc;
    rc = check_params(params);
    if (rc) return rc;
    fill_tab(shape, params, tab);
    for (int p = 0; p < shape->n_prompts; ++p) {
        const int64_t N = shape->cu_seqlens[p + 1] - shape->cu_seqlens[p];
        const int64_t k0 = nkv_k0(N, r_per_prompt[p]);
        if (k0 < 0) return NKV_EINVAL;
        tab->k0[p] = (int32_t)k0;
        tab->m_safe[p] = (int32_t)nkv_m_safe(k0, params->safeguard);
    }
    return NKV_OK;
}

}  // namespace
}  // namespace nkv

using namespace nkv;

extern "C" {

int nkv_params_default(nkv_params *p)
{
    if (!p) return NKV_EINVAL;
    memset(p, 0, sizeof(*p));
    p->struct_size = (uint32_t)sizeof(nkv_params);
    p->window = 64;
    p->block_div = 32;
    p->block_min = 128;
    p->block_max = 256;
    p->n_sink = 4;
    p->gate_mode = NKV_GATE_SURPRISE;
    p->surprise_mode = NKV_SURPRISE_NORMALISED;
    p->scale_mask = 7;
    p->top_frac = 0.10;
    p->prior[0] = 0.4; p->prior[1] = 0.4; p->prior[2] = 0.2;
    p->beta = 3.0;
    p->tau = 0.60;
    p->kappa = 10.0;
    p->safeguard = 0.20;
    p->near_tol = 1e-5;
    return NKV_OK;
}

int64_t nkv_block_size(int64_t N, const nkv_params *p)
{
    if (!p || N < 1 || p->block_div < 1 || p->block_min < 1 || p->block_max < p->block_min) return -1;
    int64_t b = N / p->block_div;
    if (b < p->block_min) b = p->block_min;
    if (b > p->block_max) b = p->block_max;
    return b;
}

int64_t nkv_k0(int64_t N, double r)
{
    if (N < 0 || !(r >= 0.0 && r <= 1.0)) return -1;
    int64_t k = (int64_t)floor((1.0 - r) * (double)N + 1e-9);
    return k > N ? N : k;
}

int64_t nkv_m_safe(int64_t k0, double safeguard)
{
    if (k0 < 0 || !(safeguard >= 0.0 && safeguard <= 1.0)) return -1;
    int64_t m = (int64_t)floor(safeguard * (double)k0 + 1e-9);
    return m > k0 ? k0 : m;
}

int64_t nkv_m_p(int64_t N, double top_frac)
{
    if (N < 1 || !(top_frac > 0.0 && top_frac <= 1.0)) return -1;
    int64_t m = (int64_t)floor(top_frac * (double)N + 1e-9);
    if (m < 1) m = 1;
    return m > N ? N : m;
}

int nkv_packed_rows(const nkv_shape *shape, const double *r_per_prompt, int64_t *rows)
{
    if (!r_per_prompt || !rows) return NKV_EINVAL;
    int rc = check_shape(shape);
    if (rc) return rc;
    int64_t n = 0;
    for (int p = 0; p < shape->n_prompts; ++p) {
        const int64_t k0 = nkv_k0(shape->cu_seqlens[p + 1] - shape->cu_seqlens[p], r_per_prompt[p]);
        if (k0 < 0) return NKV_EINVAL;
        n += (int64_t)shape->L * shape->H * k0;
    }
    *rows = n;
    return NKV_OK;
}

int nkv_workspace_bytes(const nkv_shape *shape, const nkv_params *params, size_t *bytes)
{
    if (!bytes) return NKV_EINVAL;
    int rc = check_shape(shape);
    if (rc) return rc;
    rc = check_params(params);
    if (rc) return rc;
    PromptTab tab;
    fill_tab(shape, params, &tab);
    const size_t a = score_ws(shape, tab, true).total_bytes, b = align_up(budget_ws_bytes(shape->L, shape->H, tab));
    const size_t c = align_up(select_wide_ws_bytes(shape->L, shape->H, tab));
    *bytes = a > b ? (a > c ? a : c) : (b > c ? b : c);
    return NKV_OK;
}

int nkv_score_raw(const void *keys, const nkv_shape *shape, const nkv_params *params, float *a_raw, void *ws,
                  size_t ws_bytes, void *hip_stream)
{
    if (!keys || !a_raw) return NKV_EINVAL;
    int rc = check_shape(shape);
    if (rc) return rc;
    rc = check_params(params);
    if (rc) return rc;
    if ((uintptr_t)keys % 16) return NKV_EINVAL;
    PromptTab tab;
    fill_tab(shape, params, &tab);
    const ScoreWs lay = score_ws(shape, tab, false);
    rc = check_ws(ws, ws_bytes, lay.total_bytes);
    if (rc) return rc;
    return run_raw(keys, shape, params, tab, a_raw, (char *)ws, lay, (hipStream_t)hip_stream);
}

int nkv_score(const void *keys, const nkv_shape *shape, const nkv_params *params, float *scores, void *ws,
              size_t ws_bytes, void *hip_stream)
{
    if (!keys || !scores) return NKV_EINVAL;
    int rc = check_shape(shape);
    if (rc) return rc;
    rc = check_params(params);
    if (rc) return rc;
    if ((uintptr_t)keys % 16) return NKV_EINVAL;
    PromptTab tab;
    fill_tab(shape, params, &tab);
    const ScoreWs lay = score_ws(shape, tab, true);
    rc = check_ws(ws, ws_bytes, lay.total_bytes);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)hip_stream;
    float *a_raw = (float *)((char *)ws + lay.a_raw);
    rc = run_raw(keys, shape, params, tab, a_raw, (char *)ws, lay, st);
    if (rc) return rc;
    LearnerConsts lc;
    lc.scale_mask = params->scale_mask ? params->scale_mask : 7;
    for (int k = 0; k < 3; ++k)                                            // -inf: no weight in the blend
        lc.log_prior[k] = (lc.scale_mask >> k) & 1 ? log(params->prior[k]) : -INFINITY;
    lc.beta = params->beta;
    lc.tau = (float)params->tau;
    lc.kappa = (float)params->kappa;
    lc.n_sink = params->n_sink;
    lc.gate_mode = params->gate_mode;
    lc.surprise_mode = params->surprise_mode;
    const Prof prof{params->prof_start, params->prof_stop};
    return launch_finalize(a_raw, shape->L, shape->H, tab, lc, scores, (float *)((char *)ws + lay.stats),
                           (char *)ws + lay.wide, (params->flags & NKV_FLAG_STATS_PER_HEAD) != 0, prof,
                           st) == hipSuccess
               ? NKV_OK : NKV_EHIP;
}

int nkv_budget(const float *scores, const nkv_shape *shape, const nkv_params *params, const double *r_per_prompt,
               int32_t *k_per_head, void *ws, size_t ws_bytes, void *hip_stream)
{
    PromptTab tab;
    int rc = prepare_budget(scores, shape, params, r_per_prompt, k_per_head, &tab);
    if (rc) return rc;
    if (ws != nullptr) {
        rc = check_ws(ws, ws_bytes, budget_ws_bytes(shape->L, shape->H, tab));
        if (rc) return rc;
    }
    const Prof prof{params->prof_start, params->prof_stop};
    return launch_budget(scores, shape->L, shape->H, tab, k_per_head, ws,
                         (params->flags & NKV_FLAG_BUDGET_PER_HEAD) != 0, prof, (hipStream_t)hip_stream) == hipSuccess
               ? NKV_OK : NKV_EHIP;
}

int nkv_budget_noalloc(const float *scores, const nkv_shape *shape, const nkv_params *params,
                       const double *r_per_prompt, int32_t *k_per_head, void *hip_stream)
{
    PromptTab tab;
    int rc = prepare_budget(scores, shape, params, r_per_prompt, k_per_head, &tab);
    if (rc) return rc;
    if (budget_ws_bytes(shape->L, shape->H, tab) > (size_t)NKV_STATIC_SCRATCH_BYTES) return NKV_ESCRATCH;
    void *ws = nullptr;
    rc = static_scratch(&ws);
    if (rc) return rc;
    // The budget kernels write every word of their scratch before they read it, so nothing of the previous
    // call's contents has to be cleared.
    const Prof prof{params->prof_start, params->prof_stop};
    return launch_budget(scores, shape->L, shape->H, tab, k_per_head, ws,
                         (params->flags & NKV_FLAG_BUDGET_PER_HEAD) != 0, prof, (hipStream_t)hip_stream) == hipSuccess
               ? NKV_OK : NKV_EHIP;
}

int nkv_select_compact(const void *keys, const void *values, const float *scores, const int32_t *k_per_head,
                       const nkv_shape *shape, const nkv_params *params, void *packed_k, void *packed_v,
                       int32_t *kept_idx, int64_t *head_off, int64_t row_capacity, int64_t *near_threshold_count,
                       void *ws, size_t ws_bytes, void *hip_stream)
{
    if (!keys || !values || !scores || !k_per_head || !head_off || row_capacity < 0) return NKV_EINVAL;
    int rc = check_shape(shape);
    if (rc) return rc;
    rc = check_params(params);
    if (rc) return rc;
    const bool in_place = (params->flags & NKV_FLAG_COMPACT_IN_PLACE) != 0;
    if (in_place ? (packed_k || packed_v) : (row_capacity > 0 && (!packed_k || !packed_v))) return NKV_EINVAL;
    if (row_capacity > 0 && !kept_idx) return NKV_EINVAL;
    if (in_place) {                                                   // rows of 32 .. 1024 bytes, a power of two
        for (const int bytes : {shape->d * esize_of(shape->dtype), shape->dv * esize_of(shape->dtype)})
            if (bytes < 32 || bytes > 1024 || (bytes & (bytes - 1))) return NKV_EUNSUPPORTED;
    }
    if ((uintptr_t)keys % 16 || (uintptr_t)values % 16 || (uintptr_t)packed_k % 16 || (uintptr_t)packed_v % 16)
        return NKV_EINVAL;
    PromptTab tab;
    fill_tab(shape, params, &tab);
    RowMap km, vm;
    rc = fill_map(shape, shape->key_strides, shape->key_layer_offsets, shape->d, &km);
    if (rc) return rc;
    rc = fill_map(shape, shape->value_strides, shape->value_layer_offsets, shape->dv, &vm);
    if (rc) return rc;
    if (ws != nullptr) {
        rc = check_ws(ws, ws_bytes, select_wide_ws_bytes(shape->L, shape->H, tab));
        if (rc) return rc;
    }
    return launch_select_compact(keys, values, km, vm, (params->flags & NKV_FLAG_SELECT_PER_HEAD) ? nullptr : ws,
                                 scores, k_per_head, shape->L, shape->H, shape->d, shape->dv,
                                 esize_of(shape->dtype), tab, (float)params->near_tol, packed_k, packed_v,
                                 kept_idx, head_off, row_capacity, near_threshold_count, in_place,
                                 Prof{params->prof_start, params->prof_stop}, (hipStream_t)hip_stream) == hipSuccess
               ? NKV_OK : NKV_EHIP;
}

int nkv_decode_workspace_bytes(const nkv_shape *shape, int32_t n_q_heads, int64_t rows, size_t *bytes)
{
    if (!bytes || rows < 0) return NKV_EINVAL;
    int rc = check_shape(shape);
    if (rc) return rc;
    if (n_q_heads < shape->H || n_q_heads % shape->H) return NKV_EINVAL;
    if (shape->dtype == NKV_DTYPE_F8_E4M3) return NKV_EUNSUPPORTED;
    *bytes = decode_ws_bytes(shape->dtype, shape->d, shape->dv, n_q_heads / shape->H,
                             (int64_t)shape->n_prompts * shape->L * shape->H, rows);
    return NKV_OK;
}

int nkv_decode_attention(const void *q, const void *packed_k, const void *packed_v, const int64_t *head_off,
                         int64_t rows, const nkv_shape *shape, const nkv_params *params, int32_t n_q_heads,
                         double scale, float *out, float *lse, void *ws, size_t ws_bytes, void *hip_stream)
{
    if (!q || !head_off || !out || rows < 0 || !isfinite(scale)) return NKV_EINVAL;
    if (rows > 0 && (!packed_k || !packed_v)) return NKV_EINVAL;
    int rc = check_shape(shape);
    if (rc) return rc;
    rc = check_params(params);
    if (rc) return rc;
    if (n_q_heads < shape->H || n_q_heads % shape->H) return NKV_EINVAL;
    if (shape->dtype == NKV_DTYPE_F8_E4M3) return NKV_EUNSUPPORTED;  // needs the cache's scale factors
    if ((uintptr_t)q % 16 || (uintptr_t)packed_k % 16 || (uintptr_t)packed_v % 16) return NKV_EINVAL;
    const int G = n_q_heads / shape->H;
    const int64_t n_units = (int64_t)shape->n_prompts * shape->L * shape->H;
    if (n_units * G >= (1ll << 31) || rows / 256 + n_units >= (1ll << 31)) return NKV_ESHAPE;
    rc = check_ws(ws, ws_bytes, decode_ws_bytes(shape->dtype, shape->d, shape->dv, G, n_units, rows));
    if (rc) return rc;
    return launch_decode(q, packed_k, packed_v, head_off, shape->dtype, (int)n_units, G, shape->d, shape->dv, rows,
                         scale, out, lse, ws, Prof{params->prof_start, params->prof_stop},
                         (hipStream_t)hip_stream) == hipSuccess
               ? NKV_OK : NKV_EHIP;
}

int nkv_copy_probe(void *dst, const void *src, size_t bytes, void *hip_stream)
{
    if (!src || bytes % 16 || (uintptr_t)dst % 16 || (uintptr_t)src % 16) return NKV_EINVAL;
    return launch_copy_probe(dst, src, bytes, (hipStream_t)hip_stream) == hipSuccess ? NKV_OK : NKV_EHIP;
}

const char *nkv_strerror(int status)
{
    switch (status) {
    case NKV_OK: return "ok";
    case NKV_EINVAL: return "invalid argument (null pointer, misaligned tensor, parameter or ratio out of range)";
    case NKV_ESHAPE: return "invalid shape (L, H, d, dv, prompt count or cu_seqlens)";
    case NKV_EWORKSPACE: return "workspace missing, misaligned or too small";
    case NKV_EHIP: return "HIP runtime error while enqueuing kernels";
    case NKV_EUNSUPPORTED: return "request not covered by the kernels";
    case NKV_ESCRATCH: return "shape needs more scratch than the library's static array holds (NKV_STATIC_SCRATCH_BYTES)";
    default: return "unknown status";
    }
}

int nkv_version(void) { return 100; }

}  // extern "C"
