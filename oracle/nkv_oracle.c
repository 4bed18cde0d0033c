/*
 * NestedKV prefill compression pass -- plain CPU oracle.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, step-by-step statement of
 * what the pass computes, written from the paper (Sections 2.1-2.6 and
 * Appendix A "Implementation Details"), in fp64, with naive sums and full
 * sorts.  It shares no code with the HIP library and is called only by the
 * tests, by the smoke check and by the benchmark's cpu_baseline leg.  It is
 * never tuned; OpenMP over the independent KV heads of a layer is the only
 * concession to running time.
 *
 * Conventions (0-based token index i, one prompt, one layer at a time):
 *   keys   [H][N][d]  float  (bf16 inputs are widened exactly by the caller)
 *   scores [H][N]     float  (the fp64 result a* rounded once to fp32)
 *
 * Readings of points the paper leaves open (all listed in the design notes):
 *   - norms are clamped below by EPS = 1e-12 (zero key => k_hat = 0, cos = 0);
 *   - the current window [max(0, i-W+1), i] includes token i;
 *   - blocks start at token 0, the last one may be short and divides by its
 *     own length; N <= b means a single block;
 *   - min-max runs over all N tokens of the head (sinks included); a range
 *     below FLAT = 1e-6 means the reading carries no ranking and gives all
 *     zeros (a division by such a range would only amplify rounding noise);
 *   - top/bottom sets of the reliability gap hold m_p = max(1, floor(p*N+1e-9));
 *   - std is the population one (ddof = 0) unless told otherwise;
 *   - scale_mask (bit k set: scale k takes part; stable, episodic, current = bits 0, 1, 2): a scale that is
 *     switched off is left out of the blend (the softmax runs over the others), of the winner and of the
 *     standard deviation alike: the Appendix's component ablation "Stable + episodic (no current)" is mask 3;
 *   - surprise_mode 0: min-max within the head, subtract the head mean, clamp
 *     at zero (Appendix A), then gate; surprise_mode 1: gate the raw std
 *     (Section 2.4 taken literally);
 *   - the first min(n_sink, N) scores are overwritten with PIN = 3.0e38f as the
 *     last step of scoring;
 *   - layer budget = H * k0, k0 = floor((1-r)*N + 1e-9); per-head safeguard
 *     m_safe = floor(safeguard * k0 + 1e-9);
 *   - ties: higher score first, then lower head, then lower token index;
 *     kept indices are returned in ascending token order.
 *
 * parity: every function here is pinned by tests/test_oracle_*.py (closed
 * forms, invariants, special cases checked against numpy/scipy routines and
 * brute force).  What no test can pin -- agreement with the authors' own code
 * on the readings above -- is "parity unpinned" and is said so there.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define NKVO_EPS 1e-12
#define NKVO_FLAT 1e-6
#define NKVO_PIN 3.0e38f

typedef struct {
    int32_t window;        /* W, Section 2.2 "Current memory" (64)            */
    int32_t block_div;     /* 32  } b = clip(floor(N/div), min, max),        */
    int32_t block_min;     /* 128 } Section 2.2 "Episodic memory"            */
    int32_t block_max;     /* 256 }                                          */
    int32_t n_sink;        /* 4, Section 2.3                                 */
    int32_t gate_mode;     /* 0 surprise gate, 1 only average, 2 only max    */
    int32_t surprise_mode; /* see header                                     */
    int32_t std_ddof;      /* 0 population, 1 sample                         */
    int32_t scale_mask;    /* bits 0..2: stable, episodic, current take part */
    int32_t pad_;
    double top_frac;       /* p = 0.10, Section 2.4                          */
    double prior[3];       /* (0.4, 0.4, 0.2) order stable, episodic, current*/
    double beta, tau, kappa; /* 3.0, 0.60, 10.0, Appendix A                  */
} nkvo_params;

/* Optional intermediates; any pointer may be NULL. */
typedef struct {
    double *mu_s;     /* [H][d]                 stable anchor                 */
    double *mu_e;     /* [H][nblk][d]           one episodic anchor per block */
    double *mu_c;     /* [H][N][d]              current anchor per token      */
    double *a_raw;    /* [3][H][N]              a_s, a_e, a_c                 */
    double *a_tilde;  /* [3][H][N]              after per-head min-max        */
    double *delta;    /* [H][3]                 reliability gaps              */
    double *w;        /* [H][3]                 blend weights                 */
    double *surprise; /* [H][N]                 s(i) as gated (after mode)    */
    double *alpha;    /* [H][N]                 gate                          */
    double *blend;    /* [H][N]                                               */
    double *win;      /* [H][N]                                               */
} nkvo_debug;

void nkvo_params_default(nkvo_params *p)
{
    p->window = 64; p->block_div = 32; p->block_min = 128; p->block_max = 256;
    p->n_sink = 4; p->gate_mode = 0; p->surprise_mode = 0; p->std_ddof = 0;
    p->scale_mask = 7; p->pad_ = 0;
    p->top_frac = 0.10;
    p->prior[0] = 0.4; p->prior[1] = 0.4; p->prior[2] = 0.2;
    p->beta = 3.0; p->tau = 0.60; p->kappa = 10.0;
}

/* Section 2.2, block-size schedule. */
int64_t nkvo_block_size(int64_t N, const nkvo_params *p)
{
    int64_t b = N / p->block_div;
    if (b < p->block_min) b = p->block_min;
    if (b > p->block_max) b = p->block_max;
    return b;
}

/* Appendix A: retained positions per head before competition, floor((1-r)N). */
int64_t nkvo_k0(int64_t N, double r)
{
    return (int64_t)floor((1.0 - r) * (double)N + 1e-9);
}

/* Appendix A: per-head safeguard floor(alpha_s * k0). */
int64_t nkvo_m_safe(int64_t k0, double safeguard)
{
    return (int64_t)floor(safeguard * (double)k0 + 1e-9);
}

/* Section 2.4: size of the top / bottom sets. */
int64_t nkvo_m_p(int64_t N, double top_frac)
{
    int64_t m = (int64_t)floor(top_frac * (double)N + 1e-9);
    return m < 1 ? 1 : m;
}

static double dotd(const double *a, const double *b, int d)
{
    double s = 0.0;
    for (int c = 0; c < d; ++c) s += a[c] * b[c];
    return s;
}

static double clamp_eps(double x) { return x < NKVO_EPS ? NKVO_EPS : x; }

/* Section 2.3: a = -cos(k_hat, mu), norms clamped. */
static double neg_cos(const double *kh, const double *mu, int d)
{
    double nk = sqrt(dotd(kh, kh, d));
    double nm = sqrt(dotd(mu, mu, d));
    return -dotd(kh, mu, d) / (clamp_eps(nk) * clamp_eps(nm));
}

static int cmp_double_asc(const void *x, const void *y)
{
    double a = *(const double *)x, b = *(const double *)y;
    return (a > b) - (a < b);
}

static void minmax_normalise(const double *a, double *out, int64_t N)
{
    double lo = a[0], hi = a[0];
    for (int64_t i = 1; i < N; ++i) { if (a[i] < lo) lo = a[i]; if (a[i] > hi) hi = a[i]; }
    double range = hi - lo;
    for (int64_t i = 0; i < N; ++i) out[i] = range < NKVO_FLAT ? 0.0 : (a[i] - lo) / range;
}

static int score_head(const float *K, int64_t N, int d, const nkvo_params *p, float *scores,
                      int h, int H, const nkvo_debug *dbg)
{
    const int64_t W = p->window;
    const int64_t b = nkvo_block_size(N, p);
    const int64_t nblk = (N + b - 1) / b;
    double *kh = (double *)malloc(sizeof(double) * N * d);
    double *mu = (double *)malloc(sizeof(double) * d);
    double *a[3], *at[3];
    for (int k = 0; k < 3; ++k) {
        a[k] = (double *)malloc(sizeof(double) * N);
        at[k] = (double *)malloc(sizeof(double) * N);
    }
    double *srt = (double *)malloc(sizeof(double) * N);
    double *s = (double *)malloc(sizeof(double) * N);
    if (!kh || !mu || !a[2] || !at[2] || !srt || !s) return -1;

    /* Section 2.1: k_hat = k / ||k||. */
    for (int64_t i = 0; i < N; ++i) {
        double ss = 0.0;
        for (int c = 0; c < d; ++c) { double x = (double)K[i * d + c]; ss += x * x; }
        double nrm = clamp_eps(sqrt(ss));
        for (int c = 0; c < d; ++c) kh[i * d + c] = (double)K[i * d + c] / nrm;
    }

    /* Stable memory: mean over the whole prompt. */
    for (int c = 0; c < d; ++c) mu[c] = 0.0;
    for (int64_t i = 0; i < N; ++i)
        for (int c = 0; c < d; ++c) mu[c] += kh[i * d + c];
    for (int c = 0; c < d; ++c) mu[c] /= (double)N;
    if (dbg && dbg->mu_s) memcpy(dbg->mu_s + (size_t)h * d, mu, sizeof(double) * d);
    for (int64_t i = 0; i < N; ++i) a[0][i] = neg_cos(kh + i * d, mu, d);

    /* Episodic memory: mean over the block holding i. */
    for (int64_t blk = 0; blk < nblk; ++blk) {
        int64_t lo = blk * b, hi = lo + b < N ? lo + b : N;
        for (int c = 0; c < d; ++c) mu[c] = 0.0;
        for (int64_t j = lo; j < hi; ++j)
            for (int c = 0; c < d; ++c) mu[c] += kh[j * d + c];
        for (int c = 0; c < d; ++c) mu[c] /= (double)(hi - lo);
        if (dbg && dbg->mu_e) memcpy(dbg->mu_e + ((size_t)h * nblk + blk) * d, mu, sizeof(double) * d);
        for (int64_t i = lo; i < hi; ++i) a[1][i] = neg_cos(kh + i * d, mu, d);
    }

    /* Current memory: causal window ending at i, summed directly. */
    for (int64_t i = 0; i < N; ++i) {
        int64_t lo = i - W + 1 < 0 ? 0 : i - W + 1;
        for (int c = 0; c < d; ++c) mu[c] = 0.0;
        for (int64_t j = lo; j <= i; ++j)
            for (int c = 0; c < d; ++c) mu[c] += kh[j * d + c];
        for (int c = 0; c < d; ++c) mu[c] /= (double)(i - lo + 1);
        if (dbg && dbg->mu_c) memcpy(dbg->mu_c + ((size_t)h * N + i) * d, mu, sizeof(double) * d);
        a[2][i] = neg_cos(kh + i * d, mu, d);
    }

    /* Section 2.3: per-head min-max of each scale. */
    for (int k = 0; k < 3; ++k) {
        minmax_normalise(a[k], at[k], N);
        if (dbg && dbg->a_raw) memcpy(dbg->a_raw + ((size_t)k * H + h) * N, a[k], sizeof(double) * N);
        if (dbg && dbg->a_tilde) memcpy(dbg->a_tilde + ((size_t)k * H + h) * N, at[k], sizeof(double) * N);
    }

    /* Section 2.4: reliability gaps and head-adaptive weights, over the scales that take part. */
    const int64_t mp = nkvo_m_p(N, p->top_frac) > N ? N : nkvo_m_p(N, p->top_frac);
    int on[3], n_on = 0;
    for (int k = 0; k < 3; ++k) { on[k] = (p->scale_mask >> k) & 1; n_on += on[k]; }
    double delta[3], w[3], z[3], zmax = -INFINITY, zsum = 0.0;
    for (int k = 0; k < 3; ++k) {
        memcpy(srt, at[k], sizeof(double) * N);
        qsort(srt, (size_t)N, sizeof(double), cmp_double_asc);
        double top = 0.0, bot = 0.0;
        for (int64_t j = 0; j < mp; ++j) { bot += srt[j]; top += srt[N - 1 - j]; }
        delta[k] = top / (double)mp - bot / (double)mp;
        z[k] = on[k] ? log(p->prior[k]) + p->beta * delta[k] : -INFINITY;
        if (z[k] > zmax) zmax = z[k];
    }
    for (int k = 0; k < 3; ++k) { w[k] = on[k] ? exp(z[k] - zmax) : 0.0; zsum += w[k]; }
    for (int k = 0; k < 3; ++k) w[k] /= zsum;
    if (dbg && dbg->delta) memcpy(dbg->delta + (size_t)h * 3, delta, sizeof(delta));
    if (dbg && dbg->w) memcpy(dbg->w + (size_t)h * 3, w, sizeof(w));

    /* Compression-induced surprise: std over the normalised readings that take part. */
    for (int64_t i = 0; i < N; ++i) {
        double m = 0.0, v = 0.0;
        for (int k = 0; k < 3; ++k) if (on[k]) m += at[k][i];
        m /= (double)n_on;
        for (int k = 0; k < 3; ++k) if (on[k]) v += (at[k][i] - m) * (at[k][i] - m);
        s[i] = n_on - p->std_ddof > 0 ? sqrt(v / (double)(n_on - p->std_ddof)) : 0.0;
    }
    if (p->surprise_mode == 0) {
        minmax_normalise(s, s, N);
        double mean = 0.0;
        for (int64_t i = 0; i < N; ++i) mean += s[i];
        mean /= (double)N;
        for (int64_t i = 0; i < N; ++i) s[i] = s[i] - mean > 0.0 ? s[i] - mean : 0.0;
    }

    /* Routed score. */
    for (int64_t i = 0; i < N; ++i) {
        double blend = 0.0, win = -INFINITY;
        for (int k = 0; k < 3; ++k) {
            if (!on[k]) continue;
            blend += w[k] * at[k][i];
            if (at[k][i] > win) win = at[k][i];
        }
        double alpha = 1.0 / (1.0 + exp(-p->kappa * (s[i] - p->tau)));
        double star;
        if (p->gate_mode == 1) star = blend;
        else if (p->gate_mode == 2) star = win;
        else star = (1.0 - alpha) * blend + alpha * win;
        scores[i] = (float)star;
        if (dbg && dbg->surprise) dbg->surprise[(size_t)h * N + i] = s[i];
        if (dbg && dbg->alpha) dbg->alpha[(size_t)h * N + i] = alpha;
        if (dbg && dbg->blend) dbg->blend[(size_t)h * N + i] = blend;
        if (dbg && dbg->win) dbg->win[(size_t)h * N + i] = win;
    }
    /* Sink pinning, the last step before selection. */
    for (int64_t i = 0; i < N && i < p->n_sink; ++i) scores[i] = NKVO_PIN;

    free(kh); free(mu); free(srt); free(s);
    for (int k = 0; k < 3; ++k) { free(a[k]); free(at[k]); }
    return 0;
}

/* Scores of one prompt at one layer: keys [H][N][d] -> scores [H][N]. */
int nkvo_score_layer(const float *keys, int H, int64_t N, int d, const nkvo_params *p,
                     float *scores, const nkvo_debug *dbg)
{
    if (!keys || !p || !scores || H < 1 || N < 1 || d < 1 || (p->scale_mask & 7) == 0) return -2;
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int h = 0; h < H; ++h) {
        int e = score_head(keys + (size_t)h * N * d, N, d, p, scores + (size_t)h * N, h, H, dbg);
        if (e) {
#pragma omp atomic write
            err = e;
        }
    }
    return err;
}

typedef struct { float s; int32_t h; int64_t i; } nkvo_item;

/* score descending, then head ascending, then index ascending */
static int cmp_item(const void *x, const void *y)
{
    const nkvo_item *a = (const nkvo_item *)x, *b = (const nkvo_item *)y;
    if (a->s > b->s) return -1;
    if (a->s < b->s) return 1;
    if (a->h != b->h) return a->h < b->h ? -1 : 1;
    if (a->i != b->i) return a->i < b->i ? -1 : 1;
    return 0;
}

/*
 * Section 2.6 + Appendix A: each head first keeps its own m_safe best tokens,
 * the remaining H*k0 - H*m_safe slots go to the best unprotected (head, token)
 * pairs of the layer; B_h counts what head h ends up with.
 */
int nkvo_budget_layer(const float *scores, int H, int64_t N, int64_t k0, int64_t m_safe, int32_t *B)
{
    if (!scores || !B || H < 1 || N < 1 || k0 < 0 || k0 > N || m_safe < 0 || m_safe > k0) return -2;
    nkvo_item *head = (nkvo_item *)malloc(sizeof(nkvo_item) * N);
    nkvo_item *pool = (nkvo_item *)malloc(sizeof(nkvo_item) * (size_t)H * N);
    if (!head || !pool) return -1;
    int64_t npool = 0;
    for (int h = 0; h < H; ++h) {
        for (int64_t i = 0; i < N; ++i) { head[i].s = scores[(size_t)h * N + i]; head[i].h = h; head[i].i = i; }
        qsort(head, (size_t)N, sizeof(nkvo_item), cmp_item);
        for (int64_t j = m_safe; j < N; ++j) pool[npool++] = head[j];   /* the unprotected ones */
        B[h] = (int32_t)m_safe;
    }
    qsort(pool, (size_t)npool, sizeof(nkvo_item), cmp_item);
    int64_t rest = (int64_t)H * k0 - (int64_t)H * m_safe;
    for (int64_t j = 0; j < rest; ++j) B[pool[j].h] += 1;
    free(head); free(pool);
    return 0;
}

/* Section 2.5: the B best positions of one head, returned in ascending order. */
int nkvo_select_head(const float *scores, int64_t N, int64_t B, int32_t *kept)
{
    if (!scores || N < 1 || B < 0 || B > N || (B > 0 && !kept)) return -2;
    nkvo_item *it = (nkvo_item *)malloc(sizeof(nkvo_item) * N);
    if (!it) return -1;
    for (int64_t i = 0; i < N; ++i) { it[i].s = scores[i]; it[i].h = 0; it[i].i = i; }
    qsort(it, (size_t)N, sizeof(nkvo_item), cmp_item);
    char *keep = (char *)calloc((size_t)N, 1);
    for (int64_t j = 0; j < B; ++j) keep[it[j].i] = 1;
    int64_t n = 0;
    for (int64_t i = 0; i < N; ++i) if (keep[i]) kept[n++] = (int32_t)i;
    free(it); free(keep);
    return 0;
}

/* Retained rows are bitwise copies: out[j] = rows[kept[j]]. */
int nkvo_gather_rows(const void *rows, int64_t row_bytes, const int32_t *kept, int64_t B, void *out)
{
    if ((!rows || !out || !kept) && B > 0) return -2;
    for (int64_t j = 0; j < B; ++j)
        memcpy((char *)out + j * row_bytes, (const char *)rows + (int64_t)kept[j] * row_bytes, (size_t)row_bytes);
    return 0;
}
