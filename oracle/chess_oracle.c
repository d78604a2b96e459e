/*
 * CHESS decode hot path -- plain CPU oracle.
 *
 * TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only the tests, the smoke check and
 * the benchmark's cpu_baseline leg may call into this file.  It shares no
 * code, header, table or helper with the HIP library; it is written straight
 * from the paper (CHESS, arxiv 2602.20732) so that a reader can check every
 * function against the passage it cites.
 *
 * Arithmetic: every floating-point accumulation is fp64, taken in the index
 * order the formula states; values the method stores (summary vectors, the
 * attention output) are rounded once to fp32.
 *
 * What each function follows:
 *   oracle_summarize  Sec. 3.1, Eq. 1 (page vector = mean of the page's key
 *                     rows) and Eq. 2 (chunk / grid vector = mean of children)
 *   oracle_scores     Sec. 3.2, Eq. 4 (dot product of probe and unit vector); the probe is the group's
 *                     query sum or the key-derived anchor of Eq. 3
 *   oracle_select     Sec. 3.2 cascade text and Alg. 1 stage 2 (grid -> chunk
 *                     -> page, a child is ranked only if its parent was kept),
 *                     then the union with sink and recent-window pages
 *   oracle_anchor     Sec. 3.2, Eq. 3 as an output of its own (the anchor of every sequence and KV head)
 *   oracle_select_shared  the same cascade under the paper's own scope: Eq. 1 flattens the states of all
 *                     layers and heads into one vector per unit, so one score per unit (Eq. 4 on the
 *                     flattened vectors = the sum of the per-layer, per-head dots) and one page set per
 *                     sequence, shared by every layer and head
 *   oracle_entropy    Sec. 3.3: the entropy of a step's output distribution (softmax of the logits)
 *   oracle_page_trigger  Sec. 3.3: average entropy and variance of the entropy over the steps of one
 *                     generated page, and the decision to reselect when either exceeds its threshold
 *   oracle_attend     softmax attention restricted to the listed pages: the
 *                     textbook definition, the paper's "Full-KV" when every
 *                     page is listed (Sec. 5.1 Baselines)
 *
 * Readings where the paper is silent (all restated in the design notes):
 *   - one layer, one page set per KV head; the probe of a KV head is the sum
 *     of its query-group rows (a dot of concatenated heads is the sum of the
 *     per-head dots, Eq. 1's Flatten restricted to the group);
 *   - a partial tail page / last chunk / last grid is averaged over the
 *     members that exist;
 *   - Sec. 3.1 calls a summary a compact vector and gives no storage type (Eq. 1-2 define the means only): fp32
 *     (the fp64 mean rounded once), or bf16 (that fp32 value rounded to nearest-even bf16; Eq. 2's parents average the
 *     children as stored, so that a refresh from stored siblings equals a full pass): a switch, default fp32;
 *   - "top rho fraction" keeps exactly ceil(rho * n) of the n units that are
 *     active at that level (the reading under which Table 1's budgets are the
 *     products of the three ratios); rank order is score descending, index
 *     ascending; an inactive unit is never ranked (no zero fill);
 *   - sink and window pages are not candidates at page level, the budget is
 *     on top of them.
 *   - ORACLE_CUT_THRESHOLD is Alg. 1 stage 2 as printed (keep S >= tau), with tau the score of the
 *     ceil(rho * n)-th active unit in rank order (the paper leaves the quantile's interpolation open);
 *     ORACLE_CUT_COUNT is the exact-count rule the benchmark spec asks for.
 *   - Sec. 3.3 names its two metrics "average Entropy" H_p and "Varentropy" Var(H)_p of a page p and says the
 *     second captures temporal instability: read here as the mean and the population variance, over the
 *     steps that generated page p, of the per-step entropy; reselection fires when either is above its
 *     threshold (the thresholds are inputs: the paper calibrates them on data this build does not have);
 * Parity unpinned (our reading only, the paper cannot arbitrate): N_c / N_g
 * defaults, ceil vs interpolated quantile count, group-sum probe, exclusion
 * of safety pages from the candidates, partial-unit means, the oversampling
 * factors of the budget plan.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_PLAN_BUDGET = 0, ORACLE_PLAN_RATIO = 1, ORACLE_PLAN_FLAT = 2 };
enum { ORACLE_PROBE_QUERY = 0, ORACLE_PROBE_ANCHOR = 1 };
enum { ORACLE_CUT_COUNT = 0, ORACLE_CUT_THRESHOLD = 1 };
enum { ORACLE_SUMMARY_F32 = 0, ORACLE_SUMMARY_BF16 = 1 };

typedef struct {
    int32_t n_q_heads;       /* H_q                                        */
    int32_t n_kv_heads;      /* H_kv, divides H_q                          */
    int32_t head_dim;        /* d                                          */
    int32_t page_size;       /* B tokens per page                          */
    int32_t pages_per_chunk; /* N_c                                        */
    int32_t chunks_per_grid; /* N_g                                        */
    int32_t max_pages;       /* row stride of the block table and of the
                                per-level summary arrays (in pages)        */
    int32_t summary_dtype;   /* ORACLE_SUMMARY_*: how a summary vector is stored.  F32: the fp64 mean rounded to
                                fp32 once.  BF16: that fp32 value rounded to the nearest bf16 (ties to even); a
                                chunk / grid then averages its children AS STORED.  The arrays stay float
                                either way (a bf16 value is a float whose low 16 bits are zero)            */
} oracle_geom;

typedef struct {
    int32_t plan;          /* ORACLE_PLAN_*                                 */
    int32_t sink_pages;    /* s                                             */
    int32_t window_pages;  /* w                                             */
    int32_t budget_pages;  /* > 0: k for every sequence                     */
    int32_t budget_bp;     /* else k = max(1, ceil(P * bp / 10000))         */
    int32_t over_chunk;    /* budget plan: chunk oversampling               */
    int32_t over_grid;     /* budget plan: grid oversampling                */
    int32_t rho_g_bp, rho_c_bp, rho_p_bp; /* ratio plan, basis points       */
    int32_t probe;         /* ORACLE_PROBE_*: what the units are scored against */
    int32_t cut_rule;      /* ORACLE_CUT_COUNT: a level keeps exactly k units (ties to the lower index);
                              ORACLE_CUT_THRESHOLD: Alg. 1 stage 2 as printed, tau = the k-th largest score of the
                              level's active units and every active unit with S >= tau is kept (ties at the cut
                              are all kept, so the count can exceed k) */
} oracle_plan;

static double bf16_value(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

/* a mean as the summaries store it (finite values): fp32, or fp32 rounded to the nearest bf16, ties to even */
static float stored_mean(double mean, int summary_dtype)
{
    float f = (float)mean;
    if (summary_dtype == ORACLE_SUMMARY_BF16) {
        uint32_t u;
        memcpy(&u, &f, sizeof u);
        u += 0x7fffu + ((u >> 16) & 1u);
        u &= 0xffff0000u;
        memcpy(&f, &u, sizeof f);
    }
    return f;
}

/* max row counts of the chunk and grid arrays for a given page stride */
static int64_t chunk_stride(const oracle_geom *g) { return ceil_div(g->max_pages, g->pages_per_chunk); }
static int64_t grid_stride(const oracle_geom *g) { return ceil_div(chunk_stride(g), g->chunks_per_grid); }

/* K pool layout: [physical page][kv head][token in page][dim], bf16. */
static double k_at(const uint16_t *k_pool, const oracle_geom *g, int64_t phys, int h, int tok, int dim)
{
    int64_t off = (((phys * g->n_kv_heads + h) * g->page_size) + tok) * g->head_dim + dim;
    return bf16_value(k_pool[off]);
}

/* V pool layout: [physical page][kv head][dim][token in page], bf16. */
static double v_at(const uint16_t *v_pool, const oracle_geom *g, int64_t phys, int h, int tok, int dim)
{
    int64_t off = (((phys * g->n_kv_heads + h) * g->head_dim) + dim) * g->page_size + tok;
    return bf16_value(v_pool[off]);
}

/*
 * Eq. 1 and Eq. 2.  page_vec [batch][H_kv][max_pages][d], chunk_vec
 * [batch][H_kv][ceil(max_pages/N_c)][d], grid_vec [batch][H_kv][ceil(.../N_g)][d],
 * all fp32; rows past a sequence's own counts are left untouched.
 */
void oracle_summarize(const uint16_t *k_pool, const int32_t *block_table, const int32_t *seq_lens,
                      int32_t batch, const oracle_geom *g, float *page_vec, float *chunk_vec, float *grid_vec)
{
    const int d = g->head_dim, B = g->page_size, Nc = g->pages_per_chunk, Ng = g->chunks_per_grid;
    const int64_t cs = chunk_stride(g), gs = grid_stride(g);
    for (int b = 0; b < batch; ++b) {
        const int64_t L = seq_lens[b];
        const int64_t P = ceil_div(L, B), nc = ceil_div(P, Nc), ng = ceil_div(nc, Ng);
        for (int h = 0; h < g->n_kv_heads; ++h) {
            float *pv = page_vec + ((int64_t)b * g->n_kv_heads + h) * g->max_pages * d;
            float *cv = chunk_vec + ((int64_t)b * g->n_kv_heads + h) * cs * d;
            float *gv = grid_vec + ((int64_t)b * g->n_kv_heads + h) * gs * d;
            for (int64_t j = 0; j < P; ++j) {                /* Eq. 1 */
                const int64_t phys = block_table[(int64_t)b * g->max_pages + j];
                const int64_t n = (j == P - 1) ? L - j * B : B;
                for (int i = 0; i < d; ++i) {
                    double acc = 0.0;
                    for (int t = 0; t < n; ++t) acc += k_at(k_pool, g, phys, h, t, i);
                    pv[j * d + i] = stored_mean(acc / (double)n, g->summary_dtype);
                }
            }
            for (int64_t c = 0; c < nc; ++c) {               /* Eq. 2, chunks */
                const int64_t lo = c * Nc, hi = (lo + Nc < P) ? lo + Nc : P;
                for (int i = 0; i < d; ++i) {
                    double acc = 0.0;
                    for (int64_t j = lo; j < hi; ++j) acc += (double)pv[j * d + i];
                    cv[c * d + i] = stored_mean(acc / (double)(hi - lo), g->summary_dtype);
                }
            }
            for (int64_t k = 0; k < ng; ++k) {               /* Eq. 2, grids */
                const int64_t lo = k * Ng, hi = (lo + Ng < nc) ? lo + Ng : nc;
                for (int i = 0; i < d; ++i) {
                    double acc = 0.0;
                    for (int64_t c = lo; c < hi; ++c) acc += (double)cv[c * d + i];
                    gv[k * d + i] = stored_mean(acc / (double)(hi - lo), g->summary_dtype);
                }
            }
        }
    }
}

/* probe of KV head h: sum of its group's query rows, g ascending */
static void probe_of(const uint16_t *q, const oracle_geom *g, int b, int h, double *probe)
{
    const int G = g->n_q_heads / g->n_kv_heads, d = g->head_dim;
    for (int i = 0; i < d; ++i) {
        double acc = 0.0;
        for (int r = 0; r < G; ++r)
            acc += bf16_value(q[((int64_t)b * g->n_q_heads + h * G + r) * d + i]);
        probe[i] = acc;
    }
}

/*
 * Sec. 3.2, Eq. 3: the query anchor, the mean of the page vectors of the recent
 * window W (the last min(w, P) pages of the sequence), per KV head like every
 * other vector here.  Summed in page order in fp64, divided by |W|, rounded to
 * fp32 once like the other stored means of Eq. 1-2.
 */
static void anchor_of(const float *page_vec, const oracle_geom *g, int64_t row, int64_t P, int64_t w, double *probe)
{
    const int d = g->head_dim;
    const int64_t W = w < P ? w : P;
    for (int i = 0; i < d; ++i) {
        double acc = 0.0;
        for (int64_t j = P - W; j < P; ++j) acc += (double)page_vec[(row * g->max_pages + j) * d + i];
        probe[i] = (double)(float)(acc / (double)W);
    }
}

/* the probe the plan asks for (pl == NULL: the query probe) */
static void probe_for(const oracle_plan *pl, const uint16_t *q, const float *page_vec, const oracle_geom *g,
                      int b, int h, int64_t P, double *probe)
{
    if (pl && pl->probe == ORACLE_PROBE_ANCHOR)
        anchor_of(page_vec, g, (int64_t)b * g->n_kv_heads + h, P, pl->window_pages, probe);
    else
        probe_of(q, g, b, h, probe);
}

static double dot_probe(const double *probe, const float *vec, int d)
{
    double acc = 0.0;
    for (int i = 0; i < d; ++i) acc += probe[i] * (double)vec[i];
    return acc;
}

/*
 * Eq. 4 for every unit of every level (Alg. 1 stage 1 scores the whole
 * hierarchy; the cascade below only ever looks at active units).
 * Outputs fp64, same row strides as the summary arrays.
 */
void oracle_scores(const uint16_t *q, const float *page_vec, const float *chunk_vec, const float *grid_vec,
                   const int32_t *seq_lens, int32_t batch, const oracle_geom *g, const oracle_plan *pl,
                   double *page_s, double *chunk_s, double *grid_s)
{
    const int d = g->head_dim, B = g->page_size, Nc = g->pages_per_chunk, Ng = g->chunks_per_grid;
    const int64_t cs = chunk_stride(g), gs = grid_stride(g);
    double *probe = (double *)malloc(sizeof(double) * d);
    for (int b = 0; b < batch; ++b) {
        const int64_t P = ceil_div(seq_lens[b], B), nc = ceil_div(P, Nc), ng = ceil_div(nc, Ng);
        for (int h = 0; h < g->n_kv_heads; ++h) {
            const int64_t row = (int64_t)b * g->n_kv_heads + h;
            if (P == 0) continue;
            probe_for(pl, q, page_vec, g, b, h, P, probe);
            for (int64_t j = 0; j < P; ++j)
                page_s[row * g->max_pages + j] = dot_probe(probe, page_vec + (row * g->max_pages + j) * d, d);
            for (int64_t c = 0; c < nc; ++c)
                chunk_s[row * cs + c] = dot_probe(probe, chunk_vec + (row * cs + c) * d, d);
            for (int64_t k = 0; k < ng; ++k)
                grid_s[row * gs + k] = dot_probe(probe, grid_vec + (row * gs + k) * d, d);
        }
    }
    free(probe);
}

typedef struct { double score; int64_t index; } ranked;

/* rank order of the cascade: larger score first, then smaller index */
static int ranked_cmp(const void *a, const void *b)
{
    const ranked *x = (const ranked *)a, *y = (const ranked *)b;
    if (x->score > y->score) return -1;
    if (x->score < y->score) return 1;
    return (x->index > y->index) - (x->index < y->index);
}

/*
 * Keep k of n candidates; mark them in keep[index]; returns how many were kept.
 * ORACLE_CUT_COUNT: the first k in rank order.  ORACLE_CUT_THRESHOLD (Alg. 1 stage 2: tau = Quantile, mask
 * S >= tau): tau is the score of the k-th candidate in rank order and every candidate with score >= tau is kept.
 */
static int64_t keep_top(ranked *cand, int64_t n, int64_t k, int cut_rule, uint8_t *keep)
{
    qsort(cand, (size_t)n, sizeof *cand, ranked_cmp);
    if (k > n) k = n;
    if (k <= 0) return 0;
    int64_t kept = k;
    if (cut_rule == ORACLE_CUT_THRESHOLD) {
        const double tau = cand[k - 1].score;
        while (kept < n && cand[kept].score >= tau) ++kept;
    }
    for (int64_t i = 0; i < kept; ++i) keep[cand[i].index] = 1;
    return kept;
}

/* the page budget k of sequence b: its own entry of budget_per_seq when that is given and positive, else the
 * plan's fixed budget, else the plan's fraction of the sequence's P pages (at least one page) */
static int64_t ceil_bp(int64_t n, int64_t bp);
static int64_t clamp_i(int64_t x, int64_t lo, int64_t hi);
static int64_t budget_of(const oracle_plan *pl, const int32_t *budget_per_seq, int b, int64_t P)
{
    if (budget_per_seq && budget_per_seq[b] > 0) return budget_per_seq[b];
    return pl->budget_pages > 0 ? pl->budget_pages : clamp_i(ceil_bp(P, pl->budget_bp), 1, P);
}

static int64_t ceil_bp(int64_t n, int64_t bp) { return (n * bp + 9999) / 10000; }
static int64_t clamp_i(int64_t x, int64_t lo, int64_t hi) { return x < lo ? lo : (x > hi ? hi : x); }

/*
 * The cascade of Sec. 3.2 / Alg. 1 stage 2, then the union with the safety
 * pages.  page_ids [batch][H_kv][max_sel] ascending, padded with -1;
 * n_selected [batch][H_kv].  Optional outputs (may be NULL): kept_grid /
 * kept_chunk masks (uint8, summary-array strides) and counts[row*3 + {0,1,2}]
 * = k_g, k_c, k_p actually used.
 * Returns 0, or -1 if a row would need more than max_sel ids.
 */
int oracle_select(const uint16_t *q, const float *page_vec, const float *chunk_vec, const float *grid_vec,
                  const int32_t *seq_lens, int32_t batch, const oracle_geom *g, const oracle_plan *pl,
                  const int32_t *budget_per_seq, int32_t max_sel, int32_t *page_ids, int32_t *n_selected,
                  uint8_t *kept_grid, uint8_t *kept_chunk, int32_t *counts)
{
    const int d = g->head_dim, B = g->page_size, Nc = g->pages_per_chunk, Ng = g->chunks_per_grid;
    const int64_t cs = chunk_stride(g), gs = grid_stride(g);
    const int64_t s = pl->sink_pages, w = pl->window_pages;
    double *probe = (double *)malloc(sizeof(double) * d);
    ranked *cand = (ranked *)malloc(sizeof(ranked) * (size_t)(g->max_pages + 1));
    uint8_t *kg = (uint8_t *)malloc((size_t)gs + 1), *kc = (uint8_t *)malloc((size_t)cs + 1);
    uint8_t *kp = (uint8_t *)malloc((size_t)g->max_pages + 1);
    int rc = 0;

    for (int b = 0; b < batch && rc == 0; ++b) {
        const int64_t L = seq_lens[b];
        const int64_t P = ceil_div(L, B), nc = ceil_div(P, Nc), ng = ceil_div(nc, Ng);
        for (int h = 0; h < g->n_kv_heads; ++h) {
            const int64_t row = (int64_t)b * g->n_kv_heads + h;
            int32_t *ids = page_ids + row * max_sel;
            for (int i = 0; i < max_sel; ++i) ids[i] = -1;
            memset(kg, 0, (size_t)gs + 1); memset(kc, 0, (size_t)cs + 1); memset(kp, 0, (size_t)g->max_pages + 1);
            int64_t k_g = 0, k_c = 0, k_p = 0, n = 0;

            if (P <= s + w) {                       /* safety pages cover the sequence */
                if (P > max_sel) { rc = -1; break; }
                for (int64_t j = 0; j < P; ++j) ids[n++] = (int32_t)j;
            } else {
                const int64_t k = budget_of(pl, budget_per_seq, b, P);
                const int64_t kc_target = ceil_div((int64_t)pl->over_chunk * k, Nc);
                probe_for(pl, q, page_vec, g, b, h, P, probe);

                /* level 1: every grid is a candidate */
                int64_t m = 0;
                for (int64_t u = 0; u < ng; ++u) {
                    cand[m].score = dot_probe(probe, grid_vec + (row * gs + u) * d, d);
                    cand[m++].index = u;
                }
                if (pl->plan == ORACLE_PLAN_RATIO) k_g = clamp_i(ceil_bp(m, pl->rho_g_bp), 1, m);
                else if (pl->plan == ORACLE_PLAN_FLAT) k_g = m;
                else k_g = clamp_i(ceil_div((int64_t)pl->over_grid * kc_target, Ng), 0, m);
                k_g = keep_top(cand, m, k_g, pl->cut_rule, kg);

                /* level 2: chunks whose parent grid was kept */
                m = 0;
                for (int64_t u = 0; u < nc; ++u) if (kg[u / Ng]) {
                    cand[m].score = dot_probe(probe, chunk_vec + (row * cs + u) * d, d);
                    cand[m++].index = u;
                }
                if (pl->plan == ORACLE_PLAN_RATIO) k_c = clamp_i(ceil_bp(m, pl->rho_c_bp), 1, m);
                else if (pl->plan == ORACLE_PLAN_FLAT) k_c = m;
                else k_c = clamp_i(kc_target, 0, m);
                k_c = keep_top(cand, m, k_c, pl->cut_rule, kc);

                /* level 3: pages whose parent chunk was kept, safety pages excluded */
                m = 0;
                for (int64_t u = s; u < P - w; ++u) if (kc[u / Nc]) {
                    cand[m].score = dot_probe(probe, page_vec + (row * g->max_pages + u) * d, d);
                    cand[m++].index = u;
                }
                if (pl->plan == ORACLE_PLAN_RATIO) k_p = m == 0 ? 0 : clamp_i(ceil_bp(m, pl->rho_p_bp), 1, m);
                else k_p = clamp_i(k, 0, m);
                k_p = keep_top(cand, m, k_p, pl->cut_rule, kp);

                /* union with sinks and the recent window, ascending */
                if (s + k_p + w > max_sel) { rc = -1; break; }
                for (int64_t j = 0; j < P; ++j)
                    if (j < s || j >= P - w || kp[j]) ids[n++] = (int32_t)j;
            }
            n_selected[row] = (int32_t)n;
            if (kept_grid) memcpy(kept_grid + row * gs, kg, (size_t)gs);
            if (kept_chunk) memcpy(kept_chunk + row * cs, kc, (size_t)cs);
            if (counts) { counts[row * 3] = (int32_t)k_g; counts[row * 3 + 1] = (int32_t)k_c; counts[row * 3 + 2] = (int32_t)k_p; }
        }
    }
    free(probe); free(cand); free(kg); free(kc); free(kp);
    return rc;
}

/*
 * Sec. 3.2, Eq. 3 for every (sequence, KV head): anchor [batch][H_kv][d] fp32, the mean of the page
 * vectors of the last min(w, P) pages (zero for an empty sequence).
 */
void oracle_anchor(const float *page_vec, const int32_t *seq_lens, int32_t batch, const oracle_geom *g,
                   int32_t window_pages, float *anchor)
{
    const int d = g->head_dim;
    double *probe = (double *)malloc(sizeof(double) * d);
    for (int b = 0; b < batch; ++b) {
        const int64_t P = ceil_div(seq_lens[b], g->page_size);
        for (int h = 0; h < g->n_kv_heads; ++h) {
            const int64_t row = (int64_t)b * g->n_kv_heads + h;
            if (P > 0) anchor_of(page_vec, g, row, P, window_pages, probe);
            for (int i = 0; i < d; ++i) anchor[row * d + i] = P > 0 ? (float)probe[i] : 0.0f;
        }
    }
    free(probe);
}

/*
 * Eq. 4 on the flattened vectors of Eq. 1: the unit vector of the model is the concatenation, over layers
 * l and KV heads h, of the per-(l, h) unit vectors, and the probe is flattened the same way, so
 * S(u) = sum_l sum_h sum_i probe[l][b][h][i] * vec[l][b][h][u][i]   (one fp64 sum, in that order).
 * vecs[l] has `stride` units per (sequence, head) row; probes[l] is fp32 [batch][H_kv][d].
 */
static double shared_score(int32_t n_layers, const float *const *probes, const float *const *vecs,
                           const oracle_geom *g, int b, int64_t stride, int64_t u)
{
    const int d = g->head_dim;
    double acc = 0.0;
    for (int l = 0; l < n_layers; ++l)
        for (int h = 0; h < g->n_kv_heads; ++h) {
            const int64_t row = (int64_t)b * g->n_kv_heads + h;
            const float *pr = probes[l] + row * d, *v = vecs[l] + (row * stride + u) * d;
            for (int i = 0; i < d; ++i) acc += (double)pr[i] * (double)v[i];
        }
    return acc;
}

/*
 * The cascade of Sec. 3.2 under the model-wide scope of Eq. 1: the three levels, their keep-counts, the
 * rank order and the union with the safety pages are those of oracle_select; only the score differs
 * (shared_score), and there is one list per sequence: page_ids [batch][max_sel], n_selected [batch],
 * counts [batch][3] (may be NULL).  Returns 0, or -1 if a sequence would need more than max_sel ids.
 */
int oracle_select_shared(int32_t n_layers, const float *const *probes, const float *const *page_vec,
                         const float *const *chunk_vec, const float *const *grid_vec, const int32_t *seq_lens,
                         int32_t batch, const oracle_geom *g, const oracle_plan *pl, const int32_t *budget_per_seq,
                         int32_t max_sel, int32_t *page_ids, int32_t *n_selected, int32_t *counts)
{
    const int B = g->page_size, Nc = g->pages_per_chunk, Ng = g->chunks_per_grid;
    const int64_t cs = chunk_stride(g), gs = grid_stride(g);
    const int64_t s = pl->sink_pages, w = pl->window_pages;
    ranked *cand = (ranked *)malloc(sizeof(ranked) * (size_t)(g->max_pages + 1));
    uint8_t *kg = (uint8_t *)malloc((size_t)gs + 1), *kc = (uint8_t *)malloc((size_t)cs + 1);
    uint8_t *kp = (uint8_t *)malloc((size_t)g->max_pages + 1);
    int rc = 0;

    for (int b = 0; b < batch && rc == 0; ++b) {
        const int64_t P = ceil_div(seq_lens[b], B), nc = ceil_div(P, Nc), ng = ceil_div(nc, Ng);
        int32_t *ids = page_ids + (int64_t)b * max_sel;
        for (int i = 0; i < max_sel; ++i) ids[i] = -1;
        memset(kg, 0, (size_t)gs + 1); memset(kc, 0, (size_t)cs + 1); memset(kp, 0, (size_t)g->max_pages + 1);
        int64_t k_g = 0, k_c = 0, k_p = 0, n = 0;

        if (P <= s + w) {                           /* safety pages cover the sequence */
            if (P > max_sel) { rc = -1; break; }
            for (int64_t j = 0; j < P; ++j) ids[n++] = (int32_t)j;
        } else {
            const int64_t k = budget_of(pl, budget_per_seq, b, P);
            const int64_t kc_target = ceil_div((int64_t)pl->over_chunk * k, Nc);

            int64_t m = 0;                          /* level 1: every grid */
            for (int64_t u = 0; u < ng; ++u) {
                cand[m].score = shared_score(n_layers, probes, grid_vec, g, b, gs, u);
                cand[m++].index = u;
            }
            if (pl->plan == ORACLE_PLAN_RATIO) k_g = clamp_i(ceil_bp(m, pl->rho_g_bp), 1, m);
            else if (pl->plan == ORACLE_PLAN_FLAT) k_g = m;
            else k_g = clamp_i(ceil_div((int64_t)pl->over_grid * kc_target, Ng), 0, m);
            k_g = keep_top(cand, m, k_g, pl->cut_rule, kg);

            m = 0;                                  /* level 2: chunks of kept grids */
            for (int64_t u = 0; u < nc; ++u) if (kg[u / Ng]) {
                cand[m].score = shared_score(n_layers, probes, chunk_vec, g, b, cs, u);
                cand[m++].index = u;
            }
            if (pl->plan == ORACLE_PLAN_RATIO) k_c = clamp_i(ceil_bp(m, pl->rho_c_bp), 1, m);
            else if (pl->plan == ORACLE_PLAN_FLAT) k_c = m;
            else k_c = clamp_i(kc_target, 0, m);
            k_c = keep_top(cand, m, k_c, pl->cut_rule, kc);

            m = 0;                                  /* level 3: pages of kept chunks, safety pages excluded */
            for (int64_t u = s; u < P - w; ++u) if (kc[u / Nc]) {
                cand[m].score = shared_score(n_layers, probes, page_vec, g, b, g->max_pages, u);
                cand[m++].index = u;
            }
            if (pl->plan == ORACLE_PLAN_RATIO) k_p = m == 0 ? 0 : clamp_i(ceil_bp(m, pl->rho_p_bp), 1, m);
            else k_p = clamp_i(k, 0, m);
            k_p = keep_top(cand, m, k_p, pl->cut_rule, kp);

            if (s + k_p + w > max_sel) { rc = -1; break; }
            for (int64_t j = 0; j < P; ++j)
                if (j < s || j >= P - w || kp[j]) ids[n++] = (int32_t)j;
        }
        n_selected[b] = (int32_t)n;
        if (counts) { counts[b * 3] = (int32_t)k_g; counts[b * 3 + 1] = (int32_t)k_c; counts[b * 3 + 2] = (int32_t)k_p; }
    }
    free(cand); free(kg); free(kc); free(kp);
    return rc;
}

/*
 * Softmax attention over the valid tokens of the listed pages, one query row
 * per q head: z_t = sm_scale * q . K_t ; p = exp(z - max z) / sum ; out = sum p_t V_t.
 * page_ids NULL means every page of the sequence (Full-KV).  weights (may be
 * NULL) receives the normalised p of row 0 of the batch, q head `weights_head`,
 * in listed-token order, for the softmax checks.  out fp32 [batch][H_q][d].
 */
void oracle_attend(const uint16_t *q, const uint16_t *k_pool, const uint16_t *v_pool,
                   const int32_t *block_table, const int32_t *seq_lens,
                   const int32_t *page_ids, const int32_t *n_selected, int32_t max_sel,
                   int32_t batch, const oracle_geom *g, double sm_scale, float *out,
                   double *weights, int32_t weights_head)
{
    const int d = g->head_dim, B = g->page_size, G = g->n_q_heads / g->n_kv_heads;
    double *z = (double *)malloc(sizeof(double) * (size_t)g->max_pages * B + 8);
    double *acc = (double *)malloc(sizeof(double) * d);
    for (int b = 0; b < batch; ++b) {
        const int64_t L = seq_lens[b], P = ceil_div(L, B);
        for (int hq = 0; hq < g->n_q_heads; ++hq) {
            const int h = hq / G;
            const int64_t row = (int64_t)b * g->n_kv_heads + h;
            const int64_t n_pages = page_ids ? n_selected[row] : P;
            const uint16_t *qrow = q + ((int64_t)b * g->n_q_heads + hq) * d;
            float *o = out + ((int64_t)b * g->n_q_heads + hq) * d;
            int64_t T = 0;
            double zmax = -INFINITY;
            for (int64_t e = 0; e < n_pages; ++e) {
                const int64_t j = page_ids ? page_ids[row * max_sel + e] : e;
                const int64_t phys = block_table[(int64_t)b * g->max_pages + j];
                const int64_t n = (j == P - 1) ? L - j * B : B;
                for (int t = 0; t < n; ++t) {
                    double s = 0.0;
                    for (int i = 0; i < d; ++i) s += bf16_value(qrow[i]) * k_at(k_pool, g, phys, h, t, i);
                    z[T] = sm_scale * s;
                    if (z[T] > zmax) zmax = z[T];
                    ++T;
                }
            }
            double denom = 0.0;
            for (int64_t t = 0; t < T; ++t) { z[t] = exp(z[t] - zmax); denom += z[t]; }
            for (int i = 0; i < d; ++i) acc[i] = 0.0;
            T = 0;
            for (int64_t e = 0; e < n_pages; ++e) {
                const int64_t j = page_ids ? page_ids[row * max_sel + e] : e;
                const int64_t phys = block_table[(int64_t)b * g->max_pages + j];
                const int64_t n = (j == P - 1) ? L - j * B : B;
                for (int t = 0; t < n; ++t) {
                    const double p = z[T] / denom;
                    if (weights && b == 0 && hq == weights_head) weights[T] = p;
                    for (int i = 0; i < d; ++i) acc[i] += p * v_at(v_pool, g, phys, h, t, i);
                    ++T;
                }
            }
            for (int i = 0; i < d; ++i) o[i] = (T > 0) ? (float)acc[i] : 0.0f;
        }
    }
    free(z); free(acc);
}

/*
 * Sec. 3.3: entropy (nats) of the output distribution of one decode step, per sequence:
 * p = softmax(logits), H = -sum_v p_v log p_v, with the terms of p_v = 0 taken as 0.
 * logits bf16 [batch][row_stride], the first `vocab` of each row used.
 */
void oracle_entropy(const uint16_t *logits, int32_t batch, int32_t vocab, int64_t row_stride, double *H)
{
    for (int b = 0; b < batch; ++b) {
        const uint16_t *z = logits + (int64_t)b * row_stride;
        double m = -INFINITY, Z = 0.0, acc = 0.0;
        for (int v = 0; v < vocab; ++v) { const double x = bf16_value(z[v]); if (x > m) m = x; }
        for (int v = 0; v < vocab; ++v) Z += exp(bf16_value(z[v]) - m);
        for (int v = 0; v < vocab; ++v) {
            const double p = exp(bf16_value(z[v]) - m) / Z;
            if (p > 0.0) acc -= p * log(p);
        }
        H[b] = acc;
    }
}

/*
 * Sec. 3.3 over one generated page: H[0..n) are the entropies of its steps (fp32, as the step stores them).
 * mean = (1/n) sum H, var = (1/n) sum (H - mean)^2 (both fp64, index order); fire = mean > tau_h || var > tau_v.
 */
void oracle_page_trigger(const float *H, int32_t n, double tau_h, double tau_v, double *mean, double *var, int32_t *fire)
{
    double s = 0.0, q = 0.0;
    for (int i = 0; i < n; ++i) s += (double)H[i];
    const double mu = s / (double)n;
    for (int i = 0; i < n; ++i) { const double d = (double)H[i] - mu; q += d * d; }
    *mean = mu;
    *var = q / (double)n;
    *fire = (*mean > tau_h || *var > tau_v) ? 1 : 0;
}
