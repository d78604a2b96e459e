/*
 * Test infrastructure: runs every function of the CPU oracle (oracle/chess_oracle.c, compiled into this
 * executable with -fsanitize=address,undefined) on inputs a test wrote to a file, and writes the results to
 * another file, so that an out-of-bounds access, a use of uninitialised heap memory the sanitizers can see, a
 * signed overflow or a misaligned access in the oracle ends the run with a report instead of passing silently.
 * The test (tests/test_oracle_sanitized.py) then compares the results with those of the ordinary build.
 *
 * File format, both ways: records of [int64 byte count][payload], in the fixed order read / written below.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct { int32_t n_q_heads, n_kv_heads, head_dim, page_size, pages_per_chunk, chunks_per_grid, max_pages, summary_dtype; } geom_t;
typedef struct { int32_t plan, sink_pages, window_pages, budget_pages, budget_bp, over_chunk, over_grid, rho_g_bp, rho_c_bp,
                 rho_p_bp, probe, cut_rule; } plan_t;

void oracle_summarize(const uint16_t *, const int32_t *, const int32_t *, int32_t, const geom_t *, float *, float *, float *);
void oracle_scores(const uint16_t *, const float *, const float *, const float *, const int32_t *, int32_t, const geom_t *,
                   const plan_t *, double *, double *, double *);
int oracle_select(const uint16_t *, const float *, const float *, const float *, const int32_t *, int32_t, const geom_t *,
                  const plan_t *, const int32_t *, int32_t, int32_t *, int32_t *, uint8_t *, uint8_t *, int32_t *);
void oracle_anchor(const float *, const int32_t *, int32_t, const geom_t *, int32_t, float *);
int oracle_select_shared(int32_t, const float *const *, const float *const *, const float *const *, const float *const *,
                         const int32_t *, int32_t, const geom_t *, const plan_t *, const int32_t *, int32_t, int32_t *,
                         int32_t *, int32_t *);
void oracle_attend(const uint16_t *, const uint16_t *, const uint16_t *, const int32_t *, const int32_t *, const int32_t *,
                   const int32_t *, int32_t, int32_t, const geom_t *, double, float *, double *, int32_t);
void oracle_entropy(const uint16_t *, int32_t, int32_t, int64_t, double *);
void oracle_page_trigger(const float *, int32_t, double, double, double *, double *, int32_t *);

static void *get(FILE *f, int64_t *n)
{
    if (fread(n, sizeof *n, 1, f) != 1) { fprintf(stderr, "driver: short read\n"); exit(3); }
    void *p = malloc(*n > 0 ? (size_t)*n : 1);           /* exactly the payload: an overrun is a heap overflow */
    if (*n > 0 && fread(p, 1, (size_t)*n, f) != (size_t)*n) { fprintf(stderr, "driver: short read\n"); exit(3); }
    return p;
}

static void put(FILE *f, const void *p, int64_t n)
{
    fwrite(&n, sizeof n, 1, f);
    fwrite(p, 1, (size_t)n, f);
}

static int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

int main(int argc, char **argv)
{
    if (argc != 3) return 2;
    FILE *in = fopen(argv[1], "rb"), *out = fopen(argv[2], "wb");
    if (!in || !out) return 2;
    int64_t n;
    geom_t *g = get(in, &n);
    int64_t n_plans;
    plan_t *plans = get(in, &n_plans);
    n_plans /= (int64_t)sizeof(plan_t);
    int32_t *sl = get(in, &n);
    const int32_t batch = (int32_t)(n / 4);
    int32_t *bt = get(in, &n);
    uint16_t *K = get(in, &n), *V = get(in, &n), *Q = get(in, &n);
    int32_t *per = get(in, &n);
    if (n == 0) { free(per); per = NULL; }
    int64_t n_logits;
    uint16_t *logits = get(in, &n_logits);
    int32_t *vocab = get(in, &n);
    float *H = get(in, &n);
    const int32_t n_H = (int32_t)(n / 4);

    const int64_t rows = (int64_t)batch * g->n_kv_heads, d = g->head_dim;
    const int64_t cs = cdiv(g->max_pages, g->pages_per_chunk), gs = cdiv(cs, g->chunks_per_grid);
    const int32_t max_sel = g->max_pages;
    float *pv = calloc((size_t)(rows * g->max_pages * d), 4), *cv = calloc((size_t)(rows * cs * d), 4),
          *gv = calloc((size_t)(rows * gs * d), 4);
    oracle_summarize(K, bt, sl, batch, g, pv, cv, gv);
    put(out, pv, rows * g->max_pages * d * 4); put(out, cv, rows * cs * d * 4); put(out, gv, rows * gs * d * 4);

    float *anc = calloc((size_t)(rows * d), 4);
    oracle_anchor(pv, sl, batch, g, plans[0].window_pages, anc);
    put(out, anc, rows * d * 4);

    int32_t *ids = malloc((size_t)(rows * max_sel) * 4), *nsel = malloc((size_t)rows * 4), *cnt = malloc((size_t)rows * 12);
    uint8_t *kg = malloc((size_t)(rows * gs)), *kc = malloc((size_t)(rows * cs));
    float *o = malloc((size_t)((int64_t)batch * g->n_q_heads * d) * 4);
    double *ps = malloc((size_t)(rows * g->max_pages) * 8), *cs_s = malloc((size_t)(rows * cs) * 8), *gs_s = malloc((size_t)(rows * gs) * 8);
    double *wts = calloc((size_t)((int64_t)g->max_pages * g->page_size + 8), 8);
    for (int64_t i = 0; i < n_plans; ++i) {
        const plan_t *pl = &plans[i];
        for (int64_t j = 0; j < rows * g->max_pages; ++j) ps[j] = 0.0;
        for (int64_t j = 0; j < rows * cs; ++j) cs_s[j] = 0.0;
        for (int64_t j = 0; j < rows * gs; ++j) gs_s[j] = 0.0;
        oracle_scores(Q, pv, cv, gv, sl, batch, g, pl, ps, cs_s, gs_s);
        put(out, ps, rows * g->max_pages * 8);
        int rc = oracle_select(Q, pv, cv, gv, sl, batch, g, pl, per, max_sel, ids, nsel, kg, kc, cnt);
        put(out, &rc, 4); put(out, ids, rows * max_sel * 4); put(out, nsel, rows * 4); put(out, cnt, rows * 12);
        oracle_attend(Q, K, V, bt, sl, ids, nsel, max_sel, batch, g, 1.0 / sqrt((double)d), o, wts, 1);
        put(out, o, (int64_t)batch * g->n_q_heads * d * 4);
        /* the model-wide scope on two "layers" (this one twice), one list per sequence */
        const float *probes[2] = {anc, anc}, *p2[2] = {pv, pv}, *c2[2] = {cv, cv}, *g2[2] = {gv, gv};
        int32_t *sid = malloc((size_t)((int64_t)batch * max_sel) * 4), *sn = malloc((size_t)batch * 4), *sc = malloc((size_t)batch * 12);
        rc = oracle_select_shared(2, probes, p2, c2, g2, sl, batch, g, pl, per, max_sel, sid, sn, sc);
        put(out, &rc, 4); put(out, sid, (int64_t)batch * max_sel * 4); put(out, sn, (int64_t)batch * 4);
        free(sid); free(sn); free(sc);
    }
    oracle_attend(Q, K, V, bt, sl, NULL, NULL, 0, batch, g, 1.0 / sqrt((double)d), o, NULL, 0);     /* Full-KV */
    put(out, o, (int64_t)batch * g->n_q_heads * d * 4);

    const int32_t lb = (int32_t)(n_logits / 2 / vocab[1]);
    double *ent = malloc((size_t)lb * 8);
    oracle_entropy(logits, lb, vocab[0], vocab[1], ent);
    put(out, ent, (int64_t)lb * 8);
    double tr[2];
    int32_t fire;
    oracle_page_trigger(H, n_H, 1.0, 0.5, &tr[0], &tr[1], &fire);
    put(out, tr, 16); put(out, &fire, 4);

    free(g); free(plans); free(sl); free(bt); free(K); free(V); free(Q); free(per); free(logits); free(vocab); free(H);
    free(pv); free(cv); free(gv); free(anc); free(ids); free(nsel); free(cnt); free(kg); free(kc); free(o); free(ps);
    free(cs_s); free(gs_s); free(wts); free(ent);
    fclose(in);
    return fclose(out) == 0 ? 0 : 4;
}
