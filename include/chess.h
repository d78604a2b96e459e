/*
 * libchess -- the decode-step hot path of CHESS (context-aware hierarchical KV selection,
 * arxiv 2602.20732) for AMD MI355X (gfx950): per-page key summaries over a paged bf16 KV cache,
 * probe-against-summary scoring, Grid -> Chunk -> Page top-k page selection that always keeps
 * sink and recent-window pages, and block-sparse decode attention that reads the selected pages
 * in place (no KV copy, only page indices change: Sec. 1, Sec. 4.1, App. B "Zero-Copy Logic").
 *
 * C ABI.  Every data pointer is a DEVICE pointer owned by the caller unless it says "host".
 * The library never allocates or frees device memory; only chess_append_kv and chess_reuse_step write the K/V
 * pools (the appended token's rows, nothing else).  Every call is
 * asynchronous on `stream` (a hipStream_t passed as void*, NULL = the default stream), does no
 * host synchronisation, and can be captured in a HIP graph.  A context caches launch shapes: calls on one
 * context must not run concurrently from several host threads (use one context per thread).
 *
 * Return value: 0 on success, a negative CHESS_E* code on misuse the host can detect (null
 * pointers, shapes outside the configuration).  Data the host cannot see (sequence lengths,
 * block-table entries) is trusted: block-table entries of existing pages must be valid physical
 * page numbers.  A sequence of length 0 is defined: n_selected = 0, out = 0.
 *
 * Layouts (one layer; d = head_dim = 128, B = page_size, H = n_kv_heads, G = n_q_heads / H):
 *   K pool       bf16 [physical page][H][B][d]
 *   V pool       bf16 [physical page][H][d][B]        (token-minor inside a page)
 *   block table  int32 [batch][max_pages_per_seq]     logical page -> physical page
 *   seq_lens     int32 [batch]                        tokens in each sequence
 *   q            bf16 [batch][n_q_heads][d]           q head hq belongs to KV head hq / G
 *   summaries    fp32 (or bf16, see chess_config.summary_dtype), three arrays in one buffer (byte offsets from
 *                chess_summary_layout):
 *                  pages  [batch][H][max_pages_per_seq][d]
 *                  chunks [batch][H][ceil(max_pages_per_seq / N_c)][d]
 *                  grids  [batch][H][ceil(max_chunks / N_g)][d]       all in logical order
 *   page_ids     int32 [batch][H][max_selected_pages] logical page numbers, ascending, -1 padded
 *   n_selected   int32 [batch][H]
 *   out          fp32 [batch][n_q_heads][d]
 */
#ifndef CHESS_H
#define CHESS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CHESS_OK        0
#define CHESS_EINVAL   (-1)  /* null pointer, bad shape, size outside the configuration       */
#define CHESS_ENOTSUP  (-2)  /* valid request this build cannot serve (e.g. too many candidates for LDS) */
#define CHESS_EHIP     (-3)  /* the HIP runtime reported an error at launch                   */
#define CHESS_ENOMEM   (-4)  /* host allocation of the context failed                         */
#define CHESS_ESCRATCH (-5)  /* chess_sparse_decode_static: the call needs more than CHESS_STATIC_SCRATCH_BYTES */

/* How the per-level keep-counts of the cascade are derived (Sec. 3.2; Alg. 1 stage 2). */
#define CHESS_PLAN_BUDGET 0  /* page budget k; chunk / grid counts from oversampling factors  */
#define CHESS_PLAN_RATIO  1  /* the paper's retention ratios rho_g, rho_c, rho_p              */
#define CHESS_PLAN_FLAT   2  /* keep every grid and chunk: plain top-k over pages             */

/* What a unit's vector is scored against (Sec. 3.2). */
#define CHESS_PROBE_QUERY  0 /* the sum of the KV head's G query rows (the decode query)                   */
#define CHESS_PROBE_ANCHOR 1 /* Eq. 3: the mean of the page vectors of the recent window (the last          */
                             /* window_pages pages), keys only; q is then not read and may be NULL          */

/* How many units a level keeps once its count k is known (Alg. 1 stage 2 thresholds at a quantile). */
#define CHESS_CUT_COUNT     0 /* exactly k units; ties at the cut go to the lower index                      */
#define CHESS_CUT_THRESHOLD 1 /* every unit whose score is >= the k-th largest score (S >= tau as printed in */
                              /* Alg. 1): ties at the cut are all kept, so a level may keep more than k.     */
                              /* Grid and chunk lists are sized for every unit; a page list that outgrows    */
                              /* max_selected_pages is cut short (lowest pages first) and the launch raises  */
                              /* CHESS_FLAG_OVERFLOW in the workspace's error word                           */

/* Bits of the word chess_workspace_error reads. */
#define CHESS_FLAG_WAIT     1 /* a bounded wait between workgroups was given up: results undefined          */
#define CHESS_FLAG_OVERFLOW 2 /* CHESS_CUT_THRESHOLD kept more pages than a page_ids row holds: list cut short */

/* Storage type of the summary vectors (the paper only says "compact vector"). */
#define CHESS_SUMMARY_F32  0  /* fp32: the fp64 mean rounded once                                            */
#define CHESS_SUMMARY_BF16 1  /* bf16: that fp32 value rounded to nearest-even bf16; parents average the     */
                              /* stored (bf16) child vectors; half the bytes the selection reads             */

#define CHESS_MAX_LAYERS 64   /* most layers one chess_select_shared call can take */

#define CHESS_STATIC_SCRATCH_BYTES (4u << 20)   /* device scratch chess_sparse_decode_static owns, per GPU */

typedef struct chess_ctx chess_ctx; /* opaque; small host-side state only */

typedef struct {
    int32_t n_q_heads;          /* multiple of n_kv_heads, group size G <= 16               */
    int32_t n_kv_heads;
    int32_t head_dim;           /* must be 128                                               */
    int32_t page_size;          /* B: 16 or 32 tokens (Sec. 4.3 uses 16, Sec. 5.1 uses 32)   */
    int32_t pages_per_chunk;    /* N_c (Sec. 3.1)                                            */
    int32_t chunks_per_grid;    /* N_g (Sec. 3.1); N_c * N_g <= 256                          */
    int32_t max_batch;
    int32_t max_pages_per_seq;  /* row stride of the block table and of the page summaries   */
    int32_t max_selected_pages; /* row stride of page_ids                                    */
    float   sm_scale;           /* softmax scale; 0 means 1 / sqrt(head_dim)                 */
    int32_t summary_dtype;      /* CHESS_SUMMARY_*                                           */
    int32_t shared_device;      /* non-zero: other work may run on this GPU at the same time.  chess_select,
                                   chess_decode_step and chess_select_shared then give every (sequence, KV head)
                                   (every sequence) to ONE workgroup: no workgroup ever waits for another, so no
                                   launch depends on what else is resident.  0: the device is this library's
                                   while a call runs, and short batches are spread over cooperating workgroups */
} chess_config;

typedef struct {
    int32_t plan;               /* CHESS_PLAN_*                                              */
    int32_t sink_pages;         /* s: pages [0, s) are always kept (Sec. 3.2, attention sinks) */
    int32_t window_pages;       /* w: the last w pages are always kept (recent window)       */
    int32_t budget_pages;       /* > 0: page budget k for every sequence                     */
    int32_t budget_bp;          /* else k = max(1, ceil(P * budget_bp / 10000)), P = pages of the sequence */
    int32_t over_chunk;         /* PLAN_BUDGET: keep ceil(over_chunk * k / N_c) chunks       */
    int32_t over_grid;          /* PLAN_BUDGET: keep ceil(over_grid * that / N_g) grids      */
    int32_t rho_g_bp;           /* PLAN_RATIO: ratios in basis points; a level keeps         */
    int32_t rho_c_bp;           /*   clamp(ceil(n * rho), 1, n) of its n active units        */
    int32_t rho_p_bp;
    int32_t probe;              /* CHESS_PROBE_*; the anchor needs window_pages >= 1         */
    int32_t cut_rule;           /* CHESS_CUT_*                                               */
    const int32_t* budget_per_seq; /* DEVICE int32 [batch] or NULL: a value > 0 replaces budget_pages / budget_bp
                                   for that sequence (clamped to max_selected_pages - s - w); <= 0 keeps the
                                   plan's own budget.  Ignored by CHESS_PLAN_RATIO.  With it the host sizes every
                                   level for the largest budget the configuration allows */
} chess_select_plan;

/* Create / destroy the host-side context.  `cfg` is a host pointer and is copied.  Queries the
 * current HIP device once (LDS per workgroup, CU count).  CHESS_EINVAL on an unsupported shape. */
int chess_create(const chess_config* cfg, chess_ctx** out);
void chess_destroy(chess_ctx* ctx);

/* Size in bytes of the summaries buffer (for max_batch sequences) the caller must allocate, and
 * the byte offsets of its three level arrays. */
int chess_summary_bytes(const chess_ctx* ctx, size_t* bytes);
int chess_summary_layout(const chess_ctx* ctx, size_t* page_off, size_t* chunk_off, size_t* grid_off);

/* Size in bytes of the workspace (split partials of decode, published keys and kept-unit lists of
 * select, arrival counters); allocate 256-byte aligned.  chess_workspace_init must run once on a
 * fresh allocation (it clears the arrival counters with a small fill kernel; the kernels re-arm
 * them themselves afterwards).  A workspace carries no results between calls, but two calls that
 * share one must not overlap in time (use one workspace per stream). */
int chess_workspace_bytes(const chess_ctx* ctx, size_t* bytes);
int chess_workspace_init(chess_ctx* ctx, void* workspace, void* stream);

/*
 * Hierarchical summaries (Sec. 3.1).  Page vector = mean of the page's key rows (Eq. 1, per KV
 * head of this layer); chunk / grid vector = mean of the child vectors that exist (Eq. 2).  A
 * partial tail page is averaged over its own tokens.  Accumulation is fp64 in index order, one
 * rounding to fp32 per stored vector (with CHESS_SUMMARY_BF16 that fp32 value is rounded once more, to
 * nearest-even bf16, and a parent averages its children as stored).
 * from_page: device int32 [batch] or NULL.  NULL recomputes everything.  Otherwise only pages
 * >= from_page[b] and the chunks / grids containing them are recomputed; vectors below that must
 * be valid from an earlier call on the same prefix.
 */
int chess_summarize(chess_ctx* ctx, const void* k_pool, const int32_t* block_table, const int32_t* seq_lens,
                    int32_t batch, const int32_t* from_page, void* summaries, void* stream);

/*
 * The append of a decode step (the paper's decode loop grows the paged cache by one token per step, Sec. 4.3;
 * the layouts are this library's): writes the new token's key and value rows, bf16 [batch][H_kv][128], at
 * position seq_lens[b] of sequence b -- K row-major in its page, V token-minor -- through the block table, which
 * must already map that page.  seq_lens holds the lengths BEFORE the append and is not changed (the caller adds
 * one); a sequence with no room left (seq_lens[b] >= max_pages_per_seq * page_size) or a negative length is
 * skipped.  The only call that writes the pools.  Follow it with chess_summarize_tail (or chess_decode_step
 * with refresh_tail) on the new lengths to bring the summaries up to date.
 * page_ids / n_selected (both or neither; may be NULL): the lists that are being reused are extended in the same
 * launch as chess_extend_window would for the lengths after the append.
 */
int chess_append_kv(chess_ctx* ctx, const void* k_new, const void* v_new, void* k_pool, void* v_pool,
                    const int32_t* block_table, const int32_t* seq_lens, int32_t batch, int32_t* page_ids,
                    int32_t* n_selected, void* stream);

/* The per-decode-step refresh: chess_summarize with from_page[b] = (pages of sequence b) - 1,
 * i.e. the tail page and its chunk and grid, launched on batch * H workgroups only. */
int chess_summarize_tail(chess_ctx* ctx, const void* k_pool, const int32_t* block_table, const int32_t* seq_lens,
                         int32_t batch, void* summaries, void* stream);

/* The catch-up before a reselection (Sec. 3.3: between reselections nothing reads the summaries): chess_summarize
 * with from_page[b] = max(0, (pages of sequence b) - recent_pages), launched only on the grids those pages can
 * touch.  recent_pages >= 1 is a host value: an upper bound on the pages any sequence has gained or changed since
 * its summaries were last current (recent_pages = 1 is chess_summarize_tail). */
int chess_summarize_recent(chess_ctx* ctx, const void* k_pool, const int32_t* block_table, const int32_t* seq_lens,
                           int32_t batch, int32_t recent_pages, void* summaries, void* stream);

/*
 * Coarse-to-fine selection (Sec. 3.2, Eq. 4, Alg. 1).  Per (sequence, KV head): the probe is the
 * sum of the group's G query rows; a unit's score is probe . unit vector (fp64).  Level 1 keeps
 * the top k_g grids; level 2 ranks only chunks of kept grids and keeps k_c; level 3 ranks only
 * pages of kept chunks that are neither sink nor window pages and keeps k_p.  Rank order: score
 * descending, then index ascending (plan->cut_rule: exactly k units per level, or every unit that ties
 * with the k-th).  Result: sinks, kept pages, window pages as one ascending
 * list of logical page numbers; if the sequence has at most s + w pages, all of them.
 * `plan` is a host pointer.  CHESS_EINVAL if s + w + (largest possible k_p) exceeds
 * max_selected_pages; CHESS_ENOTSUP if a level can have more candidates than fit in LDS.
 * Uses the workspace (published keys, a counter per sequence and KV head).
 */
int chess_select(chess_ctx* ctx, const void* q, const void* summaries, const int32_t* seq_lens, int32_t batch,
                 const chess_select_plan* plan, int32_t* page_ids, int32_t* n_selected, void* workspace,
                 void* stream);

/*
 * The query anchor of Sec. 3.2, Eq. 3 for every (sequence, KV head) of n_layers layers, one launch: the mean of
 * the page vectors of the last min(window_pages, P) pages (fp64 sum in page order, rounded to fp32 once; zero
 * for an empty sequence).  summaries, anchors: HOST arrays of n_layers DEVICE pointers (read during the call
 * only); anchors[l]: fp32 [batch][H_kv][128], 16-byte aligned, written.  Asynchronous on `stream`.
 * CHESS_EINVAL on null / misaligned pointers, n_layers outside [1, CHESS_MAX_LAYERS], batch outside
 * [1, max_batch], window_pages < 1.
 */
int chess_anchor(chess_ctx* ctx, const void* const* summaries, int32_t n_layers, const int32_t* seq_lens, int32_t batch,
                 int32_t window_pages, float* const* anchors, void* stream);

/*
 * The selection under the paper's own scope (Sec. 3.1, Eq. 1 flattens the key means of all layers and heads
 * into one vector per unit; Sec. 3.2, Eq. 3-4): a unit's score is the sum, over the n_layers layers and the H_kv
 * heads, of probe[l][b][h] . unit vector[l][b][h] (fp64), and the cascade of chess_select runs once per
 * sequence on those scores: one page list per sequence, for every layer and head of the model.
 * probes, summaries: HOST arrays of n_layers DEVICE pointers (read during the call only): probes[l] fp32
 * [batch][H_kv][128] (what chess_anchor writes for layer l, or any other probe), summaries[l] a summary buffer
 * of this context's geometry; 16-byte aligned.  All layers share seq_lens.
 * page_ids / n_selected: the layout chess_sparse_decode reads, [batch][H_kv][max_selected_pages] and
 * [batch][H_kv]; the sequence's list is written for each of its KV heads, so the decode calls of every layer
 * take them as they are.  plan->probe is ignored (the probes are given).
 * CHESS_EINVAL as for chess_select, or n_layers outside [1, CHESS_MAX_LAYERS], or a null / misaligned table
 * entry; CHESS_ENOTSUP as for chess_select, or batch above the number of compute units.
 * Uses the workspace like chess_select (rows of the first KV head of each sequence).
 */
int chess_select_shared(chess_ctx* ctx, const float* const* probes, const void* const* summaries, int32_t n_layers,
                        const int32_t* seq_lens, int32_t batch, const chess_select_plan* plan, int32_t* page_ids,
                        int32_t* n_selected, void* workspace, void* stream);

/*
 * Between reselections (Sec. 3.3) a page list is reused while the sequence grows; the recent window of Sec. 3.2
 * is relative to the current position, so the pages generated since the selection belong to the list.  This call
 * appends to every list the pages after its last entry up to the sequence's current last page (seq_lens: the
 * current lengths); an empty list starts at page 0.  A row stops growing when it holds max_selected_pages ids:
 * size the configuration for the longest stretch between reselections.  page_ids / n_selected: as written by
 * chess_select / chess_decode_step / chess_select_shared, updated in place.
 */
int chess_extend_window(chess_ctx* ctx, const int32_t* seq_lens, int32_t batch, int32_t* page_ids, int32_t* n_selected,
                        void* stream);

/*
 * The step between reselections (Sec. 3.3) as ONE launch: what chess_append_kv (with the lists) followed by
 * chess_sparse_decode on the lengths + 1 computes, with the same results bit for bit.  The new token's rows go from
 * k_new / v_new straight into the attention (they do not make a round trip through the pools); the last workgroup of
 * a (sequence, KV head) to finish stores them in the pools and, when the token opens a page, adds the page to
 * the list.  seq_lens: the lengths BEFORE the token (not changed; the caller adds one afterwards).  A sequence with no
 * room left is attended as it is.  Precondition: every list ends with the tail page of seq_lens (as a selection on
 * these lengths, chess_append_kv with the lists, chess_extend_window or this call leave it); an empty list
 * belongs to an empty sequence.  Arguments and errors as for the two calls.
 */
int chess_reuse_step(chess_ctx* ctx, const void* q, const void* k_new, const void* v_new, void* k_pool, void* v_pool,
                     const int32_t* block_table, const int32_t* seq_lens, int32_t* page_ids, int32_t* n_selected,
                     int32_t batch, float* out, void* workspace, void* stream);

/*
 * The quality monitor of Sec. 3.3, first half: the entropy (nats) of the output distribution of one decode step,
 * H[b] = -sum_v p_v log p_v with p = softmax(logits[b]).  logits: device, bf16 [batch][row_stride], the first
 * `vocab` entries of a row are used (-inf entries count as probability 0); 16-byte aligned, row_stride a multiple
 * of 8.  entropy: device fp32 [batch], written.  fp32 arithmetic (absolute error around 1e-5).  Uses the workspace.
 * CHESS_EINVAL on null / misaligned pointers, batch outside [1, max_batch], vocab < 1, row_stride < vocab or not
 * a multiple of 8.
 */
int chess_entropy(chess_ctx* ctx, const void* logits, int32_t batch, int32_t vocab, int64_t row_stride, float* entropy,
                  void* workspace, void* stream);

/*
 * Sec. 3.3, second half: one call per decode step.  Appends entropy[b] to the history of the page sequence b is
 * generating; when that makes page_steps entries, takes their mean and population variance (fp64, in step order),
 * sets fire[b] = (mean > tau_entropy || variance > tau_variance), writes stats[b] = {mean, variance} (if stats is
 * not NULL) and starts a new page; otherwise fire[b] = 0.  The thresholds are inputs (the paper takes the 99th
 * percentiles of a calibration run).  history: device fp32 [batch][page_steps]; count: device int32 [batch], zero
 * before a sequence's first step; fire: device int32 [batch]; stats: device fp64 [batch][2] or NULL.  A caller
 * reselects (chess_select / chess_decode_step) for the sequences whose flag is set and reuses the page list for
 * the others.  CHESS_EINVAL on null pointers, batch outside [1, max_batch], page_steps < 1.
 */
int chess_trigger_update(chess_ctx* ctx, const float* entropy, int32_t batch, int32_t page_steps, double tau_entropy,
                         double tau_variance, float* history, int32_t* count, int32_t* fire, double* stats, void* stream);

/* chess_entropy and chess_trigger_update in one launch (same results): the thread that ends up with a sequence's
 * entropy also updates that sequence's page statistics.  entropy (fp32 [batch]) is still written. */
int chess_monitor_step(chess_ctx* ctx, const void* logits, int32_t batch, int32_t vocab, int64_t row_stride,
                       int32_t page_steps, double tau_entropy, double tau_variance, float* entropy, float* history,
                       int32_t* count, int32_t* fire, double* stats, void* workspace, void* stream);

/*
 * Block-sparse decode attention over the listed pages, read in place (Sec. 4.3 takes a paged
 * decode kernel over page indices; App. B).  Per q head: softmax(sm_scale * q . K_t) weighted sum
 * of V_t over the valid tokens of the listed pages.  bf16 inputs, fp32 accumulation, fp32 out.
 * page_ids entries must be distinct valid logical pages of the sequence.
 */
int chess_sparse_decode(chess_ctx* ctx, const void* q, const void* k_pool, const void* v_pool,
                        const int32_t* block_table, const int32_t* seq_lens, const int32_t* page_ids,
                        const int32_t* n_selected, int32_t batch, float* out, void* workspace, void* stream);

/* The same attention over every page of each sequence: the paper's Full-KV baseline (Sec. 5.1). */
int chess_dense_decode(chess_ctx* ctx, const void* q, const void* k_pool, const void* v_pool,
                       const int32_t* block_table, const int32_t* seq_lens, int32_t batch, float* out,
                       void* workspace, void* stream);

/*
 * One decode step of a layer in a single launch: chess_select followed by chess_sparse_decode over the
 * list it produces (Sec. 3.2 then Sec. 4.3), with the same results as the two calls: the page list is
 * the one chess_select writes, `out` is attention over exactly those pages.  The list stays on chip
 * between the two stages; it is also written to page_ids / n_selected unless those are NULL (pass them
 * to reuse the list in later steps, as the paper does between reselections, Sec. 3.3).
 * Arguments, layouts and errors as for the two calls.
 * With CHESS_PROBE_ANCHOR the attention still uses q; the selection does not.  (The anchor reads the window's
 * page vectors before anything else, so it cannot be combined with refresh_tail: CHESS_ENOTSUP.)
 * refresh_tail != 0: the launch first does what chess_summarize_tail does (Sec. 3.1, Eq. 1-2: the vectors of
 * the tail page, its chunk and its grid are recomputed from the K pool, written to `summaries`, and are the
 * ones the selection scores), so a decode step is this one call.  refresh_tail == 0: `summaries` is only read
 * and must be current.
 */
int chess_decode_step(chess_ctx* ctx, const void* q, const void* k_pool, const void* v_pool,
                      const int32_t* block_table, const int32_t* seq_lens, void* summaries, int32_t refresh_tail,
                      int32_t batch, const chess_select_plan* plan, int32_t* page_ids, int32_t* n_selected, float* out,
                      void* workspace, void* stream);

/* Synchronous check: copies the workspace's error word back on `stream` and waits for that stream (so it sees
 * every launch made on it before; work on other streams is not waited for).  *flag receives CHESS_FLAG_* bits,
 * which stay set until chess_workspace_init.  CHESS_FLAG_WAIT: a kernel using this workspace gave up a bounded
 * wait -- which cannot happen unless the device was shared with work that kept this library's workgroups from
 * becoming resident together (see chess_config.shared_device).  Results written by such a launch are undefined,
 * and published words are left behind: check the flag (or re-initialise the workspace) before the workspace is
 * used again.  CHESS_FLAG_OVERFLOW: see CHESS_CUT_THRESHOLD; the workspace stays usable. */
int chess_workspace_error(chess_ctx* ctx, const void* workspace, int32_t* flag, void* stream);

/*
 * chess_sparse_decode for callers that cannot allocate device memory (code under HIP graph capture that was not
 * handed a workspace, tight serving loops, harnesses that forbid hipMalloc): the same kernels and results, with
 * the split partials and arrival counters in a device array the library owns (CHESS_STATIC_SCRATCH_BYTES per
 * GPU, alive until the process ends) instead of a caller's workspace.  No allocation of any kind happens in the
 * call.  CHESS_ESCRATCH if batch * H_kv * (splits chosen for this shape) needs more than the array holds.
 * Every call on one GPU uses that GPU's one array: calls that overlap in time on the same GPU (two streams, two
 * contexts) race; calls on one stream are safe.
 */
int chess_sparse_decode_static(chess_ctx* ctx, const void* q, const void* k_pool, const void* v_pool,
                               const int32_t* block_table, const int32_t* seq_lens, const int32_t* page_ids,
                               const int32_t* n_selected, int32_t batch, float* out, void* stream);

const char* chess_strerror(int code);
int chess_version(void);

#ifdef __cplusplus
}
#endif
#endif /* CHESS_H */
