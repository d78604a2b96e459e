// The C ABI of libchess: argument checks, buffer sizing and launch-shape decisions on the host;
// every step of the path itself runs in the kernels of summarize.hip, select.hip and decode.hip.
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <initializer_list>
#include <mutex>
#include <new>

#include "chess_internal.h"

// Device memory chess_sparse_decode_static works in instead of a caller's workspace: split partials and arrival
// counters.  Every GPU the library runs on holds its own copy at its own address, for the life of the process.
// In host code this name is only a handle for hipGetSymbolAddress: kernels and fills get the looked-up address.
static __device__ __align__(256) unsigned char scratch[CHESS_STATIC_SCRATCH_BYTES];

namespace {

using chess::kHeadDim;

// Per device: the address of that device's copy of `scratch`, looked up once (by chess_create, with the device
// current).
constexpr int kMaxDevices = 64;
void* g_scratch_of_device[kMaxDevices];
std::mutex g_scratch_mutex;

void* scratch_of_current_device(int dev)
{
    if (dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_of_device[dev] == nullptr) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) {
            (void)hipGetLastError();                    // leave no sticky error behind; the static entry point reports it
            return nullptr;
        }
        g_scratch_of_device[dev] = p;
    }
    return g_scratch_of_device[dev];
}

inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline int64_t ceil_bp(int64_t n, int64_t bp) { return (n * bp + 9999) / 10000; }
inline int64_t clampi(int64_t x, int64_t lo, int64_t hi) { return x < lo ? lo : (x > hi ? hi : x); }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Largest keep-counts any sequence of at most max_pages pages can reach under `pl`.
struct Bounds { int64_t kg, kc, kp, kp_exact, slots, lists; };

bool plan_bounds(const chess_ctx* ctx, const chess_select_plan* pl, Bounds* out)
{
    const chess::Geom& g = ctx->geom;
    const int64_t P = g.max_pages, nc = g.max_chunks, ng = g.max_grids;
    if (pl->sink_pages < 0 || pl->window_pages < 0) return false;
    if (pl->probe != CHESS_PROBE_QUERY && pl->probe != CHESS_PROBE_ANCHOR) return false;
    if (pl->probe == CHESS_PROBE_ANCHOR && pl->window_pages < 1) return false;
    if (pl->cut_rule != CHESS_CUT_COUNT && pl->cut_rule != CHESS_CUT_THRESHOLD) return false;
    const int64_t cand = std::max<int64_t>(0, P - pl->sink_pages - pl->window_pages);   // pages that may compete
    int64_t kmax = 0;
    if (pl->plan != CHESS_PLAN_RATIO) {
        if (pl->budget_pages < 0 || (pl->budget_pages == 0 && (pl->budget_bp < 1 || pl->budget_bp > 10000))) return false;
        kmax = pl->budget_pages > 0 ? pl->budget_pages : clampi(ceil_bp(P, pl->budget_bp), 1, P);
        // budgets the host cannot see: size every level for the largest one a page_ids row can hold
        if (pl->budget_per_seq != nullptr)
            kmax = std::max<int64_t>(kmax, std::max<int64_t>(1, (int64_t)g.max_sel - pl->sink_pages - pl->window_pages));
    }
    Bounds b{};
    switch (pl->plan) {
    case CHESS_PLAN_BUDGET: {
        if (pl->over_chunk < 1 || pl->over_grid < 1) return false;
        const int64_t kct = cdiv((int64_t)pl->over_chunk * kmax, g.n_c);
        b.kg = std::min<int64_t>(ng, cdiv((int64_t)pl->over_grid * kct, g.n_g));
        b.kc = std::min<int64_t>(std::min<int64_t>(nc, kct), b.kg * g.n_g);
        b.kp = std::min<int64_t>(kmax, std::min<int64_t>(cand, b.kc * g.n_c));
        break;
    }
    case CHESS_PLAN_RATIO: {
        for (int32_t r : {pl->rho_g_bp, pl->rho_c_bp, pl->rho_p_bp})
            if (r < 1 || r > 10000) return false;
        b.kg = clampi(ceil_bp(ng, pl->rho_g_bp), 1, ng);
        b.kc = clampi(ceil_bp(std::min<int64_t>(nc, b.kg * g.n_g), pl->rho_c_bp), 1, nc);
        b.kp = cand == 0 ? 0 : clampi(ceil_bp(std::min<int64_t>(cand, b.kc * g.n_c), pl->rho_p_bp), 1, cand);
        break;
    }
    case CHESS_PLAN_FLAT:
        b.kg = ng; b.kc = nc; b.kp = std::min<int64_t>(kmax, cand);
        break;
    default:
        return false;
    }
    b.kp_exact = b.kp;
    if (pl->cut_rule == CHESS_CUT_THRESHOLD) {
        // ties at a cut are all kept, so a level can keep up to everything it has: the lists and the page slots are
        // sized for that, and only a page list that outgrows its page_ids row is an error (reported by the kernels)
        b.kg = ng;
        b.kc = nc;
        b.kp = std::min<int64_t>(cand, std::max<int64_t>(0, (int64_t)g.max_sel - pl->sink_pages - pl->window_pages));
    }
    // grid keys and, behind them, chunk keys by unit (merged) or N_g slots per kept grid (lazy); then the page slots
    b.slots = std::max<int64_t>(ng + std::max<int64_t>(nc, b.kg * g.n_g), b.kc * g.n_c);
    b.lists = std::max<int64_t>(b.kg, b.kc);
    *out = b;
    return true;
}

struct SplitShape { int n_splits, waves; };

// Split-K shape.  Every workgroup has four waves; tiles are dealt round-robin over splits and waves.
// Dense (every page): enough workgroups to cover the chip a few times over; the workgroup that finishes last merges
// ns partial rows per output, tile time falls as 1/ns and merge time grows as G*ns/32 (in units of one memory
// round trip), so the best split count is about sqrt(8*tiles/G), within what is resident at once.
// A page list (tens to hundreds of pages): the fixed latencies dominate, and the measured optimum (sweeps at batch
// 1 .. 32, 21 .. 415 pages, G = 1 .. 7) is: no split once there is a (sequence, head) per compute unit; otherwise one
// workgroup per compute unit, at least two tiles per workgroup, and at most 1.6 x the merge-balanced count.
SplitShape choose_splits(const chess_ctx* ctx, int batch, int64_t max_list_pages, bool listed)
{
    const chess::Geom& g = ctx->geom;
    const int ppt = chess::kTileTokens / g.page_size;
    const int64_t tiles = std::max<int64_t>(1, cdiv(max_list_pages, ppt));
    const int64_t pairs = (int64_t)batch * g.n_kv_heads;
    const int64_t target = 4LL * ctx->n_cu;
    if (ctx->force_splits > 0) return {ctx->force_splits, ctx->force_waves};
    const int waves = 4;
    // all workgroups resident at once: a second round of workgroups would double a short kernel
    const int64_t resident = (int64_t)ctx->dec_blocks4 * ctx->n_cu;
    const double balanced = std::sqrt(8.0 * (double)tiles / g.group);
    int64_t ns;
    if (listed) {
        ns = std::min<int64_t>(ctx->n_cu / pairs, cdiv(tiles, 2));
        ns = std::min<int64_t>(ns, (int64_t)std::llround(1.6 * balanced));
        ns = std::max<int64_t>(ns, 1);
    } else {
        ns = (int64_t)std::llround(balanced);
        ns = std::min<int64_t>(ns, std::max<int64_t>(1, resident / pairs));
        ns = clampi(ns, 1, cdiv(tiles, waves));
    }
    ns = std::min<int64_t>(ns, std::min<int64_t>(ctx->max_splits, 1024 / g.group));
    while (ns > 1 && pairs * ns > target + pairs) --ns;            // stay inside the workspace
    return {(int)ns, waves};
}

int decode_common(chess_ctx* ctx, const void* q, const void* k_pool, const void* v_pool, const int32_t* block_table,
                  const int32_t* seq_lens, const int32_t* page_ids, const int32_t* n_selected, int32_t batch,
                  float* out, void* workspace, void* stream)
{
    if (!ctx || !q || !k_pool || !v_pool || !block_table || !seq_lens || !out || !workspace) return CHESS_EINVAL;
    if (batch < 1 || batch > ctx->cfg.max_batch) return CHESS_EINVAL;
    if ((reinterpret_cast<uintptr_t>(k_pool) | reinterpret_cast<uintptr_t>(v_pool) | reinterpret_cast<uintptr_t>(q) |
         reinterpret_cast<uintptr_t>(out) | reinterpret_cast<uintptr_t>(workspace)) & 15) return CHESS_EINVAL;
    const SplitShape sh = choose_splits(ctx, batch, page_ids ? ctx->geom.max_sel : ctx->geom.max_pages, page_ids != nullptr);
    float* ws_acc = reinterpret_cast<float*>(static_cast<char*>(workspace) + ctx->ws_acc_off);
    float* ws_ml = reinterpret_cast<float*>(static_cast<char*>(workspace) + ctx->ws_ml_off);
    int32_t* arrivals = reinterpret_cast<int32_t*>(static_cast<char*>(workspace) + ctx->ws_cnt_off);
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = chess::launch_decode(ctx, static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k_pool),
                                        static_cast<const uint16_t*>(v_pool), block_table, seq_lens, page_ids,
                                        n_selected, batch, sh.n_splits, sh.waves, out, ws_acc, ws_ml, arrivals, s);
    return e == hipSuccess ? CHESS_OK : CHESS_EHIP;
}

}  // namespace

extern "C" {

int chess_create(const chess_config* cfg, chess_ctx** out)
{
    if (!cfg || !out) return CHESS_EINVAL;
    *out = nullptr;
    if (cfg->head_dim != kHeadDim) return CHESS_EINVAL;
    if (cfg->page_size != 16 && cfg->page_size != 32) return CHESS_EINVAL;
    if (cfg->n_kv_heads < 1 || cfg->n_q_heads < 1 || cfg->n_q_heads % cfg->n_kv_heads) return CHESS_EINVAL;
    if (cfg->n_q_heads / cfg->n_kv_heads > chess::kMaxGroup) return CHESS_EINVAL;
    if (cfg->pages_per_chunk < 1 || cfg->chunks_per_grid < 1 ||
        (int64_t)cfg->pages_per_chunk * cfg->chunks_per_grid > 256) return CHESS_EINVAL;
    if (cfg->max_batch < 1 || cfg->max_pages_per_seq < 1 || cfg->max_selected_pages < 1) return CHESS_EINVAL;
    if (cfg->max_selected_pages > cfg->max_pages_per_seq) return CHESS_EINVAL;
    if (!(cfg->sm_scale >= 0.f) || !std::isfinite(cfg->sm_scale)) return CHESS_EINVAL;
    if (cfg->summary_dtype != CHESS_SUMMARY_F32 && cfg->summary_dtype != CHESS_SUMMARY_BF16) return CHESS_EINVAL;

    chess_ctx* c = new (std::nothrow) chess_ctx();
    if (!c) return CHESS_ENOMEM;
    c->cfg = *cfg;
    chess::Geom& g = c->geom;
    g.n_q_heads = cfg->n_q_heads; g.n_kv_heads = cfg->n_kv_heads; g.group = cfg->n_q_heads / cfg->n_kv_heads;
    g.page_size = cfg->page_size; g.n_c = cfg->pages_per_chunk; g.n_g = cfg->chunks_per_grid;
    g.max_pages = cfg->max_pages_per_seq;
    g.max_chunks = (int32_t)cdiv(g.max_pages, g.n_c);
    g.max_grids = (int32_t)cdiv(g.max_chunks, g.n_g);
    g.max_sel = cfg->max_selected_pages;
    g.inv_nc = g.n_c > 1 ? (uint32_t)((0x100000000ull + g.n_c - 1) / g.n_c) : 0u;
    g.inv_ng = g.n_g > 1 ? (uint32_t)((0x100000000ull + g.n_g - 1) / g.n_g) : 0u;
    c->sm_scale = cfg->sm_scale > 0.f ? cfg->sm_scale : 1.0f / std::sqrt((float)kHeadDim);

    int dev = 0, v = 0;
    if (hipGetDevice(&dev) != hipSuccess) { delete c; return CHESS_EHIP; }
    c->device = dev;
    c->n_cu = hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0 ? v : 256;
    c->lds_per_block = hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) == hipSuccess && v > 0 ? v : 65536;

    const size_t rows = (size_t)cfg->max_batch * g.n_kv_heads;
    const size_t vec = kHeadDim * sizeof(float);
    const size_t svec = kHeadDim * (cfg->summary_dtype == CHESS_SUMMARY_BF16 ? sizeof(uint16_t) : sizeof(float));
    c->page_off = 0;
    c->chunk_off = align_up(c->page_off + rows * g.max_pages * svec, 256);
    c->grid_off = align_up(c->chunk_off + rows * g.max_chunks * svec, 256);
    c->summary_bytes = align_up(c->grid_off + rows * g.max_grids * svec, 256);

    c->max_splits = 256;
    const size_t part_rows = (size_t)(4 * c->n_cu + rows) * g.group;       // see choose_splits
    c->ws_acc_off = 0;
    c->ws_ml_off = align_up(part_rows * vec, 256);
    c->ws_keys_off = align_up(c->ws_ml_off + part_rows * 2 * sizeof(float), 256);
    c->key_stride = (int64_t)g.max_grids * (1 + g.n_g) + (int64_t)g.max_chunks * g.n_c;
    c->ws_tail_off = align_up(c->ws_keys_off + rows * c->key_stride * sizeof(uint64_t), 256);
    c->ws_meta_off = align_up(c->ws_tail_off + rows * 4 * sizeof(uint64_t), 256);
    c->ws_cnt_off = align_up(c->ws_meta_off + rows * chess::kSelMetaStride * sizeof(int32_t), 256);
    c->ws_err_off = align_up(c->ws_cnt_off + rows * sizeof(int32_t), 256);
    c->ws_ent_off = align_up(c->ws_err_off + 256, 256);
    c->ws_entcnt_off = align_up(c->ws_ent_off + (size_t)cfg->max_batch * chess::kEntMaxSplits * 4 * sizeof(float), 256);
    c->workspace_bytes = align_up(c->ws_entcnt_off + (size_t)cfg->max_batch * sizeof(int32_t), 256);
    c->dec_blocks4 = c->dec_blocks1 = 2;
    if (chess::decode_occupancy(g.page_size, 4, g.group, &v) == hipSuccess && v > 0) c->dec_blocks4 = v;
    if (chess::decode_occupancy(g.page_size, 1, g.group, &v) == hipSuccess && v > 0) c->dec_blocks1 = v;
    c->force_cluster = 0;
    c->force_schedule = 0;
    c->force_general_cut = 0;
    c->poll_limit = 0;
    c->occ_lds = -1;
    c->occ_blocks = 0;
    c->shared_occ_lds = -1;
    c->shared_occ_blocks = 0;
    c->step_occ_lds = -1;
    c->step_occ_blocks = 0;
    c->ws_zero_off = c->ws_keys_off;
    c->ws_zero_bytes = c->workspace_bytes - c->ws_keys_off;
    c->ws_prof_off = c->workspace_bytes;
#ifdef CHESS_PROF
    c->workspace_bytes += align_up(rows * 2 * 24 * sizeof(int32_t), 256);   // profiling builds: two timelines of 24 stamps per row, at the end
#endif
    c->force_splits = 0;
    c->force_waves = 4;
    c->static_scratch = scratch_of_current_device(dev);
    *out = c;
    return CHESS_OK;
}

void chess_destroy(chess_ctx* ctx) { delete ctx; }

int chess_summary_bytes(const chess_ctx* ctx, size_t* bytes)
{
    if (!ctx || !bytes) return CHESS_EINVAL;
    *bytes = ctx->summary_bytes;
    return CHESS_OK;
}

int chess_summary_layout(const chess_ctx* ctx, size_t* page_off, size_t* chunk_off, size_t* grid_off)
{
    if (!ctx || !page_off || !chunk_off || !grid_off) return CHESS_EINVAL;
    *page_off = ctx->page_off; *chunk_off = ctx->chunk_off; *grid_off = ctx->grid_off;
    return CHESS_OK;
}

int chess_workspace_bytes(const chess_ctx* ctx, size_t* bytes)
{
    if (!ctx || !bytes) return CHESS_EINVAL;
    *bytes = ctx->workspace_bytes;
    return CHESS_OK;
}

static int summarize_common(chess_ctx* ctx, const void* k_pool, const int32_t* block_table, const int32_t* seq_lens,
                            int32_t batch, const int32_t* from_page, int recent, void* summaries, void* stream)
{
    if (!ctx || !k_pool || !block_table || !seq_lens || !summaries) return CHESS_EINVAL;
    if (batch < 1 || batch > ctx->cfg.max_batch) return CHESS_EINVAL;
    if ((reinterpret_cast<uintptr_t>(k_pool) | reinterpret_cast<uintptr_t>(summaries)) & 15) return CHESS_EINVAL;
    char* sb = static_cast<char*>(summaries);
    hipError_t e = chess::launch_summarize(ctx, static_cast<const uint16_t*>(k_pool), block_table, seq_lens, batch,
                                           from_page, recent, sb + ctx->page_off, sb + ctx->chunk_off, sb + ctx->grid_off,
                                           static_cast<hipStream_t>(stream));
    return e == hipSuccess ? CHESS_OK : CHESS_EHIP;
}

int chess_summarize(chess_ctx* ctx, const void* k_pool, const int32_t* block_table, const int32_t* seq_lens,
                    int32_t batch, const int32_t* from_page, void* summaries, void* stream)
{
    return summarize_common(ctx, k_pool, block_table, seq_lens, batch, from_page, 0, summaries, stream);
}

int chess_summarize_tail(chess_ctx* ctx, const void* k_pool, const int32_t* block_table, const int32_t* seq_lens,
                         int32_t batch, void* summaries, void* stream)
{
    return summarize_common(ctx, k_pool, block_table, seq_lens, batch, nullptr, 1, summaries, stream);
}

int chess_summarize_recent(chess_ctx* ctx, const void* k_pool, const int32_t* block_table, const int32_t* seq_lens,
                           int32_t batch, int32_t recent_pages, void* summaries, void* stream)
{
    if (recent_pages < 1) return CHESS_EINVAL;
    return summarize_common(ctx, k_pool, block_table, seq_lens, batch, nullptr, recent_pages, summaries, stream);
}

int chess_workspace_init(chess_ctx* ctx, void* workspace, void* stream)
{
    if (!ctx || !workspace || (reinterpret_cast<uintptr_t>(workspace) & 15)) return CHESS_EINVAL;
    hipError_t e = chess::launch_zero(ctx, reinterpret_cast<int32_t*>(static_cast<char*>(workspace) + ctx->ws_zero_off),
                                      ctx->ws_zero_bytes / sizeof(int32_t), static_cast<hipStream_t>(stream));
    return e == hipSuccess ? CHESS_OK : CHESS_EHIP;
}

// Workgroups that cooperate on one (sequence, KV head).  Measured on MI355X (batch 1 .. 32, 16K .. 256K tokens):
// once there is a (sequence, head) per compute unit, splitting them further only adds exchanges; below that, more
// members keep paying off until each wave has about two tiles of the list left, between 8 and 12 members.
// All workgroups of the grid have to fit on the device at once (the members wait for each other's keys).
static int64_t choose_cluster(const chess_ctx* ctx, int64_t pairs, int64_t capacity)
{
    if (pairs >= ctx->n_cu || ctx->cfg.shared_device != 0) return 1;
    const int64_t tiles = cdiv(ctx->geom.max_sel, chess::kTileTokens / ctx->geom.page_size);
    return std::max<int64_t>(1, std::min<int64_t>(capacity / pairs, clampi(cdiv(tiles, 8), 8, 12)));
}

// Which schedule the levels run on (select_device.h).  merged: all chunks are scored with the grids, which saves a
// dependent memory phase and an exchange for n_c - k_g N_g more chunk vectors; it pays while the launch is bound by
// its chain of memory round trips rather than by bytes.  Otherwise lazy, and every member scores all grids itself
// when they are few.
static void choose_schedule(const chess_ctx* ctx, int64_t pairs, int64_t cluster, chess::SelectParams* sp)
{
    const int svec = kHeadDim * (ctx->cfg.summary_dtype == CHESS_SUMMARY_BF16 ? 2 : 4);
    // measured on MI355X: merged wins when several workgroups share a (sequence, head) (an exchange is saved, not only
    // a phase) and all chunk vectors of the launch stay below about 24 MB (cfg4a: bf16 summaries yes, fp32 no)
    const int64_t chunk_bytes = pairs * ctx->geom.max_chunks * svec;
    sp->merged = ctx->force_schedule > 0 ? ctx->force_schedule == 2 : (cluster > 1 && chunk_bytes <= (24LL << 20));
    sp->local_grids = pairs * cluster * ctx->geom.max_grids * svec <= (4LL << 20);   // repeated grid reads stay small (measured: at 33 MB it costs 3 us)   // repeated grid reads stay small
}

// Checks a plan against the configuration and fills the kernel-side parameters.
static int prepare_select(chess_ctx* ctx, const chess_select_plan* plan, chess::SelectParams* out)
{
    Bounds bd;
    if (!plan_bounds(ctx, plan, &bd)) return CHESS_EINVAL;
    if ((int64_t)plan->sink_pages + plan->window_pages + bd.kp_exact > ctx->geom.max_sel) return CHESS_EINVAL;
    chess::SelectParams sp{};
    sp.plan = plan->plan; sp.sink = plan->sink_pages; sp.window = plan->window_pages;
    sp.budget_pages = plan->budget_pages; sp.budget_bp = plan->budget_bp;
    sp.over_chunk = plan->over_chunk; sp.over_grid = plan->over_grid;
    sp.rho_g_bp = plan->rho_g_bp; sp.rho_c_bp = plan->rho_c_bp; sp.rho_p_bp = plan->rho_p_bp;
    sp.cap2 = (int32_t)(bd.kg * ctx->geom.n_g);
    sp.cap3 = (int32_t)(bd.kc * ctx->geom.n_c);
    sp.cap_keys = (int32_t)bd.slots;
    sp.cap_kg = (int32_t)bd.kg;
    sp.cap_kc = (int32_t)bd.kc;
    sp.probe = plan->probe;
    sp.poll_limit = ctx->poll_limit > 0 ? ctx->poll_limit : ctx->poll_limit < 0 ? 0 : (1 << 15);   // < 0: every wait fails at once
    sp.general_cut = ctx->force_general_cut;
    sp.budget_per_seq = plan->plan == CHESS_PLAN_RATIO ? nullptr : plan->budget_per_seq;
    sp.keep_ties = plan->cut_rule == CHESS_CUT_THRESHOLD;
    *out = sp;
    return CHESS_OK;
}

static chess::SelectWs select_ws(const chess_ctx* ctx, void* workspace)
{
    char* wb = static_cast<char*>(workspace);
    return chess::SelectWs{reinterpret_cast<uint64_t*>(wb + ctx->ws_keys_off), ctx->key_stride,
                           reinterpret_cast<uint64_t*>(wb + ctx->ws_tail_off),
                           reinterpret_cast<int32_t*>(wb + ctx->ws_meta_off), reinterpret_cast<int32_t*>(wb + ctx->ws_err_off)
#ifdef CHESS_PROF
                           , reinterpret_cast<int32_t*>(wb + ctx->ws_prof_off)
#endif
    };
}

int chess_select(chess_ctx* ctx, const void* q, const void* summaries, const int32_t* seq_lens, int32_t batch,
                 const chess_select_plan* plan, int32_t* page_ids, int32_t* n_selected, void* workspace, void* stream)
{
    if (!ctx || !summaries || !seq_lens || !plan || !page_ids || !n_selected || !workspace) return CHESS_EINVAL;
    if (!q && plan->probe != CHESS_PROBE_ANCHOR) return CHESS_EINVAL;
    if (batch < 1 || batch > ctx->cfg.max_batch) return CHESS_EINVAL;
    if ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(summaries) | reinterpret_cast<uintptr_t>(workspace)) & 15)
        return CHESS_EINVAL;
    chess::SelectParams sp;
    if (int rc = prepare_select(ctx, plan, &sp)) return rc;
    const size_t lds = chess::select_lds_bytes(sp, ctx->geom.max_sel);
    if (lds + 8192 > (size_t)ctx->lds_per_block) return CHESS_ENOTSUP;   // the kernel's static LDS is below 8 KB

    // cluster size: the members of a cluster wait for each other's keys, so every workgroup of the grid has to fit
    // on the device at once
    const bool bf16 = ctx->cfg.summary_dtype == CHESS_SUMMARY_BF16;
    if (ctx->occ_lds != (int)lds) {
        int blocks = 0;
        if (chess::select_occupancy(bf16, (int)lds, &blocks) != hipSuccess) return CHESS_EHIP;
        ctx->occ_lds = (int)lds;
        ctx->occ_blocks = blocks;
    }
    const int64_t pairs = (int64_t)batch * ctx->geom.n_kv_heads;
    const int64_t capacity = (int64_t)ctx->occ_blocks * ctx->n_cu;
    int64_t cluster = choose_cluster(ctx, pairs, capacity);
    if (ctx->force_cluster > 0) cluster = std::min<int64_t>(ctx->force_cluster, capacity / pairs);
    cluster = ctx->cfg.shared_device != 0 ? 1 : clampi(cluster, 1, chess::kSelMaxCluster);

    choose_schedule(ctx, pairs, cluster, &sp);
    const chess::SelectWs ws = select_ws(ctx, workspace);
    const char* sb = static_cast<const char*>(summaries);
    hipError_t e = chess::launch_select(ctx, static_cast<const uint16_t*>(q), sb + ctx->page_off, sb + ctx->chunk_off,
                                        sb + ctx->grid_off, seq_lens, batch, (int)cluster,
                                        sp, ws, lds, page_ids, n_selected, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? CHESS_OK : CHESS_EHIP;
}

int chess_reuse_step(chess_ctx* ctx, const void* q, const void* k_new, const void* v_new, void* k_pool, void* v_pool,
                     const int32_t* block_table, const int32_t* seq_lens, int32_t* page_ids, int32_t* n_selected,
                     int32_t batch, float* out, void* workspace, void* stream)
{
    if (!ctx || !q || !k_new || !v_new || !k_pool || !v_pool || !block_table || !seq_lens || !page_ids || !n_selected ||
        !out || !workspace)
        return CHESS_EINVAL;
    if (batch < 1 || batch > ctx->cfg.max_batch) return CHESS_EINVAL;
    if ((reinterpret_cast<uintptr_t>(k_pool) | reinterpret_cast<uintptr_t>(v_pool) | reinterpret_cast<uintptr_t>(q) |
         reinterpret_cast<uintptr_t>(k_new) | reinterpret_cast<uintptr_t>(v_new) | reinterpret_cast<uintptr_t>(out) |
         reinterpret_cast<uintptr_t>(workspace)) & 15)
        return CHESS_EINVAL;
    SplitShape sh = choose_splits(ctx, batch, ctx->geom.max_sel, true);
    if (sh.waves != 4) sh.waves = 4;
    char* wb = static_cast<char*>(workspace);
    hipError_t e = chess::launch_reuse(ctx, static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k_new),
                                       static_cast<const uint16_t*>(v_new), static_cast<uint16_t*>(k_pool),
                                       static_cast<uint16_t*>(v_pool), block_table, seq_lens, page_ids, n_selected, batch,
                                       sh.n_splits, out, reinterpret_cast<float*>(wb + ctx->ws_acc_off),
                                       reinterpret_cast<float*>(wb + ctx->ws_ml_off),
                                       reinterpret_cast<int32_t*>(wb + ctx->ws_cnt_off), static_cast<hipStream_t>(stream));
    return e == hipSuccess ? CHESS_OK : CHESS_EHIP;
}

int chess_extend_window(chess_ctx* ctx, const int32_t* seq_lens, int32_t batch, int32_t* page_ids, int32_t* n_selected,
                        void* stream)
{
    if (!ctx || !seq_lens || !page_ids || !n_selected) return CHESS_EINVAL;
    if (batch < 1 || batch > ctx->cfg.max_batch) return CHESS_EINVAL;
    hipError_t e = chess::launch_extend(ctx, seq_lens, batch, page_ids, n_selected, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? CHESS_OK : CHESS_EHIP;
}

static int entropy_common(chess_ctx* ctx, const void* logits, int32_t batch, int32_t vocab, int64_t row_stride, float* entropy,
                          int32_t page_steps, double tau_h, double tau_v, float* history, int32_t* count, int32_t* fire,
                          double* stats, void* workspace, void* stream)
{
    if (!ctx || !logits || !entropy || !workspace) return CHESS_EINVAL;
    if (batch < 1 || batch > ctx->cfg.max_batch || vocab < 1 || row_stride < vocab || (row_stride & 7)) return CHESS_EINVAL;
    if ((reinterpret_cast<uintptr_t>(logits) | reinterpret_cast<uintptr_t>(workspace)) & 15) return CHESS_EINVAL;
    // enough workgroups to fill the device, each with at least 4096 logits
    const int64_t by_size = std::max<int64_t>(1, vocab / 4096);
    const int splits = (int)clampi(std::min<int64_t>(by_size, cdiv(2 * ctx->n_cu, batch)), 1, chess::kEntMaxSplits);
    char* wb = static_cast<char*>(workspace);
    hipError_t e = chess::launch_entropy(ctx, static_cast<const uint16_t*>(logits), batch, vocab, row_stride, splits, entropy,
                                         reinterpret_cast<float*>(wb + ctx->ws_ent_off),
                                         reinterpret_cast<int32_t*>(wb + ctx->ws_entcnt_off), page_steps, tau_h, tau_v,
                                         history, count, fire, stats, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? CHESS_OK : CHESS_EHIP;
}

int chess_entropy(chess_ctx* ctx, const void* logits, int32_t batch, int32_t vocab, int64_t row_stride, float* entropy,
                  void* workspace, void* stream)
{
    return entropy_common(ctx, logits, batch, vocab, row_stride, entropy, 0, 0.0, 0.0, nullptr, nullptr, nullptr, nullptr,
                          workspace, stream);
}

int chess_monitor_step(chess_ctx* ctx, const void* logits, int32_t batch, int32_t vocab, int64_t row_stride,
                       int32_t page_steps, double tau_entropy, double tau_variance, float* entropy, float* history,
                       int32_t* count, int32_t* fire, double* stats, void* workspace, void* stream)
{
    if (!history || !count || !fire || page_steps < 1) return CHESS_EINVAL;
    return entropy_common(ctx, logits, batch, vocab, row_stride, entropy, page_steps, tau_entropy, tau_variance, history,
                          count, fire, stats, workspace, stream);
}

int chess_trigger_update(chess_ctx* ctx, const float* entropy, int32_t batch, int32_t page_steps, double tau_entropy,
                         double tau_variance, float* history, int32_t* count, int32_t* fire, double* stats, void* stream)
{
    if (!ctx || !entropy || !history || !count || !fire) return CHESS_EINVAL;
    if (batch < 1 || batch > ctx->cfg.max_batch || page_steps < 1) return CHESS_EINVAL;
    hipError_t e = chess::launch_trigger(entropy, batch, page_steps, tau_entropy, tau_variance, history, count, fire, stats,
                                         static_cast<hipStream_t>(stream));
    return e == hipSuccess ? CHESS_OK : CHESS_EHIP;
}

int chess_append_kv(chess_ctx* ctx, const void* k_new, const void* v_new, void* k_pool, void* v_pool,
                    const int32_t* block_table, const int32_t* seq_lens, int32_t batch, int32_t* page_ids,
                    int32_t* n_selected, void* stream)
{
    if (!ctx || !k_new || !v_new || !k_pool || !v_pool || !block_table || !seq_lens) return CHESS_EINVAL;
    if ((page_ids == nullptr) != (n_selected == nullptr)) return CHESS_EINVAL;
    if (batch < 1 || batch > ctx->cfg.max_batch) return CHESS_EINVAL;
    hipError_t e = chess::launch_append(ctx, static_cast<const uint16_t*>(k_new), static_cast<const uint16_t*>(v_new),
                                        static_cast<uint16_t*>(k_pool), static_cast<uint16_t*>(v_pool), block_table,
                                        seq_lens, batch, page_ids, n_selected, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? CHESS_OK : CHESS_EHIP;
}

int chess_anchor(chess_ctx* ctx, const void* const* summaries, int32_t n_layers, const int32_t* seq_lens, int32_t batch,
                 int32_t window_pages, float* const* anchors, void* stream)
{
    if (!ctx || !summaries || !seq_lens || !anchors) return CHESS_EINVAL;
    if (n_layers < 1 || n_layers > CHESS_MAX_LAYERS) return CHESS_EINVAL;
    if (batch < 1 || batch > ctx->cfg.max_batch || window_pages < 1) return CHESS_EINVAL;
    chess::AnchorTable tab{};
    for (int l = 0; l < n_layers; ++l) {
        if (!summaries[l] || !anchors[l]) return CHESS_EINVAL;
        if ((reinterpret_cast<uintptr_t>(summaries[l]) | reinterpret_cast<uintptr_t>(anchors[l])) & 15) return CHESS_EINVAL;
        tab.summaries[l] = static_cast<const char*>(summaries[l]);
        tab.anchors[l] = anchors[l];
    }
    tab.page_off = ctx->page_off;
    hipError_t e = chess::launch_anchor(ctx, tab, n_layers, seq_lens, batch, window_pages, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? CHESS_OK : CHESS_EHIP;
}

int chess_select_shared(chess_ctx* ctx, const float* const* probes, const void* const* summaries, int32_t n_layers,
                        const int32_t* seq_lens, int32_t batch, const chess_select_plan* plan, int32_t* page_ids,
                        int32_t* n_selected, void* workspace, void* stream)
{
    if (!ctx || !probes || !summaries || !seq_lens || !plan || !page_ids || !n_selected || !workspace) return CHESS_EINVAL;
    if (n_layers < 1 || n_layers > CHESS_MAX_LAYERS) return CHESS_EINVAL;
    if (batch < 1 || batch > ctx->cfg.max_batch) return CHESS_EINVAL;
    if (reinterpret_cast<uintptr_t>(workspace) & 15) return CHESS_EINVAL;
    chess::SharedTable tab{};
    for (int l = 0; l < n_layers; ++l) {
        if (!probes[l] || !summaries[l]) return CHESS_EINVAL;
        if ((reinterpret_cast<uintptr_t>(probes[l]) | reinterpret_cast<uintptr_t>(summaries[l])) & 15) return CHESS_EINVAL;
        tab.probes[l] = probes[l];
        tab.summaries[l] = static_cast<const char*>(summaries[l]);
    }
    tab.page_off = ctx->page_off; tab.chunk_off = ctx->chunk_off; tab.grid_off = ctx->grid_off;
    tab.n_layers = n_layers;
    chess::SelectParams sp;
    if (int rc = prepare_select(ctx, plan, &sp)) return rc;
    const size_t lds = chess::select_lds_bytes(sp, ctx->geom.max_sel);
    if (lds + 10240 > (size_t)ctx->lds_per_block) return CHESS_ENOTSUP;  // the kernel's static LDS is below 10 KB
    if (ctx->shared_occ_lds != (int)lds) {
        int blocks = 0;
        if (chess::select_shared_occupancy(ctx->cfg.summary_dtype == CHESS_SUMMARY_BF16, (int)lds, &blocks) != hipSuccess) return CHESS_EHIP;
        ctx->shared_occ_lds = (int)lds;
        ctx->shared_occ_blocks = blocks;
    }
    // a unit's vector is n_layers * H_kv rows, so the more members the better, as long as all fit at once; two
    // workgroups per compute unit cover each other's drains between passes (measured 4 % faster than one)
    const int64_t capacity = (int64_t)std::min(ctx->shared_occ_blocks, 2) * ctx->n_cu;
    if (capacity < batch) return CHESS_ENOTSUP;
    int64_t cluster = capacity / batch;
    if (ctx->force_cluster > 0) cluster = std::min<int64_t>(ctx->force_cluster, cluster);
    cluster = ctx->cfg.shared_device != 0 ? 1 : clampi(cluster, 1, chess::kSharedMaxCluster);
    sp.local_grids = 0;
    sp.merged = 0;                                   // a unit is n_layers * H_kv rows here: the launch is bound by bytes
    const chess::SelectWs ws = select_ws(ctx, workspace);
    hipError_t e = chess::launch_select_shared(ctx, tab, seq_lens, batch, (int)cluster, sp, ws, lds, page_ids, n_selected,
                                               static_cast<hipStream_t>(stream));
    return e == hipSuccess ? CHESS_OK : CHESS_EHIP;
}

int chess_decode_step(chess_ctx* ctx, const void* q, const void* k_pool, const void* v_pool,
                      const int32_t* block_table, const int32_t* seq_lens, void* summaries, int32_t refresh_tail,
                      int32_t batch, const chess_select_plan* plan, int32_t* page_ids, int32_t* n_selected, float* out,
                      void* workspace, void* stream)
{
    if (!ctx || !q || !k_pool || !v_pool || !block_table || !seq_lens || !summaries || !plan || !out || !workspace)
        return CHESS_EINVAL;
    if (batch < 1 || batch > ctx->cfg.max_batch) return CHESS_EINVAL;
    if ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k_pool) | reinterpret_cast<uintptr_t>(v_pool) |
         reinterpret_cast<uintptr_t>(summaries) | reinterpret_cast<uintptr_t>(out) | reinterpret_cast<uintptr_t>(workspace)) & 15)
        return CHESS_EINVAL;
    chess::SelectParams sp;
    if (int rc = prepare_select(ctx, plan, &sp)) return rc;
    if (sp.probe == CHESS_PROBE_ANCHOR && refresh_tail != 0) return CHESS_ENOTSUP;
    int union_off = 0;
    const size_t lds = chess::step_lds_bytes(sp, ctx->geom.max_sel, &union_off);
    if (lds + 8192 > (size_t)ctx->lds_per_block) return CHESS_ENOTSUP;

    if (ctx->step_occ_lds != (int)lds) {
        int blocks = 0;
        if (chess::step_occupancy(ctx->geom.page_size, ctx->cfg.summary_dtype == CHESS_SUMMARY_BF16, (int)lds, &blocks) != hipSuccess) return CHESS_EHIP;
        ctx->step_occ_lds = (int)lds;
        ctx->step_occ_blocks = blocks;
    }
    if (ctx->step_occ_blocks < 1) return CHESS_ENOTSUP;
    const int64_t pairs = (int64_t)batch * ctx->geom.n_kv_heads;
    const int64_t capacity = (int64_t)ctx->step_occ_blocks * ctx->n_cu;
    int64_t cluster = choose_cluster(ctx, pairs, capacity);
    if (ctx->force_cluster > 0) cluster = std::min<int64_t>(ctx->force_cluster, capacity / pairs);
    cluster = ctx->cfg.shared_device != 0 ? 1 : clampi(cluster, 1, chess::kSelMaxCluster);
    if (pairs * cluster > 4LL * ctx->n_cu + pairs) return CHESS_ENOTSUP;   // partial rows of the workspace
    choose_schedule(ctx, pairs, cluster, &sp);

    const chess::SelectWs ws = select_ws(ctx, workspace);
    char* sb = static_cast<char*>(summaries);
    char* wb = static_cast<char*>(workspace);
    chess::StepLaunch sl{static_cast<const uint16_t*>(q), sb + ctx->page_off, sb + ctx->chunk_off, sb + ctx->grid_off,
                         static_cast<const uint16_t*>(k_pool), static_cast<const uint16_t*>(v_pool), block_table, seq_lens,
                         page_ids, n_selected, out, reinterpret_cast<float*>(wb + ctx->ws_acc_off),
                         reinterpret_cast<float*>(wb + ctx->ws_ml_off), reinterpret_cast<int32_t*>(wb + ctx->ws_cnt_off),
                         refresh_tail != 0};
    hipError_t e = chess::launch_step(ctx, sl, batch, (int)cluster, sp, ws, lds, union_off, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? CHESS_OK : CHESS_EHIP;
}

int chess_workspace_error(chess_ctx* ctx, const void* workspace, int32_t* flag, void* stream)
{
    if (!ctx || !workspace || !flag) return CHESS_EINVAL;
    // ordered behind everything launched on the caller's stream (a copy on the null stream would not wait for
    // work on a non-blocking stream)
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e = hipMemcpyAsync(flag, static_cast<const char*>(workspace) + ctx->ws_err_off, sizeof(int32_t),
                                  hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    return e == hipSuccess ? CHESS_OK : CHESS_EHIP;
}

int chess_debug_force_cluster(chess_ctx* ctx, int32_t cluster)
{
    if (!ctx || cluster < 0 || cluster > chess::kSelMaxCluster) return CHESS_EINVAL;
    ctx->force_cluster = cluster;
    return CHESS_OK;
}

int chess_debug_force_schedule(chess_ctx* ctx, int32_t schedule)
{
    if (!ctx || schedule < 0 || schedule > 2) return CHESS_EINVAL;
    ctx->force_schedule = schedule;
    return CHESS_OK;
}

int chess_debug_force_general_cut(chess_ctx* ctx, int32_t on)
{
    if (!ctx || (on != 0 && on != 1)) return CHESS_EINVAL;
    ctx->force_general_cut = on;
    return CHESS_OK;
}

int chess_debug_set_poll_limit(chess_ctx* ctx, int32_t polls)
{
    if (!ctx) return CHESS_EINVAL;
    ctx->poll_limit = polls;
    return CHESS_OK;
}

int chess_sparse_decode(chess_ctx* ctx, const void* q, const void* k_pool, const void* v_pool,
                        const int32_t* block_table, const int32_t* seq_lens, const int32_t* page_ids,
                        const int32_t* n_selected, int32_t batch, float* out, void* workspace, void* stream)
{
    if (!page_ids || !n_selected) return CHESS_EINVAL;
    return decode_common(ctx, q, k_pool, v_pool, block_table, seq_lens, page_ids, n_selected, batch, out, workspace, stream);
}

int chess_sparse_decode_static(chess_ctx* ctx, const void* q, const void* k_pool, const void* v_pool,
                               const int32_t* block_table, const int32_t* seq_lens, const int32_t* page_ids,
                               const int32_t* n_selected, int32_t batch, float* out, void* stream)
{
    if (!ctx || !q || !k_pool || !v_pool || !block_table || !seq_lens || !page_ids || !n_selected || !out) return CHESS_EINVAL;
    if (batch < 1 || batch > ctx->cfg.max_batch) return CHESS_EINVAL;
    if ((reinterpret_cast<uintptr_t>(k_pool) | reinterpret_cast<uintptr_t>(v_pool) | reinterpret_cast<uintptr_t>(q) |
         reinterpret_cast<uintptr_t>(out)) & 15) return CHESS_EINVAL;
    // the array's address was looked up for the device the context was created on
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev != ctx->device || ctx->static_scratch == nullptr) return CHESS_EHIP;
    const SplitShape sh = choose_splits(ctx, batch, ctx->geom.max_sel, true);
    // layout inside the array: arrival counters [rows] | partial rows [rows][splits][G][128] | (m, l) [rows][splits][G]
    const size_t rows = (size_t)batch * ctx->geom.n_kv_heads;
    const size_t part_rows = sh.n_splits > 1 ? rows * sh.n_splits * ctx->geom.group : 0;
    const size_t acc_off = align_up(rows * sizeof(int32_t), 256);
    const size_t ml_off = align_up(acc_off + part_rows * kHeadDim * sizeof(float), 256);
    const size_t need = ml_off + part_rows * 2 * sizeof(float);
    if (need > (size_t)CHESS_STATIC_SCRATCH_BYTES) return CHESS_ESCRATCH;
    char* base = static_cast<char*>(ctx->static_scratch);
    hipStream_t s = static_cast<hipStream_t>(stream);
    // whatever the previous call on this GPU left where the counters are (another context's partials, say) goes
    // first: a small fill kernel, not a memset node, so that the call can be captured in a graph
    hipError_t e = chess::launch_zero(ctx, reinterpret_cast<int32_t*>(base), rows, s);
    if (e != hipSuccess) return CHESS_EHIP;
    e = chess::launch_decode(ctx, static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k_pool),
                             static_cast<const uint16_t*>(v_pool), block_table, seq_lens, page_ids, n_selected, batch,
                             sh.n_splits, sh.waves, out, reinterpret_cast<float*>(base + acc_off),
                             reinterpret_cast<float*>(base + ml_off), reinterpret_cast<int32_t*>(base), s);
    return e == hipSuccess ? CHESS_OK : CHESS_EHIP;
}

int chess_dense_decode(chess_ctx* ctx, const void* q, const void* k_pool, const void* v_pool,
                       const int32_t* block_table, const int32_t* seq_lens, int32_t batch, float* out,
                       void* workspace, void* stream)
{
    return decode_common(ctx, q, k_pool, v_pool, block_table, seq_lens, nullptr, nullptr, batch, out, workspace, stream);
}

int chess_debug_force_splits(chess_ctx* ctx, int32_t n_splits, int32_t waves)
{
    if (!ctx || n_splits < 0 || n_splits > ctx->max_splits || (waves != 1 && waves != 4)) return CHESS_EINVAL;
    if (n_splits * ctx->geom.group > 1024) return CHESS_EINVAL;
    const int64_t rows = (int64_t)ctx->cfg.max_batch * ctx->geom.n_kv_heads;
    if (rows * n_splits > 4LL * ctx->n_cu + rows) return CHESS_EINVAL;
    ctx->force_splits = n_splits;
    ctx->force_waves = waves;
    return CHESS_OK;
}

const char* chess_strerror(int code)
{
    switch (code) {
    case CHESS_OK: return "ok";
    case CHESS_EINVAL: return "invalid argument (null pointer, misaligned buffer, or shape outside the configuration)";
    case CHESS_ENOTSUP: return "not supported (a selection level would have more candidates than fit in LDS)";
    case CHESS_EHIP: return "HIP runtime error at kernel launch";
    case CHESS_ENOMEM: return "out of host memory";
    case CHESS_ESCRATCH: return "the call needs more device scratch than chess_sparse_decode_static owns (CHESS_STATIC_SCRATCH_BYTES)";
    default: return "unknown error code";
    }
}

int chess_version(void) { return 1; }

}  // extern "C"
