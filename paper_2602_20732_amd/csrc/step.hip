// The whole decode step of one layer in one launch: coarse-to-fine page selection (Sec. 3.2, Alg. 1 stage 2)
// followed at once by block-sparse attention over the selected pages, read in place (Sec. 4.3, App. B).
//
// A cluster of C workgroups per (sequence, KV head) runs the three selection levels (select_device.h); every
// member ends up with the same page list in its LDS, so the list never travels through memory: member m
// goes straight on to decode tiles m, m + C, ... of it (decode_device.h) as split m of C, and the last
// member to finish merges the C partials.  Compared with chess_select + chess_sparse_decode this saves a
// kernel boundary, the round trip of the list through HBM and the second kernel's start-up loads.
// Member 0 also writes the list to page_ids / n_selected when the caller wants it.
#include "decode_device.h"
#include "select_device.h"

namespace chess {

static_assert(kSelThreads % kWave == 0 && kSelThreads >= 256, "the fused step decodes with every wave of the workgroup");
constexpr int kStepWaves = kSelThreads / kWave;

struct StepArgs {
    const uint16_t* q;
    void* pages;             // summaries (fp32 or bf16): read; the tail units are rewritten when refresh_tail is set
    void* chunks;
    void* grids;
    const uint16_t* k_pool;
    const uint16_t* v_pool;
    const int32_t* block_table;
    const int32_t* seq_lens;
    int32_t* page_ids;       // may be null
    int32_t* n_selected;     // may be null
    float* out;
    float* ws_acc;
    float* ws_ml;
    int32_t* arrivals;
    float scale_log2;
    int32_t union_off;       // byte offset of the LDS region selection and decode share (after the page list)
    int32_t refresh_tail;    // recompute the summaries of the tail page, its chunk and its grid first
};

// The per-step refresh of the summaries (Sec. 3.1, Eq. 1-2) of the tail page, its chunk and its grid, done by one
// workgroup per (sequence, KV head) inside the step: thread c < 128 owns column c and adds in the same order as
// the summarize kernel (tokens, then the chunk's pages, then the grid's chunks, ascending, fp64, one rounding to
// the storage type per vector; a parent averages its children as they are stored), so the vectors are the ones
// chess_summarize_tail writes.  They go to the summaries and to `fresh` (LDS, [3][128]: page, chunk, grid); their
// scores against the probe are published as keys in tail_words[0..2] (grid, chunk, page) when `publish` is set (a
// cluster of one has nobody to tell) and kept in sh.tail_key.  Every thread of the workgroup must call it.
template <int B, class T>
__device__ __forceinline__ void refresh_tail_units(const uint16_t* __restrict__ k_pool, int64_t phys, T* pages_row,
                                                   T* chunks_row, T* grids_row, int h, int H, int L, int P,
                                                   const Geom& g, const double (&pr)[8], T* fresh,
                                                   uint64_t* tail_words, bool publish, Shared& sh)
{
    const int tid = threadIdx.x;
    const int tp = P - 1, tc = div_by(tp, g.n_c, g.inv_nc), tg = div_by(tc, g.n_g, g.inv_ng);
    const int n_tok = L - tp * B;
    if (tid < kHeadDim) {
        const int c = tid;
        // the page's key rows, all requested at once (rows past the last token repeat it and are not added)
        const uint16_t* rows = k_pool + ((phys * H + h) * B) * kHeadDim + c;
        uint16_t kr[B];
#pragma unroll
        for (int t = 0; t < B; ++t) kr[t] = rows[(size_t)min(t, n_tok - 1) * kHeadDim];
        // the other pages of the chunk and the other chunks of the grid (the tail unit is the last child of each),
        // eight at a time and the first eight of each together with the key rows: one round trip for the usual
        // hierarchy of 8 x 8
        constexpr int kSib = 8;
        const int p_lo = tc * g.n_c, c_lo = tg * g.n_g;
        T sp[kSib], sc[kSib];
#pragma unroll
        for (int x = 0; x < kSib; ++x) {
            sp[x] = pages_row[(size_t)min(p_lo + x, tp) * kHeadDim + c];
            sc[x] = chunks_row[(size_t)min(c_lo + x, tc) * kHeadDim + c];
        }
        double acc_c = 0.0, acc_g = 0.0;
#pragma unroll
        for (int x = 0; x < kSib; ++x) {
            if (p_lo + x < tp) acc_c += loaded(sp[x]);
            if (c_lo + x < tc) acc_g += loaded(sc[x]);
        }
        for (int j0 = p_lo + kSib; j0 < tp; j0 += kSib) {
#pragma unroll
            for (int x = 0; x < kSib; ++x) sp[x] = pages_row[(size_t)min(j0 + x, tp) * kHeadDim + c];
#pragma unroll
            for (int x = 0; x < kSib; ++x)
                if (j0 + x < tp) acc_c += loaded(sp[x]);
        }
        for (int j0 = c_lo + kSib; j0 < tc; j0 += kSib) {
#pragma unroll
            for (int x = 0; x < kSib; ++x) sc[x] = chunks_row[(size_t)min(j0 + x, tc) * kHeadDim + c];
#pragma unroll
            for (int x = 0; x < kSib; ++x)
                if (j0 + x < tc) acc_g += loaded(sc[x]);
        }
        double acc_p = 0.0;
#pragma unroll
        for (int t = 0; t < B; ++t)
            if (t < n_tok) acc_p += loaded(kr[t]);
        const T vp = stored<T>(acc_p / (double)n_tok);
        const T vc = stored<T>((acc_c + loaded(vp)) / (double)(tp - tc * g.n_c + 1));
        const T vg = stored<T>((acc_g + loaded(vc)) / (double)(tc - tg * g.n_g + 1));
        pages_row[(size_t)tp * kHeadDim + c] = vp;
        chunks_row[(size_t)tc * kHeadDim + c] = vc;
        grids_row[(size_t)tg * kHeadDim + c] = vg;
        fresh[c] = vp;
        fresh[kHeadDim + c] = vc;
        fresh[2 * kHeadDim + c] = vg;
    }
    __syncthreads();
    // scores of the three vectors, one 16-lane group each, with the arithmetic of score_rows
    const int g16 = tid >> 4, ln = tid & 15;
    if (g16 < 3) {
        Vec<T> v;
        v.load(fresh + g16 * kHeadDim, ln);
        const double d = row16_sum(dot8<T>(pr, v));
        if (ln == 15) {
            const uint64_t key = order_key(d);
            const int level = 2 - g16;                            // fresh[0] is the page, fresh[2] the grid
            if (publish) publish_u64(tail_words + level, key);
            sh.tail_key[level] = key;
        }
    }
    __syncthreads();
}

// grid = (C, H_kv, batch); T = storage type of the summaries (float or bf16 bits)
template <int B, class T>
__global__ __launch_bounds__(kSelThreads) __attribute__((amdgpu_waves_per_eu(2))) void step_kernel(StepArgs a, Geom g, SelectParams sp, SelectWs ws)
{
    constexpr int PPT = 32 / B;
    extern __shared__ unsigned long long lds_raw[];
    int32_t* ids_l = reinterpret_cast<int32_t*>(lds_raw);                                  // [max_sel] the page list
    int32_t* phys_l = ids_l + g.max_sel;                                                   // [max_sel] their physical pages
    T* fresh = reinterpret_cast<T*>(reinterpret_cast<char*>(lds_raw) + a.union_off - 3 * kHeadDim * sizeof(float));   // [3][128]
    char* un = reinterpret_cast<char*>(lds_raw) + a.union_off;
    uint64_t* keys = reinterpret_cast<uint64_t*>(un);                                      // selection's view
    int32_t* kept_grids = reinterpret_cast<int32_t*>(keys + sp.cap_keys);
    int32_t* kept_chunks = kept_grids + sp.cap_kg;
    int32_t* phys_by_slot = kept_chunks + sp.cap_kc;                                       // [cap3]
    DecodeLds<kStepWaves> dl(reinterpret_cast<float*>(un));                                // decode's view
    __shared__ Shared sh;

    const int m = blockIdx.x, C = gridDim.x, h = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6, m16 = lane & 15, grp = lane >> 4;
    const int G = g.group, H = g.n_kv_heads;
    Prof prof;
    prof.mark(0);
    const size_t row = (size_t)b * H + h;
    const uint16_t* q_rows = a.q + ((size_t)b * g.n_q_heads + (size_t)h * G) * kHeadDim;
    float* out_rows = a.out + ((size_t)b * g.n_q_heads + (size_t)h * G) * kHeadDim;
    const int L_raw = a.seq_lens[b];
    const int k_fixed = fixed_budget(sp, g, b);
    double pr[8];
    if (sp.probe == CHESS_PROBE_QUERY) load_probe<T>(q_rows, G, pr);  // requested before anything waits on the length
    init_shared(sh, sp.poll_limit);
    const int L = min(max(L_raw, 0), g.max_pages * B);
    const int P = (L + B - 1) / B;
    const int s = sp.sink, w = sp.window;
    const int32_t* bt_row = a.block_table + (size_t)b * g.max_pages;
    if (P == 0) {                                                     // empty sequence: no pages, zero output
        if (m == 0) {
            if (a.page_ids) for (int i = tid; i < g.max_sel; i += kSelThreads) a.page_ids[row * g.max_sel + i] = -1;
            if (a.n_selected && tid == 0) a.n_selected[row] = 0;
            for (int i = tid; i < G * kHeadDim; i += kSelThreads) out_rows[i] = 0.f;
        }
        return;
    }
    T* pages_row = static_cast<T*>(a.pages) + row * g.max_pages * kHeadDim;
    T* chunks_row = static_cast<T*>(a.chunks) + row * g.max_chunks * kHeadDim;
    T* grids_row = static_cast<T*>(a.grids) + row * g.max_grids * kHeadDim;
    if (sp.probe == CHESS_PROBE_ANCHOR) load_anchor<T>(pages_row, P, w, pr);
    // member 0 refreshes the tail units: its block-table entry is requested now
    const bool tail_on = a.refresh_tail != 0;
    uint64_t* tail_words = tail_on ? ws.tail + row * 4 : nullptr;
    int tail_phys = 0;
    if (tail_on && m == 0) tail_phys = bt_row[P - 1];
    auto refresh_tail = [&]() {
        refresh_tail_units<B, T>(a.k_pool, tail_phys, pages_row, chunks_row, grids_row, h, H, L, P, g, pr, fresh, tail_words, C > 1, sh);
    };
    __syncthreads();
    prof.mark(1);                                                     // prologue done

        // ---- the page list, in every member's LDS
    const PubLayout pubs = pub_layout(ws.keys + row * ws.key_stride, g);
    CascadeResult res;
    res.n_kp = 0; res.n_a = 0; res.n_p = 0; res.overflow = false;
    int n_sel;
    if (P <= s + w) {                                                 // safety pages cover the sequence
        n_sel = min(P, g.max_sel);
        for (int i = tid; i < n_sel; i += kSelThreads) { ids_l[i] = i; phys_l[i] = bt_row[i]; }
        if (tail_on && m == 0) refresh_tail();                        // nobody reads the keys; the summaries are kept current
    } else {
        // the block-table entries of the safety pages are requested now and used after the selection
        const bool safety_early = s + w <= kSelThreads;
        const int safety_lp = tid < s ? tid : P - w + (tid - s);
        int safety_phys = 0;
        if (safety_early && tid < s + w) safety_phys = bt_row[safety_lp];
        // kept pages and their physical pages go straight to their places in the list, behind the sinks
        const bool ok = cascade<true, T>(pages_row, chunks_row, grids_row, pr, P, g, sp, pubs, m, C, true, keys, kept_grids,
                                         kept_chunks, ids_l + s, sh, &res, prof, tail_words, refresh_tail, k_fixed, bt_row,
                                         phys_by_slot, phys_l + s);
        if (!ok) {
            if (tid == 0) __hip_atomic_fetch_or(ws.error, kErrWait, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return;
        }
        if (res.overflow && m == 0 && tid == 0) __hip_atomic_fetch_or(ws.error, kErrOverflow, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // union with the safety pages: sinks, kept pages, window -- already ascending
        const int n_kp = res.n_kp;
        n_sel = s + n_kp + w;
        if (safety_early) {
            if (tid < s + w) {
                const int at = tid < s ? tid : n_kp + tid;
                ids_l[at] = safety_lp;
                phys_l[at] = safety_phys;
            }
        } else {
            for (int i = tid; i < s + w; i += kSelThreads) {
                const int lp = i < s ? i : P - w + (i - s), at = i < s ? i : n_kp + i;
                ids_l[at] = lp;
                phys_l[at] = bt_row[lp];
            }
        }
    }
    __syncthreads();
    if (m == 0) {
        if (a.page_ids) for (int i = tid; i < g.max_sel; i += kSelThreads) a.page_ids[row * g.max_sel + i] = i < n_sel ? ids_l[i] : -1;
        if (a.n_selected && tid == 0) a.n_selected[row] = n_sel;
    }
    prof.mark(14);                                                    // list built

    // ---- attention over this member's tiles of the list: split m of C
    const int n_tiles = (n_sel + PPT - 1) / PPT;
    const int stride = C * kStepWaves;
    const int t = m + C * wave;
    int raw_cur[PPT], raw_nxt[PPT];
    fetch_ids<B, true>(raw_cur, t, ids_l, max(n_sel, 1));
    fetch_ids<B, true>(raw_nxt, t + stride, ids_l, max(n_sel, 1));
    WaveAcc<B> acc;
    acc.init(q_rows, G, m16, grp);
    run_tiles<B, true, true>(acc, t, stride, n_tiles, n_sel, raw_cur, raw_nxt, ids_l, max(n_sel, 1), bt_row, phys_l, a.k_pool, a.v_pool, H, h, L, P,
                 a.scale_log2, m16, grp);
    prof.mark(15);                                                    // tiles done
    if (!combine_waves<kStepWaves>(acc.o, acc.m_run, acc.l_run, dl, G, C, m, row, out_rows, a.ws_acc, a.ws_ml)) return;
    prof.mark(16);                                                    // partial published
    // (profiling builds keep two timelines per row: member 0's and that of the member that merges)
    if (!arrive_last(a.arrivals + row, C, &sh.flag)) {
#ifdef CHESS_PROF
        prof.mark(17);
        if (tid == 0 && m == 0) prof.store(ws.prof + (row * 2) * Prof::kSlots);
#endif
        return;
    }
    prof.mark(17);                                                    // last to arrive
    merge_splits<kStepWaves>(G, C, row, out_rows, a.ws_acc, a.ws_ml);
    if (C > 1) clear_published(pubs, res, tail_words);                    // every member is done with the key words
#ifdef CHESS_PROF
    prof.mark(18);
    if (tid == 0) prof.store(ws.prof + (row * 2 + 1) * Prof::kSlots);
    if (tid == 0 && m == 0) prof.store(ws.prof + (row * 2) * Prof::kSlots);
#endif
}

using StepKernel = void (*)(StepArgs, Geom, SelectParams, SelectWs);
static StepKernel step_kernel_of(int page_size, bool bf16)
{
    if (bf16) return page_size == 16 ? step_kernel<16, uint16_t> : step_kernel<32, uint16_t>;
    return page_size == 16 ? step_kernel<16, float> : step_kernel<32, float>;
}

// Dynamic LDS of the fused kernel and where its shared region starts.
size_t step_lds_bytes(const SelectParams& sp, int max_sel, int* union_off)
{
    const size_t list = ((size_t)max_sel * 2 * 4 + 15) / 16 * 16 + 3 * kHeadDim * sizeof(float);   // page list, physical pages, refreshed tail vectors
    const size_t sel = (size_t)sp.cap_keys * 8 + ((size_t)(sp.cap_kg + sp.cap_kc + sp.cap3) * 4 + 7) / 8 * 8;
    const size_t dec = (size_t)DecodeLds<kStepWaves>::kFloats * sizeof(float);
    *union_off = (int)list;
    return list + (sel > dec ? sel : dec);
}

hipError_t step_occupancy(int page_size, bool bf16, int lds_bytes, int* blocks_per_cu)
{
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(step_kernel_of(page_size, bf16)),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (e != hipSuccess) return e;
    return hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, step_kernel_of(page_size, bf16), kSelThreads, lds_bytes);
}

hipError_t launch_step(chess_ctx* ctx, const StepLaunch& sl, int batch, int cluster, const SelectParams& sp,
                       const SelectWs& ws, size_t lds_bytes, int union_off, hipStream_t stream)
{
    const Geom& g = ctx->geom;
    StepArgs a;
    a.q = sl.q; a.pages = sl.pages; a.chunks = sl.chunks; a.grids = sl.grids; a.k_pool = sl.k_pool; a.v_pool = sl.v_pool;
    a.block_table = sl.block_table; a.seq_lens = sl.seq_lens; a.page_ids = sl.page_ids; a.n_selected = sl.n_selected;
    a.out = sl.out; a.ws_acc = sl.ws_acc; a.ws_ml = sl.ws_ml; a.arrivals = sl.arrivals;
    a.scale_log2 = ctx->sm_scale * 1.4426950408889634f;
    a.union_off = union_off;
    a.refresh_tail = sl.refresh_tail;
    const dim3 grid(cluster, g.n_kv_heads, batch), block(kSelThreads);
    return launch(step_kernel_of(g.page_size, ctx->cfg.summary_dtype == CHESS_SUMMARY_BF16), grid, block, lds_bytes, stream, a, g, sp, ws);
}

}  // namespace chess
