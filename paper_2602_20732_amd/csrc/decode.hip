// Paged decode attention over a list of pages read in place (sparse: the selected page ids; dense: every
// page), split-K with an online-softmax merge; the arithmetic is in decode_device.h.
#include "decode_device.h"

namespace chess {

// Three workgroups of four waves per compute unit (at most 170 registers a lane): see run_tiles_with, kSingle.
template <int B, int NW, bool kList>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(3))) void decode_kernel(const uint16_t* __restrict__ q,
                                                         const uint16_t* __restrict__ k_pool,
                                                         const uint16_t* __restrict__ v_pool,
                                                         const int32_t* __restrict__ block_table,
                                                         const int32_t* __restrict__ seq_lens,
                                                         const int32_t* __restrict__ page_ids,
                                                         const int32_t* __restrict__ n_selected, Geom g,
                                                         float scale_log2, int n_splits, float* __restrict__ out,
                                                         float* __restrict__ ws_acc, float* __restrict__ ws_ml,
                                                         int32_t* __restrict__ arrivals
                                                         )
{
    constexpr int PPT = 32 / B;
    extern __shared__ float lds_f[];                  // DecodeLds<NW>::floats(G)
    __shared__ int lds_last;
    DecodeLds<NW> lds(lds_f, g.group);

    const int split = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m16 = lane & 15, grp = lane >> 4;
    const int G = g.group, H = g.n_kv_heads;
    const size_t row = (size_t)b * H + h;
    const int32_t* ids = kList ? page_ids + row * g.max_sel : nullptr;
    const int32_t* bt_row = block_table + (size_t)b * g.max_pages;
    // tiles are dealt round-robin: tile = split + n_splits * (wave + NW * i), so the first tile of a wave
    // is known before the list length is, and its page numbers can be fetched alongside the lengths
    const int stride = n_splits * NW;
    const int t = split + n_splits * wave;
    int raw_cur[PPT], raw_nxt[PPT];
    const int L_raw = seq_lens[b];
    const int n_raw = kList ? n_selected[row] : 0;
    fetch_ids<B, kList>(raw_cur, t, ids, g.max_sel);
    fetch_ids<B, kList>(raw_nxt, t + stride, ids, g.max_sel);
    const int L = min(max(L_raw, 0), g.max_pages * B);
    const int P = (L + B - 1) / B;
    const int n_pages = P == 0 ? 0 : (kList ? min(max(n_raw, 0), g.max_sel) : P);
    const int n_tiles = (n_pages + PPT - 1) / PPT;

    WaveAcc<B> acc;
    acc.init(q + ((size_t)b * g.n_q_heads + (size_t)h * G) * kHeadDim, G, m16, grp);
    NewToken<B> none;
    none.tile = -1;
    run_tiles_with<B, kList, false, false, true>(acc, t, stride, n_tiles, n_pages, raw_cur, raw_nxt, ids, g.max_sel, bt_row, nullptr,
                                                 k_pool, v_pool, H, h, L, P, scale_log2, m16, grp, none, 1 << 30);

    float* out_rows = out + ((size_t)b * g.n_q_heads + (size_t)h * G) * kHeadDim;
    if (!combine_waves<NW>(acc.o, acc.m_run, acc.l_run, lds, G, n_splits, split, row, out_rows, ws_acc, ws_ml)) return;
    if (!arrive_last(arrivals + row, n_splits, &lds_last)) return;
    merge_splits<NW>(G, n_splits, row, out_rows, ws_acc, ws_ml);
}

// The step between reselections (Sec. 3.3) in one launch: attention over the kept list for the sequence WITH the
// token that is being appended, whose key / value rows are not in the pools yet.  Every split takes them from
// k_new / v_new straight into the operands of the tile that holds the tail page; the last split of a (sequence,
// KV head) to finish -- after which nobody reads the tail page or the list any more -- writes the rows to the pools
// and, when the token opens a new page, the page to the list.  The lists must end with the tail page of seq_lens
// (as a selection on these lengths, chess_append_kv with the lists, or this call leave them).
// grid = (n_splits, H_kv, batch), four waves.
// kSingle: one tile in registers at a time; faster while a wave has only a few tiles (the host decides).
// Two workgroups per compute unit either way (squeezed into the registers of three, the kernel was slower).
template <int B, bool kSingle>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void reuse_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k_new,
                                                    const uint16_t* __restrict__ v_new, uint16_t* __restrict__ k_pool,
                                                    uint16_t* __restrict__ v_pool, const int32_t* __restrict__ block_table,
                                                    const int32_t* __restrict__ seq_lens, int32_t* __restrict__ page_ids,
                                                    int32_t* __restrict__ n_selected, Geom g, float scale_log2, int n_splits,
                                                    float* __restrict__ out, float* __restrict__ ws_acc,
                                                    float* __restrict__ ws_ml, int32_t* __restrict__ arrivals)
{
    constexpr int PPT = 32 / B, NW = 4;
    extern __shared__ float lds_f[];
    __shared__ int lds_last;
    DecodeLds<NW> lds(lds_f, g.group);

    const int split = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m16 = lane & 15, grp = lane >> 4;
    const int G = g.group, H = g.n_kv_heads;
    const size_t row = (size_t)b * H + h;
    int32_t* ids = page_ids + row * g.max_sel;
    const int32_t* bt_row = block_table + (size_t)b * g.max_pages;
    const int stride = n_splits * NW;
    const int t = split + n_splits * wave;
    int raw_cur[PPT], raw_nxt[PPT];
    const int L_before = seq_lens[b];
    const int n_raw = n_selected[row];
    fetch_ids<B, true>(raw_cur, t, ids, g.max_sel);
    fetch_ids<B, true>(raw_nxt, t + stride, ids, g.max_sel);
    NewToken<B> nt;
    nt.k_row = k_new + row * kHeadDim;
    nt.v_row = v_new + row * kHeadDim;

    const bool room = L_before >= 0 && L_before < g.max_pages * B;
    const int L = room ? L_before + 1 : min(max(L_before, 0), g.max_pages * B);
    const int P = (L + B - 1) / B;
    const int n_stored = min(max(n_raw, 0), g.max_sel);
    const bool grow = room && L_before % B == 0 && n_stored < g.max_sel;     // the token opens a page
    const int n_pages = P == 0 ? 0 : n_stored + (grow ? 1 : 0);
    const int n_tiles = (n_pages + PPT - 1) / PPT;
    // the tail page is the list's last entry -- unless the token opens a page and the row has no room for it: then
    // (and in the steps after: run_tiles_with looks at the entry) the token is stored but not attended, as with
    // chess_append_kv + chess_sparse_decode
    nt.tile = room && n_pages > 0 && (grow || L_before % B != 0) ? (n_pages - 1) / PPT : -1;
    nt.T = ((n_pages - 1) % PPT) * B + L_before % B;

    WaveAcc<B> acc;
    acc.init(q + ((size_t)b * g.n_q_heads + (size_t)h * G) * kHeadDim, G, m16, grp);
    run_tiles_with<B, true, false, true, kSingle>(acc, t, stride, n_tiles, n_pages, raw_cur, raw_nxt, ids, g.max_sel, bt_row, nullptr, k_pool,
                                         v_pool, H, h, L, P, scale_log2, m16, grp, nt, n_stored);

    float* out_rows = out + ((size_t)b * g.n_q_heads + (size_t)h * G) * kHeadDim;
    const bool split_up = combine_waves<NW>(acc.o, acc.m_run, acc.l_run, lds, G, n_splits, split, row, out_rows, ws_acc, ws_ml);
    if (split_up && !arrive_last(arrivals + row, n_splits, &lds_last)) return;
    // every split of the row is past its reads: the token and the page go where the next step looks for them
    if (room) {
        const int tid = threadIdx.x;
        if (tid < kHeadDim) {
            const int64_t phys = bt_row[L_before / B];
            const size_t blk = ((size_t)phys * H + h) * B * kHeadDim;
            const int tok = L_before % B;
            k_pool[blk + (size_t)tok * kHeadDim + tid] = k_new[row * kHeadDim + tid];
            v_pool[blk + (size_t)tid * B + tok] = v_new[row * kHeadDim + tid];
        }
        if (grow && tid == 0) {
            ids[n_stored] = P - 1;
            n_selected[row] = n_stored + 1;
        }
    }
    if (split_up) merge_splits<NW>(G, n_splits, row, out_rows, ws_acc, ws_ml);
}

hipError_t launch_reuse(chess_ctx* ctx, const uint16_t* q, const uint16_t* k_new, const uint16_t* v_new, uint16_t* k_pool,
                        uint16_t* v_pool, const int32_t* block_table, const int32_t* seq_lens, int32_t* page_ids,
                        int32_t* n_selected, int batch, int n_splits, float* out, float* ws_acc, float* ws_ml,
                        int32_t* arrivals, hipStream_t stream)
{
    const Geom& g = ctx->geom;
    const float scale_log2 = ctx->sm_scale * 1.4426950408889634f;
    const dim3 grid(n_splits, g.n_kv_heads, batch), block(256);
    const size_t lds = (size_t)(4 * g.group * kHeadDim + 2 * 4 * g.group) * sizeof(float);
    // without the prefetch of the next tile while a wave has at most four tiles of the longest possible list
    const int tiles = (g.max_sel + kTileTokens / g.page_size - 1) / (kTileTokens / g.page_size);
    const bool single = tiles <= 4 * 4 * n_splits;
    auto kern = g.page_size == 16 ? (single ? reuse_kernel<16, true> : reuse_kernel<16, false>)
                                  : (single ? reuse_kernel<32, true> : reuse_kernel<32, false>);
    return launch(kern, grid, block, lds, stream, q, k_new, v_new, k_pool, v_pool, block_table, seq_lens, page_ids, n_selected,
                  g, scale_log2, n_splits, out, ws_acc, ws_ml, arrivals);
}

hipError_t launch_decode(chess_ctx* ctx, const uint16_t* q, const uint16_t* k_pool, const uint16_t* v_pool,
                         const int32_t* block_table, const int32_t* seq_lens, const int32_t* page_ids,
                         const int32_t* n_selected, int batch, int n_splits, int waves, float* out,
                         float* ws_acc, float* ws_ml, int32_t* arrivals, hipStream_t stream)
{
    const Geom& g = ctx->geom;
    const float scale_log2 = ctx->sm_scale * 1.4426950408889634f;
    const dim3 grid(n_splits, g.n_kv_heads, batch), block(64 * waves);
    const size_t lds = (size_t)(waves * g.group * kHeadDim + 2 * waves * g.group) * sizeof(float);
    using Kern = void (*)(const uint16_t*, const uint16_t*, const uint16_t*, const int32_t*, const int32_t*, const int32_t*,
                          const int32_t*, Geom, float, int, float*, float*, float*, int32_t*);
    // [page size 16 / 32][waves 4 / 1][list / every page]
    static const Kern table[2][2][2] = {
        {{decode_kernel<16, 4, true>, decode_kernel<16, 4, false>}, {decode_kernel<16, 1, true>, decode_kernel<16, 1, false>}},
        {{decode_kernel<32, 4, true>, decode_kernel<32, 4, false>}, {decode_kernel<32, 1, true>, decode_kernel<32, 1, false>}}};
    const Kern kern = table[g.page_size == 16 ? 0 : 1][waves == 4 ? 0 : 1][page_ids ? 0 : 1];
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    return launch(kern, grid, block, lds, stream, q, k_pool, v_pool, block_table, seq_lens,
                  page_ids, n_selected, g, scale_log2, n_splits, out, ws_acc, ws_ml, arrivals);
}

hipError_t decode_occupancy(int page_size, int waves, int group, int* blocks_per_cu)
{
    // (the list variant: it is the one whose split count depends on what fits)
    const size_t lds = (size_t)(waves * group * kHeadDim + 2 * waves * group) * sizeof(float);
    if (page_size == 16)
        return waves == 4 ? hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, decode_kernel<16, 4, true>, 256, lds)
                          : hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, decode_kernel<16, 1, true>, 64, lds);
    return waves == 4 ? hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, decode_kernel<32, 4, true>, 256, lds)
                      : hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, decode_kernel<32, 1, true>, 64, lds);
}

// One new token per sequence into the paged pools: K row-major [phys][H][B][128], V token-minor [phys][H][128][B].
// grid = batch * H_kv workgroups of 128 threads, thread = dim.
__global__ __launch_bounds__(kHeadDim) void append_kernel(const uint16_t* __restrict__ k_new, const uint16_t* __restrict__ v_new,
                                                          uint16_t* __restrict__ k_pool, uint16_t* __restrict__ v_pool,
                                                          const int32_t* __restrict__ block_table,
                                                          const int32_t* __restrict__ seq_lens, Geom g,
                                                          int32_t* __restrict__ page_ids, int32_t* __restrict__ n_selected)
{
    const int row = blockIdx.x, b = row / g.n_kv_heads, h = row - b * g.n_kv_heads, dim = threadIdx.x;
    const int L = seq_lens[b], B = g.page_size;
    if (L < 0 || L >= g.max_pages * B) return;        // no room: the sequence is left as it is
    if (page_ids != nullptr && dim == 0) {            // the row's list follows the tail (what extend_kernel does)
        const int P = L / B + 1;                      // pages once the token is in
        int32_t* ids = page_ids + (size_t)row * g.max_sel;
        int n = min(max(n_selected[row], 0), g.max_sel);
        int last = n > 0 ? ids[n - 1] : -1;
        while (last < P - 1 && n < g.max_sel) ids[n++] = ++last;
        n_selected[row] = n;
    }
    const int64_t phys = block_table[(size_t)b * g.max_pages + L / B];
    const int t = L % B;
    const size_t blk = ((size_t)phys * g.n_kv_heads + h) * B * kHeadDim;
    k_pool[blk + (size_t)t * kHeadDim + dim] = k_new[(size_t)row * kHeadDim + dim];
    v_pool[blk + (size_t)dim * B + t] = v_new[(size_t)row * kHeadDim + dim];
}

hipError_t launch_append(chess_ctx* ctx, const uint16_t* k_new, const uint16_t* v_new, uint16_t* k_pool, uint16_t* v_pool,
                         const int32_t* block_table, const int32_t* seq_lens, int batch, int32_t* page_ids,
                         int32_t* n_selected, hipStream_t stream)
{
    return launch(append_kernel, dim3(batch * ctx->geom.n_kv_heads), dim3(kHeadDim), 0, stream, k_new, v_new, k_pool, v_pool,
                  block_table, seq_lens, ctx->geom, page_ids, n_selected);
}

// Between reselections the recent window follows the tail: every list is extended by the pages after its last
// entry, up to the sequence's current last page (as far as the row has room).  One thread per (sequence, KV head).
__global__ void extend_kernel(const int32_t* __restrict__ seq_lens, int rows, Geom g, int32_t* __restrict__ page_ids,
                              int32_t* __restrict__ n_selected)
{
    const int row = blockIdx.x * blockDim.x + threadIdx.x;
    if (row >= rows) return;
    const int L = min(max(seq_lens[row / g.n_kv_heads], 0), g.max_pages * g.page_size);
    const int P = (L + g.page_size - 1) / g.page_size;
    int32_t* ids = page_ids + (size_t)row * g.max_sel;
    int n = min(max(n_selected[row], 0), g.max_sel);
    int last = n > 0 ? ids[n - 1] : -1;
    while (last < P - 1 && n < g.max_sel) ids[n++] = ++last;
    n_selected[row] = n;
}

hipError_t launch_extend(chess_ctx* ctx, const int32_t* seq_lens, int batch, int32_t* page_ids, int32_t* n_selected,
                         hipStream_t stream)
{
    const int rows = batch * ctx->geom.n_kv_heads;
    return launch(extend_kernel, dim3((rows + 63) / 64), dim3(64), 0, stream, seq_lens, rows, ctx->geom, page_ids, n_selected);
}

__global__ void zero_kernel(int32_t* p, size_t n)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

hipError_t launch_zero(chess_ctx* ctx, int32_t* p, size_t n_words, hipStream_t stream)
{
    (void)ctx;
    hipLaunchKernelGGL(zero_kernel, dim3((unsigned)((n_words + 255) / 256)), dim3(256), 0, stream, p, n_words);
    return hipGetLastError();
}

}  // namespace chess
