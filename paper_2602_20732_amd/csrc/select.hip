// Coarse-to-fine page selection (Sec. 3.2, Eq. 4, Alg. 1 stage 2) as a call of its own: one launch, a
// cluster of C workgroups per (sequence, KV head); the levels themselves are in select_device.h.
// Member 0 of a cluster writes the list: sink pages, kept pages, window pages.
#include "select_device.h"

namespace chess {

// grid = (C, H_kv, batch); T = storage type of the summaries (float or bf16 bits)
template <class T>
__global__ __launch_bounds__(kSelThreads) void select_kernel(const uint16_t* __restrict__ q,
                                                             const T* __restrict__ pages,
                                                             const T* __restrict__ chunks,
                                                             const T* __restrict__ grids,
                                                             const int32_t* __restrict__ seq_lens, Geom g,
                                                             SelectParams sp, SelectWs ws,
                                                             int32_t* __restrict__ page_ids,
                                                             int32_t* __restrict__ n_selected)
{
    extern __shared__ unsigned long long lds_raw[];
    uint64_t* keys = reinterpret_cast<uint64_t*>(lds_raw);                    // [cap_keys]
    int32_t* kept_grids = reinterpret_cast<int32_t*>(keys + sp.cap_keys);     // [cap_kg]
    int32_t* kept_chunks = kept_grids + sp.cap_kg;                            // [cap_kc]
    int32_t* sel_pages = kept_chunks + sp.cap_kc;                             // [max_sel]
    __shared__ Shared sh;

    const int m = blockIdx.x, C = gridDim.x, h = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
    Prof prof;
    prof.mark(0);
    const size_t row = (size_t)b * g.n_kv_heads + h;
    int32_t* ids = page_ids + row * g.max_sel;
    const int B = g.page_size;
    const int L_raw = seq_lens[b];
    const int k_fixed = fixed_budget(sp, g, b);
    double pr[8];
    if (sp.probe == CHESS_PROBE_QUERY)                                // requested before anything waits on the length
        load_probe<T>(q + ((size_t)b * g.n_q_heads + (size_t)h * g.group) * kHeadDim, g.group, pr);
    init_shared(sh, sp.poll_limit);
    const int L = min(max(L_raw, 0), g.max_pages * B);
    const int P = (L + B - 1) / B;
    const int s = sp.sink, w = sp.window;
    if (P <= s + w) {                                                 // safety pages cover the sequence
        if (m == 0) {
            for (int i = tid; i < g.max_sel; i += kSelThreads) ids[i] = i < P ? i : -1;
            if (tid == 0) n_selected[row] = min(P, g.max_sel);
        }
        return;
    }
    if (sp.probe == CHESS_PROBE_ANCHOR) load_anchor<T>(pages + row * g.max_pages * kHeadDim, P, w, pr);
    __syncthreads();
    prof.mark(1);                                                     // prologue done

    const PubLayout pubs = pub_layout(ws.keys + row * ws.key_stride, g);
    CascadeResult res;
    const bool ok = cascade<false, T>(pages + row * g.max_pages * kHeadDim, chunks + row * g.max_chunks * kHeadDim,
                                      grids + row * g.max_grids * kHeadDim, pr, P, g, sp, pubs, m, C, m == 0, keys,
                                      kept_grids, kept_chunks, sel_pages, sh, &res, prof, nullptr, [] {}, k_fixed);
    if (!ok) {
        if (tid == 0) __hip_atomic_fetch_or(ws.error, kErrWait, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return;
    }
    if (C > 1) {
        // whoever is last to be done with the published words clears them for the next launch
        if (arrive_last(ws.meta + row * kSelMetaStride, C, &sh.flag)) clear_published(pubs, res);
    }
    if (m != 0) return;
    if (res.overflow && tid == 0) __hip_atomic_fetch_or(ws.error, kErrOverflow, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

    // ---- union with the safety pages: sinks, kept pages, window -- already ascending
    const int n_kp = res.n_kp, n_sel = s + n_kp + w;
    for (int i = tid; i < g.max_sel; i += kSelThreads) {
        int v = -1;
        if (i < s) v = i;
        else if (i < s + n_kp) v = sel_pages[i - s];
        else if (i < n_sel) v = P - w + (i - s - n_kp);
        ids[i] = v;
    }
    if (tid == 0) n_selected[row] = n_sel;
#ifdef CHESS_PROF
    prof.mark(15);
    if (tid == 0) prof.store(ws.prof + row * Prof::kSlots);
#endif
}

size_t select_lds_bytes(const SelectParams& sp, int max_sel)
{
    return (size_t)sp.cap_keys * 8 + ((size_t)(sp.cap_kg + sp.cap_kc + max_sel) * 4 + 7) / 8 * 8;
}

hipError_t select_occupancy(bool bf16, int lds_bytes, int* blocks_per_cu)
{
    const void* kern = bf16 ? reinterpret_cast<const void*>(select_kernel<uint16_t>) : reinterpret_cast<const void*>(select_kernel<float>);
    if (lds_bytes > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return e;
    }
    return bf16 ? hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, select_kernel<uint16_t>, kSelThreads, lds_bytes)
                : hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, select_kernel<float>, kSelThreads, lds_bytes);
}

hipError_t launch_select(chess_ctx* ctx, const uint16_t* q, const void* pages, const void* chunks,
                         const void* grids, const int32_t* seq_lens, int batch, int cluster, const SelectParams& sp,
                         const SelectWs& ws, size_t lds_bytes, int32_t* page_ids, int32_t* n_selected,
                         hipStream_t stream)
{
    const dim3 grid(cluster, ctx->geom.n_kv_heads, batch), block(kSelThreads);
    if (ctx->cfg.summary_dtype == CHESS_SUMMARY_BF16)
        return launch(select_kernel<uint16_t>, grid, block, lds_bytes, stream, q, static_cast<const uint16_t*>(pages),
                      static_cast<const uint16_t*>(chunks), static_cast<const uint16_t*>(grids), seq_lens, ctx->geom, sp, ws,
                      page_ids, n_selected);
    return launch(select_kernel<float>, grid, block, lds_bytes, stream, q, static_cast<const float*>(pages),
                  static_cast<const float*>(chunks), static_cast<const float*>(grids), seq_lens, ctx->geom, sp, ws, page_ids,
                  n_selected);
}

}  // namespace chess
