// The selection under the paper's own scope (Sec. 3.1, Eq. 1: a unit's vector is the concatenation, over all
// layers and heads, of the per-layer, per-head means) with the key anchor of Sec. 3.2, Eq. 3 as the probe:
// one score per unit, S(u) = sum over layers l and KV heads h of probe[l][h] . v[l][h][u] (Eq. 4 on the
// flattened vectors), one page set per sequence for the whole model.
//
// anchor_kernel: Eq. 3 for every (sequence, KV head) of one layer, as an output of its own.
// select_shared_kernel: a cluster of C workgroups per sequence runs the three levels of select_device.h; only the
// scoring differs.  A unit's vector is n_layers * H_kv rows of 512 bytes in as many arrays, so all 16 lane
// groups of a workgroup work on the same few slots: group j takes the rows r = j, j + 16, ... (row r = layer
// r / H_kv, head r % H_kv), eight slots at a time (eight vectors in flight per group and row), fp64 partial
// sums; the groups' partials are added in group order through LDS.  The order of the additions is fixed, so a
// unit's score does not depend on the launch shape.
#include "select_device.h"

namespace chess {

// grid = ceil(rows / 16), 256 threads: a 16-lane group per (sequence, KV head)
__global__ __launch_bounds__(256) void anchor_kernel(const float* __restrict__ pages, const int32_t* __restrict__ seq_lens,
                                                     int rows, Geom g, int window, float* __restrict__ anchor)
{
    const int row = blockIdx.x * 16 + (threadIdx.x >> 4), ln = threadIdx.x & 15;
    if (row >= rows) return;
    const int b = row / g.n_kv_heads;
    const int L = min(max(seq_lens[b], 0), g.max_pages * g.page_size);
    const int P = (L + g.page_size - 1) / g.page_size;
    double pr[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (P > 0) load_anchor(pages + (size_t)row * g.max_pages * kHeadDim, P, window, pr);
    float4* dst = reinterpret_cast<float4*>(anchor + (size_t)row * kHeadDim);
    dst[ln] = make_float4((float)pr[0], (float)pr[1], (float)pr[2], (float)pr[3]);
    dst[16 + ln] = make_float4((float)pr[4], (float)pr[5], (float)pr[6], (float)pr[7]);
}

hipError_t launch_anchor(chess_ctx* ctx, const float* pages, const int32_t* seq_lens, int batch, int window,
                         float* anchor, hipStream_t stream)
{
    const int rows = batch * ctx->geom.n_kv_heads;
    return launch(anchor_kernel, dim3((rows + 15) / 16), dim3(256), 0, stream, pages, seq_lens, rows, ctx->geom, window,
                  anchor);
}

constexpr int kSharedSlots = 8;                      // slots a workgroup scores together

struct SharedScorer {
    static constexpr int kShareRound = 1;
    const SharedTable& tab;
    int b;
    const Geom& g;
    double* red;                                     // LDS [16 groups][kSharedSlots]

    template <class Map>
    __device__ __forceinline__ void operator()(int level, int lo, int hi, Map unit_of, bool local, uint64_t* keys,
                                               uint64_t* pub) const
    {
        const int tid = threadIdx.x, g16 = tid >> 4, ln = tid & 15;
        const int H = g.n_kv_heads, R = tab.n_layers * H;
        const size_t level_off = level == 0 ? tab.grid_off : level == 1 ? tab.chunk_off : tab.page_off;
        const size_t units = level == 0 ? g.max_grids : level == 1 ? g.max_chunks : g.max_pages;
        for (int s0 = lo; s0 < hi; s0 += kSharedSlots) {
            int unit[kSharedSlots];
            double part[kSharedSlots];
#pragma unroll
            for (int x = 0; x < kSharedSlots; ++x) {
                unit[x] = s0 + x < hi ? unit_of(s0 + x) : -1;
                part[x] = 0.0;
            }
            for (int r = g16; r < R; r += kSelGroups) {
                const int l = r / H, h = r - l * H;
                const size_t row = (size_t)b * H + h;
                const float4* prow = reinterpret_cast<const float4*>(tab.probes[l] + row * kHeadDim);
                const float4 pa = prow[ln], pb = prow[16 + ln];
                const float* base = reinterpret_cast<const float*>(tab.summaries[l] + level_off) + row * units * kHeadDim;
                float4 va[kSharedSlots], vb[kSharedSlots];
#pragma unroll
                for (int x = 0; x < kSharedSlots; ++x) {
                    // always load (unit 0 when the slot has no unit): all eight stay in flight
                    const float4* p = reinterpret_cast<const float4*>(base + (size_t)max(unit[x], 0) * kHeadDim) + ln;
                    va[x] = p[0];
                    vb[x] = p[16];
                }
#pragma unroll
                for (int x = 0; x < kSharedSlots; ++x) {
                    double d = part[x];
                    d = fma((double)pa.x, (double)va[x].x, d); d = fma((double)pa.y, (double)va[x].y, d);
                    d = fma((double)pa.z, (double)va[x].z, d); d = fma((double)pa.w, (double)va[x].w, d);
                    d = fma((double)pb.x, (double)vb[x].x, d); d = fma((double)pb.y, (double)vb[x].y, d);
                    d = fma((double)pb.z, (double)vb[x].z, d); d = fma((double)pb.w, (double)vb[x].w, d);
                    part[x] = d;
                }
            }
#pragma unroll
            for (int x = 0; x < kSharedSlots; ++x) {
                const double d = row16_sum(part[x]);
                if (ln == 15) red[g16 * kSharedSlots + x] = d;
            }
            __syncthreads();
            if (tid < kSharedSlots && s0 + tid < hi) {
                double d = 0.0;
#pragma unroll
                for (int j = 0; j < kSelGroups; ++j) d += red[j * kSharedSlots + tid];
                const int u = unit_of(s0 + tid);
                if (local) keys[s0 + tid] = u >= 0 ? order_key(d) : 0ull;
                else publish_u64(pub + s0 + tid, u >= 0 ? order_key(d) : kAbsentKey);
            }
            __syncthreads();                          // red is reused by the next pass
        }
    }
};

// grid = (C, 1, batch)
__global__ __launch_bounds__(kSelThreads) void select_shared_kernel(SharedTable tab, const int32_t* __restrict__ seq_lens,
                                                                    Geom g, SelectParams sp, SelectWs ws,
                                                                    int32_t* __restrict__ page_ids,
                                                                    int32_t* __restrict__ n_selected)
{
    extern __shared__ unsigned long long lds_raw[];
    uint64_t* keys = reinterpret_cast<uint64_t*>(lds_raw);                    // [cap_keys]
    int32_t* kept_grids = reinterpret_cast<int32_t*>(keys + sp.cap_keys);     // [cap_kg]
    int32_t* kept_chunks = kept_grids + sp.cap_kg;                            // [cap_kc]
    int32_t* sel_pages = kept_chunks + sp.cap_kc;                             // [max_sel]
    __shared__ Shared sh;
    __shared__ double red[kSelGroups * kSharedSlots];

    const int m = blockIdx.x, C = gridDim.x, b = blockIdx.z, tid = threadIdx.x;
    const int H = g.n_kv_heads, B = g.page_size;
    Prof prof;
    for (int i = tid; i < kBins; i += kSelThreads) sh.hist[i] = 0;   // as cut_in_registers wants it
    if (tid == 0) sh.n_mem = 0;
    if (tid < 3) sh.tail_key[tid] = 0ull;
    if (tid == 0) sh.poll_limit = sp.poll_limit;
    const int L = min(max(seq_lens[b], 0), g.max_pages * B);
    const int P = (L + B - 1) / B;
    const int s = sp.sink, w = sp.window;
    // the list is the same for every KV head of the sequence: it is written H times, in the layout the
    // decode calls read
    if (P <= s + w) {                                                 // safety pages cover the sequence
        if (m == 0) {
            for (int i = tid; i < H * g.max_sel; i += kSelThreads) {
                const int at = i % g.max_sel;
                page_ids[(size_t)b * H * g.max_sel + i] = at < P ? at : -1;
            }
            if (tid < H) n_selected[b * H + tid] = min(P, g.max_sel);
        }
        return;
    }
    __syncthreads();

    const PubLayout pubs = pub_layout(ws.keys + (size_t)b * ws.key_stride, g, sp);
    CascadeResult res;
    const SharedScorer scorer{tab, b, g, red};
    const bool ok = cascade_with<false>(scorer, P, g, sp, pubs, m, C, m == 0, keys, kept_grids, kept_chunks, sel_pages, sh,
                                        &res, prof, nullptr, [] {});
    if (!ok) {
        if (tid == 0) __hip_atomic_store(ws.error, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return;
    }
    if (C > 1) {
        // whoever is last to be done with the published words clears them for the next launch
        if (arrive_last(ws.meta + (size_t)b * kSelMetaStride, C, &sh.flag)) clear_published(pubs, res);
    }
    if (m != 0) return;

    const int n_kp = res.n_kp, n_sel = s + n_kp + w;
    for (int i = tid; i < H * g.max_sel; i += kSelThreads) {
        const int at = i % g.max_sel;
        int v = -1;
        if (at < s) v = at;
        else if (at < s + n_kp) v = sel_pages[at - s];
        else if (at < n_sel) v = P - w + (at - s - n_kp);
        page_ids[(size_t)b * H * g.max_sel + i] = v;
    }
    if (tid < H) n_selected[b * H + tid] = n_sel;
}

hipError_t select_shared_occupancy(int lds_bytes, int* blocks_per_cu)
{
    if (lds_bytes > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(select_shared_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return e;
    }
    return hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, select_shared_kernel, kSelThreads, lds_bytes);
}

hipError_t launch_select_shared(chess_ctx* ctx, const SharedTable& tab, const int32_t* seq_lens, int batch, int cluster,
                                const SelectParams& sp, const SelectWs& ws, size_t lds_bytes, int32_t* page_ids,
                                int32_t* n_selected, hipStream_t stream)
{
    const dim3 grid(cluster, 1, batch), block(kSelThreads);
    return launch(select_shared_kernel, grid, block, lds_bytes, stream, tab, seq_lens, ctx->geom, sp, ws, page_ids,
                  n_selected);
}

}  // namespace chess
