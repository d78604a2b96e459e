// The selection under the paper's own scope (Sec. 3.1, Eq. 1: a unit's vector is the concatenation, over all
// layers and heads, of the per-layer, per-head means) with the key anchor of Sec. 3.2, Eq. 3 as the probe:
// one score per unit, S(u) = sum over layers l and KV heads h of probe[l][h] . v[l][h][u] (Eq. 4 on the
// flattened vectors), one page set per sequence for the whole model.
//
// anchor_kernel: Eq. 3 for every (layer, sequence, KV head), as an output of its own.
// select_shared_kernel: a cluster of C workgroups per sequence runs the three levels of select_device.h; only the
// scoring differs.  A unit's vector is n_layers * H_kv rows of 512 bytes in as many arrays, so all 16 lane
// groups of a workgroup work on the same few slots: group j takes the rows r = j, j + 16, ... (row r = layer
// r / H_kv, head r % H_kv), eight slots and two rows at a time (sixteen vectors in flight per group), fp64
// partial sums; the groups' partials are added in group order through LDS.  The order of the additions is fixed, so a
// unit's score does not depend on the launch shape.
#include "select_device.h"

namespace chess {

// grid = (ceil(rows / 16), n_layers), 256 threads: a 16-lane group per (layer, sequence, KV head)
__global__ __launch_bounds__(256) void anchor_kernel(AnchorTable tab, const int32_t* __restrict__ seq_lens, int rows, Geom g,
                                                     int window)
{
    const int row = blockIdx.x * 16 + (threadIdx.x >> 4), ln = threadIdx.x & 15, l = blockIdx.y;
    if (row >= rows) return;
    const int b = row / g.n_kv_heads;
    const int L = min(max(seq_lens[b], 0), g.max_pages * g.page_size);
    const int P = (L + g.page_size - 1) / g.page_size;
    const float* pages = reinterpret_cast<const float*>(tab.summaries[l] + tab.page_off);
    double pr[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (P > 0) load_anchor(pages + (size_t)row * g.max_pages * kHeadDim, P, window, pr);
    float4* dst = reinterpret_cast<float4*>(tab.anchors[l] + (size_t)row * kHeadDim);
    dst[ln] = make_float4((float)pr[0], (float)pr[1], (float)pr[2], (float)pr[3]);
    dst[16 + ln] = make_float4((float)pr[4], (float)pr[5], (float)pr[6], (float)pr[7]);
}

hipError_t launch_anchor(chess_ctx* ctx, const AnchorTable& tab, int n_layers, const int32_t* seq_lens, int batch,
                         int window, hipStream_t stream)
{
    const int rows = batch * ctx->geom.n_kv_heads;
    return launch(anchor_kernel, dim3((rows + 15) / 16, n_layers), dim3(256), 0, stream, tab, seq_lens, rows, ctx->geom,
                  window);
}

constexpr int kSharedSlots = 8;                      // slots a workgroup scores together

struct SharedScorer {
    static constexpr int kShareRound = 1;
    const SharedTable& tab;
    int b;
    const Geom& g;
    double* red;                                     // LDS [16 groups][kSharedSlots]

    // One pass: the N slots s0 .. s0 + N - 1 (N is a template parameter so that exactly N vectors per row are
    // requested, all before the first is used: a run-time count would make the compiler wait for each).
    template <int N, class Map>
    __device__ __forceinline__ void pass(int level, int s0, Map unit_of, bool local, uint64_t* keys, uint64_t* pub) const
    {
        const int tid = threadIdx.x, g16 = tid >> 4, ln = tid & 15;
        const int H = g.n_kv_heads, R = tab.n_layers * H;
        const size_t level_off = level == 0 ? tab.grid_off : level == 1 ? tab.chunk_off : tab.page_off;
        const size_t units = level == 0 ? g.max_grids : level == 1 ? g.max_chunks : g.max_pages;
        int unit[N];
        double part[N];
#pragma unroll
        for (int x = 0; x < N; ++x) {
            unit[x] = unit_of(s0 + x);
            part[x] = 0.0;
        }
        // two rows per trip: 2 N vectors in flight per group.  A trip's second row may not exist: it then reads the
        // first row again with a zero probe (adding exact zeros)
        for (int r = g16; r < R; r += 2 * kSelGroups) {
            float4 pa[2], pb[2];
            const float* base[2];
#pragma unroll
            for (int y = 0; y < 2; ++y) {
                const bool have = r + y * kSelGroups < R;
                const int ry = have ? r + y * kSelGroups : r;
                const int l = ry / H, h = ry - l * H;
                const size_t row = (size_t)b * H + h;
                const float4* p0 = reinterpret_cast<const float4*>(tab.probes[l] + row * kHeadDim);
                base[y] = reinterpret_cast<const float*>(tab.summaries[l] + level_off) + row * units * kHeadDim;
                pa[y] = p0[ln];
                pb[y] = p0[16 + ln];
                if (!have) { pa[y] = make_float4(0.f, 0.f, 0.f, 0.f); pb[y] = pa[y]; }
            }
            float4 va[2][N], vb[2][N];
#pragma unroll
            for (int y = 0; y < 2; ++y) {
#pragma unroll
                for (int x = 0; x < N; ++x) {
                    // always load (unit 0 when the slot has no unit): all stay in flight
                    const float4* p = reinterpret_cast<const float4*>(base[y] + (size_t)max(unit[x], 0) * kHeadDim) + ln;
                    va[y][x] = p[0];
                    vb[y][x] = p[16];
                }
            }
#pragma unroll
            for (int y = 0; y < 2; ++y) {
#pragma unroll
                for (int x = 0; x < N; ++x) {
                    double d = part[x];
                    d = fma((double)pa[y].x, (double)va[y][x].x, d); d = fma((double)pa[y].y, (double)va[y][x].y, d);
                    d = fma((double)pa[y].z, (double)va[y][x].z, d); d = fma((double)pa[y].w, (double)va[y][x].w, d);
                    d = fma((double)pb[y].x, (double)vb[y][x].x, d); d = fma((double)pb[y].y, (double)vb[y][x].y, d);
                    d = fma((double)pb[y].z, (double)vb[y][x].z, d); d = fma((double)pb[y].w, (double)vb[y][x].w, d);
                    part[x] = d;
                }
            }
        }
#pragma unroll
        for (int x = 0; x < N; ++x) {
            const double d = row16_sum(part[x]);
            if (ln == 15) red[g16 * kSharedSlots + x] = d;
        }
        __syncthreads();
        if (tid < N) {
            double d = 0.0;
#pragma unroll
            for (int j = 0; j < kSelGroups; ++j) d += red[j * kSharedSlots + tid];
            const int u = unit_of(s0 + tid);
            if (local) keys[s0 + tid] = u >= 0 ? order_key(d) : 0ull;
            else publish_u64(pub + s0 + tid, u >= 0 ? order_key(d) : kAbsentKey);
        }
        __syncthreads();                              // red is reused by the next pass
    }

    template <class Map>
    __device__ __forceinline__ void operator()(int level, int lo, int hi, Map unit_of, bool local, uint64_t* keys,
                                               uint64_t* pub) const
    {
        // the share in passes of equal size (the last may be shorter), at most kSharedSlots slots each
        const int n_pass = (hi - lo + kSharedSlots - 1) / kSharedSlots;
        const int per_pass = n_pass > 0 ? (hi - lo + n_pass - 1) / n_pass : 0;
        for (int s0 = lo; s0 < hi; s0 += per_pass) {
            switch (min(per_pass, hi - s0)) {             // uniform over the workgroup
            case 1: pass<1>(level, s0, unit_of, local, keys, pub); break;
            case 2: pass<2>(level, s0, unit_of, local, keys, pub); break;
            case 3: pass<3>(level, s0, unit_of, local, keys, pub); break;
            case 4: pass<4>(level, s0, unit_of, local, keys, pub); break;
            case 5: pass<5>(level, s0, unit_of, local, keys, pub); break;
            case 6: pass<6>(level, s0, unit_of, local, keys, pub); break;
            case 7: pass<7>(level, s0, unit_of, local, keys, pub); break;
            default: pass<8>(level, s0, unit_of, local, keys, pub); break;
            }
        }
    }
};
static_assert(kSharedSlots == 8, "the dispatch in SharedScorer lists the pass sizes");

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
    const int k_fixed = fixed_budget(sp, g, b);
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
                                        &res, prof, nullptr, [] {}, k_fixed);
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
