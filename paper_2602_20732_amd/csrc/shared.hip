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
template <class T>
__global__ __launch_bounds__(256) void anchor_kernel(AnchorTable tab, const int32_t* __restrict__ seq_lens, int rows, Geom g,
                                                     int window)
{
    const int row = blockIdx.x * 16 + (threadIdx.x >> 4), ln = threadIdx.x & 15, l = blockIdx.y;
    if (row >= rows) return;
    const int b = row / g.n_kv_heads;
    const int L = min(max(seq_lens[b], 0), g.max_pages * g.page_size);
    const int P = (L + g.page_size - 1) / g.page_size;
    const T* pages = reinterpret_cast<const T*>(tab.summaries[l] + tab.page_off);
    double pr[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (P > 0) load_anchor<T>(pages + (size_t)row * g.max_pages * kHeadDim, P, window, pr);
    // the anchor is an fp32 vector [128] in dim order, whatever arrangement the lanes hold it in
    float* dst = tab.anchors[l] + (size_t)row * kHeadDim;
#pragma unroll
    for (int i = 0; i < 8; ++i) dst[Vec<T>::lane_dim(ln, i)] = (float)pr[i];
}

hipError_t launch_anchor(chess_ctx* ctx, const AnchorTable& tab, int n_layers, const int32_t* seq_lens, int batch,
                         int window, hipStream_t stream)
{
    const int rows = batch * ctx->geom.n_kv_heads;
    if (ctx->cfg.summary_dtype == CHESS_SUMMARY_BF16)
        return launch(anchor_kernel<uint16_t>, dim3((rows + 15) / 16, n_layers), dim3(256), 0, stream, tab, seq_lens, rows,
                      ctx->geom, window);
    return launch(anchor_kernel<float>, dim3((rows + 15) / 16, n_layers), dim3(256), 0, stream, tab, seq_lens, rows, ctx->geom,
                  window);
}

constexpr int kSharedSlots = 8;                      // slots a workgroup scores together

template <class T>
struct SharedScorer {
    static constexpr int kShareRound = 1;
    static constexpr int kTrip = kSharedSlots;
    const SharedTable& tab;
    int b;
    const Geom& g;
    double* red;                                     // LDS [16 groups][kSharedSlots]

    // One pass: the N work slots s0 .. s0 + N - 1, all of one level (N is a template parameter so that exactly N
    // vectors per row are requested, all before the first is used: a run-time count would make the compiler wait
    // for each).
    template <int N, class Target>
    __device__ __forceinline__ void pass(int s0, Target target, bool local, uint64_t* keys, uint64_t* pub) const
    {
        const int tid = threadIdx.x, g16 = tid >> 4, ln = tid & 15;
        const int H = g.n_kv_heads, R = tab.n_layers * H;
        const int level = target(s0).array;          // (never the merged schedule: a pass stays inside one array)
        const size_t level_off = level == 0 ? tab.grid_off : level == 1 ? tab.chunk_off : tab.page_off;
        const size_t units = level == 0 ? g.max_grids : level == 1 ? g.max_chunks : g.max_pages;
        int unit[N];
        double part[N];
#pragma unroll
        for (int x = 0; x < N; ++x) {
            unit[x] = target(s0 + x).unit;
            part[x] = 0.0;
        }
        // two rows per trip: 2 N vectors in flight per group.  A trip's second row may not exist: it then reads the
        // first row again with a zero probe (adding exact zeros)
        for (int r = g16; r < R; r += 2 * kSelGroups) {
            double pr[2][8];
            const T* base[2];
#pragma unroll
            for (int y = 0; y < 2; ++y) {
                const bool have = r + y * kSelGroups < R;
                const int ry = have ? r + y * kSelGroups : r;
                const int l = ry / H, h = ry - l * H;
                const size_t row = (size_t)b * H + h;
                const float* p0 = tab.probes[l] + row * kHeadDim;
                base[y] = reinterpret_cast<const T*>(tab.summaries[l] + level_off) + row * units * kHeadDim;
                // the probe in the arrangement the vectors are held in (two runs of four consecutive dims)
                const float4 pa = *reinterpret_cast<const float4*>(p0 + Vec<T>::lane_dim(ln, 0));
                const float4 pb = *reinterpret_cast<const float4*>(p0 + Vec<T>::lane_dim(ln, 4));
                pr[y][0] = have ? (double)pa.x : 0.0; pr[y][1] = have ? (double)pa.y : 0.0;
                pr[y][2] = have ? (double)pa.z : 0.0; pr[y][3] = have ? (double)pa.w : 0.0;
                pr[y][4] = have ? (double)pb.x : 0.0; pr[y][5] = have ? (double)pb.y : 0.0;
                pr[y][6] = have ? (double)pb.z : 0.0; pr[y][7] = have ? (double)pb.w : 0.0;
            }
            Vec<T> v[2][N];
#pragma unroll
            for (int y = 0; y < 2; ++y) {
#pragma unroll
                for (int x = 0; x < N; ++x)       // always load (unit 0 when the slot has no unit): all stay in flight
                    v[y][x].load(base[y] + (size_t)max(unit[x], 0) * kHeadDim, ln);
            }
#pragma unroll
            for (int y = 0; y < 2; ++y) {
#pragma unroll
                for (int x = 0; x < N; ++x) part[x] = dot8<T>(pr[y], v[y][x], part[x]);
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
            const SlotRef ref = target(s0 + tid);
            if (ref.dest >= 0) {
                if (local) keys[ref.dest] = ref.unit >= 0 ? order_key(d) : 0ull;
                else publish_u64(pub + ref.dest, ref.unit >= 0 ? order_key(d) : kAbsentKey);
            }
        }
        __syncthreads();                              // red is reused by the next pass
    }

    template <class Target>
    __device__ __forceinline__ void operator()(int lo, int hi, Target target, bool local, uint64_t* keys, uint64_t* pub) const
    {
        // the share in passes of equal size (the last may be shorter), at most kSharedSlots slots each
        const int n_pass = (hi - lo + kSharedSlots - 1) / kSharedSlots;
        const int per_pass = n_pass > 0 ? (hi - lo + n_pass - 1) / n_pass : 0;
        for (int s0 = lo; s0 < hi; s0 += per_pass) {
            switch (min(per_pass, hi - s0)) {             // uniform over the workgroup
            case 1: pass<1>(s0, target, local, keys, pub); break;
            case 2: pass<2>(s0, target, local, keys, pub); break;
            case 3: pass<3>(s0, target, local, keys, pub); break;
            case 4: pass<4>(s0, target, local, keys, pub); break;
            case 5: pass<5>(s0, target, local, keys, pub); break;
            case 6: pass<6>(s0, target, local, keys, pub); break;
            case 7: pass<7>(s0, target, local, keys, pub); break;
            default: pass<8>(s0, target, local, keys, pub); break;
            }
        }
    }
};
static_assert(kSharedSlots == 8, "the dispatch in SharedScorer lists the pass sizes");

// grid = (C, 1, batch); T = storage type of the summaries
template <class T>
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
    init_shared(sh, sp.poll_limit);
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

    const PubLayout pubs = pub_layout(ws.keys + (size_t)b * ws.key_stride, g);
    CascadeResult res;
    const SharedScorer<T> scorer{tab, b, g, red};
    const bool ok = cascade_with<false>(scorer, P, g, sp, pubs, m, C, m == 0, keys, kept_grids, kept_chunks, sel_pages, sh,
                                        &res, prof, nullptr, [] {}, k_fixed);
    if (!ok) {
        if (tid == 0) __hip_atomic_fetch_or(ws.error, kErrWait, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return;
    }
    if (C > 1) {
        // whoever is last to be done with the published words clears them for the next launch
        if (arrive_last(ws.meta + (size_t)b * kSelMetaStride, C, &sh.flag)) clear_published(pubs, res);
    }
    if (m != 0) return;
    if (res.overflow && tid == 0) __hip_atomic_fetch_or(ws.error, kErrOverflow, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

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

hipError_t select_shared_occupancy(bool bf16, int lds_bytes, int* blocks_per_cu)
{
    const void* kern = bf16 ? reinterpret_cast<const void*>(select_shared_kernel<uint16_t>)
                            : reinterpret_cast<const void*>(select_shared_kernel<float>);
    if (lds_bytes > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return e;
    }
    return bf16 ? hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, select_shared_kernel<uint16_t>, kSelThreads, lds_bytes)
                : hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, select_shared_kernel<float>, kSelThreads, lds_bytes);
}

hipError_t launch_select_shared(chess_ctx* ctx, const SharedTable& tab, const int32_t* seq_lens, int batch, int cluster,
                                const SelectParams& sp, const SelectWs& ws, size_t lds_bytes, int32_t* page_ids,
                                int32_t* n_selected, hipStream_t stream)
{
    const dim3 grid(cluster, 1, batch), block(kSelThreads);
    if (ctx->cfg.summary_dtype == CHESS_SUMMARY_BF16)
        return launch(select_shared_kernel<uint16_t>, grid, block, lds_bytes, stream, tab, seq_lens, ctx->geom, sp, ws, page_ids,
                      n_selected);
    return launch(select_shared_kernel<float>, grid, block, lds_bytes, stream, tab, seq_lens, ctx->geom, sp, ws, page_ids,
                  n_selected);
}

}  // namespace chess
