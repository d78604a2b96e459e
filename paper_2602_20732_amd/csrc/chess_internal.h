// Internal declarations shared by the HIP translation units of libchess (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/chess.h"
#include "../../include/chess_debug.h"

namespace chess {

constexpr int kHeadDim = 128;        // d
constexpr int kWave = 64;            // CDNA wavefront
constexpr int kMaxGroup = 16;        // q heads per KV head: one MFMA N-tile
constexpr int kTileTokens = 32;      // tokens per decode tile = K extent of one 16x16x32 MFMA

// Geometry every kernel needs, passed by value.
struct Geom {
    int32_t n_q_heads, n_kv_heads, group;
    int32_t page_size;               // B
    int32_t n_c, n_g;                // pages per chunk, chunks per grid
    int32_t max_pages, max_chunks, max_grids;   // row strides of block table / summary arrays
    int32_t max_sel;                 // row stride of page_ids
    uint32_t inv_nc, inv_ng;         // ceil(2^32 / n_c), ceil(2^32 / n_g) (0 for 1): divisions by n_c / n_g as a multiply-high
};

struct SelectParams {
    int32_t plan, sink, window, budget_pages, budget_bp, over_chunk, over_grid, rho_g_bp, rho_c_bp, rho_p_bp;
    int32_t cap2, cap3;              // most candidate slots level 2 / level 3 can have (host bound)
    int32_t cap_keys, cap_kg, cap_kc;   // LDS capacities: keys of one level, kept grids, kept chunks
    int32_t probe;                   // CHESS_PROBE_*
    int32_t poll_limit;              // polls before a wait for published keys is given up
    int32_t general_cut;             // test hook: every level takes the general (LDS radix) cut
    int32_t local_grids;             // every member scores all grids itself (no exchange at the grid level)
    int32_t merged;                  // all chunks are scored together with the grids (one memory phase and one exchange fewer)
    int32_t keep_ties;               // the threshold rule: a level keeps every unit that ties with its k-th
    const int32_t* budget_per_seq;   // device [batch] or null: a value > 0 is that sequence's page budget
};

// The page budget the plan fixes for sequence b, or 0 when it is derived from the sequence's page count:
// budget_per_seq[b] when given and positive (clamped to what a page_ids row can hold), else budget_pages.
__device__ __forceinline__ int fixed_budget(const SelectParams& sp, const Geom& g, int b)
{
    const int per = sp.budget_per_seq != nullptr ? sp.budget_per_seq[b] : 0;
    const int room = g.max_sel - sp.sink - sp.window;
    return per > 0 ? (per < room ? per : (room > 1 ? room : 1)) : sp.budget_pages;
}

#ifndef CHESS_SEL_THREADS
#define CHESS_SEL_THREADS 256
#endif
constexpr int kSelThreads = CHESS_SEL_THREADS;   // workgroup of the selection kernels
constexpr int kSelMaxCluster = 32;   // most workgroups per (sequence, KV head)
constexpr int kSelMetaStride = 8;    // int32 per (sequence, KV head): [0] members that are done with the published keys

// Select scratch in the caller's workspace (device pointers).
struct SelectWs {
    uint64_t* keys;                  // [rows][key_stride]  published candidate keys: grids | chunk slots | page slots;
    int64_t key_stride;              //   all zero between launches
    uint64_t* tail;                  // [rows][4] keys of the refreshed tail grid / chunk / page; zero between launches
    int32_t* meta;                   // [rows][kSelMetaStride], zero between launches
    int32_t* error;                  // one word of kErr* bits
#ifdef CHESS_PROF
    int32_t* prof;                   // [rows][Prof::kSlots] phase timestamps in 10 ns ticks (profiling builds only)
#endif
};
constexpr int kErrWait = 1;          // a wait for published keys was given up
constexpr int kErrOverflow = 2;      // the threshold rule kept more units than a list has room for (the list was cut short)

// Values that cross workgroups inside one launch travel as agent-scope atomics: on gfx950 these are loads and
// stores with the sc1 bit, which do not live in the per-XCD L2s as cached copies (a store is written through to
// the memory side that all eight XCDs share before it is acknowledged, a load is served from there), so they are
// coherent across the device without any cache maintenance.  Two kinds of message:
//  * a published word that IS the message (a key, polled until it is non-zero) needs no ordering against anything
//    else;
//  * data announced by something else (split partials by the arrival counter): the writer's waves wait until their
//    sc1 stores are acknowledged (s_waitcnt 0: by then they are at the shared memory side) before the workgroup's
//    barrier and the arrival, and the reader's sc1 loads, issued after it has seen the last arrival, are served from
//    that same place.  The language-level equivalent, a release fence before and an acquire fence after the arrival
//    at agent scope, was measured: it compiles to a write-back and an invalidate of the whole L2 (buffer_wbl2 sc1 /
//    buffer_inv sc1), which these accesses do not need, and costs 12 us per sparse-decode launch (14 -> 26 us).  So
//    the ordering rests on the hardware behaviour above, with relaxed atomics, not on the abstract memory model.
__device__ __forceinline__ void publish_u64(uint64_t* p, uint64_t v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t observe_u64(const uint64_t* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void publish_f32(float* p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float observe_f32(const float* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Called by every thread of a workgroup after its publish_* stores.  Returns true (to every thread)
// in the workgroup that arrives last of `expected`; that workgroup also re-arms the counter for the
// next launch.  Nobody waits.  The counter must be 0 before the first launch.
__device__ __forceinline__ bool arrive_last(int32_t* counter, int expected, int* lds_flag)
{
    __builtin_amdgcn_s_waitcnt(0);                   // this wave's published stores are acknowledged, its loads have returned
    __syncthreads();
    if (threadIdx.x == 0) {
        const int old = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int last = old == expected - 1;
        if (last) __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *lds_flag = last;
    }
    __syncthreads();
    return *lds_flag != 0;
}

}  // namespace chess

struct chess_ctx {
    chess_config cfg;
    chess::Geom geom;
    float sm_scale;
    int device;
    int n_cu;
    int lds_per_block;
    size_t page_off, chunk_off, grid_off, summary_bytes;   // bytes
    int max_splits;
    int force_splits, force_waves;                         // 0 = automatic
    size_t ws_acc_off, ws_ml_off, workspace_bytes;
    size_t ws_ent_off, ws_entcnt_off;                      // entropy partials, their arrival counters
    size_t ws_keys_off, ws_tail_off, ws_meta_off, ws_cnt_off, ws_err_off, ws_prof_off;   // select scratch, decode arrival counters, error word
    int64_t key_stride;
    int force_cluster;                                     // 0 = automatic
    int force_schedule;                                    // 0 = automatic, 1 = lazy, 2 = merged
    int force_general_cut;                                 // 0 = automatic
    int poll_limit;                                        // 0 = the default
    int dec_blocks4, dec_blocks1;                          // decode workgroups per CU with 4 waves / 1 wave
    int occ_lds, occ_blocks;                               // cached occupancy query of the select kernel
    int step_occ_lds, step_occ_blocks;                     // ... and of the fused step kernel
    int shared_occ_lds, shared_occ_blocks;                 // ... and of the model-wide select kernel
    size_t ws_zero_off, ws_zero_bytes;                     // the part chess_workspace_init clears
    void* static_scratch;                                  // this device's copy of the library's own scratch array (or null)
};

namespace chess {

// Launch `kernel` on `stream` and report the launch status.
template <typename... KArgs, typename... Args>
inline hipError_t launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds, hipStream_t stream, Args... args)
{
    hipLaunchKernelGGL(kernel, grid, block, lds, stream, args...);
    return hipGetLastError();
}

// Launchers (each returns a hipError_t from the launch).
// (summary arrays travel as void*: fp32 or bf16 by the context's summary_dtype)
hipError_t launch_summarize(chess_ctx* ctx, const uint16_t* k_pool, const int32_t* block_table,
                            const int32_t* seq_lens, int batch, const int32_t* from_page, int recent,
                            void* pages, void* chunks, void* grids, hipStream_t stream);

hipError_t launch_select(chess_ctx* ctx, const uint16_t* q, const void* pages, const void* chunks,
                         const void* grids, const int32_t* seq_lens, int batch, int cluster, const SelectParams& sp,
                         const SelectWs& ws, size_t lds_bytes, int32_t* page_ids, int32_t* n_selected,
                         hipStream_t stream);
// Device pointers of one fused decode-step launch.
struct StepLaunch {
    const uint16_t* q;
    void* pages;
    void* chunks;
    void* grids;
    const uint16_t* k_pool;
    const uint16_t* v_pool;
    const int32_t* block_table;
    const int32_t* seq_lens;
    int32_t* page_ids;
    int32_t* n_selected;
    float* out;
    float* ws_acc;
    float* ws_ml;
    int32_t* arrivals;
    int32_t refresh_tail;
};
hipError_t launch_step(chess_ctx* ctx, const StepLaunch& sl, int batch, int cluster, const SelectParams& sp,
                       const SelectWs& ws, size_t lds_bytes, int union_off, hipStream_t stream);
size_t step_lds_bytes(const SelectParams& sp, int max_sel, int* union_off);
hipError_t step_occupancy(int page_size, bool bf16, int lds_bytes, int* blocks_per_cu);
hipError_t select_occupancy(bool bf16, int lds_bytes, int* blocks_per_cu);

// The model-wide scope: per-layer probes (fp32 [batch][H_kv][128]) and summary buffers, passed by value.
constexpr int kMaxLayers = CHESS_MAX_LAYERS;
constexpr int kSharedMaxCluster = 128;
struct SharedTable {
    const float* probes[kMaxLayers];
    const char* summaries[kMaxLayers];
    size_t page_off, chunk_off, grid_off;            // bytes into a summary buffer
    int n_layers;
};
struct AnchorTable {
    const char* summaries[kMaxLayers];
    float* anchors[kMaxLayers];
    size_t page_off;
};
hipError_t launch_anchor(chess_ctx* ctx, const AnchorTable& tab, int n_layers, const int32_t* seq_lens, int batch,
                         int window, hipStream_t stream);
hipError_t select_shared_occupancy(bool bf16, int lds_bytes, int* blocks_per_cu);
hipError_t launch_select_shared(chess_ctx* ctx, const SharedTable& tab, const int32_t* seq_lens, int batch, int cluster,
                                const SelectParams& sp, const SelectWs& ws, size_t lds_bytes, int32_t* page_ids,
                                int32_t* n_selected, hipStream_t stream);
size_t select_lds_bytes(const SelectParams& sp, int max_sel);
hipError_t decode_occupancy(int page_size, int waves, int group, int* blocks_per_cu);
hipError_t launch_append(chess_ctx* ctx, const uint16_t* k_new, const uint16_t* v_new, uint16_t* k_pool, uint16_t* v_pool,
                         const int32_t* block_table, const int32_t* seq_lens, int batch, int32_t* page_ids,
                         int32_t* n_selected, hipStream_t stream);
hipError_t launch_reuse(chess_ctx* ctx, const uint16_t* q, const uint16_t* k_new, const uint16_t* v_new, uint16_t* k_pool,
                        uint16_t* v_pool, const int32_t* block_table, const int32_t* seq_lens, int32_t* page_ids,
                        int32_t* n_selected, int batch, int n_splits, float* out, float* ws_acc, float* ws_ml,
                        int32_t* arrivals, hipStream_t stream);
hipError_t launch_extend(chess_ctx* ctx, const int32_t* seq_lens, int batch, int32_t* page_ids, int32_t* n_selected,
                         hipStream_t stream);
constexpr int kEntMaxSplits = 32;
// page_steps > 0: the thread that ends up with a sequence's entropy also does that sequence's trigger update
hipError_t launch_entropy(chess_ctx* ctx, const uint16_t* logits, int batch, int vocab, int64_t row_stride, int splits,
                          float* H, float* partials, int32_t* arrivals, int page_steps, double tau_h, double tau_v,
                          float* history, int32_t* count, int32_t* fire, double* stats, hipStream_t stream);
hipError_t launch_trigger(const float* H, int batch, int page_steps, double tau_h, double tau_v, float* history,
                          int32_t* count, int32_t* fire, double* stats, hipStream_t stream);
hipError_t launch_zero(chess_ctx* ctx, int32_t* p, size_t n_words, hipStream_t stream);

// page_ids == nullptr: every page of the sequence.  n_splits >= 1; the last split of a (sequence,
// KV head) to finish merges the partials and writes `out`.  `arrivals`: int32 [rows], zero before first use.
hipError_t launch_decode(chess_ctx* ctx, const uint16_t* q, const uint16_t* k_pool, const uint16_t* v_pool,
                         const int32_t* block_table, const int32_t* seq_lens, const int32_t* page_ids,
                         const int32_t* n_selected, int batch, int n_splits, int waves, float* out,
                         float* ws_acc, float* ws_ml, int32_t* arrivals, hipStream_t stream);

}  // namespace chess
