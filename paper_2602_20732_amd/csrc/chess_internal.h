// Internal declarations shared by the HIP translation units of libchess (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "../../include/chess.h"

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
};

struct SelectParams {
    int32_t plan, sink, window, budget_pages, budget_bp, over_chunk, over_grid, rho_g_bp, rho_c_bp, rho_p_bp;
    int32_t slot_cap;                // u64 key slots available in LDS
    int32_t list_cap;                // entries of each kept-parent list in LDS
};

struct KernelTimer {                 // one per kernel kind; events recycled in a ring
    static constexpr int kRing = 64;
    hipEvent_t start[kRing], stop[kRing];
    int pending = 0;
    double total_ms = 0.0;
    int64_t launches = 0;
    bool ready = false;
};

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
    bool timing;
    chess::KernelTimer timers[CHESS_K_COUNT];
};

namespace chess {

// Collect the finished event pairs of one timer into its totals (synchronises on them).
inline hipError_t drain_timer(KernelTimer& t)
{
    for (int i = 0; i < t.pending; ++i) {
        hipError_t e = hipEventSynchronize(t.stop[i]);
        if (e != hipSuccess) return e;
        float ms = 0.f;
        e = hipEventElapsedTime(&ms, t.start[i], t.stop[i]);
        if (e != hipSuccess) return e;
        t.total_ms += ms;
        t.launches += 1;
    }
    t.pending = 0;
    return hipSuccess;
}

// Launch `kernel`; with timing on, bracket exactly this dispatch with start / stop events so the
// elapsed time is the kernel's own duration (no launch gaps).
template <typename... KArgs, typename... Args>
inline hipError_t timed_launch(chess_ctx* ctx, int which, void (*kernel)(KArgs...), dim3 grid, dim3 block,
                               size_t lds, hipStream_t stream, Args... args)
{
    if (!ctx->timing) {
        hipLaunchKernelGGL(kernel, grid, block, lds, stream, args...);
        return hipGetLastError();
    }
    KernelTimer& t = ctx->timers[which];
    if (!t.ready) {
        for (int i = 0; i < KernelTimer::kRing; ++i) {
            hipError_t e = hipEventCreate(&t.start[i]);
            if (e == hipSuccess) e = hipEventCreate(&t.stop[i]);
            if (e != hipSuccess) return e;
        }
        t.ready = true;
    }
    if (t.pending == KernelTimer::kRing) {
        hipError_t e = drain_timer(t);
        if (e != hipSuccess) return e;
    }
    const int i = t.pending++;
    hipExtLaunchKernelGGL(kernel, grid, block, lds, stream, t.start[i], t.stop[i], 0, args...);
    return hipGetLastError();
}

// Launchers (each returns a hipError_t from the launch).
hipError_t launch_summarize(chess_ctx* ctx, const uint16_t* k_pool, const int32_t* block_table,
                            const int32_t* seq_lens, int batch, const int32_t* from_page, bool tail_only,
                            float* pages, float* chunks, float* grids, hipStream_t stream);

hipError_t launch_select(chess_ctx* ctx, const uint16_t* q, const float* pages, const float* chunks,
                         const float* grids, const int32_t* seq_lens, int batch, const SelectParams& sp,
                         size_t lds_bytes, int32_t* page_ids, int32_t* n_selected, hipStream_t stream);

// page_ids == nullptr: every page of the sequence.  n_splits >= 1; with n_splits == 1 the decode
// kernel writes `out` itself and no merge is launched.
hipError_t launch_decode(chess_ctx* ctx, const uint16_t* q, const uint16_t* k_pool, const uint16_t* v_pool,
                         const int32_t* block_table, const int32_t* seq_lens, const int32_t* page_ids,
                         const int32_t* n_selected, int batch, int n_splits, int waves, float* out,
                         float* ws_acc, float* ws_ml, hipStream_t stream);
hipError_t launch_merge(chess_ctx* ctx, int batch, int n_splits, const float* ws_acc, const float* ws_ml,
                        float* out, hipStream_t stream);

}  // namespace chess
