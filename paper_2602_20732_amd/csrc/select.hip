// Coarse-to-fine page selection (Sec. 3.2, Eq. 4, Alg. 1 stage 2): one kernel launch per level
// (grids, chunks of kept grids, pages of kept chunks), many workgroups per (sequence, KV head).
//
// The paper scores the whole hierarchy with one GEMM and prunes with masks.  Here scoring is lazy --
// a level reads only the 512-byte vectors of its candidates -- and it is spread over the chip: a
// workgroup scores a slice of 32 candidate slots (a 16-lane group per unit: two 128-bit loads per
// lane, fp64 multiply-add, 4-step butterfly) and publishes order-preserving 64-bit keys.  The last
// workgroup of a (sequence, head) to arrive pulls that row's keys into LDS, finds the k-th largest
// with an 8-bit radix select, resolves ties at the cut towards the lowest slots (= lowest indices:
// candidates are enumerated in index order) and compacts the keep mask, in order, into the
// ascending list of kept units that the next level's launch enumerates.  Level 3 writes the final
// page list: sinks, kept pages, window pages.
//
// Keys cross workgroups through agent-scope atomic stores / loads (coherent across the XCDs' L2s)
// and an arrival counter; nobody waits, so there is nothing to deadlock.
#include "chess_internal.h"

namespace chess {

constexpr int kSelThreads = 256;
constexpr int kSelWaves = kSelThreads / kWave;
constexpr int kSlice = 32;                  // candidate slots per workgroup: 16 lane groups x 2 units

// Monotone map double -> uint64 (larger score = larger key); every finite or infinite score maps
// to a key >= 1, so 0 marks an empty slot.  -0.0 is folded onto +0.0 first.
__device__ __forceinline__ uint64_t order_key(double s)
{
    s += 0.0;
    const uint64_t u = (uint64_t)__double_as_longlong(s);
    return (u >> 63) ? ~u : (u | 0x8000000000000000ull);
}

__device__ __forceinline__ int ceil_div_i(int a, int b) { return (a + b - 1) / b; }
__device__ __forceinline__ int ceil_bp(int n, int bp) { return (int)(((int64_t)n * bp + 9999) / 10000); }
__device__ __forceinline__ int clamp_i(int x, int lo, int hi) { return x < lo ? lo : (x > hi ? hi : x); }

struct Shared {
    int hist[256];
    int wave_tot[kSelWaves];
    int digit, rem, cnt, n_valid, k, last;
    unsigned long long thr;
};

// Exclusive prefix sum of `v` over the workgroup in thread order; *total receives the sum.
__device__ __forceinline__ int block_excl_scan(int v, Shared& sh, int* total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int incl = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int up = __shfl_up(incl, off);
        if (lane >= off) incl += up;
    }
    if (lane == 63) sh.wave_tot[wave] = incl;
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) {
        const int t = sh.wave_tot[w];
        if (w < wave) base += t;
        tot += t;
    }
    __syncthreads();
    *total = tot;
    return base + incl - v;
}

__device__ __forceinline__ double dot8(const double (&pr)[8], const float4& a, const float4& b)
{
    double d = 0.0;
    d = fma(pr[0], (double)a.x, d); d = fma(pr[1], (double)a.y, d);
    d = fma(pr[2], (double)a.z, d); d = fma(pr[3], (double)a.w, d);
    d = fma(pr[4], (double)b.x, d); d = fma(pr[5], (double)b.y, d);
    d = fma(pr[6], (double)b.z, d); d = fma(pr[7], (double)b.w, d);
    return d;
}

// Find the cut of the top-k among the non-empty keys (in LDS).  k = k_of(number of non-empty keys).
// On return (uniform over the workgroup): a slot is kept iff key > thr, or key == thr and it is
// among the first `ties` such slots.
template <class KFn>
__device__ __forceinline__ void radix_cut(const uint64_t* keys, int n_slots, KFn k_of, Shared& sh,
                                          uint64_t* thr_out, int* ties_out)
{
    const int tid = threadIdx.x;
    uint64_t prefix = 0, mask = 0;
    int rem = 0;
    for (int pass = 7; pass >= 0; --pass) {
        const int shift = pass * 8;
        sh.hist[tid] = 0;                              // kSelThreads == 256 bins
        __syncthreads();
        for (int i = tid; i < n_slots; i += kSelThreads) {
            const uint64_t key = keys[i];
            if (key != 0 && (key & mask) == prefix) atomicAdd(&sh.hist[(int)((key >> shift) & 255)], 1);
        }
        __syncthreads();
        if (tid < 64) {
            // lane l owns digits 255-4l .. 252-4l, so lane order is digit order descending
            const int d0 = 255 - 4 * tid;
            const int c0 = sh.hist[d0], c1 = sh.hist[d0 - 1], c2 = sh.hist[d0 - 2], c3 = sh.hist[d0 - 3];
            const int s = c0 + c1 + c2 + c3;
            int incl = s;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const int up = __shfl_up(incl, off);
                if (tid >= off) incl += up;
            }
            int want;
            if (pass == 7) {
                const int n_valid = __shfl(incl, 63);
                want = k_of(n_valid);
                if (tid == 0) { sh.n_valid = n_valid; sh.k = want; }
            } else {
                want = sh.rem;
            }
            const int excl = incl - s;
            if (want >= 1 && excl < want && want <= incl) {
                int t = excl, digit, cnt;
                if (t + c0 >= want) { digit = d0; cnt = c0; }
                else if ((t += c0) + c1 >= want) { digit = d0 - 1; cnt = c1; }
                else if ((t += c1) + c2 >= want) { digit = d0 - 2; cnt = c2; }
                else { t += c2; digit = d0 - 3; cnt = c3; }
                sh.digit = digit; sh.rem = want - t; sh.cnt = cnt;
            }
        }
        __syncthreads();
        if (pass == 7) {
            const int k = sh.k;
            if (k <= 0) { *thr_out = ~0ull; *ties_out = 0; __syncthreads(); return; }
            if (k >= sh.n_valid) { *thr_out = 0ull; *ties_out = 0; __syncthreads(); return; }
        }
        prefix |= (uint64_t)sh.digit << shift;
        mask |= 255ull << shift;
        rem = sh.rem;
        if (sh.cnt == 1 && pass > 0) {                // a single key carries this prefix: it is the cut
            for (int i = tid; i < n_slots; i += kSelThreads) {
                const uint64_t key = keys[i];
                if (key != 0 && (key & mask) == prefix) sh.thr = key;
            }
            __syncthreads();
            prefix = sh.thr;
            break;
        }
    }
    *thr_out = prefix;
    *ties_out = rem;
    __syncthreads();
}

// Ordered compaction of the kept slots: emit(pos, unit_of(slot)) in ascending slot order.
template <class Map, class Out>
__device__ __forceinline__ int compact_kept(const uint64_t* keys, int n_slots, uint64_t thr, int ties, Map unit_of,
                                            Out emit, Shared& sh)
{
    const int per = ceil_div_i(n_slots, kSelThreads);
    const int lo = min(n_slots, (int)threadIdx.x * per), hi = min(n_slots, lo + per);
    int n_eq = 0;
    for (int i = lo; i < hi; ++i) n_eq += (keys[i] == thr && thr != 0);
    int tot_eq;
    const int eq_before = block_excl_scan(n_eq, sh, &tot_eq);
    int n_keep = 0, eq_seen = eq_before;
    for (int i = lo; i < hi; ++i) {
        const uint64_t key = keys[i];
        if (key > thr) ++n_keep;
        else if (key == thr && thr != 0) { n_keep += (eq_seen < ties); ++eq_seen; }
    }
    int total;
    int pos = block_excl_scan(n_keep, sh, &total);
    eq_seen = eq_before;
    for (int i = lo; i < hi; ++i) {
        const uint64_t key = keys[i];
        bool keep = key > thr;
        if (key == thr && thr != 0) { keep = eq_seen < ties; ++eq_seen; }
        if (keep) emit(pos++, unit_of(i));
    }
    __syncthreads();
    return total;
}

// LEVEL 1: grids; 2: chunks of kept grids; 3: pages of kept chunks (sink / window pages excluded).
// grid = (slices, H_kv, batch).  `units` is the level's summary array.
template <int LEVEL>
__global__ __launch_bounds__(kSelThreads) void select_level_kernel(const uint16_t* __restrict__ q,
                                                                   const float* __restrict__ units,
                                                                   const int32_t* __restrict__ seq_lens, Geom g,
                                                                   SelectParams sp, SelectWs ws,
                                                                   int32_t* __restrict__ page_ids,
                                                                   int32_t* __restrict__ n_selected)
{
    extern __shared__ unsigned long long lds_raw[];                  // [slot cap of this level], last arriver only
    uint64_t* lds_keys = reinterpret_cast<uint64_t*>(lds_raw);
    __shared__ Shared sh;

    const int slice = blockIdx.x, h = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
    const int grp = tid >> 4, ln = tid & 15;
#ifdef CHESS_PROF_LEVEL
    const long long prof_t0 = wall_clock64();
#endif
    const size_t row = (size_t)b * g.n_kv_heads + h;
    int32_t* meta = ws.meta + row * kSelMetaStride;                  // [0] kept grids, [1] kept chunks, [2..4] arrivals
    int32_t* kept_grids = ws.kept_grids + row * g.max_grids;
    int32_t* kept_chunks = ws.kept_chunks + row * g.max_chunks;
    uint64_t* keys_g = ws.keys + row * g.max_pages;

    // independent loads first: length, parent count, this lane group's parent entries
    const int B = g.page_size;
    const int L_raw = seq_lens[b];
    const int n_parent = LEVEL == 1 ? 0 : meta[LEVEL - 2];
    const int fan = LEVEL == 2 ? g.n_g : g.n_c;                      // children per parent
    const int slot_a = slice * kSlice + grp, slot_b = slot_a + 16;
    int par_a = 0, par_b = 0;
    if (LEVEL != 1) {
        const int32_t* list = LEVEL == 2 ? kept_grids : kept_chunks;
        const int cap = LEVEL == 2 ? g.max_grids : g.max_chunks;
        par_a = list[min(slot_a / fan, cap - 1)];
        par_b = list[min(slot_b / fan, cap - 1)];
    }
    const int L = min(max(L_raw, 0), g.max_pages * B);
    const int P = (L + B - 1) / B;
    const int s = sp.sink, w = sp.window;
    int32_t* ids = page_ids + row * g.max_sel;
    if (P <= s + w) {                                                // safety pages cover the sequence
        if (slice == 0) {
            if (LEVEL == 1) {
                for (int i = tid; i < g.max_sel; i += kSelThreads) ids[i] = i < P ? i : -1;
                if (tid == 0) { n_selected[row] = min(P, g.max_sel); meta[0] = 0; }
            }
            if (LEVEL == 2 && tid == 0) meta[1] = 0;
        }
        return;
    }
    const int nc = ceil_div_i(P, g.n_c), ng = ceil_div_i(nc, g.n_g);
    const int n_slots = LEVEL == 1 ? ng : n_parent * fan;
    const int n_wg = ceil_div_i(n_slots, kSlice);
    if (slice >= n_wg) {
        if (LEVEL == 2 && n_wg == 0 && slice == 0 && tid == 0) meta[1] = 0;
        if (LEVEL == 3 && n_wg == 0 && slice == 0) {                 // no candidate chunk: safety pages only
            for (int i = tid; i < g.max_sel; i += kSelThreads) ids[i] = i < s ? i : (i < s + w ? P - w + i - s : -1);
            if (tid == 0) n_selected[row] = s + w;
        }
        return;
    }

    // slot -> unit of this level, -1 if the slot has no unit (past the end, or a safety page)
    auto unit_of = [&](int slot, int parent) {
        if (slot >= n_slots) return -1;
        if (LEVEL == 1) return slot;
        const int u = parent * fan + slot % fan;
        if (LEVEL == 2) return u < nc ? u : -1;
        return (u >= s && u < P - w) ? u : -1;
    };
    const int ua = unit_of(slot_a, par_a), ub = unit_of(slot_b, par_b);
    const size_t stride = LEVEL == 1 ? g.max_grids : (LEVEL == 2 ? g.max_chunks : g.max_pages);
    const float* base = units + row * stride * kHeadDim;
    float4 a0 = make_float4(0, 0, 0, 0), a1 = a0, b0 = a0, b1 = a0;
    if (ua >= 0) {
        const float4* p = reinterpret_cast<const float4*>(base + (size_t)ua * kHeadDim) + ln * 2;
        a0 = p[0]; a1 = p[1];
    }
    if (ub >= 0) {
        const float4* p = reinterpret_cast<const float4*>(base + (size_t)ub * kHeadDim) + ln * 2;
        b0 = p[0]; b1 = p[1];
    }
    // probe: sum of the group's query rows (dims 8*ln .. 8*ln+7 of this lane), g ascending
    double pr[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int r = 0; r < g.group; ++r) {
        const uint4 v = *reinterpret_cast<const uint4*>(q + ((size_t)b * g.n_q_heads + h * g.group + r) * kHeadDim + ln * 8);
        pr[0] += (double)__uint_as_float(v.x << 16); pr[1] += (double)__uint_as_float(v.x & 0xffff0000u);
        pr[2] += (double)__uint_as_float(v.y << 16); pr[3] += (double)__uint_as_float(v.y & 0xffff0000u);
        pr[4] += (double)__uint_as_float(v.z << 16); pr[5] += (double)__uint_as_float(v.z & 0xffff0000u);
        pr[6] += (double)__uint_as_float(v.w << 16); pr[7] += (double)__uint_as_float(v.w & 0xffff0000u);
    }
    double da = dot8(pr, a0, a1), db = dot8(pr, b0, b1);
#pragma unroll
    for (int off = 8; off >= 1; off >>= 1) {
        da += __shfl_xor(da, off);
        db += __shfl_xor(db, off);
    }
    if (ln == 0) {
        if (slot_a < n_slots) publish_u64(keys_g + slot_a, ua >= 0 ? order_key(da) : 0ull);
        if (slot_b < n_slots) publish_u64(keys_g + slot_b, ub >= 0 ? order_key(db) : 0ull);
    }
#ifdef CHESS_PROF_LEVEL
    const long long prof_t1 = wall_clock64();
#endif
    if (!arrive_last(&meta[1 + LEVEL], n_wg, &sh.last)) return;
#ifdef CHESS_PROF_LEVEL
    const long long prof_t2 = wall_clock64();
#endif

    // ---- last workgroup of this (sequence, head): cut and compact
    for (int i = tid; i < n_slots; i += kSelThreads) lds_keys[i] = observe_u64(keys_g + i);
    __syncthreads();
    const int k_budget = sp.budget_pages > 0 ? sp.budget_pages : clamp_i(ceil_bp(P, sp.budget_bp), 1, P);
    const int kc_target = ceil_div_i(sp.over_chunk * k_budget, g.n_c);
    const int plan = sp.plan;
    auto k_of = [&](int n) {
        if (LEVEL == 1) {
            const int k = plan == CHESS_PLAN_RATIO ? clamp_i(ceil_bp(n, sp.rho_g_bp), 1, n)
                        : plan == CHESS_PLAN_FLAT  ? n
                                                   : min(n, ceil_div_i(sp.over_grid * kc_target, g.n_g));
            return min(k, sp.cap2 / g.n_g);                          // never more children than level 2 has room for
        }
        if (LEVEL == 2) {
            const int k = plan == CHESS_PLAN_RATIO ? clamp_i(ceil_bp(n, sp.rho_c_bp), 1, n)
                        : plan == CHESS_PLAN_FLAT  ? n
                                                   : min(n, kc_target);
            return min(k, sp.cap3 / g.n_c);
        }
        const int k = plan == CHESS_PLAN_RATIO ? (n == 0 ? 0 : clamp_i(ceil_bp(n, sp.rho_p_bp), 1, n)) : min(n, k_budget);
        return min(k, g.max_sel - s - w);
    };
    uint64_t thr;
    int ties;
#ifdef CHESS_PROF_LEVEL
    const long long prof_t3 = wall_clock64();
#endif
    radix_cut(lds_keys, n_slots, k_of, sh, &thr, &ties);
#ifdef CHESS_PROF_LEVEL
    const long long prof_t4 = wall_clock64();
#endif
    // the parent of a slot, for the compaction's slot -> unit map (read again from the global list)
    auto unit_of_slot = [&](int slot) {
        if (LEVEL == 1) return slot;
        const int32_t* list = LEVEL == 2 ? kept_grids : kept_chunks;
        return list[slot / fan] * fan + slot % fan;
    };
    if (LEVEL == 1) {
        const int n = compact_kept(lds_keys, n_slots, thr, ties, unit_of_slot,
                                   [&](int pos, int unit) { kept_grids[pos] = unit; }, sh);
        if (tid == 0) meta[0] = n;
    } else if (LEVEL == 2) {
        const int n = compact_kept(lds_keys, n_slots, thr, ties, unit_of_slot,
                                   [&](int pos, int unit) { kept_chunks[pos] = unit; }, sh);
        if (tid == 0) meta[1] = n;
    } else {
        const int n_kp = compact_kept(lds_keys, n_slots, thr, ties, unit_of_slot,
                                      [&](int pos, int unit) { ids[s + pos] = unit; }, sh);
        // union with the safety pages: sinks, kept pages, window -- already ascending
        const int n_sel = s + n_kp + w;
        for (int i = tid; i < s; i += kSelThreads) ids[i] = i;
        for (int i = tid; i < w; i += kSelThreads) ids[s + n_kp + i] = P - w + i;
        for (int i = n_sel + tid; i < g.max_sel; i += kSelThreads) ids[i] = -1;
        if (tid == 0) n_selected[row] = n_sel;
    }
#ifdef CHESS_PROF_LEVEL
    if (LEVEL == CHESS_PROF_LEVEL && tid == 0) {      // ticks of 10 ns, last workgroup of the row only
        ws.prof[row * 8 + 0] = (int)(prof_t1 - prof_t0);          // entry -> scored and published
        ws.prof[row * 8 + 1] = (int)(prof_t2 - prof_t1);          // arrival
        ws.prof[row * 8 + 2] = (int)(prof_t3 - prof_t2);          // pull keys
        ws.prof[row * 8 + 3] = (int)(prof_t4 - prof_t3);          // radix cut
        ws.prof[row * 8 + 4] = (int)(wall_clock64() - prof_t4);   // compaction + output
    }
#endif
}

hipError_t launch_select(chess_ctx* ctx, const uint16_t* q, const float* pages, const float* chunks,
                         const float* grids, const int32_t* seq_lens, int batch, const SelectParams& sp,
                         const SelectWs& ws, int32_t* page_ids, int32_t* n_selected, hipStream_t stream)
{
    const Geom& g = ctx->geom;
    const int caps[3] = {g.max_grids, sp.cap2, sp.cap3};
    const float* units[3] = {grids, chunks, pages};
    for (int lvl = 0; lvl < 3; ++lvl) {
        const size_t lds = (size_t)caps[lvl] * 8;
        auto kern = lvl == 0 ? select_level_kernel<1> : (lvl == 1 ? select_level_kernel<2> : select_level_kernel<3>);
        if (lds > 48 * 1024) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
        }
        const dim3 grid((caps[lvl] + kSlice - 1) / kSlice, g.n_kv_heads, batch), block(kSelThreads);
        hipError_t e = launch(kern, grid, block, lds, stream, q, units[lvl], seq_lens, g, sp,
                                    ws, page_ids, n_selected);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace chess
