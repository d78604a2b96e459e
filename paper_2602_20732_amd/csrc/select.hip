// Coarse-to-fine page selection (Sec. 3.2, Eq. 4, Alg. 1 stage 2) for one (sequence, KV head) per
// workgroup of 1024 threads.
//
// The paper scores the whole hierarchy with one GEMM and prunes with masks; here scoring is lazy:
// all grids, then only the chunks of kept grids, then only the pages of kept chunks, so a level's
// HBM reads are its candidates' 512-byte vectors and nothing else.  A 16-lane group scores one unit
// (two 128-bit loads per lane, fp64 multiply-add, 4-step butterfly), writes an order-preserving
// 64-bit key to LDS; the k-th largest key is found by an 8-bit radix select over LDS, ties at the
// cut go to the lowest candidate slots (= lowest indices, candidates are enumerated in index
// order), and an ordered compaction turns the keep mask into the ascending list of kept units that
// drives the next level.  Nothing but the final page list leaves the workgroup.
#include "chess_internal.h"

namespace chess {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / kWave;

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
    int digit, rem, cnt, n_valid, k;
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

// Eq. 4 for the candidate slots [0, n_slots): slot -> unit via `unit_of` (-1 = no such unit).
template <class Map>
__device__ __forceinline__ void score_slots(const float* __restrict__ base, int n_slots, Map unit_of,
                                            const double (&pr)[8], uint64_t* keys)
{
    const int grp = threadIdx.x >> 4, ln = threadIdx.x & 15;
    constexpr int n_grp = kSelThreads / 16;
    const int n_iter = ceil_div_i(n_slots, 2 * n_grp);
    for (int it = 0; it < n_iter; ++it) {
        const int sa = grp + it * 2 * n_grp, sb = sa + n_grp;
        const int ua = sa < n_slots ? unit_of(sa) : -1;
        const int ub = sb < n_slots ? unit_of(sb) : -1;
        float4 a0 = make_float4(0, 0, 0, 0), a1 = a0, b0 = a0, b1 = a0;
        if (ua >= 0) {
            const float4* p = reinterpret_cast<const float4*>(base + (size_t)ua * kHeadDim) + ln * 2;
            a0 = p[0]; a1 = p[1];
        }
        if (ub >= 0) {
            const float4* p = reinterpret_cast<const float4*>(base + (size_t)ub * kHeadDim) + ln * 2;
            b0 = p[0]; b1 = p[1];
        }
        double da = 0.0, db = 0.0;
        da = fma(pr[0], (double)a0.x, da); da = fma(pr[1], (double)a0.y, da);
        da = fma(pr[2], (double)a0.z, da); da = fma(pr[3], (double)a0.w, da);
        da = fma(pr[4], (double)a1.x, da); da = fma(pr[5], (double)a1.y, da);
        da = fma(pr[6], (double)a1.z, da); da = fma(pr[7], (double)a1.w, da);
        db = fma(pr[0], (double)b0.x, db); db = fma(pr[1], (double)b0.y, db);
        db = fma(pr[2], (double)b0.z, db); db = fma(pr[3], (double)b0.w, db);
        db = fma(pr[4], (double)b1.x, db); db = fma(pr[5], (double)b1.y, db);
        db = fma(pr[6], (double)b1.z, db); db = fma(pr[7], (double)b1.w, db);
#pragma unroll
        for (int off = 8; off >= 1; off >>= 1) {
            da += __shfl_xor(da, off);
            db += __shfl_xor(db, off);
        }
        if (ln == 0) {
            if (sa < n_slots) keys[sa] = ua >= 0 ? order_key(da) : 0ull;
            if (sb < n_slots) keys[sb] = ub >= 0 ? order_key(db) : 0ull;
        }
    }
}

// Find the cut of the top-k among the non-empty keys.  k = k_of(number of non-empty keys).
// On return (uniform over the workgroup): a slot is kept iff key > thr, or key == thr and it is
// among the first `ties` such slots.  Returns k.
template <class KFn>
__device__ __forceinline__ int radix_cut(const uint64_t* keys, int n_slots, KFn k_of, Shared& sh,
                                         uint64_t* thr_out, int* ties_out)
{
    const int tid = threadIdx.x;
    uint64_t prefix = 0, mask = 0;
    int rem = 0, k = 0;
    for (int pass = 7; pass >= 0; --pass) {
        const int shift = pass * 8;
        if (tid < 256) sh.hist[tid] = 0;
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
                int t = excl, digit = d0, cnt = c0;
                if (t + c0 >= want) { digit = d0; cnt = c0; }
                else if ((t += c0) + c1 >= want) { digit = d0 - 1; cnt = c1; }
                else if ((t += c1) + c2 >= want) { digit = d0 - 2; cnt = c2; }
                else { t += c2; digit = d0 - 3; cnt = c3; }
                sh.digit = digit; sh.rem = want - t; sh.cnt = cnt;
            }
        }
        __syncthreads();
        if (pass == 7) {
            k = sh.k;
            if (k <= 0) { *thr_out = ~0ull; *ties_out = 0; __syncthreads(); return 0; }
            if (k >= sh.n_valid) { *thr_out = 0ull; *ties_out = 0; __syncthreads(); return sh.n_valid; }
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
    return k;
}

// Ordered compaction of the kept slots: out[pos] = unit_of(slot), ascending slot order.
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

__global__ __launch_bounds__(kSelThreads) void select_kernel(const uint16_t* __restrict__ q,
                                                             const float* __restrict__ pages,
                                                             const float* __restrict__ chunks,
                                                             const float* __restrict__ grids,
                                                             const int32_t* __restrict__ seq_lens, Geom g,
                                                             SelectParams sp, int32_t* __restrict__ page_ids,
                                                             int32_t* __restrict__ n_selected)
{
    extern __shared__ unsigned long long dyn[];
    uint64_t* keys = reinterpret_cast<uint64_t*>(dyn);               // [slot_cap]
    int32_t* kept_grids = reinterpret_cast<int32_t*>(keys + sp.slot_cap);   // [list_cap]
    int32_t* kept_chunks = kept_grids + sp.list_cap;                        // [list_cap]
    __shared__ Shared sh;

    const int h = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const size_t row = (size_t)b * g.n_kv_heads + h;
    int32_t* ids = page_ids + row * g.max_sel;
    const int B = g.page_size;
    const int L = min(max(seq_lens[b], 0), g.max_pages * B);
    const int P = (L + B - 1) / B;
    const int s = sp.sink, w = sp.window;
    if (P <= s + w) {                                                 // safety pages cover the sequence
        for (int i = tid; i < g.max_sel; i += kSelThreads) ids[i] = i < P ? i : -1;
        if (tid == 0) n_selected[row] = min(P, g.max_sel);
        return;
    }
    const int nc = ceil_div_i(P, g.n_c), ng = ceil_div_i(nc, g.n_g);

    // probe: sum of the group's query rows (dims 8*ln .. 8*ln+7 of this lane), g ascending
    double pr[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    {
        const int ln = tid & 15;
        for (int r = 0; r < g.group; ++r) {
            const uint4 v = *reinterpret_cast<const uint4*>(q + ((size_t)b * g.n_q_heads + h * g.group + r) * kHeadDim + ln * 8);
            pr[0] += (double)__uint_as_float(v.x << 16); pr[1] += (double)__uint_as_float(v.x & 0xffff0000u);
            pr[2] += (double)__uint_as_float(v.y << 16); pr[3] += (double)__uint_as_float(v.y & 0xffff0000u);
            pr[4] += (double)__uint_as_float(v.z << 16); pr[5] += (double)__uint_as_float(v.z & 0xffff0000u);
            pr[6] += (double)__uint_as_float(v.w << 16); pr[7] += (double)__uint_as_float(v.w & 0xffff0000u);
        }
    }

    const int k_budget = sp.budget_pages > 0 ? sp.budget_pages : clamp_i(ceil_bp(P, sp.budget_bp), 1, P);
    const int kc_target = ceil_div_i(sp.over_chunk * k_budget, g.n_c);
    const int plan = sp.plan;
    uint64_t thr;
    int ties;

    // ---- level 1: every grid
    {
        const float* base = grids + row * g.max_grids * kHeadDim;
        auto unit_of = [&](int slot) { return slot; };
        score_slots(base, ng, unit_of, pr, keys);
        __syncthreads();
        auto k_of = [&](int n) {
            int k = plan == CHESS_PLAN_RATIO ? clamp_i(ceil_bp(n, sp.rho_g_bp), 1, n)
                  : plan == CHESS_PLAN_FLAT  ? n
                                             : min(n, ceil_div_i(sp.over_grid * kc_target, g.n_g));
            return min(k, min(sp.list_cap, sp.slot_cap / g.n_g));
        };
        radix_cut(keys, ng, k_of, sh, &thr, &ties);
    }
    const int n_kg = compact_kept(keys, ng, thr, ties, [&](int slot) { return slot; },
                                  [&](int pos, int unit) { kept_grids[pos] = unit; }, sh);

    // ---- level 2: chunks of kept grids
    const int slots2 = n_kg * g.n_g;
    auto chunk_of = [&](int slot) {
        const int c = kept_grids[slot / g.n_g] * g.n_g + slot % g.n_g;
        return c < nc ? c : -1;
    };
    {
        const float* base = chunks + row * g.max_chunks * kHeadDim;
        score_slots(base, slots2, chunk_of, pr, keys);
        __syncthreads();
        auto k_of = [&](int n) {
            int k = plan == CHESS_PLAN_RATIO ? clamp_i(ceil_bp(n, sp.rho_c_bp), 1, n)
                  : plan == CHESS_PLAN_FLAT  ? n
                                             : min(n, kc_target);
            return min(k, min(sp.list_cap, sp.slot_cap / g.n_c));
        };
        radix_cut(keys, slots2, k_of, sh, &thr, &ties);
    }
    const int n_kc = compact_kept(keys, slots2, thr, ties, chunk_of,
                                  [&](int pos, int unit) { kept_chunks[pos] = unit; }, sh);

    // ---- level 3: pages of kept chunks, sink and window pages are not candidates
    const int slots3 = n_kc * g.n_c;
    auto page_of = [&](int slot) {
        const int p = kept_chunks[slot / g.n_c] * g.n_c + slot % g.n_c;
        return (p >= s && p < P - w) ? p : -1;
    };
    {
        const float* base = pages + row * g.max_pages * kHeadDim;
        score_slots(base, slots3, page_of, pr, keys);
        __syncthreads();
        auto k_of = [&](int n) {
            int k = plan == CHESS_PLAN_RATIO ? (n == 0 ? 0 : clamp_i(ceil_bp(n, sp.rho_p_bp), 1, n))
                                             : min(n, k_budget);
            return min(k, g.max_sel - s - w);
        };
        radix_cut(keys, slots3, k_of, sh, &thr, &ties);
    }
    const int n_kp = compact_kept(keys, slots3, thr, ties, page_of,
                                  [&](int pos, int unit) { ids[s + pos] = unit; }, sh);

    // ---- union with the safety pages: sinks, kept pages, window -- already ascending
    const int n_sel = s + n_kp + w;
    for (int i = tid; i < s; i += kSelThreads) ids[i] = i;
    for (int i = tid; i < w; i += kSelThreads) ids[s + n_kp + i] = P - w + i;
    for (int i = n_sel + tid; i < g.max_sel; i += kSelThreads) ids[i] = -1;
    if (tid == 0) n_selected[row] = n_sel;
}

hipError_t launch_select(chess_ctx* ctx, const uint16_t* q, const float* pages, const float* chunks,
                         const float* grids, const int32_t* seq_lens, int batch, const SelectParams& sp,
                         size_t lds_bytes, int32_t* page_ids, int32_t* n_selected, hipStream_t stream)
{
    if (lds_bytes > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(select_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
    }
    const dim3 grid(ctx->geom.n_kv_heads, batch), block(kSelThreads);
    return timed_launch(ctx, CHESS_K_SELECT, select_kernel, grid, block, lds_bytes, stream, q, pages, chunks, grids,
                        seq_lens, ctx->geom, sp, page_ids, n_selected);
}

}  // namespace chess
