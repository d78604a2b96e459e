// Coarse-to-fine page selection (Sec. 3.2, Eq. 4, Alg. 1 stage 2) in one launch: a cluster of C
// workgroups cooperates on each (sequence, KV head) through all three levels.
//
// The paper scores the whole hierarchy with one GEMM and prunes with masks.  Here scoring is lazy --
// a level reads only the 512-byte vectors of its candidates (all grids, chunks of kept grids, pages
// of kept chunks) -- and a level's candidates are split over the cluster so that one (sequence,
// head) draws bandwidth from C compute units.  A 16-lane group scores one unit (two 128-bit loads
// per lane, fp64 multiply-add, 4-step butterfly) and the group leader publishes an order-preserving
// 64-bit key.  After a cluster barrier every member pulls the level's keys into LDS and finds the
// cut itself (the members compute the same thing; that is cheaper than a second barrier): common
// leading bits are stripped, then an 8-bit radix select runs until the bin at the cut is taken
// whole; ties at the cut go to the lowest slots (= lowest indices: candidates are enumerated in
// index order); a ballot compaction turns the keep mask into the ascending list of kept units that
// drives the next level.  Member 0 writes the final list: sinks, kept pages, window pages.
//
// Clusters of different (sequence, head) pairs never wait for each other.  Keys cross workgroups as
// agent-scope atomics (coherent across the XCDs' L2s).  The cluster barrier spins, so the host only
// launches clusters when every workgroup of the grid can be resident at once, and the spin is
// bounded: a wait that does not end raises the workspace's error flag and the workgroup leaves.
#include "chess_internal.h"

namespace chess {

constexpr int kSelWaves = kSelThreads / kWave;
constexpr int kSpinLimit = 1 << 18;         // ~50 ms of polling before a barrier is declared dead
constexpr int kKeepAll = 0x7fffffff;

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

// Inclusive scan over the 64 lanes of a wave with DPP row shifts and row broadcasts (no LDS).
// Every lane of the wave must be active.
template <class Op>
__device__ __forceinline__ int wave_scan(int v, const int identity, Op op)
{
    v = op(v, __builtin_amdgcn_update_dpp(identity, v, 0x111, 0xf, 0xf, false));   // row_shr:1
    v = op(v, __builtin_amdgcn_update_dpp(identity, v, 0x112, 0xf, 0xf, false));   // row_shr:2
    v = op(v, __builtin_amdgcn_update_dpp(identity, v, 0x114, 0xf, 0xf, false));   // row_shr:4
    v = op(v, __builtin_amdgcn_update_dpp(identity, v, 0x118, 0xf, 0xf, false));   // row_shr:8
    v = op(v, __builtin_amdgcn_update_dpp(identity, v, 0x142, 0xa, 0xf, false));   // row_bcast:15 -> rows 1, 3
    v = op(v, __builtin_amdgcn_update_dpp(identity, v, 0x143, 0xc, 0xf, false));   // row_bcast:31 -> rows 2, 3
    return v;
}

constexpr int kBins = 1024;                 // linear score bins of the first cut pass
constexpr int kMaxMembers = 256;            // most keys the bin at the cut may hold for the exact ranking

struct Shared {
    int hist[kBins];
    uint64_t mem_key[kMaxMembers];
    int mem_slot[kMaxMembers];
    int wave_a[kSelWaves], wave_b[kSelWaves];
    int digit, rem, cnt, n_valid, ok, n_mem;
    unsigned int or_lo, or_hi, and_lo, and_hi;
    unsigned long long kmin, kmax, thr;
};

// order_key's inverse, for binning
__device__ __forceinline__ double key_score(uint64_t key)
{
    const uint64_t u = (key >> 63) ? (key & 0x7fffffffffffffffull) : ~key;
    return __longlong_as_double((long long)u);
}

// Minimum / maximum of a 64-bit value over the wave (DPP, no LDS); the result is in lane 63.
template <bool kMin>
__device__ __forceinline__ uint64_t wave_minmax(uint64_t v)
{
    const int id = kMin ? -1 : 0;
#define CHESS_MM_STEP(ctrl, rows)                                                                      \
    {                                                                                                  \
        const unsigned lo = (unsigned)__builtin_amdgcn_update_dpp(id, (int)(unsigned)v, ctrl, rows, 0xf, false); \
        const unsigned hi = (unsigned)__builtin_amdgcn_update_dpp(id, (int)(unsigned)(v >> 32), ctrl, rows, 0xf, false); \
        const uint64_t o = ((uint64_t)hi << 32) | lo;                                                  \
        v = kMin ? (o < v ? o : v) : (o > v ? o : v);                                                  \
    }
    CHESS_MM_STEP(0x111, 0xf) CHESS_MM_STEP(0x112, 0xf) CHESS_MM_STEP(0x114, 0xf) CHESS_MM_STEP(0x118, 0xf)
    CHESS_MM_STEP(0x142, 0xa) CHESS_MM_STEP(0x143, 0xc)
#undef CHESS_MM_STEP
    return v;
}

// Sum of a double over each row of 16 lanes (DPP row shifts); the total is in lane 15 of the row.
__device__ __forceinline__ double row16_sum(double d)
{
#define CHESS_RS_STEP(ctrl)                                                                            \
    {                                                                                                  \
        const uint64_t b = (uint64_t)__double_as_longlong(d);                                          \
        const unsigned lo = (unsigned)__builtin_amdgcn_update_dpp(0, (int)(unsigned)b, ctrl, 0xf, 0xf, false); \
        const unsigned hi = (unsigned)__builtin_amdgcn_update_dpp(0, (int)(unsigned)(b >> 32), ctrl, 0xf, 0xf, false); \
        d += __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));                             \
    }
    CHESS_RS_STEP(0x111) CHESS_RS_STEP(0x112) CHESS_RS_STEP(0x114) CHESS_RS_STEP(0x118)
#undef CHESS_RS_STEP
    return d;
}

struct Cut {
    uint64_t thr;   // in the shifted domain: key << shift
    int ties;       // how many of the slots whose shifted key equals thr are kept, lowest slots first
    int shift;
};

// Cut of the top-k among the non-empty keys in LDS by radix select alone: the fallback of find_cut for
// score distributions that pile more than kMaxMembers keys into one linear bin.  Same contract.
template <class KFn>
__device__ __forceinline__ Cut find_cut_radix(const uint64_t* keys, int n_slots, KFn k_of, Shared& sh)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // what the keys have in common: OR, AND and the number of non-empty ones
    unsigned int o_lo = 0, o_hi = 0, a_lo = ~0u, a_hi = ~0u;
    int nv = 0;
    for (int i = tid; i < n_slots; i += kSelThreads) {
        const uint64_t k = keys[i];
        if (k) { o_lo |= (unsigned)k; o_hi |= (unsigned)(k >> 32); a_lo &= (unsigned)k; a_hi &= (unsigned)(k >> 32); ++nv; }
    }
    if (tid == 0) { sh.or_lo = 0; sh.or_hi = 0; sh.and_lo = ~0u; sh.and_hi = ~0u; sh.n_valid = 0; }
    __syncthreads();
    auto f_or = [](int a, int b) { return a | b; };
    auto f_and = [](int a, int b) { return a & b; };
    auto f_add = [](int a, int b) { return a + b; };
    o_lo = (unsigned)wave_scan((int)o_lo, 0, f_or);   o_hi = (unsigned)wave_scan((int)o_hi, 0, f_or);
    a_lo = (unsigned)wave_scan((int)a_lo, -1, f_and); a_hi = (unsigned)wave_scan((int)a_hi, -1, f_and);
    nv = wave_scan(nv, 0, f_add);
    if (lane == 63) {
        atomicOr(&sh.or_lo, o_lo); atomicOr(&sh.or_hi, o_hi);
        atomicAnd(&sh.and_lo, a_lo); atomicAnd(&sh.and_hi, a_hi);
        atomicAdd(&sh.n_valid, nv);
    }
    __syncthreads();
    const int n_valid = sh.n_valid;
    const uint64_t all_or = ((uint64_t)sh.or_hi << 32) | sh.or_lo, all_and = ((uint64_t)sh.and_hi << 32) | sh.and_lo;
    const int k = k_of(n_valid);
    Cut cut;
    cut.shift = 0;
    if (k <= 0) { cut.thr = ~0ull; cut.ties = 0; return cut; }
    if (k >= n_valid) { cut.thr = 0ull; cut.ties = kKeepAll; return cut; }
    const uint64_t diff = all_or ^ all_and;
    if (diff == 0) { cut.thr = all_or; cut.ties = k; return cut; }    // every key is the same: first k slots
    const int shift = __clzll((long long)diff);
    cut.shift = shift;
    const int n_pass = (64 - shift + 7) / 8;
    uint64_t prefix = 0;
    int want = k;
    for (int p = 0; p < n_pass; ++p) {
        sh.hist[tid] = 0;                              // kSelThreads == 256 bins
        __syncthreads();
        for (int i = tid; i < n_slots; i += kSelThreads) {
            const uint64_t key = keys[i];
            const uint64_t sk = key << shift;
            if (key != 0 && (p == 0 || (sk >> (64 - 8 * p)) == prefix))
                atomicAdd(&sh.hist[(int)((sk >> (56 - 8 * p)) & 255)], 1);
        }
        __syncthreads();
        // thread t looks at digit 255 - t, so thread order is digit order descending
        const int c = sh.hist[255 - tid];
        const int incl_w = wave_scan(c, 0, f_add);
        if (lane == 63) sh.wave_a[wave] = incl_w;
        __syncthreads();
        int base = 0;
#pragma unroll
        for (int w = 0; w < kSelWaves; ++w) base += w < wave ? sh.wave_a[w] : 0;
        const int incl = base + incl_w, excl = incl - c;
        if (excl < want && want <= incl) { sh.digit = 255 - tid; sh.rem = want - excl; sh.cnt = c; }
        __syncthreads();
        prefix = (prefix << 8) | (uint64_t)sh.digit;
        want = sh.rem;
        if (sh.cnt == want) {                          // the whole bin at the cut is kept
            cut.thr = prefix << (56 - 8 * p);
            cut.ties = kKeepAll;
            return cut;
        }
    }
    cut.thr = n_pass >= 8 ? prefix : prefix << (64 - 8 * n_pass);
    cut.ties = want;
    return cut;
}

// Find the cut of the top-k among the non-empty keys in LDS.  k = k_of(number of non-empty keys).
// A non-empty slot is kept iff (key << shift) > thr, or (key << shift) == thr and it is among the
// first `ties` such slots.  Uniform over the workgroup; every thread must call it.
//
// One histogram pass over kBins bins that are LINEAR in the score between the smallest and the largest
// (a monotone map, so a higher bin means a strictly larger score), a scan from the top finds the bin
// the k-th largest key falls in, and the few keys of that bin are ranked exactly by (key, slot).
template <class KFn>
__device__ __forceinline__ Cut find_cut(const uint64_t* keys, int n_slots, KFn k_of, Shared& sh)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    auto f_add = [](int a, int b) { return a + b; };
    uint64_t lo_k = ~0ull, hi_k = 0ull;
    int nv = 0;
    for (int i = tid; i < n_slots; i += kSelThreads) {
        const uint64_t k = keys[i];
        if (k) { lo_k = k < lo_k ? k : lo_k; hi_k = k > hi_k ? k : hi_k; ++nv; }
    }
    if (tid == 0) { sh.kmin = ~0ull; sh.kmax = 0ull; sh.n_valid = 0; sh.n_mem = 0; }
#pragma unroll
    for (int j = 0; j < kBins / kSelThreads; ++j) sh.hist[tid + j * kSelThreads] = 0;
    __syncthreads();
    lo_k = wave_minmax<true>(lo_k);
    hi_k = wave_minmax<false>(hi_k);
    nv = wave_scan(nv, 0, f_add);
    if (lane == 63) {
        atomicMin(&sh.kmin, (unsigned long long)lo_k);
        atomicMax(&sh.kmax, (unsigned long long)hi_k);
        atomicAdd(&sh.n_valid, nv);
    }
    __syncthreads();
    const int n_valid = sh.n_valid;
    const uint64_t kmin = sh.kmin, kmax = sh.kmax;
    const int k = k_of(n_valid);
    Cut cut;
    cut.shift = 0;
    if (k <= 0) { cut.thr = ~0ull; cut.ties = 0; return cut; }
    if (k >= n_valid) { cut.thr = 0ull; cut.ties = kKeepAll; return cut; }
    if (kmin == kmax) { cut.thr = kmin; cut.ties = k; return cut; }      // every key is the same: first k slots
    const double smin = key_score(kmin);
    const double scale = (double)kBins / (key_score(kmax) - smin);
    auto bin_of = [&](uint64_t key) {
        const int b = (int)((key_score(key) - smin) * scale);
        return min(max(b, 0), kBins - 1);
    };
    for (int i = tid; i < n_slots; i += kSelThreads) {
        const uint64_t key = keys[i];
        if (key) atomicAdd(&sh.hist[bin_of(key)], 1);
    }
    __syncthreads();
    // thread t owns bins kBins-1-4t .. kBins-4-4t, so thread order is score order descending
    constexpr int kPer = kBins / kSelThreads;
    int c[kPer], own = 0;
#pragma unroll
    for (int j = 0; j < kPer; ++j) { c[j] = sh.hist[kBins - 1 - kPer * tid - j]; own += c[j]; }
    const int incl_w = wave_scan(own, 0, f_add);
    if (lane == 63) sh.wave_a[wave] = incl_w;
    __syncthreads();
    int above = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) above += w < wave ? sh.wave_a[w] : 0;
    above += incl_w - own;                                    // keys in bins above this thread's
    if (above < k && k <= above + own) {
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            if (above < k && k <= above + c[j]) { sh.digit = kBins - 1 - kPer * tid - j; sh.rem = k - above; sh.cnt = c[j]; }
            above += c[j];
        }
    }
    __syncthreads();
    const int bin = sh.digit, want = sh.rem, cnt = sh.cnt;
    if (cnt > kMaxMembers) return find_cut_radix(keys, n_slots, k_of, sh);
    for (int i = tid; i < n_slots; i += kSelThreads) {
        const uint64_t key = keys[i];
        if (key && bin_of(key) == bin) {
            const int at = atomicAdd(&sh.n_mem, 1);
            sh.mem_key[at] = key;
            sh.mem_slot[at] = i;
        }
    }
    __syncthreads();
    if (tid < cnt) {                                          // exact rank of member tid by (key desc, slot asc)
        const uint64_t mine = sh.mem_key[tid];
        const int my_slot = sh.mem_slot[tid];
        int rank = 0, n_gt = 0;
        for (int j = 0; j < cnt; ++j) {
            const uint64_t kj = sh.mem_key[j];
            n_gt += kj > mine;
            rank += kj > mine || (kj == mine && sh.mem_slot[j] < my_slot);
        }
        if (rank == want - 1) { sh.thr = mine; sh.rem = want - n_gt; }
    }
    __syncthreads();
    cut.thr = sh.thr;
    cut.ties = sh.rem;
    return cut;
}

// Ordered compaction: emit(pos, slot) for the kept slots in ascending slot order; returns their number.
// Wave w owns a contiguous quarter of the slots and walks it 64 slots at a time with ballots.
template <class Out>
__device__ __forceinline__ int compact_kept(const uint64_t* keys, int n_slots, const Cut& cut, Out emit, Shared& sh)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int quarter = ceil_div_i(ceil_div_i(n_slots, kSelWaves), 64) * 64;
    const int lo = min(n_slots, wave * quarter), hi = min(n_slots, lo + quarter);
    const uint64_t below = __lanemask_lt();
    int n_gt = 0, n_eq = 0;
    for (int r = lo; r < hi; r += 64) {
        const int i = r + lane;
        const uint64_t key = i < hi ? keys[i] : 0ull;
        const uint64_t sk = key << cut.shift;
        n_gt += __popcll(__ballot(key != 0 && sk > cut.thr));
        n_eq += __popcll(__ballot(key != 0 && sk == cut.thr));
    }
    if (lane == 0) { sh.wave_a[wave] = n_gt; sh.wave_b[wave] = n_eq; }
    __syncthreads();
    int pos = 0, eq_seen = 0, total = 0, eq_run = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) {
        const int e = sh.wave_b[w];
        const int kept = sh.wave_a[w] + clamp_i(cut.ties - eq_run, 0, e);
        if (w < wave) { pos += kept; eq_seen += e; }
        total += kept;
        eq_run += e;
    }
    for (int r = lo; r < hi; r += 64) {
        const int i = r + lane;
        const uint64_t key = i < hi ? keys[i] : 0ull;
        const uint64_t sk = key << cut.shift;
        const bool gt = key != 0 && sk > cut.thr, eq = key != 0 && sk == cut.thr;
        const uint64_t eqb = __ballot(eq);
        const bool keep = gt || (eq && eq_seen + __popcll(eqb & below) < cut.ties);
        const uint64_t kb = __ballot(keep);
        if (keep) emit(pos + __popcll(kb & below), i);
        pos += __popcll(kb);
        eq_seen += __popcll(eqb);
    }
    __syncthreads();
    return total;
}

// All members of a cluster meet here; returns false if the wait was given up.
__device__ __forceinline__ bool cluster_barrier(int32_t* counter, int target, Shared& sh)
{
    __builtin_amdgcn_s_waitcnt(0);                   // this wave's published keys are acknowledged
    __syncthreads();
    if (threadIdx.x == 0) {
        __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        int spins = 0;
        while (__hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target && spins < kSpinLimit) {
            __builtin_amdgcn_s_sleep(2);
            ++spins;
        }
        sh.ok = spins < kSpinLimit;
    }
    __syncthreads();
    return sh.ok != 0;
}

// Score the slots [lo, hi) of one level: slot -> unit through `unit_of` (-1: no unit), key to `dst[slot]`.
template <bool kDirect, class Map>
__device__ __forceinline__ void score_range(const float* __restrict__ base, int lo, int hi, Map unit_of,
                                            const double (&pr)[8], uint64_t* dst)
{
#ifndef CHESS_FLY
#define CHESS_FLY 8
#endif
    constexpr int kFly = CHESS_FLY;                  // units per 16-lane group in flight
    const int g16 = threadIdx.x >> 4, ln = threadIdx.x & 15;
    for (int s0 = lo; s0 < hi; s0 += 16 * kFly) {
        int slot[kFly], unit[kFly];
        float4 va[kFly], vb[kFly];
#pragma unroll
        for (int x = 0; x < kFly; ++x) {
            slot[x] = s0 + 16 * x + g16;
            unit[x] = slot[x] < hi ? unit_of(slot[x]) : -1;
            // always load (unit 0 when the slot has no unit): a branch here would make the compiler wait
            // for each vector before asking for the next
            const float4* p = reinterpret_cast<const float4*>(base + (size_t)max(unit[x], 0) * kHeadDim) + ln * 2;
            va[x] = p[0];
            vb[x] = p[1];
        }
#pragma unroll
        for (int x = 0; x < kFly; ++x) {
            if (s0 + 16 * x >= hi) break;             // uniform over the workgroup
            double d = 0.0;
            d = fma(pr[0], (double)va[x].x, d); d = fma(pr[1], (double)va[x].y, d);
            d = fma(pr[2], (double)va[x].z, d); d = fma(pr[3], (double)va[x].w, d);
            d = fma(pr[4], (double)vb[x].x, d); d = fma(pr[5], (double)vb[x].y, d);
            d = fma(pr[6], (double)vb[x].z, d); d = fma(pr[7], (double)vb[x].w, d);
            d = row16_sum(d);
            if (ln == 15 && slot[x] < hi) {
                const uint64_t key = unit[x] >= 0 ? order_key(d) : 0ull;
                if (kDirect) dst[slot[x]] = key;
                else publish_u64(dst + slot[x], key);
            }
        }
    }
}

// grid = (C, H_kv, batch); workgroup m of a cluster scores the m-th part of every level.
template <bool kSolo>
__global__ __launch_bounds__(kSelThreads) void select_kernel(const uint16_t* __restrict__ q,
                                                             const float* __restrict__ pages,
                                                             const float* __restrict__ chunks,
                                                             const float* __restrict__ grids,
                                                             const int32_t* __restrict__ seq_lens, Geom g,
                                                             SelectParams sp, SelectWs ws,
                                                             int32_t* __restrict__ page_ids,
                                                             int32_t* __restrict__ n_selected)
{
    extern __shared__ unsigned long long lds_raw[];
    uint64_t* keys = reinterpret_cast<uint64_t*>(lds_raw);                    // [cap_keys]
    int32_t* kept_grids = reinterpret_cast<int32_t*>(keys + sp.cap_keys);     // [cap_kg]
    int32_t* kept_chunks = kept_grids + sp.cap_kg;                            // [cap_kc]
    __shared__ Shared sh;

    const int m = blockIdx.x, C = gridDim.x, h = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
#ifdef CHESS_PROF
    long long prof_t[16];
    int prof_n = 0;
#define PROF_MARK() prof_t[prof_n++] = wall_clock64()
#else
#define PROF_MARK()
#endif
    PROF_MARK();
    const size_t row = (size_t)b * g.n_kv_heads + h;
    int32_t* meta = ws.meta + row * kSelMetaStride;                  // [0] barrier count, [1] exits
    uint64_t* pub1 = ws.keys + row * ws.key_stride;                  // published keys: grids,
    uint64_t* pub2 = pub1 + g.max_grids;                             //   chunk slots,
    uint64_t* pub3 = pub2 + sp.cap2;                                 //   page slots
    int32_t* ids = page_ids + row * g.max_sel;
    const int B = g.page_size;
    const int L_raw = seq_lens[b];
    // probe: sum of the group's query rows (dims 8*ln .. 8*ln+7 of this lane), g ascending; requested
    // before anything waits on the length
    double pr[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int r = 0; r < g.group; ++r) {
        const uint4 v = *reinterpret_cast<const uint4*>(q + ((size_t)b * g.n_q_heads + h * g.group + r) * kHeadDim + (tid & 15) * 8);
        pr[0] += (double)__uint_as_float(v.x << 16); pr[1] += (double)__uint_as_float(v.x & 0xffff0000u);
        pr[2] += (double)__uint_as_float(v.y << 16); pr[3] += (double)__uint_as_float(v.y & 0xffff0000u);
        pr[4] += (double)__uint_as_float(v.z << 16); pr[5] += (double)__uint_as_float(v.z & 0xffff0000u);
        pr[6] += (double)__uint_as_float(v.w << 16); pr[7] += (double)__uint_as_float(v.w & 0xffff0000u);
    }
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
    const int nc = ceil_div_i(P, g.n_c), ng = ceil_div_i(nc, g.n_g);

    const int k_budget = sp.budget_pages > 0 ? sp.budget_pages : clamp_i(ceil_bp(P, sp.budget_bp), 1, P);
    const int kc_target = ceil_div_i(sp.over_chunk * k_budget, g.n_c);
    const int plan = sp.plan;

    // this member's share of a level's slots: whole 16-slot rows
    auto share = [&](int n_slots, int* lo, int* hi) {
        const int per = ceil_div_i(ceil_div_i(n_slots, C), 16) * 16;
        *lo = min(n_slots, m * per);
        *hi = min(n_slots, *lo + per);
    };
    // pull a level's published keys into LDS
    auto pull = [&](const uint64_t* pub, int n_slots) {
        for (int i0 = 0; i0 < n_slots; i0 += 4 * kSelThreads) {
            uint64_t v[4];
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const int i = i0 + x * kSelThreads + tid;
                v[x] = observe_u64(pub + min(i, n_slots - 1));        // unconditional: all four stay in flight
            }
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const int i = i0 + x * kSelThreads + tid;
                if (i < n_slots) keys[i] = v[x];
            }
        }
        __syncthreads();
    };
    // barrier p of this launch, then pull
    auto meet_and_pull = [&](int p, const uint64_t* pub, int n_slots) -> bool {
        if (kSolo) { __syncthreads(); return true; }
        if (!cluster_barrier(&meta[0], p * C, sh)) {
            if (tid == 0) __hip_atomic_store(ws.error, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return false;
        }
        pull(pub, n_slots);
        return true;
    };
    int lo, hi;
    PROF_MARK();                                                      // 1: prologue done

    // ---- level 1: every grid
    share(ng, &lo, &hi);
    score_range<kSolo>(grids + row * g.max_grids * kHeadDim, lo, hi, [&](int slot) { return slot; }, pr,
                       kSolo ? keys : pub1);
    PROF_MARK();                                                      // 2: level 1 scored
    if (!meet_and_pull(1, pub1, ng)) return;
    PROF_MARK();                                                      // 3: barrier + pull
    Cut cut = find_cut(keys, ng, [&](int n) {
        const int k = plan == CHESS_PLAN_RATIO ? clamp_i(ceil_bp(n, sp.rho_g_bp), 1, n)
                    : plan == CHESS_PLAN_FLAT  ? n
                                               : min(n, ceil_div_i(sp.over_grid * kc_target, g.n_g));
        return min(k, sp.cap_kg);
    }, sh);
    PROF_MARK();                                                      // 4: cut
    const int n_kg = compact_kept(keys, ng, cut, [&](int pos, int slot) { kept_grids[pos] = slot; }, sh);
    PROF_MARK();                                                      // 5: compaction

    // ---- level 2: chunks of kept grids
    const int slots2 = n_kg * g.n_g;
    auto chunk_of = [&](int slot) {
        const int c = kept_grids[slot / g.n_g] * g.n_g + slot % g.n_g;
        return c < nc ? c : -1;
    };
    share(slots2, &lo, &hi);
    score_range<kSolo>(chunks + row * g.max_chunks * kHeadDim, lo, hi, chunk_of, pr, kSolo ? keys : pub2);
    PROF_MARK();                                                      // 6: level 2 scored
    if (!meet_and_pull(2, pub2, slots2)) return;
    PROF_MARK();                                                      // 7
    cut = find_cut(keys, slots2, [&](int n) {
        const int k = plan == CHESS_PLAN_RATIO ? clamp_i(ceil_bp(n, sp.rho_c_bp), 1, n)
                    : plan == CHESS_PLAN_FLAT  ? n
                                               : min(n, kc_target);
        return min(k, sp.cap_kc);
    }, sh);
    PROF_MARK();                                                      // 8
    const int n_kc = compact_kept(keys, slots2, cut, [&](int pos, int slot) { kept_chunks[pos] = chunk_of(slot); }, sh);

    PROF_MARK();                                                      // 9
    // ---- level 3: pages of kept chunks; sink and window pages are not candidates
    const int slots3 = n_kc * g.n_c;
    auto page_of = [&](int slot) {
        const int p = kept_chunks[slot / g.n_c] * g.n_c + slot % g.n_c;
        return (p >= s && p < P - w) ? p : -1;
    };
    share(slots3, &lo, &hi);
    score_range<kSolo>(pages + row * g.max_pages * kHeadDim, lo, hi, page_of, pr, kSolo ? keys : pub3);
    PROF_MARK();                                                      // 10: level 3 scored
    if (!kSolo) {
        // after this barrier nobody touches the counter again: the last member to leave re-arms it
        const bool ok = cluster_barrier(&meta[0], 3 * C, sh);
        if (tid == 0) {
            if (!ok) __hip_atomic_store(ws.error, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            else if (__hip_atomic_fetch_add(&meta[1], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == C - 1) {
                __hip_atomic_store(&meta[0], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(&meta[1], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        if (!ok || m != 0) return;
        pull(pub3, slots3);
    }
    __syncthreads();
    PROF_MARK();                                                      // 11: barrier + pull
    cut = find_cut(keys, slots3, [&](int n) {
        const int k = plan == CHESS_PLAN_RATIO ? (n == 0 ? 0 : clamp_i(ceil_bp(n, sp.rho_p_bp), 1, n)) : min(n, k_budget);
        return min(k, g.max_sel - s - w);
    }, sh);
    PROF_MARK();                                                      // 12
    const int n_kp = compact_kept(keys, slots3, cut, [&](int pos, int slot) { ids[s + pos] = page_of(slot); }, sh);

    // ---- union with the safety pages: sinks, kept pages, window -- already ascending
    const int n_sel = s + n_kp + w;
    for (int i = tid; i < s; i += kSelThreads) ids[i] = i;
    for (int i = tid; i < w; i += kSelThreads) ids[s + n_kp + i] = P - w + i;
    for (int i = n_sel + tid; i < g.max_sel; i += kSelThreads) ids[i] = -1;
    if (tid == 0) n_selected[row] = n_sel;
#ifdef CHESS_PROF
    PROF_MARK();                                                      // 13: end
    if (tid == 0)
        for (int i = 1; i < prof_n; ++i) ws.prof[row * 16 + i] = (int)(prof_t[i] - prof_t[i - 1]);
#endif
}

hipError_t select_occupancy(int lds_bytes, int* blocks_per_cu)
{
    if (lds_bytes > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(select_kernel<false>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(select_kernel<true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return e;
    }
    return hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, select_kernel<false>, kSelThreads, lds_bytes);
}

hipError_t launch_select(chess_ctx* ctx, const uint16_t* q, const float* pages, const float* chunks,
                         const float* grids, const int32_t* seq_lens, int batch, int cluster, const SelectParams& sp,
                         const SelectWs& ws, size_t lds_bytes, int32_t* page_ids, int32_t* n_selected,
                         hipStream_t stream)
{
    const dim3 grid(cluster, ctx->geom.n_kv_heads, batch), block(kSelThreads);
    auto kern = cluster == 1 ? select_kernel<true> : select_kernel<false>;
    return launch(kern, grid, block, lds_bytes, stream, q, pages, chunks, grids, seq_lens, ctx->geom, sp, ws, page_ids,
                  n_selected);
}

}  // namespace chess
