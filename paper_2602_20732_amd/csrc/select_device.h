// Device-side building blocks of the coarse-to-fine page selection (Sec. 3.2, Eq. 4, Alg. 1 stage 2),
// shared by the selection kernel and the fused decode-step kernel.
//
// A cluster of C workgroups cooperates on one (sequence, KV head) through all three levels.  The
// paper scores the whole hierarchy with one GEMM and prunes with masks; here scoring is lazy -- a
// level reads only the 512-byte vectors of its candidates (all grids, chunks of kept grids, pages of
// kept chunks) -- and a level's candidate slots are split over the cluster, so one (sequence, head)
// draws bandwidth from C compute units.  A 16-lane group scores one unit (two 128-bit loads per
// lane, up to 16 units in flight per group, fp64 multiply-add, DPP row sum) and the group leader
// publishes an order-preserving 64-bit key into the slot's word of the workspace.
//
// There is no barrier between the members: a key word is 0 until its owner has published it (a slot
// without a unit is published as 1), so a member simply polls the level's words until none is 0.
// One memory round trip serves as both the wait and the transfer.  Every member then finds the cut
// itself (all compute the same thing): smallest / largest key and count from its registers, one
// histogram over 1024 bins that are linear in the score between the smallest and the largest, a scan
// from the top that every wave does for itself, and an exact ranking by (key, slot) of the few keys
// in the bin the k-th largest falls in.  Ties at the cut go to the lowest slots (= lowest indices:
// candidates are enumerated in index order).  Positions in the ascending list of kept units come
// from ballots, per-run counts in LDS and the ranked members; the list drives the next level.  Score
// distributions that pile more than 64 keys into the bin at the cut (exact ties, mostly), or levels
// with more slots than the register path holds, take a general path on the LDS copy of the keys:
// radix select on the bits the keys do not share, then a ballot compaction.
//
// The words are cleared again by the workgroup that is last to be done with them, so they are all 0
// between launches.  Polls are bounded: a wait that does not end raises the workspace's error flag
// and the workgroup leaves (the workspace then needs chess_workspace_init again).
#pragma once

#include <type_traits>

#include "chess_internal.h"

namespace chess {

constexpr int kSelWaves = kSelThreads / kWave;
constexpr int kPollLimit = 1 << 15;         // polls (each a memory round trip, ~1 us) before a wait is declared dead (default)
constexpr int kKeepAll = 0x7fffffff;
constexpr uint64_t kAbsentKey = 1ull;       // published for a slot that has no unit; below every real key

// Monotone map double -> uint64 (larger score = larger key); every finite or infinite score maps
// to a key >= 2^52 - 1, so 0 can mark "not published yet" and 1 "no unit".  -0.0 is folded onto +0.0.
__device__ __forceinline__ uint64_t order_key(double s)
{
    s += 0.0;
    const uint64_t u = (uint64_t)__double_as_longlong(s);
    return (u >> 63) ? ~u : (u | 0x8000000000000000ull);
}

// order_key's inverse, for binning
__device__ __forceinline__ double key_score(uint64_t key)
{
    const uint64_t u = (key >> 63) ? (key & 0x7fffffffffffffffull) : ~key;
    return __longlong_as_double((long long)u);
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

__device__ __forceinline__ uint64_t lane_read64(uint64_t v, int src)
{
    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)v, src);
    const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(v >> 32), src);
    return ((uint64_t)hi << 32) | lo;
}

constexpr int kBins = 1024;                 // linear score bins of the cut
#ifdef CHESS_MAX_FLY
constexpr int kMaxFly = CHESS_MAX_FLY;
#else
constexpr int kMaxFly = kSelThreads >= 1024 ? 4 : 8;   // units a 16-lane group requests before it waits
#endif
constexpr int kSelGroups = kSelThreads / 16;  // 16-lane groups of a workgroup
constexpr int kFastMembers = 64;            // most keys the bin at the cut may hold on the register path
constexpr int kRegsSmall = 1024 / kSelThreads;                           // keys per thread the register path is built
constexpr int kRegsLarge = (4352 + kSelThreads - 1) / kSelThreads;       //   for: levels of up to 1024 / 4352+ slots
constexpr int kMaxRuns = kRegsLarge * kSelWaves;  // 64-slot runs of the largest level the register path holds

struct Shared {
    int hist[kBins];
    uint64_t mem_key[kFastMembers];
    int mem_slot[kFastMembers];
    int run_gt[kMaxRuns];
    int wave_a[kSelWaves], wave_b[kSelWaves];
    int digit, rem, cnt, n_valid, n_mem, flag;
    unsigned int or_lo, or_hi, and_lo, and_hi;
    unsigned st_min[kSelWaves], st_max[kSelWaves];   // upper halves of the waves' smallest / largest key of a level
    int st_cnt[kSelWaves];
    int poll_limit;         // polls before a wait is given up (kPollLimit unless a test lowered it)
    uint64_t tail_key[3];   // keys of the refreshed tail grid / chunk / page when this workgroup computed them, else 0
};

// Eq. 3: the query anchor of a (sequence, KV head), the mean of the page vectors of the recent window (the last
// min(w, P) pages): fp64 sum in page order, divided by the count, rounded to fp32 once like every stored mean.
// This lane's dims as in load_probe.  The window's vectors are requested four pages at a time.
__device__ __forceinline__ void load_anchor(const float* __restrict__ pages_row, int P, int w, double (&pr)[8])
{
    const int ln = threadIdx.x & 15;
    const int W = min(w, P), first = P - W;
    double acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int j0 = first; j0 < P; j0 += 4) {
        float4 va[4], vb[4];
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const float4* p = reinterpret_cast<const float4*>(pages_row + (size_t)min(j0 + x, P - 1) * kHeadDim) + ln;
            va[x] = p[0];
            vb[x] = p[16];
        }
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            if (j0 + x < P) {
                acc[0] += (double)va[x].x; acc[1] += (double)va[x].y; acc[2] += (double)va[x].z; acc[3] += (double)va[x].w;
                acc[4] += (double)vb[x].x; acc[5] += (double)vb[x].y; acc[6] += (double)vb[x].z; acc[7] += (double)vb[x].w;
            }
        }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) pr[i] = (double)(float)(acc[i] / (double)W);
}

struct Prof {
#ifdef CHESS_PROF
    long long t[48];
    int n = 0;
    __device__ __forceinline__ void mark() { if (n < 48) t[n++] = wall_clock64(); }
#else
    __device__ __forceinline__ void mark() {}
#endif
};

struct Cut {
    uint64_t thr;   // in the shifted domain: key << shift
    int ties;       // how many of the slots whose shifted key equals thr are kept, lowest slots first
    int shift;
};

// Cut of the top-k among the non-empty keys in LDS by radix select: k = k_of(number of non-empty keys).
// A non-empty slot is kept iff (key << shift) > thr, or (key << shift) == thr and it is among the first
// `ties` such slots.  Uniform over the workgroup; every thread must call it.
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
        if (tid < 256) sh.hist[tid] = 0;               // 256 digits
        __syncthreads();
        for (int i = tid; i < n_slots; i += kSelThreads) {
            const uint64_t key = keys[i];
            const uint64_t sk = key << shift;
            if (key != 0 && (p == 0 || (sk >> (64 - 8 * p)) == prefix))
                atomicAdd(&sh.hist[(int)((sk >> (56 - 8 * p)) & 255)], 1);
        }
        __syncthreads();
        // thread t looks at digit 255 - t, so thread order is digit order descending
        const int c = tid < 256 ? sh.hist[255 - tid] : 0;
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

// Minimum / maximum of a 32-bit unsigned value over the wave (DPP, no LDS); the result is in lane 63.
template <bool kMin>
__device__ __forceinline__ unsigned wave_minmax32(unsigned v)
{
    const int id = kMin ? -1 : 0;
#define CHESS_MM_STEP(ctrl, rows)                                                                      \
    {                                                                                                  \
        const unsigned o = (unsigned)__builtin_amdgcn_update_dpp(id, (int)v, ctrl, rows, 0xf, false);  \
        v = kMin ? min(v, o) : max(v, o);                                                              \
    }
    CHESS_MM_STEP(0x111, 0xf) CHESS_MM_STEP(0x112, 0xf) CHESS_MM_STEP(0x114, 0xf) CHESS_MM_STEP(0x118, 0xf)
    CHESS_MM_STEP(0x142, 0xa) CHESS_MM_STEP(0x143, 0xc)
#undef CHESS_MM_STEP
    return v;
}

// A key at or below the smallest key, a key at or above the largest key (both from the upper halves of the
// keys: bounds are all the binning needs) and the number of non-empty keys of a level, in two steps around one
// workgroup barrier (so that the barrier can be one the caller needs anyway): every wave leaves what it sees ...
template <int R>
__device__ __forceinline__ void wave_stats(const uint64_t (&key)[R], Shared& sh)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned a = ~0u, b = 0u;
    int n = 0;                                        // wave-uniform
#pragma unroll
    for (int x = 0; x < R; ++x) {
        const bool valid = key[x] != 0;
        const unsigned hi = (unsigned)(key[x] >> 32);
        a = valid ? min(a, hi) : a;
        b = valid ? max(b, hi) : b;
        n += __popcll(__ballot(valid));
    }
    a = wave_minmax32<true>(a);
    b = wave_minmax32<false>(b);
    if (lane == 63) { sh.st_min[wave] = a; sh.st_max[wave] = b; sh.st_cnt[wave] = n; }
}
// ... and after the barrier everybody combines them.
__device__ __forceinline__ void level_stats(const Shared& sh, uint64_t* kmin, uint64_t* kmax, int* n_valid)
{
    unsigned a = ~0u, b = 0u;
    int n = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) {
        a = min(a, sh.st_min[w]);
        b = max(b, sh.st_max[w]);
        n += sh.st_cnt[w];
    }
    *kmin = (uint64_t)a << 32;
    *kmax = ((uint64_t)b << 32) | 0xffffffffull;
    *n_valid = n;
}

// Where bin b of the histogram is stored: lane l of a wave owns bins 16 (63 - l) .. 16 (63 - l) + 15 (lane 0
// the highest scores) and reads its j-th bin from word 64 j + l, so the 64 lanes hit 64 different banks.
__device__ __forceinline__ int hist_word(int b) { return ((b & 15) << 6) | (63 - (b >> 4)); }

// Cut and ordered compaction of one level whose keys the workgroup holds in registers: thread t has
// slot x * 256 + t in key[x] (0 = empty).  k = k_of(n_valid) of the n_valid non-empty keys are kept, by
// (key descending, slot ascending); emit(pos, slot) is called for each kept slot with its position in
// ascending slot order.  Returns the number kept, or -1, having emitted nothing, when this path does not
// apply (more than kFastMembers keys share the bin at the cut).  Uniform over the workgroup: every thread
// must call it.  sh.hist must be all zero and sh.n_mem zero on entry, and they are again on a return >= 0.
//
// The kBins bins are LINEAR in the score between the scores of klo and khi (klo <= every key <= khi): a
// monotone map, so a higher bin means a strictly larger score; the scale only has to be positive, not exact.
// A scan from the top finds the bin the k-th largest key falls in, and the few keys of that bin are ranked
// exactly by (key, slot).
template <int R, class KFn, class Out>
__device__ __forceinline__ int cut_in_registers(const uint64_t (&key)[R], int n_slots, uint64_t klo, uint64_t khi,
                                                int n_valid, KFn k_of, Out emit, Shared& sh, Prof& prof)
{
    static_assert(kBins == 16 * kWave, "a lane owns 16 bins");
    static_assert(R * kSelWaves <= kMaxRuns && R * kSelWaves <= 128, "run prefix is held in two values per lane");
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint64_t below = __lanemask_lt();
    auto f_add = [](int a, int b) { return a + b; };
    const int k = k_of(n_valid);
    if (k <= 0) { __syncthreads(); return 0; }
    const bool all = k >= n_valid;

    int bin[R];
    int cutbin = -1, want = 0, cnt = 0;
    if (!all) {
        const double smin = key_score(klo);
        const double scale = (double)kBins * __builtin_amdgcn_rcp(key_score(khi) - smin);
#pragma unroll
        for (int x = 0; x < R; ++x) {
            bin[x] = -1;
            if (x * kSelThreads < n_slots && key[x] != 0) {
                const int bx = (int)((key_score(key[x]) - smin) * scale);
                bin[x] = min(max(bx, 0), kBins - 1);
                atomicAdd(&sh.hist[hist_word(bin[x])], 1);
            }
        }
        __syncthreads();
        prof.mark();
        // every wave scans the whole histogram from the top
        int own = 0;
#pragma unroll
        for (int j = 0; j < 16; ++j) own += sh.hist[64 * j + lane];
        const int incl = wave_scan(own, 0, f_add);
        const bool here = incl - own < k && k <= incl;            // true in exactly one lane
        const int src = __builtin_amdgcn_readfirstlane(__ffsll((long long)__ballot(here)) - 1);
        const int k_rem = k - (__builtin_amdgcn_readlane(incl, src) - __builtin_amdgcn_readlane(own, src));
        // the 16 bins of that lane, highest first, one per lane of the first row
        const int c = lane < 16 ? sh.hist[64 * (15 - lane) + src] : 0;
        int ci = c;
        ci += __builtin_amdgcn_update_dpp(0, ci, 0x111, 0xf, 0xf, false);
        ci += __builtin_amdgcn_update_dpp(0, ci, 0x112, 0xf, 0xf, false);
        ci += __builtin_amdgcn_update_dpp(0, ci, 0x114, 0xf, 0xf, false);
        ci += __builtin_amdgcn_update_dpp(0, ci, 0x118, 0xf, 0xf, false);
        const int at = __builtin_amdgcn_readfirstlane(__ffsll((long long)__ballot(lane < 16 && ci >= k_rem)) - 1);
        cutbin = 16 * (63 - src) + 15 - at;
        cnt = __builtin_amdgcn_readlane(c, at);
        want = k_rem - (__builtin_amdgcn_readlane(ci, at) - cnt);
        if (cnt > kFastMembers) return -1;
        prof.mark();
    } else {
#pragma unroll
        for (int x = 0; x < R; ++x) bin[x] = 0;
    }

    // keys above the cut bin are kept for sure: count them per 64-slot run; collect the cut bin's keys
    unsigned sure = 0, maybe = 0;
#pragma unroll
    for (int x = 0; x < R; ++x) {
        if (x * kSelThreads >= n_slots) break;                    // uniform
        const bool a = all ? key[x] != 0 : bin[x] > cutbin;
        const bool e = !all && bin[x] == cutbin;
        if (e) {
            const int at = atomicAdd(&sh.n_mem, 1);
            sh.mem_key[at] = key[x];
            sh.mem_slot[at] = x * kSelThreads + tid;
        }
        const uint64_t ab = __ballot(a);
        if (lane == 0) sh.run_gt[x * kSelWaves + wave] = __popcll(ab);
        sure |= (unsigned)a << x;
        maybe |= (unsigned)e << x;
    }
    __syncthreads();
    prof.mark();

    // leave the histogram clean for the next level (its readers are past the barrier above)
    for (int i = tid; i < kBins; i += kSelThreads) sh.hist[i] = 0;
    if (tid == 0) sh.n_mem = 0;

    // every wave ranks the cut bin's keys: lane j takes member j and meets the others through lane reads
    uint64_t thr = 0;
    int thr_slot = -1, my_slot = 0;
    uint64_t kept_mask = 0;
    if (cnt > 0) {
        const uint64_t mine = lane < cnt ? sh.mem_key[lane] : 0ull;
        my_slot = lane < cnt ? sh.mem_slot[lane] : 0;
        int rank = 0;
        for (int i = 0; i < cnt; ++i) {
            const uint64_t ki = lane_read64(mine, i);
            const int si = __builtin_amdgcn_readlane(my_slot, i);
            rank += ki > mine || (ki == mine && si < my_slot);
        }
        kept_mask = __ballot(lane < cnt && rank < want);
        const int src = __builtin_amdgcn_readfirstlane(__ffsll((long long)__ballot(lane < cnt && rank == want - 1)) - 1);
        thr = lane_read64(mine, src);
        thr_slot = __builtin_amdgcn_readlane(my_slot, src);
    }
    // kept members in lower slots than each of this thread's slots
    int before[R];
#pragma unroll
    for (int x = 0; x < R; ++x) before[x] = 0;
    for (uint64_t mk = kept_mask; mk != 0; mk &= mk - 1) {
        const int j = __builtin_amdgcn_readfirstlane(__ffsll((long long)mk) - 1);
        const int sj = __builtin_amdgcn_readlane(my_slot, j);
#pragma unroll
        for (int x = 0; x < R; ++x) before[x] += sj < x * kSelThreads + tid;
    }
    prof.mark();
    // sure keys in earlier runs
    const int n_runs = (n_slots + kWave - 1) / kWave;
    const int c0 = lane < n_runs ? sh.run_gt[lane] : 0;
    const int i0 = wave_scan(c0, 0, f_add);
    const int e0 = i0 - c0;
    int e1 = 0;
    if (R * kSelWaves > kWave) {
        const int c1 = lane + kWave < n_runs ? sh.run_gt[min(lane + kWave, kMaxRuns - 1)] : 0;
        const int i1 = wave_scan(c1, 0, f_add);
        e1 = i1 - c1 + __builtin_amdgcn_readlane(i0, 63);
    }
#pragma unroll
    for (int x = 0; x < R; ++x) {
        if (x * kSelThreads >= n_slots) break;                    // uniform
        const int run = x * kSelWaves + wave;
        const int base = x * kSelWaves < kWave ? __builtin_amdgcn_readlane(e0, run) : __builtin_amdgcn_readlane(e1, run - kWave);
        const bool a = (sure >> x) & 1, e = (maybe >> x) & 1;
        const int slot = x * kSelThreads + tid;
        const uint64_t ab = __ballot(a);
        const bool keep = a || (e && (key[x] > thr || (key[x] == thr && slot <= thr_slot)));
        if (keep) emit(base + __popcll(ab & below) + before[x], slot);
    }
    __syncthreads();                                              // mem_key / run_gt readers are done; emitted lists visible
    return all ? n_valid : k;
}

// Cut and ordered compaction of a small level (at most kOneWaveSlots slots) by ONE wave, with no workgroup barrier
// inside: wave 0 holds slot x * 64 + lane of the LDS copy of the keys in key[x] and does what cut_in_registers
// does -- bounds from the upper key halves, linear-bin histogram, scan from the top, exact ranking of the bin at
// the cut -- with ballots in place of the LDS lists (the other waves wait at the closing barrier; LDS operations of
// one wave complete in order, so its own histogram needs no barrier).  Same contract as cut_in_registers, keys
// from `keys` (LDS, complete: call after the pull's barrier); returns -1 (to every thread), having emitted nothing,
// when more than kFastMembers keys share the bin at the cut.
constexpr int kOneWaveRegs = 4;
constexpr int kOneWaveSlots = kOneWaveRegs * kWave;
template <class KFn, class Out>
__device__ __forceinline__ int cut_one_wave(const uint64_t* keys, int n_slots, KFn k_of, Out emit, Shared& sh)
{
    constexpr int R = kOneWaveRegs;
    const int tid = threadIdx.x, lane = tid & 63;
    if (tid < kWave) {
        const uint64_t below = __lanemask_lt();
        auto f_add = [](int a, int b) { return a + b; };
        uint64_t key[R];
        unsigned lo_h = ~0u, hi_h = 0u;
        int n_valid = 0;
#pragma unroll
        for (int x = 0; x < R; ++x) {
            const int i = x * kWave + lane;
            key[x] = i < n_slots ? keys[i] : 0ull;
            const bool valid = key[x] != 0ull;
            const unsigned h = (unsigned)(key[x] >> 32);
            lo_h = valid ? min(lo_h, h) : lo_h;
            hi_h = valid ? max(hi_h, h) : hi_h;
            n_valid += __popcll(__ballot(valid));
        }
        const int k = k_of(n_valid);
        int result;
        if (k <= 0) {
            result = 0;
        } else {
            const bool all = k >= n_valid;
            int bin[R];
            int cutbin = -1, want = 0, cnt = 0;
            bool fits = true;
            if (!all) {
                lo_h = (unsigned)__builtin_amdgcn_readlane((int)wave_minmax32<true>(lo_h), 63);
                hi_h = (unsigned)__builtin_amdgcn_readlane((int)wave_minmax32<false>(hi_h), 63);
                const double smin = key_score((uint64_t)lo_h << 32);
                const double scale = (double)kBins * __builtin_amdgcn_rcp(key_score(((uint64_t)hi_h << 32) | 0xffffffffull) - smin);
#pragma unroll
                for (int x = 0; x < R; ++x) {
                    bin[x] = -1;
                    if (key[x] != 0ull) {
                        const int bx = (int)((key_score(key[x]) - smin) * scale);
                        bin[x] = min(max(bx, 0), kBins - 1);
                        atomicAdd(&sh.hist[hist_word(bin[x])], 1);
                    }
                }
                int own = 0;
#pragma unroll
                for (int j = 0; j < 16; ++j) own += sh.hist[64 * j + lane];
                const int incl = wave_scan(own, 0, f_add);
                const bool here = incl - own < k && k <= incl;
                const int src = __builtin_amdgcn_readfirstlane(__ffsll((long long)__ballot(here)) - 1);
                const int k_rem = k - (__builtin_amdgcn_readlane(incl, src) - __builtin_amdgcn_readlane(own, src));
                const int c = lane < 16 ? sh.hist[64 * (15 - lane) + src] : 0;
                int ci = c;
                ci += __builtin_amdgcn_update_dpp(0, ci, 0x111, 0xf, 0xf, false);
                ci += __builtin_amdgcn_update_dpp(0, ci, 0x112, 0xf, 0xf, false);
                ci += __builtin_amdgcn_update_dpp(0, ci, 0x114, 0xf, 0xf, false);
                ci += __builtin_amdgcn_update_dpp(0, ci, 0x118, 0xf, 0xf, false);
                const int at = __builtin_amdgcn_readfirstlane(__ffsll((long long)__ballot(lane < 16 && ci >= k_rem)) - 1);
                cutbin = 16 * (63 - src) + 15 - at;
                cnt = __builtin_amdgcn_readlane(c, at);
                want = k_rem - (__builtin_amdgcn_readlane(ci, at) - cnt);
                fits = cnt <= kFastMembers;
                // leave the histogram clean: this wave is its only user at this level
#pragma unroll
                for (int x = 0; x < R; ++x)
                    if (bin[x] >= 0) sh.hist[hist_word(bin[x])] = 0;
            } else {
#pragma unroll
                for (int x = 0; x < R; ++x) bin[x] = 0;
            }
            if (!fits) {
                result = -1;
            } else {
                // rank the keys of the bin at the cut against each other: (key descending, slot ascending)
                uint64_t em[R];
                int rank[R];
#pragma unroll
                for (int x = 0; x < R; ++x) { em[x] = __ballot(!all && bin[x] == cutbin); rank[x] = 0; }
#pragma unroll
                for (int y = 0; y < R; ++y) {
                    for (uint64_t mk = em[y]; mk != 0ull; mk &= mk - 1) {
                        const int j = __builtin_amdgcn_readfirstlane(__ffsll((long long)mk) - 1);
                        const uint64_t kj = lane_read64(key[y], j);
                        const int sj = y * kWave + j;
#pragma unroll
                        for (int x = 0; x < R; ++x) rank[x] += kj > key[x] || (kj == key[x] && sj < x * kWave + lane);
                    }
                }
                int base = 0;
#pragma unroll
                for (int x = 0; x < R; ++x) {
                    const bool keep = all ? key[x] != 0ull : (bin[x] > cutbin || (bin[x] == cutbin && rank[x] < want));
                    const uint64_t kb = __ballot(keep);
                    if (keep) emit(base + __popcll(kb & below), x * kWave + lane);
                    base += __popcll(kb);
                }
                result = base;
            }
        }
        if (lane == 0) sh.cnt = result;
    }
    __syncthreads();
    return sh.cnt;
}

// A level of at most 64 slots: one key per lane of wave 0, each lane counts the keys that rank before its own
// (key descending, slot ascending) with 64 lane reads; no histogram, no LDS.  Same contract as cut_one_wave.
template <class KFn, class Out>
__device__ __forceinline__ int cut_one_lane_each(const uint64_t* keys, int n_slots, KFn k_of, Out emit, Shared& sh)
{
    const int tid = threadIdx.x;
    if (tid < kWave) {
        const int lane = tid;
        const uint64_t key = lane < n_slots ? keys[lane] : 0ull;
        const uint64_t valid = __ballot(key != 0ull);
        const int k = k_of(__popcll(valid));
        int rank = 0;
        for (uint64_t mk = valid; mk != 0ull; mk &= mk - 1) {
            const int j = __builtin_amdgcn_readfirstlane(__ffsll((long long)mk) - 1);
            const uint64_t kj = lane_read64(key, j);
            rank += kj > key || (kj == key && j < lane);
        }
        const uint64_t kb = __ballot(key != 0ull && rank < k);
        if ((kb >> lane) & 1ull) emit(__popcll(kb & __lanemask_lt()), lane);
        if (lane == 0) sh.cnt = __popcll(kb);
    }
    __syncthreads();
    return sh.cnt;
}

// Scores of the slots [lo, hi), kFly units per 16-lane group requested before the first is waited for.
// `unit_of(slot)` is the index of the slot's 128-float vector in `base`, or -1 when the slot has no unit.
// Lane ln of a group holds probe dims 4 ln .. 4 ln + 3 and 64 + 4 ln .. 64 + 4 ln + 3.  The key of a slot goes
// to lds_keys[slot] (0 for no unit) when the level is local, else it is published in pub[slot].  (Two pointers
// of known address space: one generic pointer for both would turn every access into a flat one.)
template <int kFly, class Map>
__device__ __forceinline__ void score_rows(const float* __restrict__ base, int lo, int hi, Map unit_of,
                                           const double (&pr)[8], bool local, uint64_t* lds_keys, uint64_t* pub)
{
    const int g16 = threadIdx.x >> 4, ln = threadIdx.x & 15;
    for (int s0 = lo; s0 < hi; s0 += kSelGroups * kFly) {
        int slot[kFly], unit[kFly];
        float4 va[kFly], vb[kFly];
#pragma unroll
        for (int x = 0; x < kFly; ++x) {
            slot[x] = s0 + kSelGroups * x + g16;
            unit[x] = slot[x] < hi ? unit_of(slot[x]) : -1;
            // always load (unit 0 when the slot has no unit): a branch here would make the compiler wait
            // for each vector before asking for the next
            const float4* p = reinterpret_cast<const float4*>(base + (size_t)max(unit[x], 0) * kHeadDim) + ln;
            va[x] = p[0];
            vb[x] = p[16];
        }
#pragma unroll
        for (int x = 0; x < kFly; ++x) {
            if (s0 + kSelGroups * x >= hi) break;     // uniform over the workgroup
            double d = 0.0;
            d = fma(pr[0], (double)va[x].x, d); d = fma(pr[1], (double)va[x].y, d);
            d = fma(pr[2], (double)va[x].z, d); d = fma(pr[3], (double)va[x].w, d);
            d = fma(pr[4], (double)vb[x].x, d); d = fma(pr[5], (double)vb[x].y, d);
            d = fma(pr[6], (double)vb[x].z, d); d = fma(pr[7], (double)vb[x].w, d);
            d = row16_sum(d);
            if (ln == 15 && slot[x] < hi) {
                if (local) lds_keys[slot[x]] = unit[x] >= 0 ? order_key(d) : 0ull;
                else publish_u64(pub + slot[x], unit[x] >= 0 ? order_key(d) : kAbsentKey);
            }
        }
    }
}

// Score the slots [lo, hi) of one level.  A share of up to kMaxFly slots per 16-lane group is requested in one
// go: one memory round trip.
template <class Map>
__device__ __forceinline__ void score_range(const float* __restrict__ base, int lo, int hi, Map unit_of,
                                            const double (&pr)[8], bool local, uint64_t* lds_keys, uint64_t* pub)
{
    score_rows<kMaxFly>(base, lo, hi, unit_of, pr, local, lds_keys, pub);
}

// One slot of a level whose key does not come from where the others' do: the unit the decode step has just
// refreshed (the tail page, its chunk, its grid), whose key one workgroup publishes in a word of its own.
struct SlotOverride {
    int slot;                 // -1: none
    const uint64_t* word;     // where the key is published
    uint64_t have;            // non-zero: the key itself (this workgroup computed it)
};

// Wait for one published word; 0 if it did not arrive within the poll limit.
__device__ __forceinline__ uint64_t poll_word(const uint64_t* word, int limit)
{
    for (int polls = 0; polls < limit; ++polls) {
        const uint64_t v = observe_u64(word);
        if (v != 0ull) return v;
        __builtin_amdgcn_s_sleep(1);
    }
    return 0ull;
}

// A level's keys into registers (thread t: slots t, t + 256, ...; 0 = empty or beyond n_slots) and into the
// LDS copy the general path works on.  local: the keys are in LDS already.  Otherwise the published words
// are polled until every one of them is there.  Ends with a workgroup barrier, before which every wave has left
// its statistics for level_stats; returns false (to every thread) if a word did not arrive within the poll limit.
template <int R>
__device__ __forceinline__ bool pull_keys(const uint64_t* pub, int n_slots, bool local, const SlotOverride& ov,
                                          uint64_t* keys, uint64_t (&key)[R], Shared& sh)
{
    const int tid = threadIdx.x;
    constexpr int kBatch = R < 8 ? R : 8;             // loads requested before the first is waited for
    bool ok = true;
#pragma unroll
    for (int x = 0; x < R; ++x) key[x] = 0ull;
    if (local) {
        __syncthreads();                              // the scores of all waves are in LDS
#pragma unroll
        for (int x = 0; x < R; ++x) {
            const int i = x * kSelThreads + tid;
            if (i < n_slots) key[x] = keys[i];
            if (i == ov.slot) {
                key[x] = ov.have != 0ull ? ov.have : poll_word(ov.word, sh.poll_limit);
                ok = key[x] != 0ull;
                keys[i] = key[x];
            }
        }
        wave_stats<R>(key, sh);
        return __syncthreads_and(ok) != 0;
    }
#pragma unroll
    for (int x0 = 0; x0 < R; x0 += kBatch) {
        if (x0 * kSelThreads >= n_slots) break;       // uniform
        int polls = 0;
        while (true) {
            bool missing = false;
#pragma unroll
            for (int x = x0; x < x0 + kBatch && x < R; ++x) {
                const int i = x * kSelThreads + tid;
                const int ic = max(min(i, n_slots - 1), 0);   // unconditional: all stay in flight
                key[x] = observe_u64(i == ov.slot ? ov.word : pub + ic);
            }
#pragma unroll
            for (int x = x0; x < x0 + kBatch && x < R; ++x)
                missing = missing || (x * kSelThreads + tid < n_slots && key[x] == 0ull);
            if (__ballot(missing) == 0ull) break;
            if (++polls >= sh.poll_limit) { ok = false; break; }
            __builtin_amdgcn_s_sleep(1);
        }
#pragma unroll
        for (int x = x0; x < x0 + kBatch && x < R; ++x) {
            const int i = x * kSelThreads + tid;
            if (i >= n_slots || key[x] == kAbsentKey) key[x] = 0ull;
            if (i < n_slots) keys[i] = key[x];
        }
    }
    wave_stats<R>(key, sh);
    return __syncthreads_and(ok) != 0;
}

// The same for a level too large for the register path: into LDS only.
__device__ __forceinline__ bool pull_keys_lds(const uint64_t* pub, int n_slots, const SlotOverride& ov, uint64_t* keys,
                                              int limit)
{
    bool ok = true;
    for (int i0 = 0; i0 < n_slots; i0 += 4 * kSelThreads) {
        uint64_t v[4];
        int polls = 0;
        while (true) {
            bool missing = false;
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const int i = i0 + x * kSelThreads + (int)threadIdx.x;
                v[x] = observe_u64(i == ov.slot ? ov.word : pub + min(i, n_slots - 1));
            }
#pragma unroll
            for (int x = 0; x < 4; ++x) missing = missing || v[x] == 0ull;
            if (__ballot(missing) == 0ull) break;
            if (++polls >= limit) { ok = false; break; }
            __builtin_amdgcn_s_sleep(1);
        }
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const int i = i0 + x * kSelThreads + threadIdx.x;
            if (i < n_slots) keys[i] = v[x] == kAbsentKey ? 0ull : v[x];
        }
    }
    return __syncthreads_and(ok) != 0;
}

// What every member does once it has scored its share of a level: the level's keys, the cut, the ordered
// list of kept slots through `emit`.  Returns the number kept, or -1 if the keys did not arrive.
template <class KFn, class Hook, class Out>
__device__ __forceinline__ int finish_level(const uint64_t* pub, int n_slots, bool local, bool general,
                                            const SlotOverride& ov, uint64_t* keys, KFn k_of, Hook after_pull, Out emit,
                                            Shared& sh, Prof& prof)
{
    int n = -1;
    if (n_slots <= kOneWaveSlots && !general) {
        uint64_t key[kRegsSmall];
        if (!pull_keys<kRegsSmall>(pub, n_slots, local, ov, keys, key, sh)) return -1;
        after_pull();
        prof.mark(); prof.mark(); prof.mark(); prof.mark(); prof.mark(); prof.mark();
        n = n_slots <= kWave ? cut_one_lane_each(keys, n_slots, k_of, emit, sh) : cut_one_wave(keys, n_slots, k_of, emit, sh);
    } else if (n_slots <= kRegsSmall * kSelThreads) {
        uint64_t key[kRegsSmall];
        if (!pull_keys<kRegsSmall>(pub, n_slots, local, ov, keys, key, sh)) return -1;
        after_pull();
        if (!general) {
            uint64_t kmin, kmax;
            int n_valid;
            prof.mark();
            level_stats(sh, &kmin, &kmax, &n_valid);
            prof.mark();
            n = cut_in_registers<kRegsSmall>(key, n_slots, kmin, kmax, n_valid, k_of, emit, sh, prof);
        }
    } else if (n_slots <= kRegsLarge * kSelThreads) {
        uint64_t key[kRegsLarge];
        if (!pull_keys<kRegsLarge>(pub, n_slots, local, ov, keys, key, sh)) return -1;
        after_pull();
        if (!general) {
            uint64_t kmin, kmax;
            int n_valid;
            level_stats(sh, &kmin, &kmax, &n_valid);
            n = cut_in_registers<kRegsLarge>(key, n_slots, kmin, kmax, n_valid, k_of, emit, sh, prof);
        }
    } else if (local) {
        __syncthreads();
        bool ok = true;
        if (ov.slot >= 0 && (int)threadIdx.x == 0) {
            const uint64_t k = ov.have != 0ull ? ov.have : poll_word(ov.word, sh.poll_limit);
            ok = k != 0ull;
            keys[ov.slot] = k;
        }
        if (ov.slot >= 0 && __syncthreads_and(ok) == 0) return -1;
        after_pull();
    } else {
        if (!pull_keys_lds(pub, n_slots, ov, keys, sh.poll_limit)) return -1;
        after_pull();
    }
    if (n >= 0) return n;
    // general path on the LDS copy of the keys
    __syncthreads();
    const Cut cut = find_cut_radix(keys, n_slots, k_of, sh);
    n = compact_kept(keys, n_slots, cut, emit, sh);
    for (int i = threadIdx.x; i < kBins; i += kSelThreads) sh.hist[i] = 0;
    if (threadIdx.x == 0) sh.n_mem = 0;
    __syncthreads();
    return n;
}

// The probe of a (sequence, KV head): the sum of the group's query rows in fp64, g ascending (Eq. 4 with
// Eq. 1's Flatten restricted to the group); this lane's dims 4 ln .. 4 ln + 3 and 64 + 4 ln .. 64 + 4 ln + 3.
__device__ __forceinline__ void load_probe(const uint16_t* __restrict__ q_rows, int group, double (&pr)[8])
{
    const int ln = threadIdx.x & 15;
#pragma unroll
    for (int i = 0; i < 8; ++i) pr[i] = 0.0;
    for (int r = 0; r < group; ++r) {
        const uint2 a = *reinterpret_cast<const uint2*>(q_rows + (size_t)r * kHeadDim + ln * 4);
        const uint2 c = *reinterpret_cast<const uint2*>(q_rows + (size_t)r * kHeadDim + 64 + ln * 4);
        pr[0] += (double)__uint_as_float(a.x << 16); pr[1] += (double)__uint_as_float(a.x & 0xffff0000u);
        pr[2] += (double)__uint_as_float(a.y << 16); pr[3] += (double)__uint_as_float(a.y & 0xffff0000u);
        pr[4] += (double)__uint_as_float(c.x << 16); pr[5] += (double)__uint_as_float(c.x & 0xffff0000u);
        pr[6] += (double)__uint_as_float(c.y << 16); pr[7] += (double)__uint_as_float(c.y & 0xffff0000u);
    }
}

struct CascadeResult {
    int n_kp;              // kept pages (their numbers, ascending, are in `sel_pages`)
    int n1, n2, n3;        // published words of the three levels (what has to be cleared afterwards)
};

// Where the three levels' published words of one (sequence, KV head) start.
struct PubLayout {
    uint64_t* grids;       // [max_grids]
    uint64_t* chunks;      // chunk slots: n_g per kept grid
    uint64_t* pages;       // page slots: n_c per kept chunk
};
__device__ __forceinline__ PubLayout pub_layout(uint64_t* row_words, const Geom& g, const SelectParams& sp)
{
    PubLayout p;
    p.grids = row_words;
    p.chunks = row_words + g.max_grids;
    p.pages = p.chunks + sp.cap2;
    return p;
}

// The three levels for one (sequence, KV head) with P > sink + window pages.  Member m of C scores the m-th
// part of every level.  With want_l3 every member ends up with the kept page numbers in sel_pages[0 .. n_kp);
// without it a member returns as soon as its level-3 keys are published (n_kp = 0).  sh.hist must be all
// zero and sh.n_mem zero on entry.  Returns false if a wait was given up.  k_fixed > 0: the page budget of this
// sequence (fixed_budget); 0: derived from its page count.
// The levels run through one copy of the code (a loop, not three inlined bodies): the kernel executes every
// instruction about once, so its time is sensitive to how much code it has to fetch.
//
// kPhys: the caller goes on to read the kept pages, so the block-table entries of all page-level candidates are
// requested behind the page-level scores (by every member, for all slots) and parked in phys_by_slot (LDS,
// one word per slot); sel_phys[i] then receives the physical page of sel_pages[i].
//
// tail_words non-null: the decode step refreshes the summaries of the tail page, its chunk and its grid in this
// launch.  `refresh_tail()` is called in member 0 once its grid-level vectors are requested; it leaves the three
// units' keys in tail_words[0..2] (grid, chunk, page) for the cluster and in sh.tail_key for itself.  Wherever one
// of these units is a candidate, its key is taken from there instead of the slot's own word (whatever was
// scored for that slot from the old vector is ignored).
//
// How a level's slots are scored is the Scorer's business: scorer(level, lo, hi, unit_of, local, keys, pub) leaves
// the keys of the slots [lo, hi) in keys[] (local) or publishes them in pub[]; a member's share of a level is a
// multiple of Scorer::kShareRound slots.
template <bool kPhys, class Scorer, class TailFn>
__device__ __forceinline__ bool cascade_with(const Scorer& scorer, int P, const Geom& g,
                                        const SelectParams& sp, const PubLayout& pubs, int m, int C, bool want_l3,
                                        uint64_t* keys, int32_t* kept_grids, int32_t* kept_chunks, int32_t* sel_pages,
                                        Shared& sh, CascadeResult* res, Prof& prof, const uint64_t* tail_words,
                                        TailFn refresh_tail, int k_fixed, const int32_t* __restrict__ bt_row = nullptr,
                                        int32_t* phys_by_slot = nullptr, int32_t* sel_phys = nullptr)
{
    const int s = sp.sink, w = sp.window;
    const int nc = ceil_div_i(P, g.n_c), ng = ceil_div_i(nc, g.n_g);
    const int k_budget = k_fixed > 0 ? k_fixed : clamp_i(ceil_bp(P, sp.budget_bp), 1, P);
    const int kc_target = ceil_div_i(sp.over_chunk * k_budget, g.n_c);
    const int plan = sp.plan;
    const bool general = sp.general_cut != 0;
    res->n_kp = 0; res->n1 = 0; res->n2 = 0; res->n3 = 0;

    int n_slots = ng;                                 // candidate slots of the current level
    const int32_t* parents = nullptr;                 // kept units of the level above, ascending
    int n_parents = 0;
    auto tail_unit = [&](int lv) { return lv == 0 ? ng - 1 : lv == 1 ? nc - 1 : P - 1; };   // (no array: a run-time index would put it in scratch memory)
#pragma unroll 1
    for (int level = 0; level < 3; ++level) {
        // level 0: every grid; level 1: chunks of kept grids; level 2: pages of kept chunks that are neither
        // sink nor window pages
        const int fan = level == 0 ? 1 : level == 1 ? g.n_g : g.n_c;
        const int u_lo = level == 2 ? s : 0;
        const int u_hi = level == 0 ? ng : level == 1 ? nc : P - w;
        int32_t* out = level == 0 ? kept_grids : level == 1 ? kept_chunks : sel_pages;
        uint64_t* pub = level == 0 ? pubs.grids : level == 1 ? pubs.chunks : pubs.pages;
        // slot / fan without a division: exact for slot < 2^24 and 2 <= fan <= 256 (the error term slot * e / 2^32
        // with e = fan * inv_fan - 2^32 < fan stays below 1 / fan)
        const uint32_t inv_fan = fan > 1 ? (uint32_t)((0x100000000ull + fan - 1) / fan) : 0u;
        auto unit_of = [&](int slot) {
            int u = slot;
            if (level != 0) {
                const int pi = fan > 1 ? (int)__umulhi((unsigned)slot, inv_fan) : slot;
                u = parents[pi] * fan + (slot - pi * fan);
            }
            return (u >= u_lo && u < u_hi) ? u : -1;
        };
        const int cap = level == 0 ? sp.cap_kg : level == 1 ? sp.cap_kc : g.max_sel - s - w;
        auto k_of = [&](int n) {
            int k;
            if (plan == CHESS_PLAN_RATIO) {
                const int rho = level == 0 ? sp.rho_g_bp : level == 1 ? sp.rho_c_bp : sp.rho_p_bp;
                k = n == 0 ? 0 : clamp_i(ceil_bp(n, rho), 1, n);
            } else if (level == 2) {
                k = min(n, k_budget);
            } else if (plan == CHESS_PLAN_FLAT) {
                k = n;
            } else {
                k = min(n, level == 0 ? ceil_div_i(sp.over_grid * kc_target, g.n_g) : kc_target);
            }
            return min(k, cap);
        };
        // A grid or chunk level that keeps every unit it has needs no scores at all: the kept list is the list of
        // the units that exist (they are a prefix of the slots: only the last grid can lack chunks, and it is the
        // last parent when it is kept).  Large budgets and ratios near 1 end up here.
        if (level < 2 && !general) {
            const int missing = (level == 1 && n_parents > 0 && parents[n_parents - 1] == ng - 1) ? ng * g.n_g - nc : 0;
            const int n_present = n_slots - missing;
            if (k_of(n_present) >= n_present) {
                if (level == 0 && tail_words != nullptr && m == 0) refresh_tail();   // the summaries are still kept current
                for (int i = threadIdx.x; i < n_present; i += kSelThreads) out[i] = unit_of(i);
                __syncthreads();
                parents = out;
                n_parents = n_present;
                n_slots = n_present * (level == 0 ? g.n_g : g.n_c);
                continue;
            }
        }
        // A level is local when nothing is exchanged for it: a cluster of one; or the grid level when all grids fit
        // in one request, which every member then scores for itself (the same vectors, so the same keys) instead
        // of waiting a round trip for the others' shares (the host allows it when the repeated reads are few).
        // Otherwise this member takes its share of the level's slots: whole 16-slot rows.
        const bool local = C == 1 || (level == 0 && sp.local_grids != 0 && n_slots <= kSelGroups * kMaxFly);
        {
            const int per = local ? n_slots : ceil_div_i(ceil_div_i(n_slots, C), Scorer::kShareRound) * Scorer::kShareRound;
            const int lo = local ? 0 : min(n_slots, m * per), hi = min(n_slots, lo + per);
            scorer(level, lo, hi, unit_of, local, keys, pub);
            if (!local) { if (level == 0) res->n1 = n_slots; else if (level == 1) res->n2 = n_slots; else res->n3 = n_slots; }
        }
        // kPhys: the block-table entries of every slot's page are requested now, behind this member's vectors, and
        // parked in LDS once the level's keys have been pulled (loads return in order: no wait of their own)
        int32_t entry[kPhys ? kRegsLarge : 1];
        if (kPhys && level == 2) {
#pragma unroll
            for (int x = 0; x < kRegsLarge; ++x) {
                const int i = x * kSelThreads + (int)threadIdx.x;
                entry[kPhys ? x : 0] = 0;
                if (x * kSelThreads < n_slots) entry[kPhys ? x : 0] = bt_row[max(i < n_slots ? unit_of(i) : -1, 0)];
            }
        }
        auto after_pull = [&]() {
            if (kPhys && level == 2) {
#pragma unroll
                for (int x = 0; x < kRegsLarge; ++x) {
                    const int i = x * kSelThreads + (int)threadIdx.x;
                    if (i < n_slots) phys_by_slot[i] = entry[kPhys ? x : 0];
                }
                for (int i = kRegsLarge * kSelThreads + threadIdx.x; i < n_slots; i += kSelThreads)
                    phys_by_slot[i] = bt_row[max(unit_of(i), 0)];
                __syncthreads();                      // the general path reads other threads' slots
            }
        };
        prof.mark();
        if (level == 2 && !want_l3) return true;
        if (level == 0 && tail_words != nullptr && m == 0) refresh_tail();

        // the slot of the refreshed tail unit, if it competes at this level: the last child of the last parent
        SlotOverride ov{-1, nullptr, 0ull};
        if (tail_words != nullptr) {
            const int u = tail_unit(level);
            if (level == 0) ov.slot = u;
            else if (n_parents > 0 && parents[n_parents - 1] == tail_unit(level - 1) && u >= u_lo && u < u_hi)
                ov.slot = (n_parents - 1) * fan + (u - tail_unit(level - 1) * fan);
            ov.word = tail_words + level;
            ov.have = sh.tail_key[level];
        }

        const int n_kept = finish_level(pub, n_slots, local, general, ov, keys, k_of, after_pull, [&](int pos, int slot) {
            out[pos] = unit_of(slot);
            if (kPhys && level == 2) sel_phys[pos] = phys_by_slot[slot];
        }, sh, prof);
        if (n_kept < 0) return false;
        prof.mark();
        parents = out;
        n_parents = n_kept;
        if (level == 0) n_slots = n_kept * g.n_g;
        else if (level == 1) n_slots = n_kept * g.n_c;
        else res->n_kp = n_kept;
    }
    return true;
}

// The scorer of one (sequence, KV head): a level's vectors are rows of one array, the probe is in registers.
struct HeadScorer {
    static constexpr int kShareRound = 16;           // whole rows of 16-lane groups
    const float* pages_row;
    const float* chunks_row;
    const float* grids_row;
    const double (&pr)[8];
    template <class Map>
    __device__ __forceinline__ void operator()(int level, int lo, int hi, Map unit_of, bool local, uint64_t* keys,
                                               uint64_t* pub) const
    {
        const float* base = level == 0 ? grids_row : level == 1 ? chunks_row : pages_row;
        score_range(base, lo, hi, unit_of, pr, local, keys, pub);
    }
};

template <bool kPhys, class TailFn>
__device__ __forceinline__ bool cascade(const float* __restrict__ pages_row, const float* __restrict__ chunks_row,
                                        const float* __restrict__ grids_row, const double (&pr)[8], int P, const Geom& g,
                                        const SelectParams& sp, const PubLayout& pubs, int m, int C, bool want_l3,
                                        uint64_t* keys, int32_t* kept_grids, int32_t* kept_chunks, int32_t* sel_pages,
                                        Shared& sh, CascadeResult* res, Prof& prof, const uint64_t* tail_words,
                                        TailFn refresh_tail, int k_fixed, const int32_t* __restrict__ bt_row = nullptr,
                                        int32_t* phys_by_slot = nullptr, int32_t* sel_phys = nullptr)
{
    const HeadScorer scorer{pages_row, chunks_row, grids_row, pr};
    return cascade_with<kPhys>(scorer, P, g, sp, pubs, m, C, want_l3, keys, kept_grids, kept_chunks, sel_pages, sh, res,
                               prof, tail_words, refresh_tail, k_fixed, bt_row, phys_by_slot, sel_phys);
}

// Clear the published words of one (sequence, KV head) after everybody is done with them.
__device__ __forceinline__ void clear_published(const PubLayout& pubs, const CascadeResult& r, uint64_t* tail_words = nullptr)
{
    if (tail_words != nullptr && threadIdx.x < 3) publish_u64(tail_words + threadIdx.x, 0ull);
    for (int i = threadIdx.x; i < r.n1; i += blockDim.x) publish_u64(pubs.grids + i, 0ull);
    for (int i = threadIdx.x; i < r.n2; i += blockDim.x) publish_u64(pubs.chunks + i, 0ull);
    for (int i = threadIdx.x; i < r.n3; i += blockDim.x) publish_u64(pubs.pages + i, 0ull);
}

}  // namespace chess
