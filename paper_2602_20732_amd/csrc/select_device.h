// Device-side building blocks of the coarse-to-fine page selection (Sec. 3.2, Eq. 4, Alg. 1 stage 2),
// shared by the selection kernels and the fused decode-step kernel.
//
// A cluster of C workgroups cooperates on one (sequence, KV head) -- or, under the model-wide scope, on one
// sequence -- through the three levels grids -> chunks -> pages.  The paper scores the whole hierarchy with one
// GEMM and prunes with masks; here a level reads only vectors it can need, and a level's work is split over the
// cluster, so one (sequence, head) draws bandwidth from C compute units.  A 16-lane group scores one unit (one or
// two 128-bit loads per lane, several units in flight per group, fp64 multiply-add, DPP row sum) and publishes an
// order-preserving 64-bit key into the unit's word of the workspace.
//
// Two schedules, chosen by the host:
//   lazy    grids; then the chunks of kept grids; then the pages of kept chunks: three dependent memory phases,
//           the fewest bytes (what a bandwidth-bound launch wants);
//   merged  grids and ALL chunks in one phase, two cuts back to back, then the pages of kept chunks: two memory
//           phases and one exchange fewer for n_c - k_g N_g more chunk vectors (what a latency-bound launch
//           wants).  The scores are the same numbers either way, so the kept sets are too.
// Grid and chunk keys live in unit order (word / LDS slot = unit index, chunks behind the grids; a chunk competes
// only if its grid was kept: the grid cut leaves a zero in the key slot of every grid it drops); page keys live in
// slot order (N_c slots per kept chunk).
//
// There is no barrier between the members: a key word is 0 until its owner has published it (a slot without a unit
// is published as 1), so a member polls the words it needs until none is 0.  One memory round trip serves as
// both the wait and the transfer.  Every member then finds the cut itself (all compute the same thing): bounds
// from the upper key halves, a histogram over 1024 bins that are linear in the (fp32-rounded) score, a scan from
// the top, an exact ranking by (key, slot) of the few keys in the bin the k-th largest falls in, ballots for the
// positions in the ascending list of kept units.  Ties at the cut go to the lowest slots (= lowest indices:
// candidates are enumerated in index order), or are all kept under the threshold rule.  A level of up to 64 slots is
// ranked by one wave with lane reads alone, up to 256 slots by one wave with four keys per lane and no barrier
// inside; larger levels keep their keys four (up to 1024 slots; the polled keys arrive in registers) or seventeen
// per thread over the whole workgroup, with LDS lists between the waves.  (One wave cutting 1024 keys, sixteen per
// lane, was measured: 8-9 us instead of 3-4, a single wave being a long chain of dependent instructions.)  Score
// distributions that pile more than 64 keys into the bin at the cut (exact ties, mostly) take a general path: radix
// select on the bits the keys do not share, then a ballot compaction.
//
// The words are cleared again by the workgroup that is last to be done with them, so they are all 0 between
// launches.  Polls are bounded: a wait that does not end raises the workspace's error flag and the workgroup
// leaves (the workspace then needs chess_workspace_init again).
#pragma once

#include <type_traits>

#include "chess_internal.h"

namespace chess {

constexpr int kSelWaves = kSelThreads / kWave;
constexpr int kPollLimit = 1 << 15;         // polls (each a memory round trip, ~1 us) before a wait is declared dead (default)
constexpr int kKeepAll = 0x7fffffff;
constexpr uint64_t kAbsentKey = 1ull;       // published for a slot that has no unit; below every real key
constexpr uint64_t kMarkKey = 2ull;         // "this grid was kept" where no real key exists; below every real key too

// Monotone map double -> uint64 (larger score = larger key); every finite or infinite score maps
// to a key >= 2^52 - 1, so 0 can mark "not published yet" and 1 "no unit".  -0.0 is folded onto +0.0.
__device__ __forceinline__ uint64_t order_key(double s)
{
    s += 0.0;
    const uint64_t u = (uint64_t)__double_as_longlong(s);
    return (u >> 63) ? ~u : (u | 0x8000000000000000ull);
}

// A float that never decreases when the key grows: the score with its lower 32 bits dropped, rounded to fp32,
// kept finite.  All the binning of a cut needs is this monotonicity (a higher bin then means a strictly larger
// score); the exact order inside a bin is settled on the 64-bit keys.
__device__ __forceinline__ float key_float(unsigned key_hi)
{
    const unsigned u = (key_hi >> 31) ? (key_hi & 0x7fffffffu) : ~key_hi;
    const float f = (float)__hiloint2double((int)u, 0);
    return fminf(fmaxf(f, -3.0e38f), 3.0e38f);
}

__device__ __forceinline__ int ceil_div_i(int a, int b) { return (a + b - 1) / b; }
__device__ __forceinline__ int ceil_bp(int n, int bp) { return (int)(((int64_t)n * bp + 9999) / 10000); }
__device__ __forceinline__ int clamp_i(int x, int lo, int hi) { return x < lo ? lo : (x > hi ? hi : x); }

// The thread's index as a value the compiler cannot see through.  The levels of a selection run through one loop
// (one copy of the code); whatever is derived from the plain thread index inside the loop body -- slot numbers, LDS
// addresses, for every unrolled instance -- is loop-invariant and would be hoisted out of the loop and kept in
// registers across all of it, to the point of spilling.  Derived from this, it is computed where it is used.
__device__ __forceinline__ int opaque_tid()
{
    int t = threadIdx.x;
    asm volatile("" : "+v"(t));
    return t;
}

// x / fan without a division: inv = ceil(2^32 / fan), computed by the host (unused for fan = 1); exact for x < 2^24 and fan <= 256 (the
// error term x * e / 2^32 with e = fan * inv - 2^32 < fan stays below 1 / fan)
__device__ __forceinline__ int div_by(int x, int fan, uint32_t inv) { return fan > 1 ? (int)__umulhi((unsigned)x, inv) : x; }

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

// Lane i of each row of 16 receives lane i + n of the row (n constant after unrolling; n = 0: the value itself).
__device__ __forceinline__ unsigned row_shl_by(unsigned v, int n)
{
#define CHESS_SHL_CASE(k) case k: return (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x100 + k, 0xf, 0xf, false);
    switch (n) {
        CHESS_SHL_CASE(1) CHESS_SHL_CASE(2) CHESS_SHL_CASE(3) CHESS_SHL_CASE(4) CHESS_SHL_CASE(5) CHESS_SHL_CASE(6) CHESS_SHL_CASE(7)
        CHESS_SHL_CASE(8) CHESS_SHL_CASE(9) CHESS_SHL_CASE(10) CHESS_SHL_CASE(11) CHESS_SHL_CASE(12) CHESS_SHL_CASE(13)
        CHESS_SHL_CASE(14) CHESS_SHL_CASE(15)
    default: return v;
    }
#undef CHESS_SHL_CASE
}

__device__ __forceinline__ uint64_t lane_read64(uint64_t v, int src)
{
    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)v, src);
    const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(v >> 32), src);
    return ((uint64_t)hi << 32) | lo;
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

// ---------------------------------------------------------------------------------------------------------------
// Summary vectors in memory.  T = float: 128 fp32, a lane of a 16-lane group holds dims 4 ln .. 4 ln + 3 and
// 64 + 4 ln .. 64 + 4 ln + 3 (two 128-bit loads).  T = uint16_t: 128 bf16, a lane holds dims 8 ln .. 8 ln + 7
// (one 128-bit load).  lane_dim gives the dim of a lane's i-th element; a probe is held in the same arrangement.
template <class T>
struct Vec;

template <>
struct Vec<float> {
    float4 a, b;
    __device__ __forceinline__ void load(const float* row, int ln)
    {
        const float4* p = reinterpret_cast<const float4*>(row) + ln;
        a = p[0];
        b = p[16];
    }
    template <int I>
    __device__ __forceinline__ double at() const
    {
        return (double)(I == 0 ? a.x : I == 1 ? a.y : I == 2 ? a.z : I == 3 ? a.w : I == 4 ? b.x : I == 5 ? b.y : I == 6 ? b.z : b.w);
    }
    static __device__ __forceinline__ int lane_dim(int ln, int i) { return i < 4 ? 4 * ln + i : 64 + 4 * ln + (i - 4); }
};

template <>
struct Vec<uint16_t> {
    uint4 v;
    __device__ __forceinline__ void load(const uint16_t* row, int ln) { v = reinterpret_cast<const uint4*>(row)[ln]; }
    template <int I>
    __device__ __forceinline__ double at() const
    {
        const uint32_t w = I < 2 ? v.x : I < 4 ? v.y : I < 6 ? v.z : v.w;
        return (double)__uint_as_float((I & 1) ? (w & 0xffff0000u) : (w << 16));
    }
    static __device__ __forceinline__ int lane_dim(int ln, int i) { return 8 * ln + i; }
};

// Eq. 4 for one unit: this lane's eight products, fp64, in element order (the 16 lanes' partial sums are then
// added by row16_sum).
template <class T>
__device__ __forceinline__ double dot8(const double (&pr)[8], const Vec<T>& v, double d = 0.0)
{
    d = fma(pr[0], v.template at<0>(), d); d = fma(pr[1], v.template at<1>(), d);
    d = fma(pr[2], v.template at<2>(), d); d = fma(pr[3], v.template at<3>(), d);
    d = fma(pr[4], v.template at<4>(), d); d = fma(pr[5], v.template at<5>(), d);
    d = fma(pr[6], v.template at<6>(), d); d = fma(pr[7], v.template at<7>(), d);
    return d;
}

// acc[i] += this lane's i-th element
template <class T>
__device__ __forceinline__ void add8(double (&acc)[8], const Vec<T>& v)
{
    acc[0] += v.template at<0>(); acc[1] += v.template at<1>(); acc[2] += v.template at<2>(); acc[3] += v.template at<3>();
    acc[4] += v.template at<4>(); acc[5] += v.template at<5>(); acc[6] += v.template at<6>(); acc[7] += v.template at<7>();
}

// A mean as the summaries store it: the fp64 value rounded to fp32 once; for bf16 summaries that fp32 value
// rounded to nearest-even bf16 (finite inputs).
template <class T>
__device__ __forceinline__ T stored(double mean);
template <>
__device__ __forceinline__ float stored<float>(double mean) { return (float)mean; }
template <>
__device__ __forceinline__ uint16_t stored<uint16_t>(double mean)
{
    const uint32_t u = __float_as_uint((float)mean);
    return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}
__device__ __forceinline__ double loaded(float v) { return (double)v; }
__device__ __forceinline__ double loaded(uint16_t v) { return (double)__uint_as_float((uint32_t)v << 16); }

constexpr int kBins = 1024;                 // linear score bins of the cut
constexpr int kSelGroups = kSelThreads / 16;  // 16-lane groups of a workgroup
constexpr int kFastMembers = 64;            // most keys the bin at the cut may hold on the histogram paths
constexpr int kRegsLarge = (4352 + kSelThreads - 1) / kSelThreads;       // keys per thread of the largest level the register path holds
constexpr int kMaxRuns = kRegsLarge * kSelWaves;  // its 64-slot runs
constexpr int kOneWaveSlots = 4 * kWave;    // largest level one wave cuts by itself

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

// What the kernels do to a Shared before the first level: the histogram all zero, no collected members.
__device__ __forceinline__ void init_shared(Shared& sh, int poll_limit)
{
    for (int i = threadIdx.x; i < kBins; i += kSelThreads) sh.hist[i] = 0;
    if (threadIdx.x == 0) { sh.n_mem = 0; sh.poll_limit = poll_limit; }
    if (threadIdx.x < 3) sh.tail_key[threadIdx.x] = 0ull;
}

// Eq. 3: the query anchor of a (sequence, KV head), the mean of the page vectors of the recent window (the last
// min(w, P) pages): fp64 sum in page order, divided by the count, rounded to fp32 once (the anchor is an fp32 vector
// whatever the summaries' storage type).  This lane's dims as Vec<T> arranges them.  Four pages per request.
template <class T>
__device__ __forceinline__ void load_anchor(const T* __restrict__ pages_row, int P, int w, double (&pr)[8])
{
    const int ln = threadIdx.x & 15;
    const int W = min(w, P), first = P - W;
    double acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int j0 = first; j0 < P; j0 += 4) {
        Vec<T> v[4];
#pragma unroll
        for (int x = 0; x < 4; ++x) v[x].load(pages_row + (size_t)min(j0 + x, P - 1) * kHeadDim, ln);
#pragma unroll
        for (int x = 0; x < 4; ++x)
            if (j0 + x < P) add8<T>(acc, v[x]);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) pr[i] = (double)(float)(acc[i] / (double)W);
}

// Phase timestamps of profiling builds (-DCHESS_PROF): mark(i) stores the clock in slot i; nothing otherwise.
struct Prof {
#ifdef CHESS_PROF
    static constexpr int kSlots = 24;
    long long t[kSlots];
    __device__ __forceinline__ Prof() { for (int i = 0; i < kSlots; ++i) t[i] = 0; }
    __device__ __forceinline__ void mark(int i) { t[i] = wall_clock64(); }
    // the clock once `value` has arrived in a register (waits for the load that produces it)
    __device__ __forceinline__ void mark_after(int i, int value) { asm volatile("" ::"v"(value)); t[i] = wall_clock64(); }
    __device__ __forceinline__ void store(int32_t* dst) const
    {
        for (int i = 0; i < kSlots; ++i) dst[i] = t[i] != 0 ? (int32_t)(t[i] - t[0]) : -1;
    }
#else
    __device__ __forceinline__ void mark(int) {}
    __device__ __forceinline__ void mark_after(int, int) {}
#endif
};

// How many units a level keeps, as data (so that the three levels run through one copy of the cut code):
// rho_bp > 0: clamp(ceil(n * rho), 1, n) (the paper's ratios); else min(n, target); never more than cap.
struct KeepRule {
    int rho_bp, target, cap;
    __device__ __forceinline__ int operator()(int n) const
    {
        const int k = rho_bp > 0 ? (n == 0 ? 0 : clamp_i(ceil_bp(n, rho_bp), 1, n)) : min(n, target);
        return min(k, cap);
    }
};

// Which slots of a level compete, as data: every slot, or slot i only if mask[i / fan] is non-zero (a chunk
// competes only if the grid cut left its grid's key in place).
struct ActiveRule {
    const uint64_t* mask;   // LDS, or null: every slot
    int fan;
    uint32_t inv;
    __device__ __forceinline__ bool operator()(int i) const { return mask == nullptr || mask[div_by(i, fan, inv)] != 0ull; }
};

// Where a kept slot goes, as data: out[pos] = the slot's unit (the slot itself, or parents[slot / fan] * fan +
// slot % fan); with phys_by_slot, sel_phys[pos] = phys_by_slot[slot] as well.
struct EmitRule {
    int32_t* out;
    const int32_t* parents;   // LDS, or null: unit = slot
    int fan;
    uint32_t inv;
    int32_t* sel_phys;
    const int32_t* phys_by_slot;
    __device__ __forceinline__ void operator()(int pos, int slot) const
    {
        int unit = slot;
        if (parents != nullptr) {
            const int pi = div_by(slot, fan, inv);
            unit = parents[pi] * fan + (slot - pi * fan);
        }
        out[pos] = unit;
        if (phys_by_slot != nullptr) sel_phys[pos] = phys_by_slot[slot];
    }
};

struct Cut {
    uint64_t thr;   // in the shifted domain: key << shift
    int ties;       // how many of the slots whose shifted key equals thr are kept, lowest slots first
    int shift;
};

// Cut of the top-k among the non-empty keys in LDS by radix select: k = k_of(number of non-empty keys).
// A non-empty slot is kept iff (key << shift) > thr, or (key << shift) == thr and it is among the first
// `ties` such slots (all of them when keep_ties is set: the threshold rule).  Uniform over the workgroup; every
// thread must call it.
__device__ __forceinline__ Cut find_cut_radix(const uint64_t* keys, int n_slots, const KeepRule& k_of, bool keep_ties, Shared& sh)
{
    const int tid = opaque_tid(), lane = tid & 63, wave = tid >> 6;
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
    const int tie_all = keep_ties ? kKeepAll : 0;
    Cut cut;
    cut.shift = 0;
    if (k <= 0) { cut.thr = ~0ull; cut.ties = 0; return cut; }
    if (k >= n_valid) { cut.thr = 0ull; cut.ties = kKeepAll; return cut; }
    const uint64_t diff = all_or ^ all_and;
    if (diff == 0) { cut.thr = all_or; cut.ties = max(k, tie_all); return cut; }    // every key is the same: first k slots
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
    cut.ties = max(want, tie_all);
    return cut;
}

// Ordered compaction: emit(pos, slot) for the kept slots in ascending slot order; returns their number.
// Wave w owns a contiguous quarter of the slots and walks it 64 slots at a time with ballots.  mark: the key
// slot of every slot that is not kept is set to zero.
__device__ __forceinline__ int compact_kept(uint64_t* keys, int n_slots, const Cut& cut, const EmitRule& emit, int cap, bool mark,
                                            Shared& sh)
{
    const int tid = opaque_tid(), lane = tid & 63, wave = tid >> 6;
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
        const int at = pos + __popcll(kb & below);
        if (keep && at < cap) emit(at, i);
        if (mark && i < hi && !keep) keys[i] = 0ull;
        pos += __popcll(kb);
        eq_seen += __popcll(eqb);
    }
    __syncthreads();
    return total;
}

// Where bin b of the histogram is stored: lane l of a wave owns bins 16 (63 - l) .. 16 (63 - l) + 15 (lane 0
// the highest scores) and reads its j-th bin from word 64 j + l, so the 64 lanes hit 64 different banks.
__device__ __forceinline__ int hist_word(int b) { return ((b & 15) << 6) | (63 - (b >> 4)); }

// The bin the k-th largest key falls in, from the histogram (a scan from the top, by one wave, all lanes active):
// returns the bin, *want = how many of that bin's keys are among the k largest, *cnt = how many keys it holds.
__device__ __forceinline__ int find_cut_bin(const int* hist, int k, int* want, int* cnt)
{
    const int lane = opaque_tid() & 63;
    auto f_add = [](int a, int b) { return a + b; };
    int own = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) own += hist[64 * j + lane];
    const int incl = wave_scan(own, 0, f_add);
    const bool here = incl - own < k && k <= incl;            // true in exactly one lane
    const int src = __builtin_amdgcn_readfirstlane(__ffsll((long long)__ballot(here)) - 1);
    const int k_rem = k - (__builtin_amdgcn_readlane(incl, src) - __builtin_amdgcn_readlane(own, src));
    // the 16 bins of that lane, highest first, one per lane of the first row
    const int c = lane < 16 ? hist[64 * (15 - lane) + src] : 0;
    int ci = c;
    ci += __builtin_amdgcn_update_dpp(0, ci, 0x111, 0xf, 0xf, false);
    ci += __builtin_amdgcn_update_dpp(0, ci, 0x112, 0xf, 0xf, false);
    ci += __builtin_amdgcn_update_dpp(0, ci, 0x114, 0xf, 0xf, false);
    ci += __builtin_amdgcn_update_dpp(0, ci, 0x118, 0xf, 0xf, false);
    const int at = __builtin_amdgcn_readfirstlane(__ffsll((long long)__ballot(lane < 16 && ci >= k_rem)) - 1);
    *cnt = __builtin_amdgcn_readlane(c, at);
    *want = k_rem - (__builtin_amdgcn_readlane(ci, at) - *cnt);
    return 16 * (63 - src) + 15 - at;
}

// Rank the members of the bin at the cut (lane j < cnt holds member j: key `mine`, slot `my_slot`) by (key
// descending, slot ascending) with lane reads; returns the key and slot of the member that is last to be kept
// (rank want - 1) and, in *kept_mask, the lanes whose members are kept: rank < want, or under the threshold rule
// every member whose key is at least that member's.
__device__ __forceinline__ void rank_members(uint64_t mine, int my_slot, int cnt, int want, bool keep_ties, uint64_t* thr,
                                             int* thr_slot, uint64_t* kept_mask)
{
    const int lane = opaque_tid() & 63;
    int rank = 0;
    for (int i = 0; i < cnt; ++i) {
        const uint64_t ki = lane_read64(mine, i);
        const int si = __builtin_amdgcn_readlane(my_slot, i);
        rank += ki > mine || (ki == mine && si < my_slot);
    }
    const int src = __builtin_amdgcn_readfirstlane(__ffsll((long long)__ballot(lane < cnt && rank == want - 1)) - 1);
    *thr = lane_read64(mine, src);
    *thr_slot = __builtin_amdgcn_readlane(my_slot, src);
    *kept_mask = __ballot(lane < cnt && (rank < want || (keep_ties && mine == *thr)));
}

// Cut and ordered compaction of one level of more than kOneWaveSlots slots, its keys R per thread over the whole
// workgroup: thread t takes slot x * 256 + t of the LDS copy in key[x] (0 = empty or not competing).  k =
// k_of(n_valid) of the n_valid competing keys are kept, by (key descending, slot ascending); emit(pos, slot) is
// called for each kept slot with its position in ascending slot order (positions at or beyond cap are dropped).
// Returns the number kept, or -1, having emitted nothing, when this path does not apply (more than kFastMembers
// keys share the bin at the cut).  Uniform over the workgroup: every thread must call it, after a barrier that
// made `keys` complete.  sh.hist must be all zero and sh.n_mem zero on entry, and they are again on a return >= 0.
//
// The kBins bins are LINEAR in key_float between the smallest and the largest key: a monotone map, so a higher bin
// means a strictly larger score.  A scan from the top finds the bin the k-th largest key falls in, and the few
// keys of that bin are ranked exactly by (key, slot).
//
// kPre: the thread's keys come in `pre` (the pull left them in registers, together with every wave's bounds and count
// in sh.st_*, before its closing barrier): nothing is re-read and the first barrier here falls away.  Only for
// levels in which every slot competes.
template <int R, bool kPre = false>
__device__ __forceinline__ int cut_in_registers(uint64_t* keys, int n_slots, const ActiveRule& active, const KeepRule& k_of,
                                                bool keep_ties, const EmitRule& emit, int cap, bool mark, Shared& sh,
                                                const uint64_t (&pre)[4])
{
    static_assert(kBins == 16 * kWave, "a lane owns 16 bins");
    static_assert(R * kSelWaves <= kMaxRuns && R * kSelWaves <= 128, "run prefix is held in two values per lane");
    const int tid = opaque_tid(), lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint64_t below = __lanemask_lt();
    auto f_add = [](int a, int b) { return a + b; };

    // this thread's keys; every wave leaves the bounds and the count of what it sees
    uint64_t key[R];
    if constexpr (kPre) {
#pragma unroll
        for (int x = 0; x < R; ++x) key[x] = pre[x < 4 ? x : 0];
    } else {
        unsigned a = ~0u, b = 0u;
        int n = 0;
#pragma unroll
        for (int x = 0; x < R; ++x) {
            key[x] = 0ull;
            if (R > 4 && x * kSelThreads >= n_slots) continue;    // uniform (a branch per key only pays when there are many)
            const int i = x * kSelThreads + tid;
            key[x] = (i < n_slots && active(i)) ? keys[i] : 0ull;
            const bool valid = key[x] != 0ull;
            const unsigned hi = (unsigned)(key[x] >> 32);
            a = valid ? min(a, hi) : a;
            b = valid ? max(b, hi) : b;
            n += __popcll(__ballot(valid));
        }
        a = wave_minmax32<true>(a);
        b = wave_minmax32<false>(b);
        if (lane == 63) { sh.st_min[wave] = a; sh.st_max[wave] = b; sh.st_cnt[wave] = n; }
        __syncthreads();
    }
    unsigned lo_h = ~0u, hi_h = 0u;
    int n_valid = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) {
        lo_h = min(lo_h, sh.st_min[w]);
        hi_h = max(hi_h, sh.st_max[w]);
        n_valid += sh.st_cnt[w];
    }
    const int k = k_of(n_valid);
    if (k <= 0) {
        if (mark) {
#pragma unroll
            for (int x = 0; x < R; ++x)
                if (x * kSelThreads + tid < n_slots) keys[x * kSelThreads + tid] = 0ull;
        }
        __syncthreads();
        return 0;
    }
    const bool all = k >= n_valid;

    int bin[R];
    int cutbin = -1, want = 0, cnt = 0;
    if (!all) {
        const float fmin = key_float(lo_h), fmax = key_float(hi_h);
        const float scale = fmax > fmin ? (float)kBins / (fmax - fmin) : 0.f;
#pragma unroll
        for (int x = 0; x < R; ++x) {
            bin[x] = -1;
            if (x * kSelThreads < n_slots && key[x] != 0) {
                bin[x] = min((int)((key_float((unsigned)(key[x] >> 32)) - fmin) * scale), kBins - 1);
                atomicAdd(&sh.hist[hist_word(bin[x])], 1);
            }
        }
        __syncthreads();
        cutbin = find_cut_bin(sh.hist, k, &want, &cnt);           // every wave scans the whole histogram
        if (cnt > kFastMembers) return -1;
    } else {
#pragma unroll
        for (int x = 0; x < R; ++x) bin[x] = 0;
    }

    // keys above the cut bin are kept for sure: count them per 64-slot run; collect the cut bin's keys
    unsigned sure = 0, maybe = 0;
#pragma unroll
    for (int x = 0; x < R; ++x) {
        if (R > 4 && x * kSelThreads >= n_slots) break;           // uniform
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
        rank_members(mine, my_slot, cnt, want, keep_ties, &thr, &thr_slot, &kept_mask);
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
    // sure keys in earlier runs
    const int n_runs = (n_slots + kWave - 1) / kWave;
    const int c0 = lane < n_runs ? sh.run_gt[lane] : 0;
    const int i0 = wave_scan(c0, 0, f_add);
    const int e0 = i0 - c0;
    int e1 = 0, sure_total = __builtin_amdgcn_readlane(i0, 63);
    if (R * kSelWaves > kWave) {
        const int c1 = lane + kWave < n_runs ? sh.run_gt[min(lane + kWave, kMaxRuns - 1)] : 0;
        const int i1 = wave_scan(c1, 0, f_add);
        e1 = i1 - c1 + __builtin_amdgcn_readlane(i0, 63);
        sure_total += __builtin_amdgcn_readlane(i1, 63);
    }
#pragma unroll
    for (int x = 0; x < R; ++x) {
        if (R > 4 && x * kSelThreads >= n_slots) break;           // uniform
        const int run = x * kSelWaves + wave;
        const int base = x * kSelWaves < kWave ? __builtin_amdgcn_readlane(e0, run) : __builtin_amdgcn_readlane(e1, run - kWave);
        const bool a = (sure >> x) & 1, e = (maybe >> x) & 1;
        const int slot = x * kSelThreads + tid;
        const uint64_t ab = __ballot(a);
        const bool keep = a || (e && (key[x] > thr || (key[x] == thr && (slot <= thr_slot || keep_ties))));
        const int at = base + __popcll(ab & below) + before[x];
        if (keep && at < cap) emit(at, slot);
        if (mark && slot < n_slots && !keep) keys[slot] = 0ull;
    }
    __syncthreads();                                              // mem_key / run_gt readers are done; emitted lists visible
    return sure_total + __popcll(kept_mask);
}

// Cut and ordered compaction of a level of at most 64 R slots by ONE wave, with no workgroup barrier inside: wave 0
// holds slot x * 64 + lane of the LDS copy of the keys in key[x] and does what cut_in_registers does -- bounds from
// the upper key halves, linear-bin histogram, scan from the top, exact ranking of the bin at the cut -- with ballots
// and lane reads in place of the LDS lists between waves (the other waves wait at the closing barrier; LDS
// operations of one wave complete in order, so its own histogram and member list need no barrier).  Same contract
// as cut_in_registers; returns -1 (to every thread), having emitted nothing, when more than kFastMembers keys share
// the bin at the cut.
template <int R>
__device__ __forceinline__ int cut_by_one_wave(uint64_t* keys, int n_slots, const ActiveRule& active, const KeepRule& k_of,
                                               bool keep_ties, const EmitRule& emit, int cap, bool mark, Shared& sh)
{
    const int tid = opaque_tid(), lane = tid & 63;
    if (tid < kWave) {
        const uint64_t below = __lanemask_lt();
        uint64_t key[R];
        unsigned lo_h = ~0u, hi_h = 0u;
        int n_valid = 0;
#pragma unroll
        for (int x = 0; x < R; ++x) {
            const int i = x * kWave + lane;
            key[x] = (i < n_slots && active(i)) ? keys[i] : 0ull;
            const bool valid = key[x] != 0ull;
            const unsigned h = (unsigned)(key[x] >> 32);
            lo_h = valid ? min(lo_h, h) : lo_h;
            hi_h = valid ? max(hi_h, h) : hi_h;
            n_valid += __popcll(__ballot(valid));
        }
        const int k = k_of(n_valid);
        const bool all = k >= n_valid;
        int result = 0;
        int bin[R];
        int cutbin = -1, want = 0, cnt = 0;
        if (k > 0 && !all) {
            lo_h = (unsigned)__builtin_amdgcn_readlane((int)wave_minmax32<true>(lo_h), 63);
            hi_h = (unsigned)__builtin_amdgcn_readlane((int)wave_minmax32<false>(hi_h), 63);
            const float fmin = key_float(lo_h), fmax = key_float(hi_h);
            const float scale = fmax > fmin ? (float)kBins / (fmax - fmin) : 0.f;
#pragma unroll
            for (int x = 0; x < R; ++x) {
                bin[x] = -1;
                if (key[x] != 0ull) {
                    bin[x] = min((int)((key_float((unsigned)(key[x] >> 32)) - fmin) * scale), kBins - 1);
                    atomicAdd(&sh.hist[hist_word(bin[x])], 1);
                }
            }
            __builtin_amdgcn_wave_barrier();
            cutbin = find_cut_bin(sh.hist, k, &want, &cnt);
            // leave the histogram clean: this wave is its only user at this level
#pragma unroll
            for (int x = 0; x < R; ++x)
                if (bin[x] >= 0) sh.hist[hist_word(bin[x])] = 0;
        } else {
#pragma unroll
            for (int x = 0; x < R; ++x) bin[x] = 0;
        }
        if (cnt > kFastMembers) {
            result = -1;
        } else if (k > 0) {
            // the keys of the bin at the cut, one per lane (through LDS, in slot order), ranked against each other
            uint64_t thr = 0ull;
            int thr_slot = -1;
            if (cnt > 0) {
                int at0 = 0;
#pragma unroll
                for (int x = 0; x < R; ++x) {
                    const bool e = bin[x] == cutbin && key[x] != 0ull;
                    const uint64_t eb = __ballot(e);
                    if (e) {
                        const int at = at0 + __popcll(eb & below);
                        sh.mem_key[at] = key[x];
                        sh.mem_slot[at] = x * kWave + lane;
                    }
                    at0 += __popcll(eb);
                }
                __builtin_amdgcn_wave_barrier();
                const uint64_t mine = lane < cnt ? sh.mem_key[lane] : 0ull;
                const int my_slot = lane < cnt ? sh.mem_slot[lane] : 0;
                uint64_t kept_mask;
                rank_members(mine, my_slot, cnt, want, keep_ties, &thr, &thr_slot, &kept_mask);
            }
            int base = 0;
#pragma unroll
            for (int x = 0; x < R; ++x) {
                if (x * kWave >= n_slots) break;                  // uniform
                const int slot = x * kWave + lane;
                const bool valid = key[x] != 0ull;
                const bool keep = all ? valid
                                      : valid && (bin[x] > cutbin ||
                                                  (bin[x] == cutbin && (key[x] > thr || (key[x] == thr && (slot <= thr_slot || keep_ties)))));
                const uint64_t kb = __ballot(keep);
                const int at = base + __popcll(kb & below);
                if (keep && at < cap) emit(at, slot);
                if (mark && slot < n_slots && !keep) keys[slot] = 0ull;
                base += __popcll(kb);
            }
            result = base;
        } else if (mark) {
#pragma unroll
            for (int x = 0; x < R; ++x)
                if (x * kWave + lane < n_slots) keys[x * kWave + lane] = 0ull;
        }
        if (lane == 0) sh.cnt = result;
    }
    __syncthreads();
    return sh.cnt;
}

// A level of at most 64 slots: one key per lane of wave 0, each lane counts the keys that rank before its own
// (key descending, slot ascending) with lane reads; no histogram, no LDS.  Same contract as cut_by_one_wave (it
// always applies).
__device__ __forceinline__ int cut_one_lane_each(uint64_t* keys, int n_slots, const ActiveRule& active, const KeepRule& k_of,
                                                 bool keep_ties, const EmitRule& emit, int cap, bool mark, Shared& sh)
{
    const int tid = opaque_tid();
    if (tid < kWave) {
        const int lane = tid;
        const uint64_t key = (lane < n_slots && active(lane)) ? keys[lane] : 0ull;
        const uint64_t valid = __ballot(key != 0ull);
        const int k = k_of(__popcll(valid));
        int rank = 0, above = 0;                        // keys that rank before this one; keys strictly larger
        for (uint64_t mk = valid; mk != 0ull; mk &= mk - 1) {
            const int j = __builtin_amdgcn_readfirstlane(__ffsll((long long)mk) - 1);
            const uint64_t kj = lane_read64(key, j);
            rank += kj > key || (kj == key && j < lane);
            above += kj > key;
        }
        // threshold rule: a key is kept when fewer than k keys are strictly larger (it ties with or beats the k-th)
        const uint64_t kb = __ballot(key != 0ull && (keep_ties ? above < k : rank < k));
        const bool keep = (kb >> lane) & 1ull;
        const int at = __popcll(kb & __lanemask_lt());
        if (keep && at < cap) emit(at, lane);
        if (mark && lane < n_slots && !keep) keys[lane] = 0ull;
        if (lane == 0) sh.cnt = __popcll(kb);
    }
    __syncthreads();
    return sh.cnt;
}

// The cut of one level whose keys are complete in `keys` (LDS; the caller's barrier has made them visible): picks
// the path by the level's size.  Returns the number kept (what would have been emitted; positions at or beyond
// `cap` are not written: the caller treats a count above cap as an overflow).  Every thread must call it.
// have_pre: the pull handed this thread's four keys over in registers (pull_keys_regs), in `pre`.
__device__ __forceinline__ int cut_level(uint64_t* keys, int n_slots, const ActiveRule& active, const KeepRule& k_of,
                                         bool keep_ties, bool general, const EmitRule& emit, int cap, bool mark, Shared& sh,
                                         bool have_pre, const uint64_t (&pre)[4])
{
    int n = -1;
    if (!general) {
        if (n_slots <= kWave) n = cut_one_lane_each(keys, n_slots, active, k_of, keep_ties, emit, cap, mark, sh);
        else if (n_slots <= kOneWaveSlots) n = cut_by_one_wave<4>(keys, n_slots, active, k_of, keep_ties, emit, cap, mark, sh);
        else if (n_slots <= 4 * kSelThreads && have_pre) n = cut_in_registers<4, true>(keys, n_slots, active, k_of, keep_ties, emit, cap, mark, sh, pre);
        else if (n_slots <= 4 * kSelThreads) n = cut_in_registers<4>(keys, n_slots, active, k_of, keep_ties, emit, cap, mark, sh, pre);
        else if (n_slots <= kRegsLarge * kSelThreads) n = cut_in_registers<kRegsLarge>(keys, n_slots, active, k_of, keep_ties, emit, cap, mark, sh, pre);
    }
    if (n >= 0) return n;
    // general path on the LDS copy of the keys: slots that do not compete are emptied first
    const int tid = opaque_tid();
    if (active.mask != nullptr) {
        for (int i = tid; i < n_slots; i += kSelThreads)
            if (!active(i)) keys[i] = 0ull;
    }
    __syncthreads();
    const Cut cut = find_cut_radix(keys, n_slots, k_of, keep_ties, sh);
    n = compact_kept(keys, n_slots, cut, emit, cap, mark, sh);
    for (int i = tid; i < kBins; i += kSelThreads) sh.hist[i] = 0;
    if (tid == 0) sh.n_mem = 0;
    __syncthreads();
    return n;
}

// One work slot of a scoring pass: where the unit's vector is (array 0 = grids, 1 = chunks, 2 = pages; unit -1 =
// the slot has no unit) and where its key goes (index into the level's key words, in LDS or in the workspace; -1 =
// nowhere).
struct SlotRef {
    int array, unit, dest;
};

// Units a 16-lane group requests before it waits: one memory round trip covers kFly * 16 work slots of a workgroup.
template <class T>
constexpr int kFlyOf = sizeof(T) == 2 ? 12 : 9;      // (what the fused step's register budget holds without spilling)

// Scores of the work slots [lo, hi).  `target(slot)` says which unit a slot is.  The key of a slot goes to
// lds_keys[dest] (0 for no unit) when the level is local, else it is published in pub[dest].  (Two pointers of
// known address space: one generic pointer for both would turn every access into a flat one.)
template <class T, class Target>
__device__ __forceinline__ void score_rows(const T* __restrict__ grids_row, const T* __restrict__ chunks_row,
                                           const T* __restrict__ pages_row, int lo, int hi, Target target,
                                           const double (&pr)[8], bool local, uint64_t* lds_keys, uint64_t* pub)
{
    constexpr int kFly = kFlyOf<T>;
    const int tid = opaque_tid(), g16 = tid >> 4, ln = tid & 15;
    for (int s0 = lo; s0 < hi; s0 += kSelGroups * kFly) {
        int unit[kFly], dest[kFly];
        Vec<T> v[kFly];
#pragma unroll
        for (int x = 0; x < kFly; ++x) {
            unit[x] = -1;
            dest[x] = -1;
            const int slot = s0 + kSelGroups * x + g16;
            const SlotRef ref = target(min(slot, hi - 1));
            unit[x] = slot < hi ? ref.unit : -1;
            dest[x] = slot < hi ? ref.dest : -1;
            // no condition on the load, per lane or per row of slots (unit 0 when the slot has no unit; rows the share
            // does not have repeat its last slot): a per-lane condition would make the compiler wait for each vector
            // before asking for the next, and a branch per row costs more than the repeated, cache-resident loads
            const T* base = ref.array == 0 ? grids_row : ref.array == 1 ? chunks_row : pages_row;
            v[x].load(base + (size_t)max(ref.unit, 0) * kHeadDim, ln);
        }
        // The total of vector x ends up in lane 15 of its group; it is handed to lane x of the group, so that one key
        // conversion and one store serve all the vectors of the trip (instead of one masked branch, conversion and
        // store per vector).
        static_assert(kFly <= 16, "a lane of the group per vector of a trip");
        double mine = 0.0;
        int my_unit = -1, my_dest = -1;
#pragma unroll
        for (int x = 0; x < kFly; ++x) {
            if (s0 + kSelGroups * x >= hi) break;     // uniform over the workgroup
            const double d = row16_sum(dot8<T>(pr, v[x]));
            const uint64_t b = (uint64_t)__double_as_longlong(d);
            const unsigned lo = row_shl_by((unsigned)b, 15 - x), hi32 = row_shl_by((unsigned)(b >> 32), 15 - x);
            if (ln == x) {
                mine = __longlong_as_double((long long)(((uint64_t)hi32 << 32) | lo));
                my_unit = unit[x];
                my_dest = dest[x];
            }
        }
        if (my_dest >= 0) {
            if (local) lds_keys[my_dest] = my_unit >= 0 ? order_key(mine) : 0ull;
            else publish_u64(pub + my_dest, my_unit >= 0 ? order_key(mine) : kAbsentKey);
        }
    }
}

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

// The published keys a level needs, into the LDS copy the cuts work on: item j of n lands in keys[dest_of(j)] (dest
// -1: the item is skipped) and comes from pub[dest], except that dest ov_dest0 / ov_dest1 (if >= 0) come from
// tail[ov_word0] / tail[ov_word1]: the keys of units the decode step has just refreshed, which one workgroup
// publishes in words of their own.  The words are polled, up to eight per thread in flight, until every one of them
// is there.  Ends with a workgroup barrier; returns false (to every thread) if a word did not arrive within the
// poll limit.
template <class DestOf>
__device__ __forceinline__ bool pull_keys(const uint64_t* pub, const uint64_t* tail, int n, DestOf dest_of, int ov_dest0,
                                          int ov_word0, int ov_dest1, int ov_word1, uint64_t* keys, int limit)
{
    bool ok = true;
    const int tid = opaque_tid();
    constexpr int kPer = 8;                           // words a thread keeps in flight: one round for levels of up to 2048 slots
    for (int j0 = 0; j0 < n; j0 += kPer * kSelThreads) {
        uint64_t v[kPer];
        int dest[kPer];
        const uint64_t* word[kPer];
        // (no branch around items beyond n: they repeat the last word, which costs a few coalesced requests; a branch per
        // item costs more)
#pragma unroll
        for (int x = 0; x < kPer; ++x) {
            const int j = j0 + x * kSelThreads + tid;
            const int d = dest_of(min(j, n - 1));
            dest[x] = j < n ? d : -1;
            word[x] = pub + max(d, 0);
            if (d >= 0 && d == ov_dest0) word[x] = tail + ov_word0;
            if (d >= 0 && d == ov_dest1) word[x] = tail + ov_word1;
        }
        int polls = 0;
        if (limit <= 0) { ok = false; break; }        // (a test asked for every wait to fail)
        while (true) {
            bool missing = false;
#pragma unroll
            for (int x = 0; x < kPer; ++x) v[x] = observe_u64(word[x]);       // unconditional: all stay in flight
#pragma unroll
            for (int x = 0; x < kPer; ++x) missing = missing || (dest[x] >= 0 && v[x] == 0ull);
            if (__ballot(missing) == 0ull) break;
            if (++polls >= limit) { ok = false; break; }
            __builtin_amdgcn_s_sleep(2);
        }
#pragma unroll
        for (int x = 0; x < kPer; ++x)
            if (dest[x] >= 0) keys[dest[x]] = v[x] == kAbsentKey ? 0ull : v[x];
    }
    return __syncthreads_and(ok) != 0;
}

// The same for a level of at most 1024 slots whose keys sit in slot order (item j lands in keys[j]): thread t polls
// words t, t + 256, t + 512, t + 768 and KEEPS them in key[0..3] (0 = empty or beyond n) for the cut that follows,
// and every wave leaves the bounds (upper key halves) and the count of what it saw in sh.st_* before the closing
// barrier, so that cut_in_registers can start at once.
__device__ __forceinline__ bool pull_keys_regs(const uint64_t* pub, const uint64_t* tail, int n, int ov_dest0, int ov_word0,
                                               int ov_dest1, int ov_word1, uint64_t* keys, uint64_t (&key)[4], int limit, Shared& sh)
{
    bool ok = limit > 0;
    const int tid = opaque_tid(), lane = tid & 63, wave = tid >> 6;
    const uint64_t* word[4];
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        key[x] = 0ull;
        word[x] = pub;
        {
            const int j = x * kSelThreads + tid;
            const int d = min(j, n - 1);
            word[x] = pub + d;
            if (d == ov_dest0) word[x] = tail + ov_word0;
            if (d == ov_dest1) word[x] = tail + ov_word1;
        }
    }
    int polls = 0;
    while (ok) {
        bool missing = false;
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            key[x] = observe_u64(word[x]);                    // unconditional (a word beyond n repeats the last one): all stay in flight
        }
#pragma unroll
        for (int x = 0; x < 4; ++x) missing = missing || key[x] == 0ull;
        if (__ballot(missing) == 0ull) break;
        if (++polls >= limit) { ok = false; break; }
        __builtin_amdgcn_s_sleep(2);
    }
    unsigned a = ~0u, b = 0u;
    int cnt = 0;
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        const int j = x * kSelThreads + tid;
        if (j >= n || key[x] == kAbsentKey || !ok) key[x] = 0ull;
        if (j < n) keys[j] = key[x];
        const bool valid = key[x] != 0ull;
        const unsigned hi = (unsigned)(key[x] >> 32);
        a = valid ? min(a, hi) : a;
        b = valid ? max(b, hi) : b;
        cnt += __popcll(__ballot(valid));
    }
    a = wave_minmax32<true>(a);
    b = wave_minmax32<false>(b);
    if (lane == 63) { sh.st_min[wave] = a; sh.st_max[wave] = b; sh.st_cnt[wave] = cnt; }
    return __syncthreads_and(ok) != 0;
}

// The probe of a (sequence, KV head): the sum of the group's query rows in fp64, g ascending (Eq. 4 with
// Eq. 1's Flatten restricted to the group); this lane's dims as Vec<T> arranges them.
template <class T>
__device__ __forceinline__ void load_probe(const uint16_t* __restrict__ q_rows, int group, double (&pr)[8])
{
    const int ln = threadIdx.x & 15;
#pragma unroll
    for (int i = 0; i < 8; ++i) pr[i] = 0.0;
    // four rows per request (a row beyond the group repeats the last one and is not added): the usual groups of up
    // to four query heads cost one memory round trip, not one per row
    for (int r0 = 0; r0 < group; r0 += 4) {
        uint2 a[4], c[4];
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const uint16_t* row = q_rows + (size_t)min(r0 + x, group - 1) * kHeadDim;
            a[x] = *reinterpret_cast<const uint2*>(row + Vec<T>::lane_dim(ln, 0));
            c[x] = *reinterpret_cast<const uint2*>(row + Vec<T>::lane_dim(ln, 4));
        }
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            if (r0 + x < group) {
                pr[0] += (double)__uint_as_float(a[x].x << 16); pr[1] += (double)__uint_as_float(a[x].x & 0xffff0000u);
                pr[2] += (double)__uint_as_float(a[x].y << 16); pr[3] += (double)__uint_as_float(a[x].y & 0xffff0000u);
                pr[4] += (double)__uint_as_float(c[x].x << 16); pr[5] += (double)__uint_as_float(c[x].x & 0xffff0000u);
                pr[6] += (double)__uint_as_float(c[x].y << 16); pr[7] += (double)__uint_as_float(c[x].y & 0xffff0000u);
            }
        }
    }
}

// Which unit a work slot of each phase is, as small structs whose operator() compiles to straight-line code (the
// scoring loop asks once per vector; a single generic version full of per-level branches cost more instructions
// than the scoring itself).
struct GridPhaseTarget {            // level 0: grids [0, n_g), then (merged) all chunks [n_g, n_g + n_c); keys by unit
    int ng;
    __device__ __forceinline__ SlotRef operator()(int slot) const
    {
        return SlotRef{slot < ng ? 0 : 1, slot < ng ? slot : slot - ng, slot};
    }
};
struct ChunkPhaseTarget {           // level 1 (lazy): N_g slots per kept grid; chunk keys by slot, behind the grid keys
    const int32_t* parents;
    int fan, ng, nc;
    uint32_t inv;
    __device__ __forceinline__ SlotRef operator()(int slot) const
    {
        const int pi = div_by(slot, fan, inv);
        const int u = parents[pi] * fan + (slot - pi * fan);
        return SlotRef{1, u < nc ? u : -1, ng + slot};
    }
};
struct PagePhaseTarget {            // level 2: N_c slots per kept chunk; sink and window pages have no unit; keys by slot
    const int32_t* parents;
    int fan, u_lo, u_hi;
    uint32_t inv;
    __device__ __forceinline__ SlotRef operator()(int slot) const
    {
        const int pi = div_by(slot, fan, inv);
        const int u = parents[pi] * fan + (slot - pi * fan);
        return SlotRef{2, (u >= u_lo && u < u_hi) ? u : -1, slot};
    }
};

struct CascadeResult {
    int n_kp;              // kept pages (their numbers, ascending, are in `sel_pages`)
    int n_a, n_p;          // published words of the grid + chunk phases and of the page phase (what has to be cleared afterwards)
    bool overflow;         // the threshold rule kept more units at some level than the configuration has room for
};

// Where the published words of one (sequence, KV head) -- one sequence under the model-wide scope -- start.
struct PubLayout {
    uint64_t* units;       // grid keys [0, n_g); behind them the chunk keys: by unit (merged) or N_g slots per kept grid (lazy)
    uint64_t* pages;       // page slots: N_c per kept chunk
};
__device__ __forceinline__ PubLayout pub_layout(uint64_t* row_words, const Geom& g)
{
    PubLayout p;
    p.units = row_words;
    p.pages = row_words + g.max_grids + g.max_grids * g.n_g;     // (chunk slots of the lazy schedule: N_g per kept grid)
    return p;
}

// The three levels for one (sequence, KV head) with P > sink + window pages.  Member m of C scores the m-th
// part of every phase.  With want_l3 every member ends up with the kept page numbers in sel_pages[0 .. n_kp);
// without it a member returns as soon as its page keys are published (n_kp = 0).  sh as init_shared leaves it.
// Returns false if a wait was given up.  k_fixed > 0: the page budget of this sequence (fixed_budget); 0: derived
// from its page count.
// The cuts run through one copy of their code (a loop over the levels with the per-level parameters as data, not
// three inlined bodies): the kernel executes every instruction about once, so its time is sensitive to how much
// code it has to fetch.
//
// keys: LDS, max(n_g + n_c, page slots) words.  kept_grids / kept_chunks: LDS lists of the kept units, ascending.
//
// kPhys: the caller goes on to read the kept pages, so the block-table entries of all page-level candidates are
// requested behind the page-level scores (by every member, for all slots) and parked in phys_by_slot (LDS,
// one word per slot); sel_phys[i] then receives the physical page of sel_pages[i].
//
// tail_words non-null: the decode step refreshes the summaries of the tail page, its chunk and its grid in this
// launch.  `refresh_tail()` is called in member 0 once its first vectors are requested; it leaves the three
// units' keys in tail_words[0..2] (grid, chunk, page) for the cluster and in sh.tail_key for itself.  Wherever one
// of these units competes, its key is taken from there instead of the unit's own word (whatever was scored for it
// from the old vector is ignored).
//
// How a phase's work slots are scored is the Scorer's business: scorer(lo, hi, target, local, keys, pub) leaves the
// keys of the work slots [lo, hi) in keys[dest] (local) or publishes them in pub[dest]; a member's share of a
// phase is a multiple of Scorer::kShareRound slots.
template <bool kPhys, class Scorer, class TailFn>
__device__ __forceinline__ bool cascade_with(const Scorer& scorer, int P, const Geom& g,
                                        const SelectParams& sp, const PubLayout& pubs, int m, int C, bool want_l3,
                                        uint64_t* keys, int32_t* kept_grids, int32_t* kept_chunks, int32_t* sel_pages,
                                        Shared& sh, CascadeResult* res, Prof& prof, const uint64_t* tail_words,
                                        TailFn refresh_tail, int k_fixed, const int32_t* __restrict__ bt_row = nullptr,
                                        int32_t* phys_by_slot = nullptr, int32_t* sel_phys = nullptr)
{
    const int s = sp.sink, w = sp.window;
    const uint32_t inv_ng = g.inv_ng, inv_nc = g.inv_nc;                 // (divisions by N_c / N_g: multiply-high, exact below 2^24)
    const int nc = div_by(P + g.n_c - 1, g.n_c, inv_nc), ng = div_by(nc + g.n_g - 1, g.n_g, inv_ng);
    const int k_budget = k_fixed > 0 ? k_fixed : clamp_i(ceil_bp(P, sp.budget_bp), 1, P);
    const int kc_target = div_by(min(sp.over_chunk * k_budget, 1 << 23) + g.n_c - 1, g.n_c, inv_nc);
    const bool ratio = sp.plan == CHESS_PLAN_RATIO, flat = sp.plan == CHESS_PLAN_FLAT;
    const bool general = sp.general_cut != 0, keep_ties = sp.keep_ties != 0;
    res->n_kp = 0; res->n_a = 0; res->n_p = 0; res->overflow = false;

    // how many units a level keeps (built where they are used: three of them alive across the loop cost registers)
    auto rule_of = [&](int level) {
        if (level == 0) return KeepRule{ratio ? sp.rho_g_bp : 0, flat ? kKeepAll : div_by(min(sp.over_grid * kc_target, 1 << 23) + g.n_g - 1, g.n_g, inv_ng), sp.cap_kg};
        if (level == 1) return KeepRule{ratio ? sp.rho_c_bp : 0, flat ? kKeepAll : kc_target, sp.cap_kc};
        return KeepRule{ratio ? sp.rho_p_bp : 0, k_budget, g.max_sel - s - w};
    };

    // A grid level that keeps every grid needs no scores at all, and neither does a chunk level that keeps every
    // chunk of all the grids: the kept list is the list of the units that exist.  Large budgets and ratios near 1
    // end up here.
    const bool all_grids = !general && rule_of(0)(ng) >= ng;
    const bool all_chunks = all_grids && rule_of(1)(nc) >= nc;
    // merged: the chunks are scored together with the grids (one memory phase and one exchange fewer)
    const bool merged = sp.merged != 0 && !all_grids;
    const bool tail_on = tail_words != nullptr;

    int n_kg = 0, n_kc = 0;                           // kept grids, kept chunks
#pragma unroll 1
    for (int level = 0; level < 3; ++level) {
        // (the thread's index as the compiler cannot see through it: what is derived from it inside a level -- slot
        // numbers, addresses -- is then computed where it is used, not hoisted out of the loop over the levels and
        // kept in registers across all of them)
        const int tid_l = opaque_tid();
        // ---- this level's work slots: the units whose scores are computed in this phase
        //  level 0: grids [0, n_g), and with them all chunks [n_g, n_g + n_c) when merged
        //  level 1: chunks of kept grids, N_g slots per kept grid (nothing when merged: they have their keys)
        //  level 2: pages of kept chunks, N_c slots per kept chunk (sink and window pages have no unit there)
        int n_work;
        if (level == 0) n_work = all_grids ? 0 : (merged ? ng + nc : ng);
        else if (level == 1) n_work = (merged || all_chunks) ? 0 : n_kg * g.n_g;
        else n_work = n_kc * g.n_c;
        const GridPhaseTarget target0{ng};
        const ChunkPhaseTarget target1{kept_grids, g.n_g, ng, nc, inv_ng};
        const PagePhaseTarget target2{kept_chunks, g.n_c, s, P - w, inv_nc};
        uint64_t* pub = level == 2 ? pubs.pages : pubs.units;
        // A phase is local when nothing is exchanged for it: a cluster of one; or the grid phase when all grids fit
        // in one request, which every member then scores for itself (the same vectors, so the same keys) instead
        // of waiting a round trip for the others' shares (the host allows it when the repeated reads are few).
        // Otherwise this member takes its share of the phase's slots.
        const bool local = C == 1 || (level == 0 && !merged && sp.local_grids != 0 && n_work <= kSelGroups * 8);
        if (n_work > 0) {
            // (the member that refreshes the tail units has a chain of dependent loads of its own to get through
            // before the first cut: it takes no share of the first phase if the others can still cover it in one
            // memory round trip each)
            const bool spare0 = tail_on && !local && level == 0 && C > 1 && ceil_div_i(n_work, C - 1) <= Scorer::kTrip;
            const int sharers = spare0 ? C - 1 : C, mine = spare0 ? m - 1 : m;
            const int per = local ? n_work : ceil_div_i(ceil_div_i(n_work, sharers), Scorer::kShareRound) * Scorer::kShareRound;
            const int lo = local ? 0 : (mine < 0 ? n_work : min(n_work, mine * per)), hi = min(n_work, lo + per);
            // (one instance of the scoring loop per phase, each with straight-line slot arithmetic)
            if (level == 0) scorer(lo, hi, target0, local, keys, pub);
            else if (level == 1) scorer(lo, hi, target1, local, keys, pub);
            else scorer(lo, hi, target2, local, keys, pub);
            if (!local) { if (level == 2) res->n_p = n_work; else res->n_a = max(res->n_a, level == 0 ? n_work : ng + n_work); }
        }
        // kPhys: the block-table entries of every page slot are requested now, behind this member's vectors, and
        // parked in LDS once the level's keys have been pulled (loads return in order: no wait of their own)
        int32_t entry[kPhys ? kRegsLarge : 1];
        if (kPhys && level == 2) {
#pragma unroll
            for (int x = 0; x < kRegsLarge; ++x) {
                const int i = x * kSelThreads + tid_l;
                entry[kPhys ? x : 0] = 0;
                if (x * kSelThreads < n_work) entry[kPhys ? x : 0] = bt_row[max(i < n_work ? target2(i).unit : -1, 0)];
            }
        }
        prof.mark(2 + 4 * level);
        if (level == 2 && !want_l3) return true;
        // member 0 refreshes the tail units once its first vectors are on their way (the summaries are kept current
        // even if no cut needs one of the three keys)
        if (tail_on && m == 0 && level == 0) refresh_tail();

        // ---- the keys this level's cut needs, into LDS; where a refreshed tail unit competes, its fresh key
        // the tail grid is unit n_g - 1, the tail chunk unit n_c - 1 (key slot n_g + n_c - 1); the tail page is the
        // last slot of the last kept chunk, if it competes at all (no window)
        int ov_dest0 = -1, ov_word0 = 0, ov_dest1 = -1, ov_word1 = 0;
        uint64_t pulled[4] = {0ull, 0ull, 0ull, 0ull};
        bool have_pulled = false;
        const bool merged_phase = merged && level == 0;
        if (tail_on && n_work > 0) {
            if (level == 0) {
                ov_dest0 = ng - 1; ov_word0 = 0;
                if (merged) { ov_dest1 = ng + nc - 1; ov_word1 = 1; }
            } else if (level == 1) {
                // (lazy: the tail chunk is the last existing slot of the last kept grid, if that is the tail grid)
                if (n_kg > 0 && kept_grids[n_kg - 1] == ng - 1) { ov_dest0 = ng + (n_kg - 1) * g.n_g + (nc - 1 - (ng - 1) * g.n_g); ov_word0 = 1; }
            } else if (w == 0 && n_kc > 0 && kept_chunks[n_kc - 1] == nc - 1) {
                ov_dest0 = (n_kc - 1) * g.n_c + (P - 1 - (nc - 1) * g.n_c); ov_word0 = 2;
            }
        }
        if (n_work > 0 && local) {
            __syncthreads();                          // the scores of all waves are in LDS
            if (ov_dest0 >= 0) {
                if (tid_l == 0) {
                    // a cluster of one computed the tail keys itself; otherwise they are polled like any other key
                    const uint64_t k0 = C == 1 ? sh.tail_key[ov_word0] : poll_word(tail_words + ov_word0, sh.poll_limit);
                    const uint64_t k1 = ov_dest1 < 0 ? kMarkKey : C == 1 ? sh.tail_key[ov_word1] : poll_word(tail_words + ov_word1, sh.poll_limit);
                    keys[ov_dest0] = k0;
                    if (ov_dest1 >= 0) keys[ov_dest1] = k1;
                    sh.flag = (k0 != 0ull && k1 != 0ull) ? 1 : 0;
                }
                __syncthreads();
                if (sh.flag == 0) return false;
            }
        } else if (n_work > 0) {
            // (every non-local phase keeps its keys in slot order; a phase of up to 1024 slots hands them to the cut
            // in registers)
            const int off = level == 1 ? ng : 0;
            const int od0 = ov_dest0 >= 0 ? ov_dest0 - off : -1, od1 = ov_dest1 >= 0 ? ov_dest1 - off : -1;
            bool ok;
            if (n_work <= 4 * kSelThreads && !merged_phase) {
                ok = pull_keys_regs(pub + off, tail_words, n_work, od0, ov_word0, od1, ov_word1, keys + off, pulled, sh.poll_limit, sh);
                have_pulled = true;
            } else {
                ok = pull_keys(pub + off, tail_words, n_work, [](int j) { return j; }, od0, ov_word0, od1, ov_word1, keys + off, sh.poll_limit);
            }
            if (!ok) return false;
        }
        if (kPhys && level == 2) {
#pragma unroll
            for (int x = 0; x < kRegsLarge; ++x) {
                if (x * kSelThreads >= n_work) break;             // uniform
                const int i = x * kSelThreads + tid_l;
                if (i < n_work) phys_by_slot[i] = entry[kPhys ? x : 0];
            }
            for (int i = kRegsLarge * kSelThreads + tid_l; i < n_work; i += kSelThreads)
                phys_by_slot[i] = bt_row[max(target2(i).unit, 0)];
            __syncthreads();                          // the cut reads other threads' slots
        }
        prof.mark(3 + 4 * level);

        // ---- the cut
        int n_kept;
        if (level == 0 && all_grids) {
            for (int i = tid_l; i < ng; i += kSelThreads) { kept_grids[i] = i; keys[i] = kMarkKey; }   // every grid lets its chunks compete
            __syncthreads();
            n_kept = ng;
        } else if (level == 1 && all_chunks) {
            for (int i = tid_l; i < nc; i += kSelThreads) kept_chunks[i] = i;
            __syncthreads();
            n_kept = nc;
        } else {
            // chunk keys: by unit, competing only under a kept grid (merged), or N_g slots per kept grid (lazy)
            uint64_t* lk = level == 1 ? keys + ng : keys;
            const int n_slots = level == 0 ? ng : level == 1 ? (merged ? nc : n_work) : n_work;
            const ActiveRule active{(level == 1 && merged) ? keys : nullptr, g.n_g, inv_ng};
            const KeepRule rule = rule_of(level);
            const bool by_parent = level == 2 || (level == 1 && !merged);
            const EmitRule emit{level == 0 ? kept_grids : level == 1 ? kept_chunks : sel_pages,
                                by_parent ? (level == 1 ? kept_grids : kept_chunks) : nullptr, level == 1 ? g.n_g : g.n_c,
                                level == 1 ? inv_ng : inv_nc,
                                (kPhys && level == 2) ? sel_phys : nullptr, (kPhys && level == 2) ? phys_by_slot : nullptr};
            const int cap = level == 0 ? sp.cap_kg : level == 1 ? sp.cap_kc : g.max_sel - s - w;
            n_kept = cut_level(lk, n_slots, active, rule, keep_ties, general, emit, cap, level == 0 && merged, sh,
                               have_pulled, pulled);
            if (n_kept > cap) { res->overflow = true; n_kept = cap; }
        }
        prof.mark(4 + 4 * level);
        if (level == 0) n_kg = n_kept;
        else if (level == 1) n_kc = n_kept;
        else res->n_kp = n_kept;
    }
    return true;
}

// The scorer of one (sequence, KV head): a level's vectors are rows of one array, the probe is in registers.
template <class T>
struct HeadScorer {
    static constexpr int kShareRound = 1;
    static constexpr int kTrip = kSelGroups * kFlyOf<T>;   // slots a member scores per memory round trip
    const T* pages_row;
    const T* chunks_row;
    const T* grids_row;
    const double (&pr)[8];
    template <class Target>
    __device__ __forceinline__ void operator()(int lo, int hi, Target target, bool local, uint64_t* keys, uint64_t* pub) const
    {
        score_rows<T>(grids_row, chunks_row, pages_row, lo, hi, target, pr, local, keys, pub);
    }
};

template <bool kPhys, class T, class TailFn>
__device__ __forceinline__ bool cascade(const T* __restrict__ pages_row, const T* __restrict__ chunks_row,
                                        const T* __restrict__ grids_row, const double (&pr)[8], int P, const Geom& g,
                                        const SelectParams& sp, const PubLayout& pubs, int m, int C, bool want_l3,
                                        uint64_t* keys, int32_t* kept_grids, int32_t* kept_chunks, int32_t* sel_pages,
                                        Shared& sh, CascadeResult* res, Prof& prof, const uint64_t* tail_words,
                                        TailFn refresh_tail, int k_fixed, const int32_t* __restrict__ bt_row = nullptr,
                                        int32_t* phys_by_slot = nullptr, int32_t* sel_phys = nullptr)
{
    const HeadScorer<T> scorer{pages_row, chunks_row, grids_row, pr};
    return cascade_with<kPhys>(scorer, P, g, sp, pubs, m, C, want_l3, keys, kept_grids, kept_chunks, sel_pages, sh, res,
                               prof, tail_words, refresh_tail, k_fixed, bt_row, phys_by_slot, sel_phys);
}

// Clear the published words of one (sequence, KV head) after everybody is done with them.
__device__ __forceinline__ void clear_published(const PubLayout& pubs, const CascadeResult& r, uint64_t* tail_words = nullptr)
{
    if (tail_words != nullptr && threadIdx.x < 3) publish_u64(tail_words + threadIdx.x, 0ull);
    for (int i = threadIdx.x; i < r.n_a; i += blockDim.x) publish_u64(pubs.units + i, 0ull);
    for (int i = threadIdx.x; i < r.n_p; i += blockDim.x) publish_u64(pubs.pages + i, 0ull);
}

}  // namespace chess
