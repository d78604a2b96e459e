// Device-side building blocks of paged decode attention over a list of pages read in place (Sec. 4.3,
// App. B), shared by the decode kernels and the fused decode-step kernel.
//
// Work unit: one wave, one tile of 32 tokens (two 16-token pages or one 32-token page), all G <= 16
// query heads of the KV head at once, so both products are dense 16 x 16 x 32 bf16 MFMA tiles:
//   S^T[token][head] = K[token][d] . Q^T[d][head]      4 MFMA per 16 tokens (d = 128)
//   O^T[d][head]    += V^T[d][token] . P[token][head]   8 MFMA per tile and per half of P
// K rows ([token][d], d contiguous) and V rows ([d][token], tokens contiguous) are both contiguous
// along the contraction index, so every lane feeds its MFMA operands with plain 128-bit global
// loads -- no LDS staging and no transpose.  The 16 token rows of the two K products are chosen so
// that the 8 softmax weights a lane ends up holding are exactly the 8 contraction slots it must
// supply to the P.V product: the weights never move between lanes.
// P is split into a bf16 head and a bf16 remainder (two MFMAs), which keeps the weights to ~2^-17
// relative; the row sum l uses the fp32 weights.
//
// Softmax state (m, l) of head j lives in the four lanes with lane % 16 == j; O^T accumulators are
// 8 x float4 per lane.  Tiles are dealt round-robin over splits and waves; the waves of a workgroup are
// merged through LDS; the last split of a (sequence, KV head) to finish merges all splits' partials, in
// split order.
#pragma once

#include "chess_internal.h"

namespace chess {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr float kNegBig = -1.0e30f;     // "no token yet" running maximum (log2 domain), finite on purpose

__device__ __forceinline__ bf16x8 as_bf16x8(const uint4& v) { return __builtin_bit_cast(bf16x8, v); }

template <int B>
struct Tile {
    uint4 k[2][4];      // [product c][d step]
    uint4 v[8];         // [16-row block of d]
    int ntok[32 / B];   // valid tokens of each page slot of the tile (0 = slot unused)
    int lp[32 / B];     // logical page of each slot (kept by the block-table path only)
};

// The logical page numbers of tile t as stored in the list (speculative: the index is clamped into the
// row, validity is decided later), so that this load does not wait for the list length.
// kList: there is a list (compile-time, so that the list's address space stays known to the compiler: a run-time
// choice between a list entry and a computed number becomes a choice between addresses, and the access a flat one).
template <int B, bool kList>
__device__ __forceinline__ void fetch_ids(int (&raw)[32 / B], int t, const int32_t* ids, int max_sel)
{
    constexpr int PPT = 32 / B;
#pragma unroll
    for (int s = 0; s < PPT; ++s) {
        if (kList) raw[s] = ids[min(t * PPT + s, max_sel - 1)];
        else raw[s] = t * PPT + s;
    }
}

// Request the K and V operands of tile t.  The physical page of a listed page comes from the block table, or,
// when the caller has them at hand, from `phys_list` (physical pages in list order, n_pages >= 1 entries).
template <int B, bool kPhysList>
__device__ __forceinline__ void load_tile(Tile<B>& tl, int t, int n_pages, const int (&raw)[32 / B], const int32_t* bt_row,
                                          const int32_t* phys_list, const uint16_t* k_pool, const uint16_t* v_pool, int H,
                                          int h, int L, int P, int m16, int grp)
{
    constexpr int PPT = 32 / B;
    int64_t phys[PPT];
#pragma unroll
    for (int s = 0; s < PPT; ++s) {
        const bool ok = t * PPT + s < n_pages;
        int lp = ok ? raw[s] : raw[0];                            // unused slot: alias the tile's first page
        lp = min(max(lp, 0), P - 1);                              // a bad id must not become a bad address
        int pp;
        if (kPhysList) pp = phys_list[min(ok ? t * PPT + s : t * PPT, n_pages - 1)];
        else pp = bt_row[lp];
        phys[s] = __builtin_amdgcn_readfirstlane(pp);
        tl.ntok[s] = ok ? (lp == P - 1 ? L - lp * B : B) : 0;
    }
    // K: row m16 of product c is token T = 8*(m16/4) + 4*c + m16%4 of the tile
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const int T = 8 * (m16 >> 2) + 4 * c + (m16 & 3);
        const int slot = T / B, tok = T % B;
        const int64_t pg = PPT == 1 ? phys[0] : (slot ? phys[PPT - 1] : phys[0]);
        const uint4* src = reinterpret_cast<const uint4*>(k_pool + ((pg * H + h) * B + tok) * kHeadDim) + grp;
#pragma unroll
        for (int st = 0; st < 4; ++st) tl.k[c][st] = src[st * 4];  // d = 32*st + 8*grp
    }
    // V^T: row d = 16*blk + m16, tokens 8*grp .. 8*grp+7 of the tile
    {
        const int T0 = 8 * grp;
        const int slot = T0 / B, tok0 = T0 % B;
        const int64_t pg = PPT == 1 ? phys[0] : (slot ? phys[PPT - 1] : phys[0]);
        const uint16_t* base = v_pool + ((pg * H + h) * kHeadDim + m16) * B + tok0;
#pragma unroll
        for (int blk = 0; blk < 8; ++blk) tl.v[blk] = *reinterpret_cast<const uint4*>(base + (size_t)blk * 16 * B);
    }
}

// The same in two steps, for the kernels that go through the block table: the block-table entries of a tile are
// requested one tile earlier than its K / V rows, so that their round trip hides behind the rows of the tile
// before (a wave's loads return in order: an entry requested just before its rows would hold them back by a
// whole round trip per tile).
template <int B>
struct PageRef {
    int pp[32 / B];     // physical pages (the same in every lane; made scalar when they are used)
    int ntok[32 / B];   // valid tokens of each page slot (0 = slot unused)
    int lp[32 / B];     // logical pages
};

template <int B>
__device__ __forceinline__ void lookup_pages(PageRef<B>& r, int t, int n_pages, const int (&raw)[32 / B],
                                             const int32_t* bt_row, int L, int P, int n_stored)
{
    constexpr int PPT = 32 / B;
#pragma unroll
    for (int s = 0; s < PPT; ++s) {
        const bool ok = t * PPT + s < n_pages;
        int lp = ok ? raw[s] : raw[0];                            // unused slot: alias the tile's first page
        if (ok && t * PPT + s >= n_stored) lp = P - 1;            // the page the list gains in this launch: the tail page
        lp = min(max(lp, 0), P - 1);                              // a bad id must not become a bad address
        r.pp[s] = bt_row[lp];
        r.ntok[s] = ok ? (lp == P - 1 ? L - lp * B : B) : 0;
        r.lp[s] = ok ? lp : -1;
    }
}

template <int B>
__device__ __forceinline__ void load_rows(Tile<B>& tl, const PageRef<B>& r, const uint16_t* k_pool, const uint16_t* v_pool,
                                          int H, int h, int m16, int grp)
{
    constexpr int PPT = 32 / B;
    int64_t phys[PPT];
#pragma unroll
    for (int s = 0; s < PPT; ++s) {
        phys[s] = __builtin_amdgcn_readfirstlane(r.pp[s]);
        tl.ntok[s] = r.ntok[s];
        tl.lp[s] = r.lp[s];
    }
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const int T = 8 * (m16 >> 2) + 4 * c + (m16 & 3);
        const int slot = T / B, tok = T % B;
        const int64_t pg = PPT == 1 ? phys[0] : (slot ? phys[PPT - 1] : phys[0]);
        const uint4* src = reinterpret_cast<const uint4*>(k_pool + ((pg * H + h) * B + tok) * kHeadDim) + grp;
#pragma unroll
        for (int st = 0; st < 4; ++st) tl.k[c][st] = src[st * 4];
    }
    {
        const int T0 = 8 * grp;
        const int slot = T0 / B, tok0 = T0 % B;
        const int64_t pg = PPT == 1 ? phys[0] : (slot ? phys[PPT - 1] : phys[0]);
        const uint16_t* base = v_pool + ((pg * H + h) * kHeadDim + m16) * B + tok0;
#pragma unroll
        for (int blk = 0; blk < 8; ++blk) tl.v[blk] = *reinterpret_cast<const uint4*>(base + (size_t)blk * 16 * B);
    }
}

// The token a launch appends (its rows are not in the pools yet) and where it sits.  `put` replaces the token's slot
// in the operands of the tile that holds the tail page; it reads this lane's parts of the two rows then (the one
// wave that needs them asks for them behind its tile's own loads: nothing waits longer than it would anyway, and no
// other wave carries them in registers).
template <int B>
struct NewToken {
    const uint16_t* k_row;   // key row, 128 bf16
    const uint16_t* v_row;   // value row
    int tile, T;             // tile of the list that holds the tail page (-1: nothing is appended), token slot in it
    __device__ __forceinline__ void put(Tile<B>& tl, int m16, int grp) const
    {
        uint4 k[4];          // d = 32 st + 8 grp .. + 7
        uint16_t v[8];       // d = 16 blk + m16
        const uint4* ks = reinterpret_cast<const uint4*>(k_row) + grp;
#pragma unroll
        for (int st = 0; st < 4; ++st) k[st] = ks[st * 4];
#pragma unroll
        for (int blk = 0; blk < 8; ++blk) v[blk] = v_row[16 * blk + m16];
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const bool mine = 8 * (m16 >> 2) + 4 * c + (m16 & 3) == T;
#pragma unroll
            for (int st = 0; st < 4; ++st) {
                tl.k[c][st].x = mine ? k[st].x : tl.k[c][st].x; tl.k[c][st].y = mine ? k[st].y : tl.k[c][st].y;
                tl.k[c][st].z = mine ? k[st].z : tl.k[c][st].z; tl.k[c][st].w = mine ? k[st].w : tl.k[c][st].w;
            }
        }
        const bool mine = (T >> 3) == grp;
        const int e = T & 7;
#pragma unroll
        for (int blk = 0; blk < 8; ++blk) {
            uint32_t w[4] = {tl.v[blk].x, tl.v[blk].y, tl.v[blk].z, tl.v[blk].w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t lo = (w[i] & 0xffff0000u) | v[blk], hi = (w[i] & 0x0000ffffu) | ((uint32_t)v[blk] << 16);
                w[i] = (mine && (e >> 1) == i) ? ((e & 1) ? hi : lo) : w[i];
            }
            tl.v[blk] = make_uint4(w[0], w[1], w[2], w[3]);
        }
    }
};

// Online-softmax state of one wave: all G heads of one KV head.
template <int B>
struct WaveAcc {
    static constexpr int PPT = 32 / B;
    bf16x8 qop[4];      // Q^T operand: head m16, d = 32*st + 8*grp .. +7; heads >= G are zero columns
    float m_run, l_run;
    f32x4 o[8];

    __device__ __forceinline__ void init(const uint16_t* __restrict__ q_rows, int G, int m16, int grp)
    {
        const uint4* src = reinterpret_cast<const uint4*>(q_rows + (size_t)(m16 < G ? m16 : 0) * kHeadDim) + grp;
        const uint32_t keep = m16 < G ? 0xffffffffu : 0u;     // (a select between the load and a zero vector made
#pragma unroll                                                //  the compiler select between two addresses instead)
        for (int st = 0; st < 4; ++st) {
            uint4 v = src[st * 4];
            v.x &= keep; v.y &= keep; v.z &= keep; v.w &= keep;
            qop[st] = as_bf16x8(v);
        }
        m_run = kNegBig;
        l_run = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // one tile: scores, online softmax, P.V
    __device__ __forceinline__ void process(Tile<B>& tl, float scale_log2, int grp)
    {
        // scores of this lane's head for tokens 8*grp + e, e = 0..7 (c = 0 gives e 0..3, c = 1 gives 4..7)
        f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(tl.k[0][st]), qop[st], s0, 0, 0, 0);
            s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(tl.k[1][st]), qop[st], s1, 0, 0, 0);
        }
        const int slot = (8 * grp) / B, tok0 = (8 * grp) % B;
        const int nt = PPT == 1 ? tl.ntok[0] : (slot ? tl.ntok[PPT - 1] : tl.ntok[0]);
        float x[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            x[e] = (tok0 + e < nt) ? s0[e] * scale_log2 : -INFINITY;
            x[4 + e] = (tok0 + 4 + e < nt) ? s1[e] * scale_log2 : -INFINITY;
        }
        float tmax = x[0];
#pragma unroll
        for (int e = 1; e < 8; ++e) tmax = fmaxf(tmax, x[e]);
        tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
        const float m_new = fmaxf(m_run, tmax);
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        m_run = m_new;
        float p[8], psum = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) { p[e] = __builtin_amdgcn_exp2f(x[e] - m_new); psum += p[e]; }
        l_run = l_run * alpha + psum;
        bf16x8 ph, pl;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const __bf16 hi = (__bf16)p[e];
            ph[e] = hi;
            pl[e] = (__bf16)(p[e] - (float)hi);
        }
        // a partly filled tile: unused token slots of V may hold anything (NaN included); zero them
        bool partial = tl.ntok[0] < B;
        if (PPT > 1) partial = partial || tl.ntok[PPT - 1] < B;
        if (partial) {
            uint32_t keep[4];
#pragma unroll
            for (int wd = 0; wd < 4; ++wd)
                keep[wd] = ((tok0 + 2 * wd < nt) ? 0x0000ffffu : 0u) | ((tok0 + 2 * wd + 1 < nt) ? 0xffff0000u : 0u);
#pragma unroll
            for (int blk = 0; blk < 8; ++blk) {
                tl.v[blk].x &= keep[0]; tl.v[blk].y &= keep[1]; tl.v[blk].z &= keep[2]; tl.v[blk].w &= keep[3];
            }
        }
#pragma unroll
        for (int blk = 0; blk < 8; ++blk) {
            f32x4 acc = o[blk] * alpha;
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(tl.v[blk]), ph, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(tl.v[blk]), pl, acc, 0, 0, 0);
            o[blk] = acc;
        }
    }
};

// This wave's tiles t0, t0 + stride, ... < n_tiles of the list `ids` (nullptr: every page), whose first two
// tiles' page numbers the caller has fetched already.
// The next tile is always requested before the current one is computed, in the same straight-line block, so
// the compiler waits only for the older loads (a load under its own branch would force a wait for everything
// outstanding).  After the last tile the "next" request repeats the current tile: it hits in cache and is dropped.
// nt (may be null): a token appended by this launch; n_stored: list entries that are in memory (the list may gain the
// tail page in this launch: entries from n_stored on are that page).
// kSingle: one tile in registers at a time (no request for the next tile while this one is computed): with a
// third less registers three workgroups fit on a compute unit instead of two, which hides more latency than the
// prefetch did (measured on lists and on whole sequences; the block-table path only).
template <int B, bool kList, bool kPhysList, bool kAppend, bool kSingle = false>
__device__ __forceinline__ void run_tiles_with(WaveAcc<B>& acc, int t, int stride, int n_tiles, int n_pages,
                                          int (&raw_cur)[32 / B], int (&raw_nxt)[32 / B], const int32_t* ids, int max_sel,
                                          const int32_t* bt_row, const int32_t* phys_list, const uint16_t* k_pool,
                                          const uint16_t* v_pool, int H, int h, int L, int P, float scale_log2, int m16,
                                          int grp, const NewToken<B>& nt, int n_stored)
{
    constexpr int PPT = 32 / B;
    if constexpr (!kPhysList) {
        if (t < n_tiles) {
            // block-table entries run one tile ahead of the rows, page numbers one tile ahead of those
            PageRef<B> pc, pn, pnn;
            int raw_nn[PPT];
            lookup_pages<B>(pc, t, n_pages, raw_cur, bt_row, L, P, n_stored);
            lookup_pages<B>(pn, t + stride, n_pages, raw_nxt, bt_row, L, P, n_stored);
            fetch_ids<B, kList>(raw_nn, t + 2 * stride, ids, max_sel);
            if constexpr (kSingle) {
                Tile<B> cur;
                for (; t < n_tiles; t += stride) {
                    load_rows<B>(cur, pc, k_pool, v_pool, H, h, m16, grp);
                    lookup_pages<B>(pnn, t + 2 * stride, n_pages, raw_nn, bt_row, L, P, n_stored);
                    fetch_ids<B, kList>(raw_nn, t + 3 * stride, ids, max_sel);
                    const int lp_tail = (PPT == 1 || nt.T < B) ? cur.lp[0] : cur.lp[PPT - 1];
                    if (kAppend && t == nt.tile && lp_tail == P - 1) nt.put(cur, m16, grp);
                    acc.process(cur, scale_log2, grp);
                    pc = pn;
                    pn = pnn;
                }
                acc.l_run += __shfl_xor(acc.l_run, 16);
                acc.l_run += __shfl_xor(acc.l_run, 32);
                return;
            }
            Tile<B> cur, nxt;
            load_rows<B>(cur, pc, k_pool, v_pool, H, h, m16, grp);
            for (; t < n_tiles; t += stride) {
                const bool more = t + stride < n_tiles;
                if (more) pc = pn;                                // after the last tile the request repeats it
                load_rows<B>(nxt, pc, k_pool, v_pool, H, h, m16, grp);
                lookup_pages<B>(pnn, t + 2 * stride, n_pages, raw_nn, bt_row, L, P, n_stored);
                fetch_ids<B, kList>(raw_nn, t + 3 * stride, ids, max_sel);
                // (the list's last entry is the tail page unless a row ran out of room: then the token is not attended)
                // (no run-time index into the tile: it would move the tile to scratch memory)
                const int lp_tail = (PPT == 1 || nt.T < B) ? cur.lp[0] : cur.lp[PPT - 1];
                if (kAppend && t == nt.tile && lp_tail == P - 1) nt.put(cur, m16, grp);
                acc.process(cur, scale_log2, grp);
                cur = nxt;
                pn = pnn;
            }
        }
        acc.l_run += __shfl_xor(acc.l_run, 16);
        acc.l_run += __shfl_xor(acc.l_run, 32);
        return;
    }
    if (t < n_tiles) {
        Tile<B> cur, nxt;
        load_tile<B, kPhysList>(cur, t, n_pages, raw_cur, bt_row, phys_list, k_pool, v_pool, H, h, L, P, m16, grp);
        for (; t < n_tiles; t += stride) {
            const bool more = t + stride < n_tiles;
            int raw_use[PPT];
#pragma unroll
            for (int s = 0; s < PPT; ++s) raw_use[s] = more ? raw_nxt[s] : raw_cur[s];
            load_tile<B, kPhysList>(nxt, more ? t + stride : t, n_pages, raw_use, bt_row, phys_list, k_pool, v_pool, H, h, L, P, m16, grp);
            fetch_ids<B, kList>(raw_nxt, t + 2 * stride, ids, max_sel);
            acc.process(cur, scale_log2, grp);
            cur = nxt;
#pragma unroll
            for (int s = 0; s < PPT; ++s) raw_cur[s] = raw_use[s];
        }
    }
    acc.l_run += __shfl_xor(acc.l_run, 16);
    acc.l_run += __shfl_xor(acc.l_run, 32);
}

template <int B, bool kList, bool kPhysList>
__device__ __forceinline__ void run_tiles(WaveAcc<B>& acc, int t, int stride, int n_tiles, int n_pages,
                                          int (&raw_cur)[32 / B], int (&raw_nxt)[32 / B], const int32_t* ids, int max_sel,
                                          const int32_t* bt_row, const int32_t* phys_list, const uint16_t* k_pool,
                                          const uint16_t* v_pool, int H, int h, int L, int P, float scale_log2, int m16,
                                          int grp)
{
    NewToken<B> none;
    none.tile = -1;
    run_tiles_with<B, kList, kPhysList, false>(acc, t, stride, n_tiles, n_pages, raw_cur, raw_nxt, ids, max_sel, bt_row,
                                               phys_list, k_pool, v_pool, H, h, L, P, scale_log2, m16, grp, none, 1 << 30);
}

// LDS the combine below needs, in floats: [NW][hs][128] accumulators, [NW][hs] maxima, [NW][hs] sums, where the
// head stride hs is 16 (one MFMA N-tile: nothing to guard) or the group size G (what a large workgroup can afford).
template <int NW>
struct DecodeLds {
    static constexpr int kFloats = NW * kMaxGroup * kHeadDim + 2 * NW * kMaxGroup;
    static constexpr int floats(int hs) { return NW * hs * kHeadDim + 2 * NW * hs; }
    float* o;   // [NW][hs][kHeadDim]
    float* m;   // [NW][hs]
    float* l;   // [NW][hs]
    int hs;
    __device__ __forceinline__ explicit DecodeLds(float* base, int head_stride = kMaxGroup)
        : o(base), m(base + NW * head_stride * kHeadDim), l(base + NW * head_stride * kHeadDim + NW * head_stride),
          hs(head_stride) {}
};

// Merge the NW waves of this workgroup through LDS.  n_splits == 1: write `out` rows and return false.
// Otherwise publish the workgroup's partial as split `split` and return true.
template <int NW>
__device__ __forceinline__ bool combine_waves(const f32x4 (&o)[8], float m_run, float l_run, DecodeLds<NW>& lds, int G,
                                              int n_splits, int split, size_t row, float* __restrict__ out_rows,
                                              float* __restrict__ ws_acc, float* __restrict__ ws_ml)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m16 = lane & 15, grp = lane >> 4;
    // lane holds O^T[d = 16*blk + 4*grp + r][head m16]
    const int hs = lds.hs;
    if (m16 < hs) {                                     // (heads beyond the group are zero columns)
#pragma unroll
        for (int blk = 0; blk < 8; ++blk)
            *reinterpret_cast<f32x4*>(&lds.o[(wave * hs + m16) * kHeadDim + 16 * blk + 4 * grp]) = o[blk];
        if (grp == 0) { lds.m[wave * hs + m16] = m_run; lds.l[wave * hs + m16] = l_run; }
    }
    __syncthreads();

    // combine this workgroup's waves; one thread per pair of adjacent d
    uint64_t* acc_g = reinterpret_cast<uint64_t*>(ws_acc);           // partial rows as pairs of floats
    uint64_t* ml_g = reinterpret_cast<uint64_t*>(ws_ml);             // (m, l) per partial row
    for (int idx = threadIdx.x; idx < G * (kHeadDim / 2); idx += 64 * NW) {
        const int head = idx / (kHeadDim / 2), d = 2 * (idx % (kHeadDim / 2));
        float M = lds.m[head];
#pragma unroll
        for (int wv = 1; wv < NW; ++wv) M = fmaxf(M, lds.m[wv * hs + head]);
        float a0 = 0.f, a1 = 0.f, l = 0.f;
#pragma unroll
        for (int wv = 0; wv < NW; ++wv) {
            const float sc = __builtin_amdgcn_exp2f(lds.m[wv * hs + head] - M);
            a0 += lds.o[(wv * hs + head) * kHeadDim + d] * sc;
            a1 += lds.o[(wv * hs + head) * kHeadDim + d + 1] * sc;
            l += lds.l[wv * hs + head] * sc;
        }
        if (n_splits == 1) {
            const float inv = l > 0.f ? 1.f / l : 0.f;
            *reinterpret_cast<float2*>(out_rows + (size_t)head * kHeadDim + d) = make_float2(a0 * inv, a1 * inv);
        } else {
            const size_t pr = (row * n_splits + split) * G + head;
            publish_u64(acc_g + pr * (kHeadDim / 2) + d / 2, __builtin_bit_cast(uint64_t, make_float2(a0, a1)));
            if (d == 0) publish_u64(ml_g + pr, __builtin_bit_cast(uint64_t, make_float2(M, l)));
        }
    }
    return n_splits != 1;
}

// What the last split of a (sequence, KV head) to finish does: merge all splits' partials,
// out = sum_s acc_s 2^(m_s - M) / sum_s l_s 2^(m_s - M), always in split order, so the result does not
// depend on which workgroup happens to be last.  A thread owns one pair of adjacent outputs of one head and
// derives that head's M and denominator itself from the (m, l) pairs (the threads of a head read the same
// words), so the partial rows and the (m, l) pairs are requested together: one round trip to memory, no LDS,
// no barrier.
template <int NW>
__device__ __forceinline__ void merge_splits(int G, int n_splits, size_t row, float* __restrict__ out_rows,
                                             const float* __restrict__ ws_acc, const float* __restrict__ ws_ml)
{
    const uint64_t* acc_g = reinterpret_cast<const uint64_t*>(ws_acc);
    const uint64_t* ml_g = reinterpret_cast<const uint64_t*>(ws_ml);
    constexpr int kChunk = 8;                          // splits in flight per thread
    const int n_items = G * (kHeadDim / 2);
    for (int idx = threadIdx.x; idx < n_items; idx += 64 * NW) {
        const int head = idx / (kHeadDim / 2), d2 = idx % (kHeadDim / 2);
        float M = kNegBig, l = 0.f, a0 = 0.f, a1 = 0.f;
        for (int s0 = 0; s0 < n_splits; s0 += kChunk) {
            uint64_t v[kChunk], ml[kChunk];
#pragma unroll
            for (int x = 0; x < kChunk; ++x) {
                const size_t pr = (row * n_splits + min(s0 + x, n_splits - 1)) * G + head;
                ml[x] = observe_u64(ml_g + pr);
                v[x] = observe_u64(acc_g + pr * (kHeadDim / 2) + d2);
            }
            // running maximum over the splits seen so far; what has been summed is rescaled to it
            float Mc = M;
#pragma unroll
            for (int x = 0; x < kChunk; ++x)
                if (s0 + x < n_splits) Mc = fmaxf(Mc, __builtin_bit_cast(float2, ml[x]).x);
            const float keep = __builtin_amdgcn_exp2f(M - Mc);
            l *= keep; a0 *= keep; a1 *= keep;
            M = Mc;
#pragma unroll
            for (int x = 0; x < kChunk; ++x) {
                if (s0 + x < n_splits) {
                    const float2 mlx = __builtin_bit_cast(float2, ml[x]);
                    const float2 f = __builtin_bit_cast(float2, v[x]);
                    const float wt = __builtin_amdgcn_exp2f(mlx.x - M);
                    l += mlx.y * wt;
                    a0 += f.x * wt;
                    a1 += f.y * wt;
                }
            }
        }
        const float inv = l > 0.f ? 1.f / l : 0.f;
        *reinterpret_cast<float2*>(out_rows + (size_t)head * kHeadDim + 2 * d2) = make_float2(a0 * inv, a1 * inv);
    }
}

}  // namespace chess
