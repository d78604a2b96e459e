// Paged decode attention over a list of pages read in place (sparse: the selected page ids;
// dense: every page), split-K with an online-softmax merge.
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
// merged through LDS;
// the last split of a (sequence, KV head) to finish merges all splits' partials, in split order.
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
};

// The logical page numbers of tile t as stored in the list (speculative: the index is clamped into the
// row, validity is decided later), so that this load does not wait for the list length.
template <int B>
__device__ __forceinline__ void fetch_ids(int (&raw)[32 / B], int t, const int32_t* ids, int max_sel)
{
    constexpr int PPT = 32 / B;
#pragma unroll
    for (int s = 0; s < PPT; ++s) raw[s] = ids ? ids[min(t * PPT + s, max_sel - 1)] : t * PPT + s;
}

template <int B>
__device__ __forceinline__ void load_tile(Tile<B>& tl, int t, int n_pages, const int (&raw)[32 / B], const int32_t* bt_row,
                                          const uint16_t* k_pool, const uint16_t* v_pool, int H, int h, int L, int P,
                                          int m16, int grp)
{
    constexpr int PPT = 32 / B;
    int64_t phys[PPT];
#pragma unroll
    for (int s = 0; s < PPT; ++s) {
        const bool ok = t * PPT + s < n_pages;
        int lp = ok ? raw[s] : raw[0];                            // unused slot: alias the tile's first page
        lp = min(max(lp, 0), P - 1);                              // a bad id must not become a bad address
        phys[s] = __builtin_amdgcn_readfirstlane(bt_row[lp]);
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

template <int B, int NW>
__global__ __launch_bounds__(64 * NW) void decode_kernel(const uint16_t* __restrict__ q,
                                                         const uint16_t* __restrict__ k_pool,
                                                         const uint16_t* __restrict__ v_pool,
                                                         const int32_t* __restrict__ block_table,
                                                         const int32_t* __restrict__ seq_lens,
                                                         const int32_t* __restrict__ page_ids,
                                                         const int32_t* __restrict__ n_selected, Geom g,
                                                         float scale_log2, int n_splits, float* __restrict__ out,
                                                         float* __restrict__ ws_acc, float* __restrict__ ws_ml,
                                                         int32_t* __restrict__ arrivals
#ifdef CHESS_PROF
                                                         , int32_t* __restrict__ prof
#endif
                                                         )
{
    constexpr int PPT = 32 / B;
    __shared__ float lds_o[NW][kMaxGroup][kHeadDim];
    __shared__ float lds_m[NW][kMaxGroup], lds_l[NW][kMaxGroup];
    __shared__ int lds_last;

    const int split = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#ifdef CHESS_PROF
    long long prof_t[8];
    int prof_n = 0;
#define DPROF_MARK() prof_t[prof_n++] = wall_clock64()
#else
#define DPROF_MARK()
#endif
    DPROF_MARK();
    const int m16 = lane & 15, grp = lane >> 4;
    const int G = g.group, H = g.n_kv_heads;
    const size_t row = (size_t)b * H + h;
    const int32_t* ids = page_ids ? page_ids + row * g.max_sel : nullptr;
    const int32_t* bt_row = block_table + (size_t)b * g.max_pages;
    // tiles are dealt round-robin: tile = split + n_splits * (wave + NW * i), so the first tile of a wave
    // is known before the list length is, and its page numbers can be fetched alongside the lengths
    const int stride = n_splits * NW;
    int t = split + n_splits * wave;
    int raw_cur[PPT], raw_nxt[PPT];
    const int L_raw = seq_lens[b];
    const int n_raw = page_ids ? n_selected[row] : 0;
    fetch_ids<B>(raw_cur, t, ids, g.max_sel);
    fetch_ids<B>(raw_nxt, t + stride, ids, g.max_sel);
    const int L = min(max(L_raw, 0), g.max_pages * B);
    const int P = (L + B - 1) / B;
    const int n_pages = P == 0 ? 0 : (page_ids ? min(max(n_raw, 0), g.max_sel) : P);
    const int n_tiles = (n_pages + PPT - 1) / PPT;

    // Q^T operand: head m16, d = 32*st + 8*grp .. +7; heads >= G are zero columns
    bf16x8 qop[4];
    {
        const uint4 z = make_uint4(0, 0, 0, 0);
        const uint4* src = reinterpret_cast<const uint4*>(q + ((size_t)b * g.n_q_heads + h * G + (m16 < G ? m16 : 0)) * kHeadDim) + grp;
#pragma unroll
        for (int st = 0; st < 4; ++st) qop[st] = as_bf16x8(m16 < G ? src[st * 4] : z);
    }

    float m_run = kNegBig, l_run = 0.f;
    f32x4 o[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = f32x4{0.f, 0.f, 0.f, 0.f};

    DPROF_MARK();                                     // 1: lengths and first page numbers known
    // one tile: scores, online softmax, P.V
    auto process = [&](Tile<B>& tl) {
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
    };
    // The next tile is always requested before the current one is computed, in the same straight-line block, so
    // the compiler waits only for the older loads (a load under its own branch would force a wait for everything
    // outstanding).  After the last tile the "next" request repeats the current tile: it hits in cache and is dropped.
    if (t < n_tiles) {
        Tile<B> cur, nxt;
        load_tile<B>(cur, t, n_pages, raw_cur, bt_row, k_pool, v_pool, H, h, L, P, m16, grp);
#ifdef CHESS_PROF_WAIT
        DPROF_MARK();                                 // block table entry read, K/V requested
        __builtin_amdgcn_s_waitcnt(0);
        DPROF_MARK();                                 // first tile arrived
#endif
        for (; t < n_tiles; t += stride) {
            const bool more = t + stride < n_tiles;
            int raw_use[PPT];
#pragma unroll
            for (int s = 0; s < PPT; ++s) raw_use[s] = more ? raw_nxt[s] : raw_cur[s];
            load_tile<B>(nxt, more ? t + stride : t, n_pages, raw_use, bt_row, k_pool, v_pool, H, h, L, P, m16, grp);
            fetch_ids<B>(raw_nxt, t + 2 * stride, ids, g.max_sel);
            process(cur);
            cur = nxt;
#pragma unroll
            for (int s = 0; s < PPT; ++s) raw_cur[s] = raw_use[s];
        }
    }
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);
    DPROF_MARK();                                     // 2: tiles done

    // merge the waves of this workgroup through LDS: lane holds O^T[d = 16*blk + 4*grp + r][head m16]
#pragma unroll
    for (int blk = 0; blk < 8; ++blk)
        *reinterpret_cast<f32x4*>(&lds_o[wave][m16][16 * blk + 4 * grp]) = o[blk];
    if (grp == 0) { lds_m[wave][m16] = m_run; lds_l[wave][m16] = l_run; }
    __syncthreads();

    // combine this workgroup's waves; one thread per pair of adjacent d
    float2* ml_buf = reinterpret_cast<float2*>(&lds_o[0][0][0]);   // reused by the merging workgroup: [n_splits][G]
    uint64_t* acc_g = reinterpret_cast<uint64_t*>(ws_acc);           // partial rows as pairs of floats
    uint64_t* ml_g = reinterpret_cast<uint64_t*>(ws_ml);             // (m, l) per partial row
    for (int idx = threadIdx.x; idx < G * (kHeadDim / 2); idx += 64 * NW) {
        const int head = idx / (kHeadDim / 2), d = 2 * (idx % (kHeadDim / 2));
        float M = lds_m[0][head];
#pragma unroll
        for (int wv = 1; wv < NW; ++wv) M = fmaxf(M, lds_m[wv][head]);
        float a0 = 0.f, a1 = 0.f, l = 0.f;
#pragma unroll
        for (int wv = 0; wv < NW; ++wv) {
            const float sc = __builtin_amdgcn_exp2f(lds_m[wv][head] - M);
            a0 += lds_o[wv][head][d] * sc;
            a1 += lds_o[wv][head][d + 1] * sc;
            l += lds_l[wv][head] * sc;
        }
        if (n_splits == 1) {
            const float inv = l > 0.f ? 1.f / l : 0.f;
            *reinterpret_cast<float2*>(out + ((size_t)b * g.n_q_heads + h * G + head) * kHeadDim + d) = make_float2(a0 * inv, a1 * inv);
        } else {
            const size_t pr = (row * n_splits + split) * G + head;
            publish_u64(acc_g + pr * (kHeadDim / 2) + d / 2, __builtin_bit_cast(uint64_t, make_float2(a0, a1)));
            if (d == 0) publish_u64(ml_g + pr, __builtin_bit_cast(uint64_t, make_float2(M, l)));
        }
    }
    if (n_splits == 1) return;
    DPROF_MARK();                                     // 3: waves combined, partial published
    if (!arrive_last(arrivals + row, n_splits, &lds_last)) return;
    DPROF_MARK();                                     // 4: arrived (last split only from here)

    // ---- the last split of this (sequence, KV head) to finish merges all of them:
    // out = sum_s acc_s 2^(m_s - M) / sum_s l_s 2^(m_s - M), always in split order, so the result does not
    // depend on which workgroup happens to be last
    constexpr int kChunk = 8;                          // partial rows in flight per output pair
    const int n_items = G * (kHeadDim / 2);
    // the first rows of this thread's first output pair are requested together with the (m, l) pairs,
    // so the merge costs one round trip to memory, not two
    uint64_t first[kChunk];
    {
        const int idx = min((int)threadIdx.x, n_items - 1);
        const int head = idx / (kHeadDim / 2), d2 = idx % (kHeadDim / 2);
#pragma unroll
        for (int x = 0; x < kChunk; ++x)
            first[x] = observe_u64(acc_g + ((row * n_splits + min(x, n_splits - 1)) * G + head) * (kHeadDim / 2) + d2);
    }
    for (int idx = threadIdx.x; idx < n_splits * G; idx += 64 * NW) {
        const int sidx = idx / G, head = idx % G;
        ml_buf[idx] = __builtin_bit_cast(float2, observe_u64(ml_g + (row * n_splits + sidx) * G + head));
    }
    __syncthreads();
    if ((int)threadIdx.x < G) {
        const int head = threadIdx.x;
        float M = kNegBig, l = 0.f;
        for (int sidx = 0; sidx < n_splits; ++sidx) M = fmaxf(M, ml_buf[sidx * G + head].x);
        for (int sidx = 0; sidx < n_splits; ++sidx) l += ml_buf[sidx * G + head].y * __builtin_amdgcn_exp2f(ml_buf[sidx * G + head].x - M);
        const float inv = l > 0.f ? 1.f / l : 0.f;
        for (int sidx = 0; sidx < n_splits; ++sidx)
            ml_buf[sidx * G + head].x = __builtin_amdgcn_exp2f(ml_buf[sidx * G + head].x - M) * inv;   // weight of split sidx
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < n_items; idx += 64 * NW) {
        const int head = idx / (kHeadDim / 2), d2 = idx % (kHeadDim / 2);
        float a0 = 0.f, a1 = 0.f;
        for (int s0 = 0; s0 < n_splits; s0 += kChunk) {
            uint64_t v[kChunk];
#pragma unroll
            for (int x = 0; x < kChunk; ++x) {
                if (s0 == 0 && idx == (int)threadIdx.x) v[x] = first[x];
                else v[x] = observe_u64(acc_g + ((row * n_splits + min(s0 + x, n_splits - 1)) * G + head) * (kHeadDim / 2) + d2);
            }
#pragma unroll
            for (int x = 0; x < kChunk; ++x) {
                if (s0 + x < n_splits) {
                    const float2 f = __builtin_bit_cast(float2, v[x]);
                    const float wt = ml_buf[(s0 + x) * G + head].x;
                    a0 += f.x * wt;
                    a1 += f.y * wt;
                }
            }
        }
        *reinterpret_cast<float2*>(out + ((size_t)b * g.n_q_heads + h * G + head) * kHeadDim + 2 * d2) = make_float2(a0, a1);
    }
#ifdef CHESS_PROF
    DPROF_MARK();                                     // 5: merged
    if (threadIdx.x == 0)
        for (int i = 1; i < prof_n; ++i) prof[row * 8 + i] = (int)(prof_t[i] - prof_t[i - 1]);
#endif
}

hipError_t launch_decode(chess_ctx* ctx, const uint16_t* q, const uint16_t* k_pool, const uint16_t* v_pool,
                         const int32_t* block_table, const int32_t* seq_lens, const int32_t* page_ids,
                         const int32_t* n_selected, int batch, int n_splits, int waves, float* out,
                         float* ws_acc, float* ws_ml, int32_t* arrivals, hipStream_t stream)
{
    const Geom& g = ctx->geom;
    const float scale_log2 = ctx->sm_scale * 1.4426950408889634f;
    const dim3 grid(n_splits, g.n_kv_heads, batch), block(64 * waves);
    void (*kern)(const uint16_t*, const uint16_t*, const uint16_t*, const int32_t*, const int32_t*, const int32_t*,
                 const int32_t*, Geom, float, int, float*, float*, float*, int32_t*
#ifdef CHESS_PROF
                 , int32_t*
#endif
                 );
    if (g.page_size == 16) kern = waves == 4 ? decode_kernel<16, 4> : decode_kernel<16, 1>;
    else                   kern = waves == 4 ? decode_kernel<32, 4> : decode_kernel<32, 1>;
    return launch(kern, grid, block, 0, stream, q, k_pool, v_pool, block_table, seq_lens,
                        page_ids, n_selected, g, scale_log2, n_splits, out, ws_acc, ws_ml, arrivals
#ifdef CHESS_PROF
                        , reinterpret_cast<int32_t*>(ws_ml) - 1024            // profiling builds: the unused end of the partial rows
#endif
                        );
}

hipError_t decode_occupancy(int page_size, int waves, int* blocks_per_cu)
{
    if (page_size == 16)
        return waves == 4 ? hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, decode_kernel<16, 4>, 256, 0)
                          : hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, decode_kernel<16, 1>, 64, 0);
    return waves == 4 ? hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, decode_kernel<32, 4>, 256, 0)
                      : hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, decode_kernel<32, 1>, 64, 0);
}

__global__ void zero_kernel(int32_t* p, size_t n)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

hipError_t launch_zero(chess_ctx* ctx, int32_t* p, size_t n_words, hipStream_t stream)
{
    (void)ctx;
    hipLaunchKernelGGL(zero_kernel, dim3((unsigned)((n_words + 255) / 256)), dim3(256), 0, stream, p, n_words);
    return hipGetLastError();
}

}  // namespace chess
