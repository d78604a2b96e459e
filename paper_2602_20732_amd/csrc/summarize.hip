// Hierarchical key summaries (Sec. 3.1): page vector = mean of the page's key rows (Eq. 1),
// chunk / grid vector = mean of the child vectors that exist (Eq. 2).
//
// One workgroup owns one (sequence, KV head, grid).  A 16-lane group streams one page: every lane
// issues 128-bit loads of 8 consecutive dims of one token row, so one wave instruction covers four
// 256-byte rows.  Each lane adds its 8 columns over the tokens in token order in fp64, so the sum
// is the same number whatever the launch shape; the mean is rounded to fp32 once.  Page vectors of
// the grid stay in LDS, chunk and grid means are formed from them without re-reading HBM.
#include <algorithm>

#include "chess_internal.h"

namespace chess {

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

__device__ __forceinline__ void add_row(double (&acc)[8], const uint4& r)
{
    acc[0] += (double)bf16_lo(r.x); acc[1] += (double)bf16_hi(r.x);
    acc[2] += (double)bf16_lo(r.y); acc[3] += (double)bf16_hi(r.y);
    acc[4] += (double)bf16_lo(r.z); acc[5] += (double)bf16_hi(r.z);
    acc[6] += (double)bf16_lo(r.w); acc[7] += (double)bf16_hi(r.w);
}

// Eight consecutive elements of a stored vector (dims 8 ln .. 8 ln + 7), to and from memory (global or LDS).
template <class T>
struct Row8;
template <>
struct Row8<float> {
    float4 lo, hi;
    __device__ __forceinline__ void set(const double (&m)[8])
    {
        lo = make_float4((float)m[0], (float)m[1], (float)m[2], (float)m[3]);
        hi = make_float4((float)m[4], (float)m[5], (float)m[6], (float)m[7]);
    }
    __device__ __forceinline__ void load(const float* p) { lo = reinterpret_cast<const float4*>(p)[0]; hi = reinterpret_cast<const float4*>(p)[1]; }
    __device__ __forceinline__ void store(float* p) const { reinterpret_cast<float4*>(p)[0] = lo; reinterpret_cast<float4*>(p)[1] = hi; }
};
template <>
struct Row8<uint16_t> {
    uint4 v;
    // fp64 mean -> fp32 -> nearest-even bf16 (finite inputs), two per word
    static __device__ __forceinline__ uint32_t bf(double m)
    {
        const uint32_t u = __float_as_uint((float)m);
        return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    }
    __device__ __forceinline__ void set(const double (&m)[8])
    {
        v = make_uint4(bf(m[0]) | (bf(m[1]) << 16), bf(m[2]) | (bf(m[3]) << 16), bf(m[4]) | (bf(m[5]) << 16), bf(m[6]) | (bf(m[7]) << 16));
    }
    __device__ __forceinline__ void load(const uint16_t* p) { v = *reinterpret_cast<const uint4*>(p); }
    __device__ __forceinline__ void store(uint16_t* p) const { *reinterpret_cast<uint4*>(p) = v; }
};

__device__ __forceinline__ double as_f64(float v) { return (double)v; }
__device__ __forceinline__ double as_f64(uint16_t v) { return (double)__uint_as_float((uint32_t)v << 16); }
__device__ __forceinline__ void put_mean(float* p, double m) { *p = (float)m; }
__device__ __forceinline__ void put_mean(uint16_t* p, double m) { *p = (uint16_t)Row8<uint16_t>::bf(m); }

// T = storage type of the summaries (float, or bf16 bits: each stored mean is the fp32 mean rounded to nearest-even
// bf16, and a parent averages its children as they are stored)
template <int B, class T>
__global__ __launch_bounds__(256) void summarize_kernel(const uint16_t* __restrict__ k_pool,
                                                        const int32_t* __restrict__ block_table,
                                                        const int32_t* __restrict__ seq_lens,
                                                        const int32_t* __restrict__ from_page, int recent, Geom g,
                                                        T* __restrict__ pages, T* __restrict__ chunks,
                                                        T* __restrict__ grids)
{
    extern __shared__ float lds_f[];                  // [n_c * n_g][128] page vectors, then [n_g][128] chunk vectors, as stored
    T* lds = reinterpret_cast<T*>(lds_f);
    const int b = blockIdx.z, h = blockIdx.y, tid = threadIdx.x;
    const int L = min(seq_lens[b], g.max_pages * B);
    if (L <= 0) return;
    const int P = (L + B - 1) / B;
    const int nc = (P + g.n_c - 1) / g.n_c, ng = (nc + g.n_g - 1) / g.n_g;
    // recent > 0: only the last `recent` pages are new; the grid's workgroups count back from the last grid
    const int gk = recent > 0 ? ng - 1 - (int)blockIdx.x : (int)blockIdx.x;
    if (gk >= ng || gk < 0) return;
    int fp = recent > 0 ? P - recent : (from_page ? from_page[b] : 0);
    fp = fp < 0 ? 0 : fp;
    const int ppg = g.n_c * g.n_g;
    if (gk < fp / ppg) return;                        // every unit of this grid is older than from_page
    const int fc = fp / g.n_c;
    const int p_lo = gk * ppg, p_hi = min(P, p_lo + ppg);
    const int c_lo = gk * g.n_g, c_hi = min(nc, c_lo + g.n_g);
    const size_t row = (size_t)b * g.n_kv_heads + h;
    T* pg = pages + row * g.max_pages * kHeadDim;
    T* cg = chunks + row * g.max_chunks * kHeadDim;
    T* gg = grids + row * g.max_grids * kHeadDim;
    T* lds_chunk = lds + (size_t)ppg * kHeadDim;

    const int grp = tid >> 4, ln = tid & 15;
    for (int j = p_lo + grp; j < p_hi; j += 16) {
        T* dst = lds + (size_t)(j - p_lo) * kHeadDim + ln * 8;
        Row8<T> r8;
        if (j >= fp) {
            const int64_t phys = block_table[(size_t)b * g.max_pages + j];
            const int n = (j == P - 1) ? L - j * B : B;
            const uint4* src = reinterpret_cast<const uint4*>(k_pool + ((phys * g.n_kv_heads + h) * B) * kHeadDim) + ln;
            double acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
            if (n == B) {
#pragma unroll
                for (int t0 = 0; t0 < B; t0 += 16) {
                    uint4 r[16];
#pragma unroll
                    for (int t = 0; t < 16; ++t) r[t] = src[(t0 + t) * 16];
#pragma unroll
                    for (int t = 0; t < 16; ++t) add_row(acc, r[t]);
                }
            } else {
                for (int t = 0; t < n; ++t) add_row(acc, src[t * 16]);
            }
            const double dn = (double)n;
            double mean[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) mean[i] = acc[i] / dn;
            r8.set(mean);
            r8.store(pg + (size_t)j * kHeadDim + ln * 8);
        } else if (j / g.n_c >= fc) {                 // unchanged page whose chunk is being refreshed
            r8.load(pg + (size_t)j * kHeadDim + ln * 8);
        } else {
            continue;
        }
        r8.store(dst);
    }
    __syncthreads();

    for (int idx = tid; idx < (c_hi - c_lo) * kHeadDim; idx += 256) {
        const int c = c_lo + idx / kHeadDim, dim = idx % kHeadDim;
        T v;
        if (c >= fc) {
            const int lo = c * g.n_c, hi = min(P, lo + g.n_c);
            double acc = 0.0;
            for (int j = lo; j < hi; ++j) acc += as_f64(lds[(size_t)(j - p_lo) * kHeadDim + dim]);
            put_mean(&v, acc / (double)(hi - lo));
            cg[(size_t)c * kHeadDim + dim] = v;
        } else {
            v = cg[(size_t)c * kHeadDim + dim];
        }
        lds_chunk[idx] = v;
    }
    __syncthreads();

    if (tid < kHeadDim) {
        double acc = 0.0;
        for (int c = 0; c < c_hi - c_lo; ++c) acc += as_f64(lds_chunk[c * kHeadDim + tid]);
        T v;
        put_mean(&v, acc / (double)(c_hi - c_lo));
        gg[(size_t)gk * kHeadDim + tid] = v;
    }
}

hipError_t launch_summarize(chess_ctx* ctx, const uint16_t* k_pool, const int32_t* block_table,
                            const int32_t* seq_lens, int batch, const int32_t* from_page, int recent,
                            void* pages, void* chunks, void* grids, hipStream_t stream)
{
    const Geom& g = ctx->geom;
    const bool bf16 = ctx->cfg.summary_dtype == CHESS_SUMMARY_BF16;
    const size_t lds = (size_t)(g.n_c * g.n_g + g.n_g) * kHeadDim * (bf16 ? sizeof(uint16_t) : sizeof(float));
    const int ppg = g.n_c * g.n_g;
    const int span = recent > 0 ? std::min(g.max_grids, (recent + ppg - 2) / ppg + 1) : g.max_grids;   // grids `recent` pages can touch
    const dim3 grid(span, g.n_kv_heads, batch), block(256);
    const void* kern = bf16 ? (g.page_size == 16 ? reinterpret_cast<const void*>(summarize_kernel<16, uint16_t>)
                                                 : reinterpret_cast<const void*>(summarize_kernel<32, uint16_t>))
                            : (g.page_size == 16 ? reinterpret_cast<const void*>(summarize_kernel<16, float>)
                                                 : reinterpret_cast<const void*>(summarize_kernel<32, float>));
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    if (bf16) {
        auto k = g.page_size == 16 ? summarize_kernel<16, uint16_t> : summarize_kernel<32, uint16_t>;
        return launch(k, grid, block, lds, stream, k_pool, block_table, seq_lens, from_page, recent, g,
                      static_cast<uint16_t*>(pages), static_cast<uint16_t*>(chunks), static_cast<uint16_t*>(grids));
    }
    auto k = g.page_size == 16 ? summarize_kernel<16, float> : summarize_kernel<32, float>;
    return launch(k, grid, block, lds, stream, k_pool, block_table, seq_lens, from_page, recent, g,
                  static_cast<float*>(pages), static_cast<float*>(chunks), static_cast<float*>(grids));
}

}  // namespace chess
