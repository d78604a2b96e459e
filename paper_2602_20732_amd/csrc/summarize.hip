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

template <int B>
__global__ __launch_bounds__(256) void summarize_kernel(const uint16_t* __restrict__ k_pool,
                                                        const int32_t* __restrict__ block_table,
                                                        const int32_t* __restrict__ seq_lens,
                                                        const int32_t* __restrict__ from_page, int recent, Geom g,
                                                        float* __restrict__ pages, float* __restrict__ chunks,
                                                        float* __restrict__ grids)
{
    extern __shared__ float lds[];                   // [n_c * n_g][128] page vectors, then [n_g][128] chunk vectors
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
    float* pg = pages + row * g.max_pages * kHeadDim;
    float* cg = chunks + row * g.max_chunks * kHeadDim;
    float* gg = grids + row * g.max_grids * kHeadDim;
    float* lds_chunk = lds + (size_t)ppg * kHeadDim;

    const int grp = tid >> 4, ln = tid & 15;
    for (int j = p_lo + grp; j < p_hi; j += 16) {
        float* dst = lds + (size_t)(j - p_lo) * kHeadDim + ln * 8;
        float4 lo4, hi4;
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
            lo4 = make_float4((float)(acc[0] / dn), (float)(acc[1] / dn), (float)(acc[2] / dn), (float)(acc[3] / dn));
            hi4 = make_float4((float)(acc[4] / dn), (float)(acc[5] / dn), (float)(acc[6] / dn), (float)(acc[7] / dn));
            float4* gdst = reinterpret_cast<float4*>(pg + (size_t)j * kHeadDim + ln * 8);
            gdst[0] = lo4;
            gdst[1] = hi4;
        } else if (j / g.n_c >= fc) {                 // unchanged page whose chunk is being refreshed
            const float4* gsrc = reinterpret_cast<const float4*>(pg + (size_t)j * kHeadDim + ln * 8);
            lo4 = gsrc[0];
            hi4 = gsrc[1];
        } else {
            continue;
        }
        reinterpret_cast<float4*>(dst)[0] = lo4;
        reinterpret_cast<float4*>(dst)[1] = hi4;
    }
    __syncthreads();

    for (int idx = tid; idx < (c_hi - c_lo) * kHeadDim; idx += 256) {
        const int c = c_lo + idx / kHeadDim, dim = idx % kHeadDim;
        float v;
        if (c >= fc) {
            const int lo = c * g.n_c, hi = min(P, lo + g.n_c);
            double acc = 0.0;
            for (int j = lo; j < hi; ++j) acc += (double)lds[(size_t)(j - p_lo) * kHeadDim + dim];
            v = (float)(acc / (double)(hi - lo));
            cg[(size_t)c * kHeadDim + dim] = v;
        } else {
            v = cg[(size_t)c * kHeadDim + dim];
        }
        lds_chunk[idx] = v;
    }
    __syncthreads();

    if (tid < kHeadDim) {
        double acc = 0.0;
        for (int c = 0; c < c_hi - c_lo; ++c) acc += (double)lds_chunk[c * kHeadDim + tid];
        gg[(size_t)gk * kHeadDim + tid] = (float)(acc / (double)(c_hi - c_lo));
    }
}

hipError_t launch_summarize(chess_ctx* ctx, const uint16_t* k_pool, const int32_t* block_table,
                            const int32_t* seq_lens, int batch, const int32_t* from_page, int recent,
                            float* pages, float* chunks, float* grids, hipStream_t stream)
{
    const Geom& g = ctx->geom;
    const size_t lds = (size_t)(g.n_c * g.n_g + g.n_g) * kHeadDim * sizeof(float);
    const int ppg = g.n_c * g.n_g;
    const int span = recent > 0 ? std::min(g.max_grids, (recent + ppg - 2) / ppg + 1) : g.max_grids;   // grids `recent` pages can touch
    const dim3 grid(span, g.n_kv_heads, batch), block(256);
    auto kern = g.page_size == 16 ? summarize_kernel<16> : summarize_kernel<32>;
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    return launch(kern, grid, block, lds, stream, k_pool, block_table, seq_lens,
                        from_page, recent, g, pages, chunks, grids);
}

}  // namespace chess
