// The quality monitor of Sec. 3.3: the entropy of each decode step's output distribution, and per generated
// page the average entropy and the variance of the entropy over the page's steps; reselection is asked for when
// either is above its threshold.
//
// entropy_kernel: grid (splits, batch).  A workgroup streams its slice of the sequence's logits row (bf16,
// 16-byte loads) keeping, per thread, the running maximum m, s0 = sum e^(z - m) and s1 = sum e^(z - m) (z - m);
// threads, then the splits (the last one to finish, in split order), merge such triplets, and
// H = log s0 - s1 / s0.  Bound: latency (a row of 150K logits is 300 KB; a batch of 32 moves 10 MB).
// trigger_kernel: one thread per sequence appends the step's entropy to the page's history and, when the page is
// complete, takes mean and population variance in fp64 in step order.
#include "chess_internal.h"

namespace chess {

struct Ent {
    float m, s0, s1;
};

__device__ __forceinline__ Ent ent_merge(const Ent& a, const Ent& b)
{
    const float M = fmaxf(a.m, b.m);
    if (M == -INFINITY) return Ent{M, 0.f, 0.f};
    const float da = a.m - M, db = b.m - M;              // <= 0; -inf for an empty side
    const float ea = a.s0 > 0.f ? __expf(da) : 0.f, eb = b.s0 > 0.f ? __expf(db) : 0.f;
    Ent r;
    r.m = M;
    r.s0 = a.s0 * ea + b.s0 * eb;
    r.s1 = (a.s0 > 0.f ? (a.s1 + da * a.s0) * ea : 0.f) + (b.s0 > 0.f ? (b.s1 + db * b.s0) * eb : 0.f);
    return r;
}

__device__ __forceinline__ void trigger_update_one(float Hb, int b, int page_steps, double tau_h, double tau_v,
                                                   float* __restrict__ history, int32_t* __restrict__ count,
                                                   int32_t* __restrict__ fire, double* __restrict__ stats);

// What the monitor call adds to the entropy kernel: the page statistics, done by the thread that has the entropy.
struct TriggerArgs {
    int page_steps;                                      // 0: entropy only
    double tau_h, tau_v;
    float* history;
    int32_t* count;
    int32_t* fire;
    double* stats;
};

constexpr int kEntThreads = 256;
constexpr int kEntFly = 4;                               // 16-byte loads per thread and trip

// partials: [batch][splits][4] floats; arrivals: [batch] int32, zero between launches
__global__ __launch_bounds__(kEntThreads) void entropy_kernel(const uint16_t* __restrict__ logits, int vocab, int64_t row_stride,
                                                              float* __restrict__ H, float* __restrict__ partials,
                                                              int32_t* __restrict__ arrivals, TriggerArgs tr)
{
    __shared__ Ent lds[kEntThreads];
    __shared__ int flag;
    const int split = blockIdx.x, n_splits = gridDim.x, b = blockIdx.y, tid = threadIdx.x;
    const uint4* row = reinterpret_cast<const uint4*>(logits + (size_t)b * row_stride);
    const int n_chunks = (vocab + 7) / 8;                                    // 8 logits per 16 bytes
    const int per = (n_chunks + n_splits - 1) / n_splits;
    const int c_lo = split * per, c_hi = min(n_chunks, c_lo + per);
    Ent acc{-INFINITY, 0.f, 0.f};
    for (int c0 = c_lo + tid; c0 < c_hi; c0 += kEntThreads * kEntFly) {
        uint4 r[kEntFly];
#pragma unroll
        for (int x = 0; x < kEntFly; ++x) r[x] = row[min(c0 + x * kEntThreads, c_hi - 1)];
        float z[kEntFly * 8];
        float mx = -INFINITY;
#pragma unroll
        for (int x = 0; x < kEntFly; ++x) {
            const int c = c0 + x * kEntThreads;
            const uint32_t w[4] = {r[x].x, r[x].y, r[x].z, r[x].w};
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float v = __uint_as_float((i & 1) ? (w[i >> 1] & 0xffff0000u) : (w[i >> 1] << 16));
                z[x * 8 + i] = (c < c_hi && c * 8 + i < vocab) ? v : -INFINITY;
                mx = fmaxf(mx, z[x * 8 + i]);
            }
        }
        if (mx == -INFINITY) continue;
        Ent e{mx, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < kEntFly * 8; ++i) {
            const float d = z[i] - mx;                    // -inf for a masked entry: contributes 0
            const float p = __expf(d);
            e.s0 += p;
            e.s1 += d > -INFINITY ? p * d : 0.f;
        }
        acc = ent_merge(acc, e);
    }
    lds[tid] = acc;
    __syncthreads();
    // the threads' triplets in thread order: 64 lanes take 4 each, then a tree over the lanes
    if (tid < 64) {
        Ent e = lds[4 * tid];
        e = ent_merge(e, lds[4 * tid + 1]);
        e = ent_merge(e, lds[4 * tid + 2]);
        e = ent_merge(e, lds[4 * tid + 3]);
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            Ent o;
            o.m = __shfl_xor(e.m, off);
            o.s0 = __shfl_xor(e.s0, off);
            o.s1 = __shfl_xor(e.s1, off);
            e = (tid & off) ? ent_merge(o, e) : ent_merge(e, o);
        }
        if (tid == 0) {
            if (n_splits == 1) {
                const float Hb = e.s0 > 0.f ? logf(e.s0) - e.s1 / e.s0 : 0.f;
                H[b] = Hb;
                if (tr.page_steps > 0) trigger_update_one(Hb, b, tr.page_steps, tr.tau_h, tr.tau_v, tr.history, tr.count, tr.fire, tr.stats);
            } else {
                float* p = partials + ((size_t)b * n_splits + split) * 4;
                publish_f32(p, e.m); publish_f32(p + 1, e.s0); publish_f32(p + 2, e.s1);
            }
        }
    }
    if (n_splits == 1) return;
    if (!arrive_last(arrivals + b, n_splits, &flag)) return;
    // the splits' triplets: lane s of wave 0 takes split s (at most kEntMaxSplits = 32 of them), then the same tree
    if (tid < 64) {
        Ent e{-INFINITY, 0.f, 0.f};
        if (tid < n_splits) {
            const float* p = partials + ((size_t)b * n_splits + tid) * 4;
            e = Ent{observe_f32(p), observe_f32(p + 1), observe_f32(p + 2)};
        }
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            Ent o;
            o.m = __shfl_xor(e.m, off);
            o.s0 = __shfl_xor(e.s0, off);
            o.s1 = __shfl_xor(e.s1, off);
            e = (tid & off) ? ent_merge(o, e) : ent_merge(e, o);
        }
        if (tid == 0) {
            const float Hb = e.s0 > 0.f ? logf(e.s0) - e.s1 / e.s0 : 0.f;
            H[b] = Hb;
            if (tr.page_steps > 0) trigger_update_one(Hb, b, tr.page_steps, tr.tau_h, tr.tau_v, tr.history, tr.count, tr.fire, tr.stats);
        }
    }
}

hipError_t launch_entropy(chess_ctx* ctx, const uint16_t* logits, int batch, int vocab, int64_t row_stride, int splits,
                          float* H, float* partials, int32_t* arrivals, int page_steps, double tau_h, double tau_v,
                          float* history, int32_t* count, int32_t* fire, double* stats, hipStream_t stream)
{
    (void)ctx;
    const TriggerArgs tr{page_steps, tau_h, tau_v, history, count, fire, stats};
    return launch(entropy_kernel, dim3(splits, batch), dim3(kEntThreads), 0, stream, logits, vocab, row_stride, H, partials,
                  arrivals, tr);
}

// The page statistics of one sequence (what trigger_kernel does per thread).
__device__ __forceinline__ void trigger_update_one(float Hb, int b, int page_steps, double tau_h, double tau_v,
                                                   float* __restrict__ history, int32_t* __restrict__ count,
                                                   int32_t* __restrict__ fire, double* __restrict__ stats)
{
    float* hist = history + (size_t)b * page_steps;
    int c = count[b];
    if (c < 0 || c >= page_steps) c = 0;                  // a state the caller did not initialise
    hist[c] = Hb;
    ++c;
    int f = 0;
    if (c == page_steps) {                                // the page is complete
        double s = 0.0, q = 0.0;
        for (int i = 0; i < page_steps - 1; ++i) s += (double)hist[i];
        s += (double)Hb;                                  // (the entry just stored, without reading it back)
        const double mu = s / (double)page_steps;
        for (int i = 0; i < page_steps; ++i) {
#pragma clang fp contract(off)                            // product rounded, then added: no fused multiply-add
            const double d = (double)(i == page_steps - 1 ? Hb : hist[i]) - mu;
            const double dd = d * d;
            q = q + dd;
        }
        const double var = q / (double)page_steps;
        f = (mu > tau_h || var > tau_v) ? 1 : 0;
        if (stats) { stats[2 * b] = mu; stats[2 * b + 1] = var; }
        c = 0;
    }
    fire[b] = f;
    count[b] = c;
}

// one thread per sequence
__global__ void trigger_kernel(const float* __restrict__ H, int batch, int page_steps, double tau_h, double tau_v,
                               float* __restrict__ history, int32_t* __restrict__ count, int32_t* __restrict__ fire,
                               double* __restrict__ stats)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= batch) return;
    trigger_update_one(H[b], b, page_steps, tau_h, tau_v, history, count, fire, stats);
}

hipError_t launch_trigger(const float* H, int batch, int page_steps, double tau_h, double tau_v, float* history,
                          int32_t* count, int32_t* fire, double* stats, hipStream_t stream)
{
    return launch(trigger_kernel, dim3((batch + 63) / 64), dim3(64), 0, stream, H, batch, page_steps, tau_h, tau_v, history,
                  count, fire, stats);
}

}  // namespace chess
