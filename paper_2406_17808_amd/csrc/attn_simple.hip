// Chunk attention and score sums with scalar fp32 arithmetic, for any element type and head
// dimension.  This is the path of the fp32 configuration; the bf16 configurations use the
// MFMA kernels instead.
#include "launch.h"

namespace ckv {

constexpr int kSimpleThreads = 128;

__device__ inline float block_reduce_max(float v, float* red)
{
    red[threadIdx.x] = v;
    __syncthreads();
    for (int s = kSimpleThreads / 2; s > 0; s >>= 1) {
        if (threadIdx.x < s) red[threadIdx.x] = fmaxf(red[threadIdx.x], red[threadIdx.x + s]);
        __syncthreads();
    }
    const float r = red[0];
    __syncthreads();
    return r;
}

__device__ inline float block_reduce_sum(float v, float* red)
{
    red[threadIdx.x] = v;
    __syncthreads();
    for (int s = kSimpleThreads / 2; s > 0; s >>= 1) {
        if (threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
        __syncthreads();
    }
    const float r = red[0];
    __syncthreads();
    return r;
}

// One workgroup per (sequence, query head, query row).  Keys are visited in tiles of 128: thread
// j computes the logit of key j of the tile, the tile's probabilities go through LDS, and thread
// e accumulates output column e (and e + 128).  Online softmax across tiles (Eq. 2).
template <typename T>
__global__ void attn_simple_kernel(Geom g, SegList sl, int Q, const T* __restrict__ Qr,
                                   const T* __restrict__ Kr, const T* __restrict__ Vc,
                                   const T* __restrict__ Krc, const T* __restrict__ Vch,
                                   T* __restrict__ out, float* __restrict__ lse)
{
    __shared__ float qs[256];
    __shared__ float ps[kSimpleThreads];
    __shared__ float red[kSimpleThreads];
    const int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int hk = h / g.G, d = g.d;
    const size_t bh = (size_t)b * g.Hkv + hk;
    float m = -INFINITY, l = 0.f, o0 = 0.f, o1 = 0.f;
    const int e0 = threadIdx.x, e1 = threadIdx.x + kSimpleThreads;
    for (int si = 0; si < sl.n; ++si) {
        const Seg sg = sl.s[si];
        const T* qrow = Qr + ((((size_t)sg.qvar * g.B + b) * g.Hq + h) * Q + i) * d;
        __syncthreads();
        for (int e = threadIdx.x; e < d; e += kSimpleThreads) qs[e] = Elem<T>::load(qrow + e);
        __syncthreads();
        const T* kbase = sg.chunk ? Krc + (bh * Q) * d : Kr + (bh * g.slots + sg.start) * d;
        const T* vbase = sg.chunk ? Vch + (bh * Q) * d : Vc + (bh * g.slots + sg.start) * d;
        const int len = sg.chunk ? min(sg.len, i + 1) : sg.len;   // causal inside the chunk
        for (int t0 = 0; t0 < len; t0 += kSimpleThreads) {
            const int j = t0 + threadIdx.x;
            float s = -INFINITY;
            if (j < len) {
                const T* kr = kbase + (size_t)j * d;
                float acc = 0.f;
                for (int e = 0; e < d; ++e) acc += qs[e] * Elem<T>::load(kr + e);
                s = acc * g.scale;
            }
            const float mt = block_reduce_max(s, red);
            const float mn = fmaxf(m, mt);
            const float p = (j < len) ? expf(s - mn) : 0.f;
            const float lt = block_reduce_sum(p, red);
            const float alpha = expf(m - mn);     // m = -inf on the first tile gives 0
            ps[threadIdx.x] = p;
            __syncthreads();
            o0 *= alpha;
            o1 *= alpha;
            const int nt = min(kSimpleThreads, len - t0);
            for (int jj = 0; jj < nt; ++jj) {
                const T* vr = vbase + (size_t)(t0 + jj) * d;
                const float pj = ps[jj];
                if (e0 < d) o0 += pj * Elem<T>::load(vr + e0);
                if (e1 < d) o1 += pj * Elem<T>::load(vr + e1);
            }
            l = l * alpha + lt;
            m = mn;
            __syncthreads();
        }
    }
    T* orow = out + (((size_t)b * Q + i) * g.Hq + h) * d;
    if (e0 < d) Elem<T>::store(orow + e0, o0 / l);
    if (e1 < d) Elem<T>::store(orow + e1, o1 / l);
    if (threadIdx.x == 0) lse[((size_t)b * g.Hq + h) * Q + i] = m + logf(l);
}

void launch_attn_simple(const Geom& g, int dtype, const DevBuffers& b, const SegList& sl, int Q,
                        int, void* out, hipStream_t s)
{
    const dim3 grid(Q, g.Hq, g.B), block(kSimpleThreads);
    if (dtype == CASCADE_F32)
        hipLaunchKernelGGL(attn_simple_kernel<float>, grid, block, 0, s, g, sl, Q, (const float*)b.Qr, (const float*)b.Kr,
                           (const float*)b.Vc, (const float*)b.Krc, (const float*)b.Vch, (float*)out, b.lse);
    else
        hipLaunchKernelGGL(attn_simple_kernel<bf16_t>, grid, block, 0, s, g, sl, Q, (const bf16_t*)b.Qr,
                           (const bf16_t*)b.Kr, (const bf16_t*)b.Vc, (const bf16_t*)b.Krc, (const bf16_t*)b.Vch,
                           (bf16_t*)out, b.lse);
}

// Score sums: one thread per key.  For every query head of the group, the exact probabilities
// (final normaliser via the stored log-sum-exp) of the last `tail` rows of the chunk are
// weighted by wrow[rows after it] and summed (Section 3.1 EMA, one step per row); heads are
// reduced by max or mean; cached tokens then get mu <- decay * mu + sum, chunk tokens start
// at their sum.
template <typename T>
__global__ void score_simple_kernel(Geom g, SegList sl, int Q, int qstride, int tail, float decay,
                                    const T* __restrict__ Qr, const T* __restrict__ Kr,
                                    const T* __restrict__ Krc, const float* __restrict__ lse,
                                    const float* __restrict__ wrow, float* __restrict__ mu,
                                    float* __restrict__ mu_chunk)
{
    const int bh = blockIdx.y, b = bh / g.Hkv, hk = bh % g.Hkv;
    int j = blockIdx.x * blockDim.x + threadIdx.x;    // index over the concatenated segments
    int si = 0;
    while (si < sl.n && j >= sl.s[si].len) { j -= sl.s[si].len; ++si; }
    if (si >= sl.n) return;
    const Seg sg = sl.s[si];
    const int d = g.d;
    const T* kr = sg.chunk ? Krc + ((size_t)bh * Q + j) * d : Kr + ((size_t)bh * g.slots + sg.start + j) * d;
    const int i_lo = max(Q - tail, sg.chunk ? j : 0);
    float red = g.head_reduce == CASCADE_REDUCE_MAX ? 0.f : 0.f;
    for (int hh = 0; hh < g.G; ++hh) {
        const int h = hk * g.G + hh;
        const T* qbase = Qr + (((size_t)sg.qvar * g.B + b) * g.Hq + h) * (size_t)Q * d;
        const float* lrow = lse + ((size_t)b * g.Hq + h) * Q;
        float sum = 0.f;
        for (int i = i_lo; i < Q; ++i) {
            const T* qrow = qbase + (size_t)i * d;
            float acc = 0.f;
            for (int e = 0; e < d; ++e) acc += Elem<T>::load(qrow + e) * Elem<T>::load(kr + e);
            sum += wrow[Q - 1 - i] * expf(acc * g.scale - lrow[i]);
        }
        if (g.head_reduce == CASCADE_REDUCE_MAX) red = hh == 0 ? sum : fmaxf(red, sum);
        else red += sum;
    }
    if (g.head_reduce == CASCADE_REDUCE_MEAN) red /= (float)g.G;
    if (sg.chunk) mu_chunk[(size_t)bh * qstride + j] = red;
    else {
        float* p = mu + (size_t)bh * g.slots + sg.start + j;
        *p = decay * *p + red;
    }
}

void launch_score_simple(const Geom& g, int dtype, const DevBuffers& b, const SegList& sl, int Q,
                         int max_chunk, int tail_rows, float decay, hipStream_t s)
{
    int total = 0;
    for (int i = 0; i < sl.n; ++i) total += sl.s[i].len;
    const dim3 grid((total + 127) / 128, g.B * g.Hkv), block(128);
    if (dtype == CASCADE_F32)
        hipLaunchKernelGGL(score_simple_kernel<float>, grid, block, 0, s, g, sl, Q, max_chunk, tail_rows, decay,
                           (const float*)b.Qr, (const float*)b.Kr, (const float*)b.Krc, b.lse, b.wrow, b.mu, b.mu_chunk);
    else
        hipLaunchKernelGGL(score_simple_kernel<bf16_t>, grid, block, 0, s, g, sl, Q, max_chunk, tail_rows, decay,
                           (const bf16_t*)b.Qr, (const bf16_t*)b.Kr, (const bf16_t*)b.Krc, b.lse, b.wrow, b.mu, b.mu_chunk);
}

}  // namespace ckv
