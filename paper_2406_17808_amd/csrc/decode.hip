// Decode step (Eq. 2): one query per sequence against the whole cache plus its own key.
// The cache is streamed once: K in decode_qk (logits), V in decode_pv (outputs + EMA scores).
// Sixteen lanes share a row; every lane owns d/16 contiguous elements of it.
#include "launch.h"

namespace ckv {

constexpr int kDecThreads = 256;
constexpr int kLanesPerRow = 16;
constexpr int kRowsPerIter = kDecThreads / kLanesPerRow;   // 16 rows per workgroup iteration
constexpr int kMaxG = 8;

template <typename T, int EPL> struct VecLoad;
template <> struct VecLoad<bf16_t, 8> {
    __device__ static void load(const bf16_t* p, float* o)
    {
        const uint4 u = *reinterpret_cast<const uint4*>(p);
        const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) { o[2 * i] = __uint_as_float(w[i] << 16); o[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u); }
    }
};
template <> struct VecLoad<bf16_t, 4> {
    __device__ static void load(const bf16_t* p, float* o)
    {
        const uint2 u = *reinterpret_cast<const uint2*>(p);
        const uint32_t w[2] = {u.x, u.y};
#pragma unroll
        for (int i = 0; i < 2; ++i) { o[2 * i] = __uint_as_float(w[i] << 16); o[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u); }
    }
};
template <> struct VecLoad<float, 8> {
    __device__ static void load(const float* p, float* o)
    {
        const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
        o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w; o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
    }
};
template <> struct VecLoad<float, 4> {
    __device__ static void load(const float* p, float* o)
    {
        const float4 a = *reinterpret_cast<const float4*>(p);
        o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w;
    }
};

// index in the concatenation of the cached segments -> (segment, offset)
__device__ inline int seg_of(const SegList& sl, int j, int* off)
{
    int si = 0;
    while (si < sl.n - 1 && j >= sl.s[si].len) { j -= sl.s[si].len; ++si; }
    *off = j;
    return si;
}

// Rotated query slices of this lane for segment `si`: the stored keys are rotated to their slot
// index, so the query turns by (own index) - (cache index - slot index), one angle per segment.
template <typename T, int EPL>
__device__ inline void load_q_rot(const Geom& g, const SegList& sl, int si, const T* __restrict__ q,
                                  const float2* __restrict__ rope, int b, int hk, int lane, float (*qr)[EPL])
{
    const int half = g.d / 2;
    const int rot = sl.qrot0[sl.s[si].qvar];
    for (int hh = 0; hh < g.G; ++hh) {
        const T* qh = q + ((size_t)b * g.Hq + hk * g.G + hh) * g.d;
#pragma unroll
        for (int x = 0; x < EPL; ++x) {
            const int e = lane * EPL + x;
            const int pe = e < half ? e : e - half;
            const float2 cs = rope[(size_t)rot * half + pe];
            const float a = Elem<T>::load(qh + pe), c = Elem<T>::load(qh + pe + half);
            qr[hh][x] = (e < half ? a * cs.x - c * cs.y : c * cs.x + a * cs.y) * g.scale;
        }
    }
}

// logits[b][h][j] = scale * <q_rot, Kr[slot(j)]> for the rows of this split; per split and head
// the running (max, sum of exp) go to `part`.  Split 0 also handles the token's own key, whose
// logit needs no rotation (query and key sit at the same index).
template <typename T, int EPL>
__global__ void decode_qk_kernel(Geom g, SegList sl, int per_split, const T* __restrict__ q,
                                 const T* __restrict__ k_new, const T* __restrict__ Kr,
                                 const float2* __restrict__ rope, float* __restrict__ logits,
                                 float* __restrict__ part, int n_splits)
{
    __shared__ float red_m[kRowsPerIter][kMaxG], red_l[kRowsPerIter][kMaxG];
    const int split = blockIdx.x, hk = blockIdx.y, b = blockIdx.z;
    const int bh = b * g.Hkv + hk;
    const int grp = threadIdx.x / kLanesPerRow, lane = threadIdx.x % kLanesPerRow;
    const int n = sl.n_cached;
    const int j0 = split * per_split, j1 = min(n, j0 + per_split);
    const size_t lstride = (size_t)n + 1;
    float qr[kMaxG][EPL];
    float m[kMaxG], l[kMaxG];
    for (int hh = 0; hh < kMaxG; ++hh) { m[hh] = -INFINITY; l[hh] = 0.f; }
    int cur_seg = -1;
    for (int jb = j0; jb < j1; jb += kRowsPerIter) {
        const int j = jb + grp;
        // segment changes are handled per row group; rows of one iteration may straddle two segments
        int off = 0, si = (j < j1) ? seg_of(sl, j, &off) : cur_seg;
        if (j < j1 && si != cur_seg) { load_q_rot<T, EPL>(g, sl, si, q, rope, b, hk, lane, qr); cur_seg = si; }
        if (j < j1) {
            const int slot = sl.s[si].start + off;
            float kv[EPL];
            VecLoad<T, EPL>::load(Kr + ((size_t)bh * g.slots + slot) * g.d + lane * EPL, kv);
            for (int hh = 0; hh < g.G; ++hh) {
                float acc = 0.f;
#pragma unroll
                for (int x = 0; x < EPL; ++x) acc += qr[hh][x] * kv[x];
#pragma unroll
                for (int w = kLanesPerRow / 2; w > 0; w >>= 1) acc += __shfl_xor(acc, w, kLanesPerRow);
                if (lane == 0) {
                    logits[((size_t)b * g.Hq + hk * g.G + hh) * lstride + j] = acc;
                    const float mn = fmaxf(m[hh], acc);
                    l[hh] = l[hh] * __expf(m[hh] - mn) + __expf(acc - mn);
                    m[hh] = mn;
                }
            }
        }
    }
    if (split == 0 && grp == 0) {
        // own key: <R(n) q, R(n) k> = <q, k>
        float kv[EPL];
        VecLoad<T, EPL>::load(k_new + ((size_t)b * g.Hkv + hk) * g.d + lane * EPL, kv);
        for (int hh = 0; hh < g.G; ++hh) {
            float qv[EPL];
            VecLoad<T, EPL>::load(q + ((size_t)b * g.Hq + hk * g.G + hh) * g.d + lane * EPL, qv);
            float acc = 0.f;
#pragma unroll
            for (int x = 0; x < EPL; ++x) acc += qv[x] * kv[x];
#pragma unroll
            for (int w = kLanesPerRow / 2; w > 0; w >>= 1) acc += __shfl_xor(acc, w, kLanesPerRow);
            acc *= g.scale;
            if (lane == 0) {
                logits[((size_t)b * g.Hq + hk * g.G + hh) * lstride + n] = acc;
                const float mn = fmaxf(m[hh], acc);
                l[hh] = l[hh] * __expf(m[hh] - mn) + __expf(acc - mn);
                m[hh] = mn;
            }
        }
    }
    if (lane == 0)
        for (int hh = 0; hh < g.G; ++hh) { red_m[grp][hh] = m[hh]; red_l[grp][hh] = l[hh]; }
    __syncthreads();
    if (threadIdx.x < g.G) {
        const int hh = threadIdx.x;
        float mm = -INFINITY, ll = 0.f;
        for (int r = 0; r < kRowsPerIter; ++r) {
            const float mr = red_m[r][hh], lr = red_l[r][hh];
            if (lr > 0.f) {
                const float mn = fmaxf(mm, mr);
                ll = ll * __expf(mm - mn) + lr * __expf(mr - mn);
                mm = mn;
            }
        }
        float* p = part + (((size_t)b * g.Hq + hk * g.G + hh) * n_splits + split) * 2;
        p[0] = mm;
        p[1] = ll;
    }
}

// Outputs and EMA scores of the rows of this split: with the exact log-sum-exp (all splits of
// decode_qk combined) p = exp(logit - lse) is final, so partial outputs simply add up, and
// mu <- beta*mu + (1-beta)*reduce_heads(p) can be applied in the same pass (Section 3.1).
template <typename T, int EPL>
__global__ void decode_pv_kernel(Geom g, SegList sl, int per_split, const T* __restrict__ Vc,
                                 const float* __restrict__ logits, const float* __restrict__ part,
                                 int n_splits, float* __restrict__ opart, float* __restrict__ mu,
                                 float* __restrict__ lse_out)
{
    __shared__ float lse_s[kMaxG];
    __shared__ float osum[kDecThreads / 64][kMaxG][kLanesPerRow * EPL];
    const int split = blockIdx.x, hk = blockIdx.y, b = blockIdx.z;
    const int bh = b * g.Hkv + hk;
    const int grp = threadIdx.x / kLanesPerRow, lane = threadIdx.x % kLanesPerRow;
    const int n = sl.n_cached;
    const size_t lstride = (size_t)n + 1;
    if (threadIdx.x < g.G) {
        const float* p = part + ((size_t)b * g.Hq + hk * g.G + threadIdx.x) * n_splits * 2;
        float mm = -INFINITY, ll = 0.f;
        for (int s = 0; s < n_splits; ++s) {
            const float ms = p[2 * s], ls = p[2 * s + 1];
            if (ls > 0.f) {
                const float mn = fmaxf(mm, ms);
                ll = ll * __expf(mm - mn) + ls * __expf(ms - mn);
                mm = mn;
            }
        }
        lse_s[threadIdx.x] = mm + __logf(ll);
        if (split == 0) lse_out[(size_t)b * g.Hq + hk * g.G + threadIdx.x] = mm + __logf(ll);
    }
    __syncthreads();
    float o[kMaxG][EPL];
    for (int hh = 0; hh < kMaxG; ++hh)
#pragma unroll
        for (int x = 0; x < EPL; ++x) o[hh][x] = 0.f;
    const int j0 = split * per_split, j1 = min(n, j0 + per_split);
    for (int jb = j0; jb < j1; jb += kRowsPerIter) {
        const int j = jb + grp;
        if (j < j1) {
            int off;
            const int si = seg_of(sl, j, &off);
            const int slot = sl.s[si].start + off;
            float vv[EPL];
            VecLoad<T, EPL>::load(Vc + ((size_t)bh * g.slots + slot) * g.d + lane * EPL, vv);
            float red = 0.f;
            for (int hh = 0; hh < g.G; ++hh) {
                const float p = __expf(logits[((size_t)b * g.Hq + hk * g.G + hh) * lstride + j] - lse_s[hh]);
#pragma unroll
                for (int x = 0; x < EPL; ++x) o[hh][x] += p * vv[x];
                red = (g.head_reduce == CASCADE_REDUCE_MAX) ? (hh == 0 ? p : fmaxf(red, p)) : red + p;
            }
            if (lane == 0) {
                if (g.head_reduce == CASCADE_REDUCE_MEAN) red /= (float)g.G;
                float* pm = mu + (size_t)bh * g.slots + slot;
                *pm = g.beta * *pm + (1.f - g.beta) * red;
            }
        }
    }
    // the four row groups of a wave first add up through lane shuffles
    for (int hh = 0; hh < g.G; ++hh)
#pragma unroll
        for (int x = 0; x < EPL; ++x) {
            float t = o[hh][x];
            t += __shfl_xor(t, 16, 64);
            t += __shfl_xor(t, 32, 64);
            if (grp % 4 == 0) osum[grp / 4][hh][lane * EPL + x] = t;
        }
    __syncthreads();
    for (int idx = threadIdx.x; idx < g.G * g.d; idx += kDecThreads) {
        const int hh = idx / g.d, e = idx % g.d;
        float s = 0.f;
        for (int r = 0; r < kDecThreads / 64; ++r) s += osum[r][hh][e];
        opart[(((size_t)b * g.Hq + hk * g.G + hh) * n_splits + split) * g.d + e] = s;
    }
}

// out = sum of the split outputs + own value weighted by its probability; the new token's
// score starts at (1-beta) * reduce_heads(p_own).
template <typename T>
__global__ void decode_finish_kernel(Geom g, int n_cached, int n_splits, int qstride,
                                     const float* __restrict__ opart, const float* __restrict__ logits,
                                     const float* __restrict__ lse, const T* __restrict__ v_new,
                                     T* __restrict__ out, float* __restrict__ mu_chunk)
{
    const int hk = blockIdx.x, b = blockIdx.y;
    const size_t lstride = (size_t)n_cached + 1;
    for (int idx = threadIdx.x; idx < g.G * g.d; idx += blockDim.x) {
        const int hh = idx / g.d, e = idx % g.d, h = hk * g.G + hh;
        const float p = __expf(logits[((size_t)b * g.Hq + h) * lstride + n_cached] - lse[(size_t)b * g.Hq + h]);
        float s = p * Elem<T>::load(v_new + ((size_t)b * g.Hkv + hk) * g.d + e);
        const float* op = opart + ((size_t)b * g.Hq + h) * n_splits * g.d + e;
        for (int sp = 0; sp < n_splits; ++sp) s += op[(size_t)sp * g.d];
        Elem<T>::store(out + ((size_t)b * g.Hq + h) * g.d + e, s);
    }
    if (threadIdx.x == 0) {
        float red = 0.f;
        for (int hh = 0; hh < g.G; ++hh) {
            const int h = hk * g.G + hh;
            const float p = __expf(logits[((size_t)b * g.Hq + h) * lstride + n_cached] - lse[(size_t)b * g.Hq + h]);
            red = (g.head_reduce == CASCADE_REDUCE_MAX) ? (hh == 0 ? p : fmaxf(red, p)) : red + p;
        }
        if (g.head_reduce == CASCADE_REDUCE_MEAN) red /= (float)g.G;
        mu_chunk[((size_t)b * g.Hkv + hk) * qstride] = (1.f - g.beta) * red;
    }
}

static int per_split_of(const DevBuffers& bf, int n)
{
    int per_split = (n + bf.dec_splits - 1) / bf.dec_splits;
    per_split = ((per_split + kRowsPerIter - 1) / kRowsPerIter) * kRowsPerIter;
    return per_split == 0 ? kRowsPerIter : per_split;
}

template <typename T, int EPL>
static void qk_typed(const Geom& g, const DevBuffers& bf, const SegList& sl, const void* q, const void* k, hipStream_t s)
{
    const dim3 grid(bf.dec_splits, g.Hkv, g.B), block(kDecThreads);
    hipLaunchKernelGGL((decode_qk_kernel<T, EPL>), grid, block, 0, s, g, sl, per_split_of(bf, sl.n_cached), (const T*)q,
                       (const T*)k, (const T*)bf.Kr, bf.rope, bf.logits, bf.part, bf.dec_splits);
}

template <typename T, int EPL>
static void pv_typed(const Geom& g, const DevBuffers& bf, const SegList& sl, hipStream_t s)
{
    const dim3 grid(bf.dec_splits, g.Hkv, g.B), block(kDecThreads);
    // the log-sum-exp of the step lives in the first B*Hq entries of the chunk scratch
    hipLaunchKernelGGL((decode_pv_kernel<T, EPL>), grid, block, 0, s, g, sl, per_split_of(bf, sl.n_cached), (const T*)bf.Vc,
                       bf.logits, bf.part, bf.dec_splits, bf.opart, bf.mu, bf.lse);
}

#define CKV_DISPATCH(fn, ...)                                                     \
    do {                                                                          \
        const int epl = g.d / kLanesPerRow;                                       \
        if (dtype == CASCADE_F32) { if (epl == 8) fn<float, 8>(__VA_ARGS__); else fn<float, 4>(__VA_ARGS__); } \
        else { if (epl == 8) fn<bf16_t, 8>(__VA_ARGS__); else fn<bf16_t, 4>(__VA_ARGS__); }                    \
    } while (0)

void launch_decode_qk(const Geom& g, int dtype, const DevBuffers& b, const SegList& sl, const void* q, const void* k,
                      hipStream_t s)
{
    CKV_DISPATCH(qk_typed, g, b, sl, q, k, s);
}

void launch_decode_pv(const Geom& g, int dtype, const DevBuffers& b, const SegList& sl, hipStream_t s)
{
    CKV_DISPATCH(pv_typed, g, b, sl, s);
}

void launch_decode_finish(const Geom& g, int dtype, const DevBuffers& b, const SegList& sl, int qstride, const void* v,
                          void* out, hipStream_t s)
{
    const dim3 grid(g.Hkv, g.B), block(256);
    if (dtype == CASCADE_F32)
        hipLaunchKernelGGL(decode_finish_kernel<float>, grid, block, 0, s, g, sl.n_cached, b.dec_splits, qstride, b.opart,
                           b.logits, b.lse, (const float*)v, (float*)out, b.mu_chunk);
    else
        hipLaunchKernelGGL(decode_finish_kernel<bf16_t>, grid, block, 0, s, g, sl.n_cached, b.dec_splits, qstride, b.opart,
                           b.logits, b.lse, (const bf16_t*)v, (bf16_t*)out, b.mu_chunk);
}

bool decode_supported(const Geom& g) { return (g.d == 64 || g.d == 128) && g.G <= kMaxG; }

}  // namespace ckv
