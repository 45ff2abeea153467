// Cache maintenance kernels: tables, query/key rotation, the score-dependent part of the
// cascade update (Alg. 2) and the row moves that carry it out.
#include "launch.h"
#include "plan_core.h"
#include "structure.h"

namespace ckv {

// ------------------------------------------------------------------ tables

// (cos, sin)(p * theta_i), theta_i = base^(-2i/d), evaluated in double so that large
// indices keep full float accuracy.
// rope_t (optional): the same values index-minor, [d/4 groups of two rotary pairs][rows], for readers whose
// lanes hold consecutive indices (the attention kernel's queries): their 16-byte loads then fall into
// a few cache lines per instruction instead of one line per lane.
__global__ void rope_table_kernel(float2* __restrict__ rope, float2* __restrict__ rope_t, int rows, int half, int d, double base)
{
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (long)rows * half) return;
    const int p = (int)(idx / half), i = (int)(idx % half);
    const double theta = pow(base, -2.0 * (double)i / (double)d);
    double s, c;
    sincos((double)p * theta, &s, &c);
    rope[idx] = make_float2((float)c, (float)s);
    if (rope_t) rope_t[((size_t)(i >> 1) * rows + p) * 2 + (i & 1)] = make_float2((float)c, (float)s);
}

void launch_rope_table(const Geom& g, float base, float2* rope, float2* rope_t, int rows, hipStream_t s)
{
    const int half = g.d / 2;
    const long n = (long)rows * half;
    hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                       rope, rope_t, rows, half, g.d, (double)base);
}

// wrow[k] = beta^k (1 - beta): weight of the query row that has k rows after it in its chunk
// (Alg. 3's coefficient; the EMA of Section 3.1 unrolled over the rows of a chunk).
__global__ void wrow_table_kernel(float* __restrict__ wrow, int n, double beta)
{
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k < n) wrow[k] = (float)(pow(beta, (double)k) * (1.0 - beta));
}

void launch_wrow_table(float beta, float* wrow, int n, hipStream_t s)
{
    hipLaunchKernelGGL(wrow_table_kernel, dim3((n + 255) / 256), dim3(256), 0, s, wrow, n, (double)beta);
}

__global__ void fill_i32_kernel(int32_t* __restrict__ p, size_t n, int32_t v)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = v;
}

void launch_fill_i32(int32_t* p, size_t n, int32_t value, hipStream_t s)
{
    if (n == 0) return;
    const unsigned blocks = (unsigned)std::min<size_t>((n + 255) / 256, 65535);
    hipLaunchKernelGGL(fill_i32_kernel, dim3(blocks), dim3(256), 0, s, p, n, value);
}

// ------------------------------------------------------------------ initial state

// Scatter a state given in cache order into the physical layout (ring heads at 0) and build
// the rotated key copy.  One thread per (row, rotary pair).
struct FillCounts { int sink; int c[kMaxCascades]; };

template <typename T>
__global__ void load_state_kernel(Geom g, FillCounts fc, int total, T* __restrict__ Kc, T* __restrict__ Kr,
                                  T* __restrict__ Vc, float* __restrict__ mu, int32_t* __restrict__ ids,
                                  const float2* __restrict__ rope,
                                  const T* __restrict__ k_in, const T* __restrict__ v_in,
                                  const float* __restrict__ mu_in, const int32_t* __restrict__ ids_in)
{
    const int half = g.d / 2;
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const long per_bh = (long)total * half;
    if (idx >= per_bh * g.B * g.Hkv) return;
    const int bh = (int)(idx / per_bh);
    const int r = (int)((idx % per_bh) / half), e = (int)(idx % half);
    // rank r in cache order -> physical slot
    int slot = -1, rr = r;
    if (rr < fc.sink) slot = rr;
    else {
        rr -= fc.sink;
        for (int c = g.N - 1; c >= 0; --c) {
            if (rr < fc.c[c]) { slot = g.base[c] + rr; break; }
            rr -= fc.c[c];
        }
    }
    const size_t src = ((size_t)bh * total + r) * g.d;
    const size_t dst = ((size_t)bh * g.slots + slot) * g.d;
    const float x0 = Elem<T>::load(k_in + src + e), x1 = Elem<T>::load(k_in + src + e + half);
    const float2 cs = rope[(size_t)slot * half + e];
    Elem<T>::store(Kc + dst + e, x0);
    Elem<T>::store(Kc + dst + e + half, x1);
    Elem<T>::store(Kr + dst + e, rot_lo(x0, x1, cs.x, cs.y));
    Elem<T>::store(Kr + dst + e + half, rot_hi(x0, x1, cs.x, cs.y));
    Vc[dst + e] = v_in[src + e];
    Vc[dst + e + half] = v_in[src + e + half];
    if (e == 0) {
        mu[(size_t)bh * g.slots + slot] = mu_in[(size_t)bh * total + r];
        ids[(size_t)bh * g.slots + slot] = ids_in[(size_t)bh * total + r];
    }
}

void launch_load_state(const Geom& g, int dtype, const DevBuffers& b, const void* k, const void* v,
                       const float* mu, const int32_t* ids, const int* counts, int total, hipStream_t s)
{
    if (total == 0) return;
    const long n = (long)g.B * g.Hkv * total * (g.d / 2);
    FillCounts fc;
    fc.sink = counts[0];
    for (int i = 0; i < kMaxCascades; ++i) fc.c[i] = i < g.N ? counts[1 + i] : 0;
    const dim3 grid((unsigned)((n + 255) / 256)), block(256);
    if (dtype == CASCADE_F32)
        hipLaunchKernelGGL(load_state_kernel<float>, grid, block, 0, s, g, fc, total, (float*)b.Kc, (float*)b.Kr,
                           (float*)b.Vc, b.mu, b.ids, b.rope, (const float*)k, (const float*)v, mu, ids);
    else
        hipLaunchKernelGGL(load_state_kernel<bf16_t>, grid, block, 0, s, g, fc, total, (bf16_t*)b.Kc, (bf16_t*)b.Kr,
                           (bf16_t*)b.Vc, b.mu, b.ids, b.rope, (const bf16_t*)k, (const bf16_t*)v, mu, ids);
}

// ------------------------------------------------------------------ per-chunk rotation

// For every rotated query copy v: Qr[v][b][h][i] = qscale * R(qrot0[v] + i) q[b][i][h] (the bf16
// MFMA kernels want the softmax scale and log2(e) folded into the queries; everybody else passes
// 1); chunk keys are rotated to their chunk index, chunk values are copied head-major.  A thread takes 8 rotary
// pairs of one row (two 16-byte pieces for bf16) and, for a query row, produces all copies.
template <typename T> struct Vec8;
template <> struct Vec8<bf16_t> {
    __device__ static void load(const bf16_t* p, float* o)
    {
        const uint4 u = *reinterpret_cast<const uint4*>(p);
        const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) { o[2 * i] = __uint_as_float(w[i] << 16); o[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u); }
    }
    __device__ static void store(bf16_t* p, const float* v)
    {
        uint4 u;
        u.x = (uint32_t)f32_to_bf16(v[0]) | ((uint32_t)f32_to_bf16(v[1]) << 16);
        u.y = (uint32_t)f32_to_bf16(v[2]) | ((uint32_t)f32_to_bf16(v[3]) << 16);
        u.z = (uint32_t)f32_to_bf16(v[4]) | ((uint32_t)f32_to_bf16(v[5]) << 16);
        u.w = (uint32_t)f32_to_bf16(v[6]) | ((uint32_t)f32_to_bf16(v[7]) << 16);
        *reinterpret_cast<uint4*>(p) = u;
    }
};
template <> struct Vec8<float> {
    __device__ static void load(const float* p, float* o)
    {
        const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
        o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w; o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
    }
    __device__ static void store(float* p, const float* v)
    {
        *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
        *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
    }
};

template <typename T>
__device__ inline void rotate8(const float* x0, const float* x1, const float2* __restrict__ cs, T* d0, T* d1)
{
    float y0[8], y1[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const float2 c = cs[i];
        y0[i] = rot_lo(x0[i], x1[i], c.x, c.y);
        y1[i] = rot_hi(x0[i], x1[i], c.x, c.y);
    }
    Vec8<T>::store(d0, y0);
    Vec8<T>::store(d1, y1);
}

template <typename T>
__global__ void prep_kernel(Geom g, SegList sl, int Q, float qscale, int q_first_row, const float2* __restrict__ rope,
                            const T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ v,
                            T* __restrict__ Qr, T* __restrict__ Krc, T* __restrict__ Vch)
{
    const int half = g.d / 2, groups = half / 8;
    // threads [0, n_kv): one per (sequence, token, K or V head, group); then one per (sequence, query row
    // that needs rotated copies, query head, group)
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const long n_kv = (long)g.B * Q * 2 * g.Hkv * groups;
    const int q_rows = Q - q_first_row;
    float x0[8], x1[8];
    if (idx < n_kv) {
        const int e = (int)(idx % groups) * 8;
        long r = idx / groups;
        const int rr = (int)(r % (2 * g.Hkv));
        r /= 2 * g.Hkv;
        const int i = (int)(r % Q), b = (int)(r / Q);
        const int h = rr % g.Hkv;
        const size_t src = (((size_t)b * Q + i) * g.Hkv + h) * g.d;
        const size_t dst = (((size_t)b * g.Hkv + h) * Q + i) * g.d;
        if (rr < g.Hkv) {
            Vec8<T>::load(k + src + e, x0);
            Vec8<T>::load(k + src + e + half, x1);
            rotate8<T>(x0, x1, rope + (size_t)i * half + e, Krc + dst + e, Krc + dst + e + half);
        } else {
            Vec8<T>::load(v + src + e, x0);
            Vec8<T>::load(v + src + e + half, x1);
            Vec8<T>::store(Vch + dst + e, x0);
            Vec8<T>::store(Vch + dst + e + half, x1);
        }
        return;
    }
    const long qidx = idx - n_kv;
    if (qidx >= (long)g.B * q_rows * g.Hq * groups) return;
    const int e = (int)(qidx % groups) * 8;
    long r = qidx / groups;
    const int h = (int)(r % g.Hq);
    r /= g.Hq;
    const int i = q_first_row + (int)(r % q_rows), b = (int)(r / q_rows);
    const size_t src = (((size_t)b * Q + i) * g.Hq + h) * g.d;
    Vec8<T>::load(q + src + e, x0);
    Vec8<T>::load(q + src + e + half, x1);
#pragma unroll
    for (int j = 0; j < 8; ++j) { x0[j] *= qscale; x1[j] *= qscale; }
    for (int vq = 0; vq < sl.n_qvar; ++vq) {
        const size_t dst = ((((size_t)vq * g.B + b) * g.Hq + h) * Q + i) * g.d;
        rotate8<T>(x0, x1, rope + (size_t)(sl.qrot0[vq] + i) * half + e, Qr + dst + e, Qr + dst + e + half);
    }
}

// head dimensions that are not a multiple of 16: one thread per rotary pair
template <typename T>
__global__ void prep_pair_kernel(Geom g, SegList sl, int Q, float qscale, int q_first_row, const float2* __restrict__ rope,
                                 const T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ v,
                                 T* __restrict__ Qr, T* __restrict__ Krc, T* __restrict__ Vch)
{
    const int half = g.d / 2;
    const int rows_per_tok = sl.n_qvar * g.Hq + 2 * g.Hkv;
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const long total = (long)g.B * Q * rows_per_tok * half;
    if (idx >= total) return;
    const int e = (int)(idx % half);
    long r = idx / half;
    const int row = (int)(r % rows_per_tok);
    r /= rows_per_tok;
    const int i = (int)(r % Q), b = (int)(r / Q);
    if (row < sl.n_qvar * g.Hq) {
        if (i < q_first_row) return;
        const int vq = row / g.Hq, h = row % g.Hq;
        const size_t src = (((size_t)b * Q + i) * g.Hq + h) * g.d;
        const size_t dst = ((((size_t)vq * g.B + b) * g.Hq + h) * Q + i) * g.d;
        const float x0 = qscale * Elem<T>::load(q + src + e), x1 = qscale * Elem<T>::load(q + src + e + half);
        const float2 cs = rope[(size_t)(sl.qrot0[vq] + i) * half + e];
        Elem<T>::store(Qr + dst + e, rot_lo(x0, x1, cs.x, cs.y));
        Elem<T>::store(Qr + dst + e + half, rot_hi(x0, x1, cs.x, cs.y));
    } else {
        const int rr = row - sl.n_qvar * g.Hq;
        const int h = rr % g.Hkv;
        const size_t src = (((size_t)b * Q + i) * g.Hkv + h) * g.d;
        const size_t dst = (((size_t)b * g.Hkv + h) * Q + i) * g.d;
        if (rr < g.Hkv) {
            const float x0 = Elem<T>::load(k + src + e), x1 = Elem<T>::load(k + src + e + half);
            const float2 cs = rope[(size_t)i * half + e];
            Elem<T>::store(Krc + dst + e, rot_lo(x0, x1, cs.x, cs.y));
            Elem<T>::store(Krc + dst + e + half, rot_hi(x0, x1, cs.x, cs.y));
        } else {
            Vch[dst + e] = v[src + e];
            Vch[dst + e + half] = v[src + e + half];
        }
    }
}

void launch_prep(const Geom& g, int dtype, const DevBuffers& b, const SegList& sl, int Q, float qscale, int q_first_row,
                 const void* q, const void* k, const void* v, hipStream_t s)
{
    const dim3 block(256);
    if (g.d % 16 == 0) {
        const long n = (long)g.B * (Q * 2 * g.Hkv + (Q - q_first_row) * g.Hq) * (g.d / 16);
        const dim3 grid((unsigned)((n + 255) / 256));
        if (dtype == CASCADE_F32)
            hipLaunchKernelGGL(prep_kernel<float>, grid, block, 0, s, g, sl, Q, qscale, q_first_row, b.rope, (const float*)q, (const float*)k,
                               (const float*)v, (float*)b.Qr, (float*)b.Krc, (float*)b.Vch);
        else
            hipLaunchKernelGGL(prep_kernel<bf16_t>, grid, block, 0, s, g, sl, Q, qscale, q_first_row, b.rope, (const bf16_t*)q, (const bf16_t*)k,
                               (const bf16_t*)v, (bf16_t*)b.Qr, (bf16_t*)b.Krc, (bf16_t*)b.Vch);
        return;
    }
    const long n = (long)g.B * Q * (sl.n_qvar * g.Hq + 2 * g.Hkv) * (g.d / 2);
    const dim3 grid((unsigned)((n + 255) / 256));
    if (dtype == CASCADE_F32)
        hipLaunchKernelGGL(prep_pair_kernel<float>, grid, block, 0, s, g, sl, Q, qscale, q_first_row, b.rope, (const float*)q, (const float*)k,
                           (const float*)v, (float*)b.Qr, (float*)b.Krc, (float*)b.Vch);
    else
        hipLaunchKernelGGL(prep_pair_kernel<bf16_t>, grid, block, 0, s, g, sl, Q, qscale, q_first_row, b.rope, (const bf16_t*)q,
                           (const bf16_t*)k, (const bf16_t*)v, (bf16_t*)b.Qr, (bf16_t*)b.Krc, (bf16_t*)b.Vch);
}

// ------------------------------------------------------------------ homogeneous heads

// Appendix "Head Policy and Head Reduction", homogeneous heads: one score per token for all heads.
// The score kernels have reduced the query heads of every KV head; here the KV heads are reduced
// in turn (max of maxima; mean of means, the groups being equally large) and every KV head gets
// the result.  All KV heads then hold the same tokens in the same slots, so the reduction runs
// slot by slot.  For the cached rows the reduction of the updated scores is the update with the
// reduced increments: before the call the scores of a slot are equal in all heads.
__global__ void share_scores_kernel(Geom g, int n_new, int qstride, float* __restrict__ mu, float* __restrict__ mu_chunk)
{
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const long per_b = (long)g.slots + n_new;
    if (idx >= per_b * g.B) return;
    const int b = (int)(idx / per_b), j = (int)(idx % per_b);
    float* p = j < g.slots ? mu + (size_t)b * g.Hkv * g.slots + j : mu_chunk + (size_t)b * g.Hkv * qstride + (j - g.slots);
    const size_t stride = j < g.slots ? (size_t)g.slots : (size_t)qstride;
    float r = p[0];
    for (int h = 1; h < g.Hkv; ++h) r = g.head_reduce == CASCADE_REDUCE_MAX ? fmaxf(r, p[h * stride]) : r + p[h * stride];
    if (g.head_reduce == CASCADE_REDUCE_MEAN) r /= (float)g.Hkv;
    for (int h = 0; h < g.Hkv; ++h) p[h * stride] = r;
}

void launch_share_scores(const Geom& g, const DevBuffers& b, int n_new, int max_chunk, hipStream_t s)
{
    const long n = ((long)g.slots + n_new) * g.B;
    hipLaunchKernelGGL(share_scores_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, g, n_new, max_chunk, b.mu, b.mu_chunk);
}

// ------------------------------------------------------------------ cascade update: who ends up where

// One workgroup per (sequence, KV head).  For every cascade in turn:
//   phase 1  the winner of every segment (see plan_core.h);
//   phase 2  every push passes the item it evicts on to the next cascade.
// winners[c][0] is the segment of the item that was newest before the update, winners[c][1+j]
// that of the j-th slot opened.
__global__ void plan_kernel(Geom g, UpdatePlan pl, int qstride, const float* __restrict__ mu,
                            const float* __restrict__ mu_chunk, int32_t* __restrict__ offers,
                            int32_t* __restrict__ winners, int32_t* __restrict__ swaps)
{
    const int bh = blockIdx.x;
    const float* mub = mu + (size_t)bh * g.slots;
    const float* muc = mu_chunk + (size_t)bh * qstride;
    int32_t* off_in = offers + (size_t)bh * 2 * qstride;
    int32_t* off_out = off_in + qstride;
    for (int c = 0; c < pl.N; ++c) {
        const CascStep cs = pl.c[c];
        if (cs.M == 0) break;
        int32_t* W = winners + ((size_t)bh * pl.N + c) * (qstride + 1);
        const int nseg = cs.J + cs.pre;
        int my_swaps = 0;
        for (int sidx = threadIdx.x; sidx < nseg; sidx += blockDim.x) {
            const int j = sidx - cs.pre;
            int sw;
            W[1 + j] = segment_winner(cs, c, j, g.slots, pl.n_to_sink, g.token_selection, off_in, mub, muc, &sw);
            my_swaps += sw;
        }
        if (my_swaps) atomicAdd(&swaps[bh * pl.N + c], my_swaps);
        __syncthreads();
        for (int i = threadIdx.x; i < cs.P; i += blockDim.x) off_out[i] = evicted_ref(cs, i, W);
        __syncthreads();
        int32_t* tmp = off_in; off_in = off_out; off_out = tmp;
    }
}

void launch_plan(const Geom& g, const DevBuffers& b, const UpdatePlan& pl, int max_chunk, hipStream_t s)
{
    const int threads = pl.Q >= 1024 ? 1024 : (pl.Q >= 256 ? 256 : 64);
    hipLaunchKernelGGL(plan_kernel, dim3(g.B * g.Hkv), dim3(threads), 0, s, g, pl, max_chunk, b.mu, b.mu_chunk,
                       b.offers, b.winners, b.swaps);
}

// ------------------------------------------------------------------ cascade update: row moves

// Final content of cascade c (c = -1: sinks).  Entry e < E names a ring position that was
// written during the update and the ref that ends up in it; one extra entry covers the item
// that was newest before the update if a competing offer replaced it.  A destination row is
// rebuilt from the un-rotated source key, re-rotated to the destination slot index.
// `lanes` threads cooperate on a row; each handles rotary pairs e, e + lanes, ...
template <typename T>
__global__ void move_kernel(Geom g, UpdatePlan pl, int c, int E, int extra, int qstride,
                            const float2* __restrict__ rope, const int32_t* __restrict__ winners,
                            T* __restrict__ Kc, T* __restrict__ Kr, T* __restrict__ Vc,
                            float* __restrict__ mu, int32_t* __restrict__ ids,
                            const float* __restrict__ mu_chunk,
                            const T* __restrict__ k_in, const T* __restrict__ v_in,
                            long tok_stride, long batch_stride, int lanes)
{
    const int bh = blockIdx.y;
    const int b = bh / g.Hkv, h = bh % g.Hkv;
    const int rows_per_block = blockDim.x / lanes;
    const int e = blockIdx.x * rows_per_block + threadIdx.x / lanes;
    const int lane = threadIdx.x % lanes;
    if (e >= E + extra) return;
    int dst, ref;
    if (c < 0) {
        dst = pl.sink_fill0 + e;
        ref = g.slots + e;
    } else {
        const int32_t* W = winners + ((size_t)bh * pl.N + c) * (qstride + 1);
        if (!final_entry(pl.c[c], e, E, W, &dst, &ref)) return;
    }
    const int half = g.d / 2;
    const size_t drow = ((size_t)bh * g.slots + dst) * g.d;
    const T *ks, *vs;
    float score;
    int id;
    if (ref < g.slots) {
        const size_t srow = ((size_t)bh * g.slots + ref) * g.d;
        ks = Kc + srow;
        vs = Vc + srow;
        score = mu[(size_t)bh * g.slots + ref];
        id = ids[(size_t)bh * g.slots + ref];
    } else {
        const int i = ref - g.slots;
        const size_t srow = (size_t)b * batch_stride + (size_t)i * tok_stride + (size_t)h * g.d;
        ks = k_in + srow;
        vs = v_in + srow;
        score = mu_chunk[(size_t)bh * qstride + i];
        id = pl.id0 + i;
    }
    for (int p = lane; p < half; p += lanes) {
        const float x0 = Elem<T>::load(ks + p), x1 = Elem<T>::load(ks + p + half);
        const float2 cs2 = rope[(size_t)dst * half + p];
        Elem<T>::store(Kc + drow + p, x0);
        Elem<T>::store(Kc + drow + p + half, x1);
        Elem<T>::store(Kr + drow + p, rot_lo(x0, x1, cs2.x, cs2.y));
        Elem<T>::store(Kr + drow + p + half, rot_hi(x0, x1, cs2.x, cs2.y));
        Vc[drow + p] = vs[p];
        Vc[drow + p + half] = vs[p + half];
    }
    if (lane == 0) {
        mu[(size_t)bh * g.slots + dst] = score;
        ids[(size_t)bh * g.slots + dst] = id;
    }
}

// The moves of all cascades in two launches.  Every entry (cascade, index) names a destination
// slot and a source; gather_kernel copies the sources that are cache rows (un-rotated key, value,
// score, id: the state before the update) into a staging array, scatter_kernel then writes every
// destination from the staging array or from the chunk's own tokens.  No launch both reads and
// writes the cache, so the order of the cascades does not matter.
struct MoveList {
    int n, total;
    int c[kMaxCascades + 1], first[kMaxCascades + 2], E[kMaxCascades + 1], extra[kMaxCascades + 1];
};

// direct: the plan is direct (plan_is_direct) and nobody has written the winners of the FIRST
// cascade: every token is accepted there (period 1), so a slot it opens takes the offer that opens it
__device__ inline bool move_entry(const Geom& g, const UpdatePlan& pl, const MoveList& ml, int eg, int bh, int qstride,
                                  const int32_t* __restrict__ winners, int* dst, int* ref, bool direct = false)
{
    int i = 0;
    while (i + 1 < ml.n && eg >= ml.first[i + 1]) ++i;
    const int c = ml.c[i], e = eg - ml.first[i];
    if (c < 0) {
        *dst = pl.sink_fill0 + e;
        *ref = g.slots + e;
        return true;
    }
    if (direct && c == 0) {              // J <= cap: entry e is slot j = e; no offer competes in the first cascade
        const CascStep& cs = pl.c[0];
        *dst = cs.base + (cs.wpos0 + e) % cs.cap;
        *ref = offer_ref_direct(pl, 0, e < cs.A ? e : cs.kp0 + (e - cs.A) * cs.pstride, g.slots);
        return true;
    }
    const int32_t* W = winners + ((size_t)bh * pl.N + c) * (qstride + 1);
    return final_entry(pl.c[c], e, ml.E[i], W, dst, ref);
}

// lanes = d/16 threads per row, each moving 8 elements of both halves of the head dimension
template <typename T>
__global__ void gather_kernel(Geom g, UpdatePlan pl, MoveList ml, int qstride, int stage_rows,
                              const int32_t* __restrict__ winners, const T* __restrict__ Kc, const T* __restrict__ Vc,
                              const float* __restrict__ mu, const int32_t* __restrict__ ids,
                              T* __restrict__ stK, T* __restrict__ stV, float* __restrict__ stMu, int32_t* __restrict__ stId)
{
    const int lanes = g.d / 16, half = g.d / 2;
    const int bh = blockIdx.y;
    const int eg = blockIdx.x * (blockDim.x / lanes) + threadIdx.x / lanes;
    const int lane = threadIdx.x % lanes;
    if (eg >= ml.total) return;
    int dst, ref;
    if (!move_entry(g, pl, ml, eg, bh, qstride, winners, &dst, &ref)) return;
    if (ref >= g.slots) return;          // a token of the chunk: read by scatter_kernel
    const size_t srow = ((size_t)bh * g.slots + ref) * g.d, trow = ((size_t)bh * stage_rows + eg) * g.d;
    float x[8];
    Vec8<T>::load(Kc + srow + lane * 8, x);          Vec8<T>::store(stK + trow + lane * 8, x);
    Vec8<T>::load(Kc + srow + half + lane * 8, x);   Vec8<T>::store(stK + trow + half + lane * 8, x);
    Vec8<T>::load(Vc + srow + lane * 8, x);          Vec8<T>::store(stV + trow + lane * 8, x);
    Vec8<T>::load(Vc + srow + half + lane * 8, x);   Vec8<T>::store(stV + trow + half + lane * 8, x);
    if (lane == 0) {
        stMu[(size_t)bh * stage_rows + eg] = mu[(size_t)bh * g.slots + ref];
        stId[(size_t)bh * stage_rows + eg] = ids[(size_t)bh * g.slots + ref];
    }
}

template <typename T>
__global__ void scatter_kernel(Geom g, UpdatePlan pl, MoveList ml, int qstride, int stage_rows,
                               const float2* __restrict__ rope, const int32_t* __restrict__ winners,
                               const T* __restrict__ stK, const T* __restrict__ stV, const float* __restrict__ stMu,
                               const int32_t* __restrict__ stId, const float* __restrict__ mu_chunk,
                               const T* __restrict__ k_in, const T* __restrict__ v_in, long tok_stride, long batch_stride,
                               T* __restrict__ Kc, T* __restrict__ Kr, T* __restrict__ Vc, float* __restrict__ mu,
                               int32_t* __restrict__ ids, bool direct)
{
    const int lanes = g.d / 16, half = g.d / 2;
    const int bh = blockIdx.y;
    const int b = bh / g.Hkv, h = bh % g.Hkv;
    const int eg = blockIdx.x * (blockDim.x / lanes) + threadIdx.x / lanes;
    const int lane = threadIdx.x % lanes;
    if (eg >= ml.total) return;
    int dst, ref;
    if (!move_entry(g, pl, ml, eg, bh, qstride, winners, &dst, &ref, direct)) return;
    const T *ks, *vs;
    float score;
    int id;
    if (ref < g.slots) {
        const size_t trow = ((size_t)bh * stage_rows + eg) * g.d;
        ks = stK + trow;
        vs = stV + trow;
        score = stMu[(size_t)bh * stage_rows + eg];
        id = stId[(size_t)bh * stage_rows + eg];
    } else {
        const int i = ref - g.slots;
        const size_t srow = (size_t)b * batch_stride + (size_t)i * tok_stride + (size_t)h * g.d;
        ks = k_in + srow;
        vs = v_in + srow;
        score = mu_chunk[(size_t)bh * qstride + i];
        id = pl.id0 + i;
    }
    const size_t drow = ((size_t)bh * g.slots + dst) * g.d;
    const int e = lane * 8;
    float x0[8], x1[8];
    Vec8<T>::load(ks + e, x0);
    Vec8<T>::load(ks + half + e, x1);
    Vec8<T>::store(Kc + drow + e, x0);
    Vec8<T>::store(Kc + drow + half + e, x1);
    rotate8<T>(x0, x1, rope + (size_t)dst * half + e, Kr + drow + e, Kr + drow + half + e);
    Vec8<T>::load(vs + e, x0);
    Vec8<T>::load(vs + half + e, x1);
    Vec8<T>::store(Vc + drow + e, x0);
    Vec8<T>::store(Vc + drow + half + e, x1);
    if (lane == 0) {
        mu[(size_t)bh * g.slots + dst] = score;
        ids[(size_t)bh * g.slots + dst] = id;
    }
}

// gather_kernel for updates whose plan is direct (plan_is_direct): the thread group of an entry
// decides its segment itself (the offers are named from the structure alone), leaves the winner
// in `winners` for scatter_kernel, counts the replacements, and stages the winner if it is a cache
// row.  No plan_kernel launch, no cascade-by-cascade dependency.  Only the cascades beyond the
// first have anything to decide or to stage (the first takes the chunk's tokens as they come):
// the launch covers their entries only, n_entries of them.
template <typename T>
__global__ void gather_direct_kernel(Geom g, UpdatePlan pl, MoveList ml, int n_entries, int qstride, int stage_rows,
                                     int32_t* __restrict__ winners, int32_t* __restrict__ swaps,
                                     const float* __restrict__ mu_chunk, const T* __restrict__ Kc, const T* __restrict__ Vc,
                                     const float* __restrict__ mu, const int32_t* __restrict__ ids,
                                     T* __restrict__ stK, T* __restrict__ stV, float* __restrict__ stMu, int32_t* __restrict__ stId)
{
    __shared__ int wg_swaps[kMaxCascades];   // replacements counted by this workgroup, per cascade
    const int lanes = g.d / 16, half = g.d / 2;
    const int bh = blockIdx.y;
    const int eg = blockIdx.x * (blockDim.x / lanes) + threadIdx.x / lanes;
    const int lane = threadIdx.x % lanes;
    if (threadIdx.x < kMaxCascades) wg_swaps[threadIdx.x] = 0;
    __syncthreads();
    int c = -1, j = 0, ref = 0, dst = 0;
    bool move = false;
    if (eg < n_entries) {                // the entries of the cascades beyond the first come first in the list
        int i = 0;
        while (i + 1 < ml.n && eg >= ml.first[i + 1]) ++i;
        c = ml.c[i];
        {
            const CascStep& cs = pl.c[c];
            // entry e < E is slot j = e of the J <= cap slots opened (final_entry); entry E is the segment of
            // the item that was newest before the update
            const int e = eg - ml.first[i];
            j = e < ml.E[i] ? e : -1;
            dst = j < 0 ? cs.base + cs.newest0 : cs.base + (cs.wpos0 + j) % cs.cap;
        }
    }
    // The segment of every entry, decided by the `lanes` threads of its group together: the same
    // first-maximum rule as segment_winner (a later offer replaces the holder only on a strictly
    // higher score), with the scores of `lanes` offers loaded at a time instead of one after the other.
    {
        const int lead = (threadIdx.x & 63) - lane;          // first lane of this group inside the wave
        int kb = 0, ke = 0, sw = 0;
        float bs = 0.f;
        const float* mub = mu + (size_t)bh * g.slots;
        const float* muc = mu_chunk + (size_t)bh * qstride;
        if (c >= 0) {
            const CascStep& cs = pl.c[c];
            if (j < 0) {
                ref = cs.base + cs.newest0;
                kb = 0;
                ke = cs.kp0 < cs.M ? cs.kp0 : cs.M;
            } else {
                const int kh = j < cs.A ? j : cs.kp0 + (j - cs.A) * cs.pstride;
                ref = offer_ref_direct(pl, c, kh, g.slots);
                kb = kh + 1;
                if (j + 1 < cs.A) ke = kb;
                else if (j + 1 == cs.A) ke = cs.kp0 < cs.M ? cs.kp0 : cs.M;
                else ke = kh + cs.pstride < cs.M ? kh + cs.pstride : cs.M;
            }
            if (!g.token_selection) ke = kb;
            if (ke > kb) bs = ref_score(ref, g.slots, mub, muc);
        }
        // rounds of `lanes` offers; groups of one wave may need different numbers of rounds
        int rounds = c >= 0 && ke > kb ? (ke - kb + lanes - 1) / lanes : 0;
        int max_rounds = rounds;
        for (int w = lanes; w < 64; w <<= 1) max_rounds = max(max_rounds, __shfl_xor(max_rounds, w, 64));
        for (int r = 0; r < max_rounds; ++r) {
            const int k = kb + r * lanes + lane;
            const bool valid = r < rounds && k < ke;
            int rk = 0;
            float s = -INFINITY;
            if (valid) {
                rk = offer_ref_direct(pl, c, k, g.slots);
                s = ref_score(rk, g.slots, mub, muc);
            }
            // highest score among the holder and the offers before this lane's
            float before = bs;
            for (int x = 0; x < lanes; ++x) {
                const float sx = __shfl(s, lead + x, 64);
                if (x < lane) before = fmaxf(before, sx);
            }
            const bool record = valid && s > before;         // this offer would replace the holder when its turn comes
            const unsigned long long rec = __ballot(record) >> lead & ((1ull << lanes) - 1ull);
            if (rec) {
                const int last = 63 - __builtin_clzll(rec);  // the last replacement of the round holds the slot after it
                ref = __shfl(rk, lead + last, 64);
                bs = __shfl(s, lead + last, 64);
                sw += __builtin_popcountll(rec);
            }
        }
        if (c >= 0 && lane == 0) {
            winners[((size_t)bh * pl.N + c) * (qstride + 1) + 1 + j] = ref;
            if (sw) atomicAdd(&wg_swaps[c], sw);
        }
    }
    move = c >= 0 && ref < g.slots && ref != dst;   // a cache row that goes somewhere else (chunk tokens are read by scatter_kernel)
    if (move) {
        const size_t srow = ((size_t)bh * g.slots + ref) * g.d, trow = ((size_t)bh * stage_rows + eg) * g.d;
        float x[8];
        Vec8<T>::load(Kc + srow + lane * 8, x);          Vec8<T>::store(stK + trow + lane * 8, x);
        Vec8<T>::load(Kc + srow + half + lane * 8, x);   Vec8<T>::store(stK + trow + half + lane * 8, x);
        Vec8<T>::load(Vc + srow + lane * 8, x);          Vec8<T>::store(stV + trow + lane * 8, x);
        Vec8<T>::load(Vc + srow + half + lane * 8, x);   Vec8<T>::store(stV + trow + half + lane * 8, x);
        if (lane == 0) {
            stMu[(size_t)bh * stage_rows + eg] = mu[(size_t)bh * g.slots + ref];
            stId[(size_t)bh * stage_rows + eg] = ids[(size_t)bh * g.slots + ref];
        }
    }
    __syncthreads();
    if (threadIdx.x < pl.N && wg_swaps[threadIdx.x]) atomicAdd(&swaps[bh * pl.N + threadIdx.x], wg_swaps[threadIdx.x]);
}

template <typename T>
static void moves_two_phase(const Geom& g, const DevBuffers& b, const UpdatePlan& pl, const MoveList& ml, int max_chunk,
                            const void* k, const void* v, int k_token_stride, int k_batch_stride, bool direct, hipStream_t s)
{
    const int lanes = g.d / 16, threads = 256, rows = threads / lanes;
    const dim3 grid((ml.total + rows - 1) / rows, g.B * g.Hkv), block(threads);
    const size_t BH = (size_t)g.B * g.Hkv;
    T* stK = (T*)b.move_stage;
    T* stV = stK + BH * b.move_stage_rows * g.d;
    float* stMu = (float*)(stV + BH * b.move_stage_rows * g.d);
    int32_t* stId = (int32_t*)(stMu + BH * b.move_stage_rows);
    if (direct) {
        int n_entries = ml.total;        // entries before those of the first cascade and of the sinks
        for (int i = 0; i < ml.n; ++i)
            if (ml.c[i] <= 0) { n_entries = ml.first[i]; break; }
        if (n_entries > 0)
            hipLaunchKernelGGL(gather_direct_kernel<T>, dim3((n_entries + rows - 1) / rows, g.B * g.Hkv), block, 0, s, g, pl, ml, n_entries,
                               max_chunk, b.move_stage_rows, b.winners, b.swaps, b.mu_chunk, (const T*)b.Kc, (const T*)b.Vc, b.mu, b.ids,
                               stK, stV, stMu, stId);
    } else
        hipLaunchKernelGGL(gather_kernel<T>, grid, block, 0, s, g, pl, ml, max_chunk, b.move_stage_rows, b.winners,
                           (const T*)b.Kc, (const T*)b.Vc, b.mu, b.ids, stK, stV, stMu, stId);
    hipLaunchKernelGGL(scatter_kernel<T>, grid, block, 0, s, g, pl, ml, max_chunk, b.move_stage_rows, b.rope, b.winners,
                       (const T*)stK, (const T*)stV, stMu, stId, b.mu_chunk, (const T*)k, (const T*)v,
                       (long)k_token_stride, (long)k_batch_stride, (T*)b.Kc, (T*)b.Kr, (T*)b.Vc, b.mu, b.ids, direct);
}

// Head dimensions that are not a multiple of 16 take one launch per cascade: destinations of
// cascade c take sources from earlier cascades or from the chunk only (items never move
// backwards), so writing the last cascade first keeps every source intact until it has been read.
bool update_is_direct(const Geom& g, const DevBuffers& b, const UpdatePlan& pl)
{
    if (!(g.d % 16 == 0 && b.move_stage) || b.opt_update_staged || !plan_is_direct(pl)) return false;
    int total = pl.n_to_sink;
    for (int c = 0; c < pl.N; ++c) {
        if (pl.c[c].M == 0) continue;
        int extra;
        total += final_entries(pl.c[c], &extra);
        total += extra;
    }
    return total <= b.move_stage_rows;
}

// `direct`: no plan_kernel has run; the gather launch decides the segments itself (update_is_direct)
void launch_moves(const Geom& g, int dtype, const DevBuffers& b, const UpdatePlan& pl, int max_chunk,
                  const void* k, const void* v, int k_token_stride, int k_batch_stride, bool direct, hipStream_t s)
{
    if (g.d % 16 == 0 && b.move_stage) {
        MoveList ml;
        ml.n = 0;
        ml.total = 0;
        for (int c = pl.N - 1; c >= -1; --c) {
            int E, extra = 0;
            if (c < 0) {
                E = pl.n_to_sink;
            } else {
                if (pl.c[c].M == 0) continue;
                E = final_entries(pl.c[c], &extra);
            }
            if (E + extra == 0) continue;
            ml.c[ml.n] = c; ml.first[ml.n] = ml.total; ml.E[ml.n] = E; ml.extra[ml.n] = extra;
            ml.total += E + extra;
            ++ml.n;
        }
        ml.first[ml.n] = ml.total;
        if (ml.total == 0) return;
        if (ml.total <= b.move_stage_rows) {
            if (dtype == CASCADE_F32) moves_two_phase<float>(g, b, pl, ml, max_chunk, k, v, k_token_stride, k_batch_stride, direct, s);
            else moves_two_phase<bf16_t>(g, b, pl, ml, max_chunk, k, v, k_token_stride, k_batch_stride, direct, s);
            return;
        }
    }
    const int lanes = 32, threads = 256, rows = threads / lanes;
    for (int c = pl.N - 1; c >= -1; --c) {
        int E, extra = 0;
        if (c < 0) {
            E = pl.n_to_sink;
        } else {
            if (pl.c[c].M == 0) continue;
            E = final_entries(pl.c[c], &extra);
        }
        if (E + extra == 0) continue;
        const dim3 grid((E + extra + rows - 1) / rows, g.B * g.Hkv), block(threads);
        if (dtype == CASCADE_F32)
            hipLaunchKernelGGL(move_kernel<float>, grid, block, 0, s, g, pl, c, E, extra, max_chunk, b.rope, b.winners,
                               (float*)b.Kc, (float*)b.Kr, (float*)b.Vc, b.mu, b.ids, b.mu_chunk,
                               (const float*)k, (const float*)v, (long)k_token_stride, (long)k_batch_stride, lanes);
        else
            hipLaunchKernelGGL(move_kernel<bf16_t>, grid, block, 0, s, g, pl, c, E, extra, max_chunk, b.rope, b.winners,
                               (bf16_t*)b.Kc, (bf16_t*)b.Kr, (bf16_t*)b.Vc, b.mu, b.ids, b.mu_chunk,
                               (const bf16_t*)k, (const bf16_t*)v, (long)k_token_stride, (long)k_batch_stride, lanes);
    }
}

}  // namespace ckv
