// Decode step (Eq. 2): one query per sequence against the whole cache plus its own key.
// The cache is streamed once from HBM: K by decode_qk (logits), V by decode_pv (outputs and
// EMA scores); the logits of a step (16 bytes per cached row at 4 query heads per KV head)
// pass through a scratch array because the EMA update needs exact probabilities.
#include <stdlib.h>

#include "async_copy.h"
#include "launch.h"
#include "small_update.h"

namespace ckv {

constexpr int kDecThreads = 256;
constexpr int kLanesPerRow = 16;                            // lanes that share one row in the VALU kernels
constexpr int kRowGroups = kDecThreads / kLanesPerRow;      // 16 row groups per workgroup
constexpr int kMaxG = 8;

// Logits of a step: [B][Hkv][n_cached + 1][MAXG] floats, MAXG = group size rounded up to 1, 2, 4
// or 8 (decode_logit_heads): the heads of a group are adjacent, so the kernel that computes them
// stores, and the kernel that consumes them loads, whole 64-byte-aligned runs of a row block.
__device__ inline size_t logit_index(const Geom& g, int maxg, size_t lrows, int b, int hk, int row, int hh)
{
    return ((((size_t)b * g.Hkv + hk) * lrows + row) * maxg) + hh;
}

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

// (max, sum of exp) pairs combine associatively
__device__ inline void ml_merge(float& m, float& l, float m2, float l2)
{
    if (l2 > 0.f) {
        const float mn = fmaxf(m, m2);
        l = l * __expf(m - mn) + l2 * __expf(m2 - mn);
        m = mn;
    }
}

// One rotated, scaled element of the query: the stored keys are rotated to their slot index,
// so the query turns by (own index) - (cache index - slot index), one angle per segment.
template <typename T>
__device__ inline float q_rot_elem(const T* __restrict__ qh, const float2* __restrict__ rope, int rot, int half_d,
                                   int e, float scale)
{
    const int pe = e < half_d ? e : e - half_d;
    const float2 cs = rope[(size_t)rot * half_d + pe];
    const float a = Elem<T>::load(qh + pe), c = Elem<T>::load(qh + pe + half_d);
    return (e < half_d ? a * cs.x - c * cs.y : c * cs.x + a * cs.y) * scale;
}

// ------------------------------------------------------------------ QK, bf16: MFMA 16x16x32
//
// v_mfma_f32_16x16x32_bf16: for lane l, A holds row l%16, B column l%16, both with the 8
// contraction indices 8*(l/16)..+7; D holds column l%16, rows 4*(l/16)..+3.  Rows are 16 keys,
// columns the query heads of the group (padded with zeros to 16), the contraction runs over the
// head dimension.  Which element of the head dimension a contraction index means is free as
// long as A and B agree: lane group c = l/16 takes elements [c*D/4 + 8*ks, +8) in step ks, so a
// lane reads D/2 contiguous bytes of a key row and four lanes cover the row.

typedef __attribute__((ext_vector_type(8))) __bf16 dbf16x8_t;
typedef __attribute__((ext_vector_type(4))) float df32x4_t;
typedef __attribute__((ext_vector_type(4))) uint32_t du32x4_t;
union DFrag {
    dbf16x8_t v;
    du32x4_t u;
};

__device__ inline uint32_t dec_pack_bf16(float lo, float hi)
{
    typedef __attribute__((ext_vector_type(2))) __bf16 b2;
    typedef __attribute__((ext_vector_type(2))) float f2;
    const f2 x = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, b2));
}

constexpr int kQkRowsPerWave = 64;   // four 16-key MFMA groups in flight per wave iteration

template <int D, int MAXG>
__global__ __launch_bounds__(kDecThreads) void decode_qk_mfma_kernel(
    Geom g, SegList sl, int per_split, const bf16_t* __restrict__ q, const bf16_t* __restrict__ k_new,
    const bf16_t* __restrict__ Kr, const float2* __restrict__ rope, float* __restrict__ logits,
    float* __restrict__ part, int n_splits)
{
    constexpr int KS = D / 32;            // MFMA steps over the head dimension
    constexpr int NG = kQkRowsPerWave / 16;
    __shared__ float red_m[kDecThreads / 64][16], red_l[kDecThreads / 64][16];
    __shared__ float stage[kDecThreads / 64][kQkRowsPerWave * MAXG];   // a wave's logits of one iteration, [row][head]
    const int split = blockIdx.x, hk = blockIdx.y, b = blockIdx.z;
    const int bh = b * g.Hkv + hk;
    const int wave = threadIdx.x >> 6, l = threadIdx.x & 63, n = l & 15, c = l >> 4;
    const int ncached = sl.n_cached;
    const int j0 = split * per_split, j1 = min(ncached, j0 + per_split);
    const size_t lrows = (size_t)ncached + 1;
    const bool head_ok = n < g.G;
    const bf16_t* qh = q + ((size_t)b * g.Hq + hk * g.G + (head_ok ? n : 0)) * D;
    float* lbase = logits + logit_index(g, MAXG, lrows, b, hk, 0, 0);
    float m = -INFINITY, lsum = 0.f;

    int seg_first = 0;                    // index of the segment's first row in the concatenation
    for (int si = 0; si < sl.n; ++si) {
        const Seg sg = sl.s[si];
        const int lo = max(j0, seg_first), hi = min(j1, seg_first + sg.len);
        if (lo < hi) {
            // B operand: this segment's rotation of the group's queries, scaled, as bf16
            DFrag qf[KS];
            const int rot = sl.qrot0[sg.qvar];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    const int e = ks * 32 + c * 8 + 2 * x;
                    const float a0 = head_ok ? q_rot_elem<bf16_t>(qh, rope, rot, D / 2, e, g.scale) : 0.f;
                    const float a1 = head_ok ? q_rot_elem<bf16_t>(qh, rope, rot, D / 2, e + 1, g.scale) : 0.f;
                    qf[ks].u[x] = dec_pack_bf16(a0, a1);
                }
            // row index = index in the concatenation of the segments
            const bf16_t* kseg = Kr + ((ptrdiff_t)bh * g.slots + sg.start - seg_first) * D;
            for (int r0 = lo + wave * kQkRowsPerWave; r0 < hi; r0 += (kDecThreads / 64) * kQkRowsPerWave) {
                DFrag kf[NG][KS];
#pragma unroll
                for (int gi = 0; gi < NG; ++gi) {
                    const int row = min(r0 + gi * 16 + n, hi - 1);      // rows past the end repeat the last one
                    const bf16_t* kp = kseg + (size_t)row * D + c * 8;
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) kf[gi][ks].u = *reinterpret_cast<const du32x4_t*>(kp + ks * 32);
                }
#pragma unroll
                for (int gi = 0; gi < NG; ++gi) {
                    df32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks)
                        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[gi][ks].v, qf[ks].v, acc, 0, 0, 0);
                    // this lane: head n, keys r0 + 16*gi + 4*c + {0..3}
                    const int rbase = r0 + gi * 16 + 4 * c;
                    if (n < MAXG) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) stage[wave][(gi * 16 + 4 * c + j) * MAXG + n] = acc[j];
                    }
                    if (head_ok) {
                        // one rescaling per four logits: the running maximum rarely moves
                        float mx = m;
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            if (rbase + j < hi) mx = fmaxf(mx, acc[j]);
                        if (mx > m) {   // (also keeps -inf - -inf out of the arithmetic)
                            lsum *= __expf(m - mx);
                            m = mx;
                        }
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            if (rbase + j < hi) lsum += __expf(acc[j] - m);
                    }
                }
                // the wave's 64 x MAXG logits leave as contiguous 256-byte stores (LDS accesses of one
                // wave are ordered; no other wave touches this stage)
#pragma unroll
                for (int i = 0; i < MAXG; ++i) {
                    const int idx = l + 64 * i;
                    if (r0 + idx / MAXG < hi) lbase[(size_t)r0 * MAXG + idx] = stage[wave][idx];
                }
            }
        }
        seg_first += sg.len;
    }
    if (split == 0 && wave == 0) {
        // own key: <R(n) q, R(n) k> = <q, k>; lanes c = 0 of the valid heads take it
        if (head_ok && c == 0) {
            const bf16_t* kn = k_new + ((size_t)b * g.Hkv + hk) * D;
            float acc = 0.f;
            for (int e = 0; e < D; ++e) acc += bf16_to_f32(qh[e]) * bf16_to_f32(kn[e]);
            acc *= g.scale;
            lbase[(size_t)ncached * MAXG + n] = acc;
            const float mn = fmaxf(m, acc);
            lsum = lsum * __expf(m - mn) + __expf(acc - mn);
            m = mn;
        }
    }
    // combine the four lane groups of a head, then the waves
#pragma unroll
    for (int w = 16; w < 64; w <<= 1) {
        const float m2 = __shfl_xor(m, w, 64), l2 = __shfl_xor(lsum, w, 64);
        ml_merge(m, lsum, m2, l2);
    }
    if (c == 0) { red_m[wave][n] = m; red_l[wave][n] = lsum; }
    __syncthreads();
    if (threadIdx.x < g.G) {
        float mm = -INFINITY, ll = 0.f;
        for (int w = 0; w < kDecThreads / 64; ++w) ml_merge(mm, ll, red_m[w][threadIdx.x], red_l[w][threadIdx.x]);
        float* p = part + (((size_t)b * g.Hq + hk * g.G + threadIdx.x) * n_splits + split) * 2;
        p[0] = mm;
        p[1] = ll;
    }
}

// ------------------------------------------------------------------ QK, any type: VALU

// Sixteen lanes share a row; every lane owns D/16 contiguous elements of it and all heads of
// the group.  Four rows per lane group are in flight.
template <typename T, int EPL, int MAXG>
__global__ __launch_bounds__(kDecThreads) void decode_qk_valu_kernel(
    Geom g, SegList sl, int per_split, const T* __restrict__ q, const T* __restrict__ k_new,
    const T* __restrict__ Kr, const float2* __restrict__ rope, float* __restrict__ logits,
    float* __restrict__ part, int n_splits)
{
    constexpr int U = 4;
    __shared__ float red_m[kRowGroups][MAXG], red_l[kRowGroups][MAXG];
    const int split = blockIdx.x, hk = blockIdx.y, b = blockIdx.z;
    const int bh = b * g.Hkv + hk;
    const int grp = threadIdx.x / kLanesPerRow, lane = threadIdx.x % kLanesPerRow;
    const int ncached = sl.n_cached, d = g.d;
    const int j0 = split * per_split, j1 = min(ncached, j0 + per_split);
    const size_t lrows = (size_t)ncached + 1;
    float m[MAXG], lsum[MAXG];
#pragma unroll
    for (int hh = 0; hh < MAXG; ++hh) { m[hh] = -INFINITY; lsum[hh] = 0.f; }

    int seg_first = 0;
    for (int si = 0; si < sl.n; ++si) {
        const Seg sg = sl.s[si];
        const int lo = max(j0, seg_first), hi = min(j1, seg_first + sg.len);
        if (lo < hi) {
            float qr[MAXG][EPL];
            const int rot = sl.qrot0[sg.qvar];
#pragma unroll
            for (int hh = 0; hh < MAXG; ++hh)
                if (hh < g.G) {
                    const T* qh = q + ((size_t)b * g.Hq + hk * g.G + hh) * d;
#pragma unroll
                    for (int x = 0; x < EPL; ++x) qr[hh][x] = q_rot_elem<T>(qh, rope, rot, d / 2, lane * EPL + x, g.scale);
                }
            const T* kseg = Kr + ((ptrdiff_t)bh * g.slots + sg.start - seg_first) * d;
            for (int r0 = lo + grp * U; r0 < hi; r0 += kRowGroups * U) {
                float kv[U][EPL];
#pragma unroll
                for (int u = 0; u < U; ++u)
                    VecLoad<T, EPL>::load(kseg + (size_t)min(r0 + u, hi - 1) * d + lane * EPL, kv[u]);
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int hh = 0; hh < MAXG; ++hh)
                        if (hh < g.G) {
                            float acc = 0.f;
#pragma unroll
                            for (int x = 0; x < EPL; ++x) acc += qr[hh][x] * kv[u][x];
#pragma unroll
                            for (int w = kLanesPerRow / 2; w > 0; w >>= 1) acc += __shfl_xor(acc, w, kLanesPerRow);
                            if (lane == 0 && r0 + u < hi) {
                                logits[logit_index(g, MAXG, lrows, b, hk, r0 + u, hh)] = acc;
                                const float mn = fmaxf(m[hh], acc);
                                lsum[hh] = lsum[hh] * __expf(m[hh] - mn) + __expf(acc - mn);
                                m[hh] = mn;
                            }
                        }
            }
        }
        seg_first += sg.len;
    }
    if (split == 0 && grp == 0) {
        // own key: <R(n) q, R(n) k> = <q, k>
        float kv[EPL];
        VecLoad<T, EPL>::load(k_new + ((size_t)b * g.Hkv + hk) * d + lane * EPL, kv);
#pragma unroll
        for (int hh = 0; hh < MAXG; ++hh)
            if (hh < g.G) {
                float qv[EPL];
                VecLoad<T, EPL>::load(q + ((size_t)b * g.Hq + hk * g.G + hh) * d + lane * EPL, qv);
                float acc = 0.f;
#pragma unroll
                for (int x = 0; x < EPL; ++x) acc += qv[x] * kv[x];
#pragma unroll
                for (int w = kLanesPerRow / 2; w > 0; w >>= 1) acc += __shfl_xor(acc, w, kLanesPerRow);
                acc *= g.scale;
                if (lane == 0) {
                    logits[logit_index(g, MAXG, lrows, b, hk, ncached, hh)] = acc;
                    const float mn = fmaxf(m[hh], acc);
                    lsum[hh] = lsum[hh] * __expf(m[hh] - mn) + __expf(acc - mn);
                    m[hh] = mn;
                }
            }
    }
    if (lane == 0) {
#pragma unroll
        for (int hh = 0; hh < MAXG; ++hh) { red_m[grp][hh] = m[hh]; red_l[grp][hh] = lsum[hh]; }
    }
    __syncthreads();
    if (threadIdx.x < g.G) {
        float mm = -INFINITY, ll = 0.f;
        for (int r = 0; r < kRowGroups; ++r) ml_merge(mm, ll, red_m[r][threadIdx.x], red_l[r][threadIdx.x]);
        float* p = part + (((size_t)b * g.Hq + hk * g.G + threadIdx.x) * n_splits + split) * 2;
        p[0] = mm;
        p[1] = ll;
    }
}

// ------------------------------------------------------------------ PV and EMA scores

// Lane N of every row of 16 lanes, to all lanes of that row (DPP row_newbcast).
template <int N> __device__ inline float row_bcast(float x)
{
    return __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(x), 0x150 + N, 0xf, 0xf, false));
}

template <int J, int NPL> __device__ inline float pair_value(const float (&pl)[NPL])
{
    return row_bcast<J % 16>(pl[J / 16]);
}

template <int HH, int U, int MAXG, int EPL, int NPL>
__device__ inline void pv_accumulate_head(const float (&pl)[NPL], const float (&vv)[U][EPL], float (&o)[MAXG][EPL],
                                          float (&red)[U], bool use_max, int G)
{
    if (HH < G) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float p;
            // the pair index must be a compile-time constant of the broadcast: spelled out per row
            switch (u) {
                case 0: p = pair_value<0 * MAXG + HH>(pl); break;
                case 1: p = pair_value<1 * MAXG + HH>(pl); break;
                case 2: p = pair_value<2 * MAXG + HH>(pl); break;
                case 3: p = pair_value<3 * MAXG + HH>(pl); break;
                case 4: p = pair_value<4 * MAXG + HH>(pl); break;
                case 5: p = pair_value<5 * MAXG + HH>(pl); break;
                case 6: p = pair_value<6 * MAXG + HH>(pl); break;
                default: p = pair_value<7 * MAXG + HH>(pl); break;
            }
#pragma unroll
            for (int x = 0; x < EPL; ++x) o[HH][x] += p * vv[u][x];
            red[u] = use_max ? fmaxf(red[u], p) : red[u] + p;
        }
    }
}

// With the exact log-sum-exp (all splits of decode_qk combined) p = exp(logit - lse) is final,
// so the partial outputs of the splits simply add up, and mu <- beta*mu + (1-beta)*reduce_heads(p)
// is applied in the same pass (Section 3.1).  Sixteen lanes share a row (each owns EPL elements
// of it), eight rows per lane group are in flight.  The probabilities of those rows (8 x MAXG
// values) are computed once, spread over the sixteen lanes, and handed round by lane broadcasts.
template <typename T, int EPL, int MAXG>
__global__ __launch_bounds__(kDecThreads) void decode_pv_kernel(
    Geom g, SegList sl, int per_split, const T* __restrict__ Vc, const float* __restrict__ logits,
    const float* __restrict__ part, int n_splits, float* __restrict__ opart, float* __restrict__ mu,
    float* __restrict__ lse_out)
{
    constexpr int U = 8;
    constexpr int NP = U * MAXG, NPL = (NP + kLanesPerRow - 1) / kLanesPerRow;
    __shared__ float lse_s[MAXG];
    __shared__ float osum[kDecThreads / 64][MAXG][kLanesPerRow * EPL];
    const int split = blockIdx.x, hk = blockIdx.y, b = blockIdx.z;
    const int bh = b * g.Hkv + hk;
    const int grp = threadIdx.x / kLanesPerRow, lane = threadIdx.x % kLanesPerRow;
    const int ncached = sl.n_cached, d = g.d;
    const size_t lrows = (size_t)ncached + 1;
    if (threadIdx.x < MAXG) {
        float v = 0.f;
        if (threadIdx.x < g.G) {
            const float* p = part + ((size_t)b * g.Hq + hk * g.G + threadIdx.x) * n_splits * 2;
            float mm = -INFINITY, ll = 0.f;
            for (int s = 0; s < n_splits; ++s) ml_merge(mm, ll, p[2 * s], p[2 * s + 1]);
            v = mm + __logf(ll);
            if (split == 0) lse_out[(size_t)b * g.Hq + hk * g.G + threadIdx.x] = v;
        }
        lse_s[threadIdx.x] = v;
    }
    __syncthreads();
    // this lane's pairs: pair j = lane + 16 t is (row j / MAXG of the eight, head j % MAXG)
    // (the pairs of eight consecutive rows are 8 x MAXG consecutive floats of the logits)
    int pu[NPL];
    float plse[NPL];
    bool pvalid[NPL];
    const float* lbase = logits + logit_index(g, MAXG, lrows, b, hk, 0, 0);
#pragma unroll
    for (int t = 0; t < NPL; ++t) {
        const int j = lane + kLanesPerRow * t, hh = j % MAXG;
        pu[t] = j / MAXG;
        pvalid[t] = j < NP && hh < g.G;
        plse[t] = lse_s[hh];
    }
    float o[MAXG][EPL];
#pragma unroll
    for (int hh = 0; hh < MAXG; ++hh)
#pragma unroll
        for (int x = 0; x < EPL; ++x) o[hh][x] = 0.f;
    const int j0 = split * per_split, j1 = min(ncached, j0 + per_split);
    const float beta = g.beta, omb = 1.f - g.beta;
    const bool use_max = g.head_reduce == CASCADE_REDUCE_MAX;

    int seg_first = 0;
    for (int si = 0; si < sl.n; ++si) {
        const Seg sg = sl.s[si];
        const int lo = max(j0, seg_first), hi = min(j1, seg_first + sg.len);
        if (lo < hi) {
            const T* vseg = Vc + ((ptrdiff_t)bh * g.slots + sg.start - seg_first) * d;
            float* museg = mu + ((ptrdiff_t)bh * g.slots + sg.start - seg_first);
            // (holding the next iteration's rows in a second register set costs more in occupancy than it gains)
            auto fetch = [&](int r0, float (&vv)[U][EPL], float (&lg)[NPL]) {
#pragma unroll
                for (int u = 0; u < U; ++u) VecLoad<T, EPL>::load(vseg + (size_t)min(r0 + u, hi - 1) * d + lane * EPL, vv[u]);
#pragma unroll
                for (int t = 0; t < NPL; ++t)
                    lg[t] = (pvalid[t] && r0 + pu[t] < hi) ? lbase[(size_t)r0 * MAXG + lane + kLanesPerRow * t] : -INFINITY;
            };
            auto consume = [&](int r0, const float (&vv)[U][EPL], const float (&lg)[NPL]) {
                float pl[NPL];
#pragma unroll
                for (int t = 0; t < NPL; ++t) pl[t] = __expf(lg[t] - plse[t]);   // exp(-inf) = 0 for pairs that do not exist
                float red[U];
#pragma unroll
                for (int u = 0; u < U; ++u) red[u] = 0.f;
                pv_accumulate_head<0, U, MAXG, EPL, NPL>(pl, vv, o, red, use_max, g.G);
                if (MAXG > 1) pv_accumulate_head<1 % MAXG, U, MAXG, EPL, NPL>(pl, vv, o, red, use_max, g.G);
                if (MAXG > 2) {
                    pv_accumulate_head<2 % MAXG, U, MAXG, EPL, NPL>(pl, vv, o, red, use_max, g.G);
                    pv_accumulate_head<3 % MAXG, U, MAXG, EPL, NPL>(pl, vv, o, red, use_max, g.G);
                }
                if (MAXG > 4) {
                    pv_accumulate_head<4 % MAXG, U, MAXG, EPL, NPL>(pl, vv, o, red, use_max, g.G);
                    pv_accumulate_head<5 % MAXG, U, MAXG, EPL, NPL>(pl, vv, o, red, use_max, g.G);
                    pv_accumulate_head<6 % MAXG, U, MAXG, EPL, NPL>(pl, vv, o, red, use_max, g.G);
                    pv_accumulate_head<7 % MAXG, U, MAXG, EPL, NPL>(pl, vv, o, red, use_max, g.G);
                }
                if (lane == 0) {
#pragma unroll
                    for (int u = 0; u < U; ++u)
                        if (r0 + u < hi) {
                            float* pm = museg + r0 + u;
                            *pm = beta * *pm + omb * (use_max ? red[u] : red[u] / (float)g.G);
                        }
                }
            };
            constexpr int STEP = kRowGroups * U;
            float vvA[U][EPL], lgA[NPL];
            int r0 = lo + grp * U;
            if (r0 < hi) fetch(r0, vvA, lgA);
            while (r0 < hi) {
                consume(r0, vvA, lgA);
                r0 += STEP;
                if (r0 < hi) fetch(r0, vvA, lgA);
            }
        }
        seg_first += sg.len;
    }
    // the four row groups of a wave first add up through lane shuffles
#pragma unroll
    for (int hh = 0; hh < MAXG; ++hh)
#pragma unroll
        for (int x = 0; x < EPL; ++x) {
            float t = o[hh][x];
            t += __shfl_xor(t, 16, 64);
            t += __shfl_xor(t, 32, 64);
            if (grp % 4 == 0) osum[grp / 4][hh][lane * EPL + x] = t;
        }
    __syncthreads();
    for (int idx = threadIdx.x; idx < g.G * d; idx += kDecThreads) {
        const int hh = idx / d, e = idx % d;
        float s = 0.f;
        for (int r = 0; r < kDecThreads / 64; ++r) s += osum[r][hh][e];
        opart[(((size_t)b * g.Hq + hk * g.G + hh) * n_splits + split) * d + e] = s;
    }
}

// out = sum of the split outputs + own value weighted by its probability; the new token's
// score starts at (1-beta) * reduce_heads(p_own).  The same workgroup then inserts the token
// (Alg. 2 for one token: small_update.h).
template <typename T>
__global__ void decode_finish_kernel(Geom g, UpdatePlan pl, UpdateBuffers upd, int n_cached, int n_splits, int qstride, int maxg,
                                     const float* __restrict__ opart, const float* __restrict__ logits,
                                     const float* __restrict__ lse, const T* __restrict__ v_new,
                                     T* __restrict__ out, float* __restrict__ mu_chunk)
{
    const int hk = blockIdx.x, b = blockIdx.y;
    const size_t lrows = (size_t)n_cached + 1;
    for (int idx = threadIdx.x; idx < g.G * g.d; idx += blockDim.x) {
        const int hh = idx / g.d, e = idx % g.d, h = hk * g.G + hh;
        const float p = __expf(logits[logit_index(g, maxg, lrows, b, hk, n_cached, hh)] - lse[(size_t)b * g.Hq + h]);
        float s = p * Elem<T>::load(v_new + ((size_t)b * g.Hkv + hk) * g.d + e);
        const float* op = opart + ((size_t)b * g.Hq + h) * n_splits * g.d + e;
        for (int sp = 0; sp < n_splits; ++sp) s += op[(size_t)sp * g.d];
        Elem<T>::store(out + ((size_t)b * g.Hq + h) * g.d + e, s);
    }
    if (threadIdx.x == 0) {
        // independent heads: the query heads of this KV head; homogeneous heads: all query heads (every
        // workgroup of the sequence computes the same value, group by group in the same order)
        const bool all = g.head_policy == CASCADE_HEADS_HOMOGENEOUS;
        float total = 0.f;
        for (int k2 = all ? 0 : hk; k2 < (all ? g.Hkv : hk + 1); ++k2) {
            float red = 0.f;
            for (int hh = 0; hh < g.G; ++hh) {
                const int h = k2 * g.G + hh;
                const float p = __expf(logits[logit_index(g, maxg, lrows, b, k2, n_cached, hh)] - lse[(size_t)b * g.Hq + h]);
                red = (g.head_reduce == CASCADE_REDUCE_MAX) ? fmaxf(red, p) : red + p;
            }
            if (g.head_reduce == CASCADE_REDUCE_MEAN) red /= (float)g.G;
            total = (g.head_reduce == CASCADE_REDUCE_MAX) ? fmaxf(total, red) : total + red;
        }
        if (all && g.head_reduce == CASCADE_REDUCE_MEAN) total /= (float)g.Hkv;
        mu_chunk[((size_t)b * g.Hkv + hk) * qstride] = (1.f - g.beta) * total;
    }
    __syncthreads();   // the token's score is written
    small_update<T>(g, pl, qstride, upd, b, hk);
}

// ------------------------------------------------------------------ PV and EMA scores, bf16: MFMA fed from LDS
//
// O^T = V^T P^T with v_mfma_f32_16x16x32_bf16: rows are 16 elements of the head dimension, columns
// the query heads of the group (padded to 16), the contraction runs over 32 cached rows.  Every
// wave streams its own 32-row tiles of V (and the tiles' logits and scores) through a private
// ring of LDS stages filled by asynchronous copies, so the bytes in flight do not depend on what
// the wave is computing and no workgroup barrier is needed inside the loop.  The A operand wants
// 8 rows of one column per lane: ds_read_b64_tr_b16 transposes on the way out of LDS.
//
// A staged V tile keeps rows of D elements; the 16-byte pieces of a row are permuted (piece ^
// swizzle(row)) so that the 8 rows one half of a wave reads in a transposing read fall into
// different banks.  The copy applies the permutation on the global side (a copy instruction
// writes LDS contiguously).
constexpr int kPvStages = 4;
constexpr int kPvRows = 32;           // cached rows per tile = contraction length of the MFMA
constexpr int kPvWaves = kDecThreads / 64;

template <int D> struct PvSwizzle;
template <> struct PvSwizzle<128> {
    __device__ static int of(int row) { return 2 * ((((row >> 3) & 1) << 2) | (row & 3)); }
};
template <> struct PvSwizzle<64> {
    __device__ static int of(int row) { return 2 * ((((row >> 3) & 1) << 1) | ((row >> 1) & 1)); }
};

typedef short pv_v4i16_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) pv_v4i16_t pv_lds_v4i16_t;

// ds_read_b64_tr_b16: the 16 lanes of a group address a 4-row x 16-column block of 16-bit
// elements (lane i: row i/4, columns 4*(i%4)..+3); lane i receives column i of the 4 rows.
__device__ inline uint2 pv_read_tr16(const unsigned char* p)
{
    const pv_v4i16_t r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((pv_lds_v4i16_t*)p);
    return __builtin_bit_cast(uint2, r);
}

// The tiles of one wave in order: inside every segment's part of [j0, j1) the tiles of 32 rows
// first, first + stride, ... counted from the start of that part.
struct WaveTiles {
    int si, seg_first, r0, hi, start, first, stride;
    bool valid;
    __device__ void seek(const SegList& sl, int j0, int j1)
    {
        while (si < sl.n) {
            const int len = sl.s[si].len;
            hi = min(j1, seg_first + len);
            r0 = max(j0, seg_first) + first;
            start = sl.s[si].start;
            if (r0 < hi) { valid = true; return; }
            seg_first += len;
            ++si;
        }
        valid = false;
    }
    __device__ void begin(const SegList& sl, int j0, int j1, int first_row, int row_stride)
    {
        si = 0; seg_first = 0; r0 = 0; hi = 0; start = 0;
        first = first_row; stride = row_stride;
        seek(sl, j0, j1);
    }
    __device__ void next(const SegList& sl, int j0, int j1)
    {
        r0 += stride;
        if (r0 >= hi) {
            seg_first += sl.s[si].len;
            ++si;
            seek(sl, j0, j1);
        }
    }
};

template <int D, int MAXG>
struct PvStage {
    static constexpr int kVBytes = kPvRows * D * 2;
    static constexpr int kLogitCopies = (kPvRows * MAXG * 4 + 255) / 256;
    static constexpr int kLgOff = kVBytes;                        // logits of the tile, [row][head]
    static constexpr int kMuOff = kLgOff + kLogitCopies * 256;    // scores of the tile's rows
    static constexpr int kBytes = kMuOff + 256;
    static constexpr int kVCopies = kVBytes / 1024;
    static constexpr int kCopies = kVCopies + kLogitCopies + 1;   // vector memory operations per tile
};

// Waits until the copies of the oldest tile in flight have landed: `ahead` later tiles (NC copies
// each) have been issued after it, and (in steady state) the stores of kPvStages - 1 tiles (NS
// each).  Counting fewer operations than are really outstanding only waits longer.
template <int NC, int NS> __device__ inline void ring_wait(int ahead, bool steady)
{
    static_assert(kPvStages == 4, "cases below");
    constexpr int ST = (kPvStages - 1) * NS;
    static_assert(3 * NC + ST < 64, "vmcnt range");
    if (steady) {
        if (ahead >= 3) wait_vm_fenced<3 * NC + ST>();
        else if (ahead == 2) wait_vm_fenced<2 * NC + ST>();
        else if (ahead == 1) wait_vm_fenced<NC + ST>();
        else wait_vm_fenced<0>();
    } else {
        if (ahead >= 3) wait_vm_fenced<3 * NC>();
        else if (ahead == 2) wait_vm_fenced<2 * NC>();
        else if (ahead == 1) wait_vm_fenced<NC>();
        else wait_vm_fenced<0>();
    }
}

template <int D, int MAXG>
__global__ __launch_bounds__(kDecThreads, 1) void decode_pv_mfma_kernel(
    Geom g, SegList sl, int per_split, const bf16_t* __restrict__ Vc, const float* __restrict__ logits,
    const float* __restrict__ part, int n_splits, float* __restrict__ opart, float* __restrict__ mu,
    float* __restrict__ lse_out)
{
    using St = PvStage<D, MAXG>;
    constexpr int DB = D / 16;                 // MFMA row blocks over the head dimension
    constexpr int PPR = D / 8;                 // 16-byte pieces per row
    constexpr int RPI = 64 / PPR;              // rows per copy instruction
    __shared__ __attribute__((aligned(1024))) unsigned char ring[kPvWaves][kPvStages][St::kBytes];
    __shared__ __attribute__((aligned(16))) bf16_t Pt[kPvWaves][MAXG][kPvRows];
    __shared__ float lse_s[MAXG];
    static_assert(sizeof(float) * kPvWaves * MAXG * D <= sizeof(ring), "the partial outputs reuse the ring");
    const int split = blockIdx.x, hk = blockIdx.y, b = blockIdx.z;
    const int bh = b * g.Hkv + hk;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), l = threadIdx.x & 63, n = l & 15, c = l >> 4;
    const int ncached = sl.n_cached;
    const size_t lrows = (size_t)ncached + 1;
    if (threadIdx.x < MAXG) {
        float v = 0.f;
        if (threadIdx.x < g.G) {
            const float* p = part + ((size_t)b * g.Hq + hk * g.G + threadIdx.x) * n_splits * 2;
            float mm = -INFINITY, ll = 0.f;
            for (int s = 0; s < n_splits; ++s) ml_merge(mm, ll, p[2 * s], p[2 * s + 1]);
            v = mm + __logf(ll);
            if (split == 0) lse_out[(size_t)b * g.Hq + hk * g.G + threadIdx.x] = v;
        }
        lse_s[threadIdx.x] = v;
    }
    __syncthreads();   // (also: every ordinary load of this kernel has returned before the first copy)

    const int j0 = split * per_split, j1 = min(ncached, j0 + per_split);
    const float* lbase = logits + logit_index(g, MAXG, lrows, b, hk, 0, 0);
    const bf16_t* vbh = Vc + (size_t)bh * g.slots * D;
    float* mubh = mu + (size_t)bh * g.slots;
    const uint32_t ring_lds = lds_address(&ring[wave][0][0]);
    unsigned char* ring_w = &ring[wave][0][0];

    // copy addressing of this lane: V copy x brings rows x*RPI + l/PPR, piece l%PPR of the LDS row
    // holds piece (l%PPR) ^ swizzle(row) of the global row
    auto issue = [&](const WaveTiles& t, int stage) {
        const int nvalid = min(kPvRows, t.hi - t.r0);          // rows past the end repeat the last one
        const uint32_t dst = ring_lds + (uint32_t)stage * St::kBytes;
        const int phys = t.start + (t.r0 - t.seg_first);       // first slot of the tile
        const bf16_t* vsrc = vbh + (size_t)phys * D;
#pragma unroll
        for (int x = 0; x < St::kVCopies; ++x) {
            const int row = x * RPI + l / PPR;
            const int piece = (l % PPR) ^ PvSwizzle<D>::of(row);
            async_copy_1k_stream(vsrc, (uint32_t)((min(row, nvalid - 1) * PPR + piece) * 16),
                                 __builtin_amdgcn_readfirstlane(dst + x * 1024u));
        }
        const float* lsrc = lbase + (size_t)t.r0 * MAXG;
#pragma unroll
        for (int x = 0; x < St::kLogitCopies; ++x)
            async_copy_256_stream(lsrc, (uint32_t)(min(x * 64 + l, nvalid * MAXG - 1) * 4),
                                  __builtin_amdgcn_readfirstlane(dst + St::kLgOff + x * 256u));
        async_copy_256(mubh + phys, (uint32_t)(min(l, nvalid - 1) * 4), __builtin_amdgcn_readfirstlane(dst + St::kMuOff));
    };

    // transposing reads of this lane: rows 8c + 4*hf + (n>>2), column block db, 8 bytes at element 4*(n&3)
    int tr_row[2], tr_sw[2];
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) {
        tr_row[hf] = 8 * c + 4 * hf + (n >> 2);
        tr_sw[hf] = PvSwizzle<D>::of(tr_row[hf]);
    }

    df32x4_t acc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) acc[db] = df32x4_t{0.f, 0.f, 0.f, 0.f};
    const float beta = g.beta, omb = 1.f - g.beta;
    const bool use_max = g.head_reduce == CASCADE_REDUCE_MAX;
    float lse_r[MAXG];
#pragma unroll
    for (int hh = 0; hh < MAXG; ++hh) lse_r[hh] = lse_s[hh];

    WaveTiles prod, cons;
    prod.begin(sl, j0, j1, wave * kPvRows, kPvWaves * kPvRows);
    cons = prod;
    int issued = 0, done = 0;
    for (; issued < kPvStages && prod.valid; ++issued) {
        issue(prod, issued);
        prod.next(sl, j0, j1);
    }
    while (cons.valid) {
        const int stage = done % kPvStages;
        ring_wait<St::kCopies, 1>(issued - done - 1, done >= kPvStages - 1);
        const unsigned char* sp = ring_w + stage * St::kBytes;
        const int nvalid = min(kPvRows, cons.hi - cons.r0);
        // probabilities of the tile: lane x < 32 takes row x and all heads
        if (l < kPvRows) {
            const float* lg = reinterpret_cast<const float*>(sp + St::kLgOff) + l * MAXG;
            float red = 0.f;
#pragma unroll
            for (int hh = 0; hh < MAXG; ++hh) {
                const float p = (hh < g.G && l < nvalid) ? __expf(lg[hh] - lse_r[hh]) : 0.f;
                red = use_max ? fmaxf(red, p) : red + p;
                Pt[wave][hh][l] = (bf16_t)(dec_pack_bf16(p, 0.f) & 0xFFFFu);
            }
            if (l < nvalid) {   // lane 0 always stores: the operation count of ring_wait relies on it
                const float old = reinterpret_cast<const float*>(sp + St::kMuOff)[l];
                const int phys = cons.start + (cons.r0 - cons.seg_first);
                counted_store_f32(mubh + phys, (uint32_t)(l * 4), beta * old + omb * (use_max ? red : red / (float)g.G));
            }
        }
        __builtin_amdgcn_wave_barrier();   // LDS accesses of one wave are executed in order
        DFrag pf;
        pf.u = du32x4_t{0u, 0u, 0u, 0u};
        if (n < MAXG) pf.u = *reinterpret_cast<const du32x4_t*>(&Pt[wave][n][8 * c]);
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            DFrag vf;
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
                const int piece = (2 * db + ((n & 3) >> 1)) ^ tr_sw[hf];
                const uint2 r = pv_read_tr16(sp + tr_row[hf] * (D * 2) + piece * 16 + (n & 1) * 8);
                vf.u[2 * hf] = r.x;
                vf.u[2 * hf + 1] = r.y;
            }
            acc[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf.v, pf.v, acc[db], 0, 0, 0);
        }
        wait_lds_reads();                  // the stage may be overwritten now
        ++done;
        cons.next(sl, j0, j1);
        if (prod.valid) {
            issue(prod, stage);
            ++issued;
            prod.next(sl, j0, j1);
        }
    }
    wait_vm_fenced<0>();
    __syncthreads();                       // every wave is done with its ring
    // this lane holds, for head n, elements 16*db + 4*c + j of the wave's partial output
    float* osum = reinterpret_cast<float*>(&ring[0][0][0]);   // [wave][MAXG][D]
    if (n < MAXG) {
#pragma unroll
        for (int db = 0; db < DB; ++db)
            *reinterpret_cast<df32x4_t*>(&osum[((size_t)wave * MAXG + n) * D + 16 * db + 4 * c]) = acc[db];
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < g.G * D; idx += kDecThreads) {
        const int hh = idx / D, e = idx % D;
        float s = 0.f;
        for (int w = 0; w < kPvWaves; ++w) s += osum[((size_t)w * MAXG + hh) * D + e];
        opart[(((size_t)b * g.Hq + hk * g.G + hh) * n_splits + split) * D + e] = s;
    }
}

// ------------------------------------------------------------------ QK, bf16: MFMA fed from LDS
//
// The same streaming structure for K: 32-row tiles through a private ring per wave, the A
// fragments (16 keys x 8 elements per lane) read with ds_read_b128.  The 16-byte pieces of a
// staged row are permuted so that the 16 rows of a fragment read fall into different banks.
// The rotated, scaled query fragments of every rotation the step uses are computed once per
// workgroup and kept in LDS, so the loop issues no ordinary load and no wait of the compiler's
// drains the ring.
template <int D> struct QkSwizzle;
template <> struct QkSwizzle<128> { __device__ static int of(int row) { return row & 15; } };
template <> struct QkSwizzle<64> { __device__ static int of(int row) { return (row >> 1) & 7; } };

template <int MAXG> struct QkLimits {
    static constexpr int kRotations = 96 / MAXG < kMaxQueryRotations ? 96 / MAXG : kMaxQueryRotations;   // query copies held in LDS
};

template <int D, int MAXG>
__global__ __launch_bounds__(kDecThreads, 1) void decode_qk_stream_kernel(
    Geom g, SegList sl, int per_split, const bf16_t* __restrict__ q, const bf16_t* __restrict__ k_new,
    const bf16_t* __restrict__ Kr, const float2* __restrict__ rope, float* __restrict__ logits,
    float* __restrict__ part, int n_splits)
{
    constexpr int KS = D / 32;                 // MFMA steps over the head dimension
    constexpr int PPR = D / 8;                 // 16-byte pieces per row
    constexpr int RPI = 64 / PPR;              // rows per copy instruction
    constexpr int kTileBytes = kPvRows * D * 2;
    constexpr int NC = kTileBytes / 1024;      // copies per tile
    constexpr int NS = (kPvRows * MAXG * 4 + 255) / 256;   // logit stores per tile
    constexpr int NR = QkLimits<MAXG>::kRotations;
    __shared__ __attribute__((aligned(1024))) unsigned char ring[kPvWaves][kPvStages][kTileBytes];
    __shared__ __attribute__((aligned(16))) du32x4_t qfr[NR][KS][4][MAXG];
    __shared__ __attribute__((aligned(16))) float stage[kPvWaves][kPvRows * MAXG];   // a tile's logits, [row][head]
    __shared__ float red_m[kPvWaves][16], red_l[kPvWaves][16];
    const int split = blockIdx.x, hk = blockIdx.y, b = blockIdx.z;
    const int bh = b * g.Hkv + hk;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), l = threadIdx.x & 63, n = l & 15, c = l >> 4;
    const int ncached = sl.n_cached;
    const size_t lrows = (size_t)ncached + 1;
    const bool head_ok = n < g.G;
    float* lbase = logits + logit_index(g, MAXG, lrows, b, hk, 0, 0);

    // B operands: every rotation of the group's queries, scaled, as bf16 (zero for padded heads)
    for (int idx = threadIdx.x; idx < sl.n_qvar * KS * 4 * MAXG; idx += kDecThreads) {
        const int hh = idx % MAXG, cc = (idx / MAXG) % 4, ks = (idx / (4 * MAXG)) % KS, v = idx / (4 * MAXG * KS);
        du32x4_t f = {0u, 0u, 0u, 0u};
        if (hh < g.G) {
            const bf16_t* qh = q + ((size_t)b * g.Hq + hk * g.G + hh) * D;
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const int e = ks * 32 + cc * 8 + 2 * x;
                f[x] = dec_pack_bf16(q_rot_elem<bf16_t>(qh, rope, sl.qrot0[v], D / 2, e, g.scale),
                                     q_rot_elem<bf16_t>(qh, rope, sl.qrot0[v], D / 2, e + 1, g.scale));
            }
        }
        qfr[v][ks][cc][hh] = f;
    }
    __syncthreads();   // (also: every ordinary load so far has returned before the first copy)

    const int j0 = split * per_split, j1 = min(ncached, j0 + per_split);
    const bf16_t* kbh = Kr + (size_t)bh * g.slots * D;
    const uint32_t ring_lds = lds_address(&ring[wave][0][0]);
    const unsigned char* ring_w = &ring[wave][0][0];

    auto issue = [&](const WaveTiles& t, int stg) {
        const int nvalid = min(kPvRows, t.hi - t.r0);          // rows past the end repeat the last one
        const uint32_t dst = ring_lds + (uint32_t)stg * kTileBytes;
        const bf16_t* ksrc = kbh + (size_t)(t.start + (t.r0 - t.seg_first)) * D;
#pragma unroll
        for (int x = 0; x < NC; ++x) {
            const int row = x * RPI + l / PPR;
            const int piece = (l % PPR) ^ QkSwizzle<D>::of(row);
            async_copy_1k_stream(ksrc, (uint32_t)((min(row, nvalid - 1) * PPR + piece) * 16),
                                 __builtin_amdgcn_readfirstlane(dst + x * 1024u));
        }
    };

    // fragment reads of this lane: key group gi, step ks: row 16*gi + n, piece 4*ks + c
    int a_off[2][KS];
#pragma unroll
    for (int gi = 0; gi < 2; ++gi)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int row = 16 * gi + n;
            a_off[gi][ks] = row * (D * 2) + (((4 * ks + c) ^ QkSwizzle<D>::of(row)) * 16);
        }

    float m = -INFINITY, lsum = 0.f;
    DFrag qf[KS];
    int q_si = -1;
    WaveTiles prod, cons;
    prod.begin(sl, j0, j1, wave * kPvRows, kPvWaves * kPvRows);
    cons = prod;
    int issued = 0, done = 0;
    for (; issued < kPvStages && prod.valid; ++issued) {
        issue(prod, issued);
        prod.next(sl, j0, j1);
    }
    while (cons.valid) {
        const int stg = done % kPvStages;
        if (cons.si != q_si) {             // uniform for the wave
            q_si = cons.si;
            const int v = sl.s[q_si].qvar;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                qf[ks].u = du32x4_t{0u, 0u, 0u, 0u};
                if (n < MAXG) qf[ks].u = qfr[v][ks][c][n];
            }
        }
        ring_wait<NC, NS>(issued - done - 1, done >= kPvStages - 1);
        const unsigned char* sp = ring_w + stg * kTileBytes;
        const int nvalid = min(kPvRows, cons.hi - cons.r0);
#pragma unroll
        for (int gi = 0; gi < 2; ++gi) {
            DFrag kf[KS];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) kf[ks].u = *reinterpret_cast<const du32x4_t*>(sp + a_off[gi][ks]);
            df32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[ks].v, qf[ks].v, acc, 0, 0, 0);
            // this lane: head n, tile rows 16*gi + 4*c + {0..3}
            const int rb = gi * 16 + 4 * c;
            if (n < MAXG) {
#pragma unroll
                for (int j = 0; j < 4; ++j) stage[wave][(rb + j) * MAXG + n] = acc[j];
            }
            if (head_ok) {
                // one rescaling per four logits: the running maximum rarely moves
                float mx = m;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (rb + j < nvalid) mx = fmaxf(mx, acc[j]);
                if (mx > m) {   // (also keeps -inf - -inf out of the arithmetic)
                    lsum *= __expf(m - mx);
                    m = mx;
                }
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (rb + j < nvalid) lsum += __expf(acc[j] - m);
            }
        }
        __builtin_amdgcn_wave_barrier();   // LDS accesses of one wave are executed in order
        // the tile's logits leave as contiguous runs; every store is issued by all lanes (lanes past
        // the end repeat the last logit), the operation count of ring_wait relies on it
        float* ltile = lbase + (size_t)cons.r0 * MAXG;
#pragma unroll
        for (int x = 0; x < NS; ++x) {
            const int idx = min(x * 64 + l, nvalid * MAXG - 1);
            counted_store_f32(ltile, (uint32_t)(idx * 4), stage[wave][idx]);
        }
        wait_lds_reads();                  // the stage may be overwritten now
        ++done;
        cons.next(sl, j0, j1);
        if (prod.valid) {
            issue(prod, stg);
            ++issued;
            prod.next(sl, j0, j1);
        }
    }
    wait_vm_fenced<0>();
    if (split == 0 && wave == 0) {
        // own key: <R(n) q, R(n) k> = <q, k>; lanes c = 0 of the valid heads take it
        if (head_ok && c == 0) {
            const bf16_t* qh = q + ((size_t)b * g.Hq + hk * g.G + n) * D;
            const bf16_t* kn = k_new + ((size_t)b * g.Hkv + hk) * D;
            float acc = 0.f;
            for (int e = 0; e < D; ++e) acc += bf16_to_f32(qh[e]) * bf16_to_f32(kn[e]);
            acc *= g.scale;
            lbase[(size_t)ncached * MAXG + n] = acc;
            const float mn = fmaxf(m, acc);
            lsum = lsum * __expf(m - mn) + __expf(acc - mn);
            m = mn;
        }
    }
    // combine the four lane groups of a head, then the waves
#pragma unroll
    for (int w = 16; w < 64; w <<= 1) {
        const float m2 = __shfl_xor(m, w, 64), l2 = __shfl_xor(lsum, w, 64);
        ml_merge(m, lsum, m2, l2);
    }
    if (c == 0) { red_m[wave][n] = m; red_l[wave][n] = lsum; }
    __syncthreads();
    if (threadIdx.x < g.G) {
        float mm = -INFINITY, ll = 0.f;
        for (int w = 0; w < kPvWaves; ++w) ml_merge(mm, ll, red_m[w][threadIdx.x], red_l[w][threadIdx.x]);
        float* p = part + (((size_t)b * g.Hq + hk * g.G + threadIdx.x) * n_splits + split) * 2;
        p[0] = mm;
        p[1] = ll;
    }
}

// ------------------------------------------------------------------ launchers

static int per_split_of(const DevBuffers& bf, int n)
{
    int per_split = (n + bf.dec_splits - 1) / bf.dec_splits;
    per_split = ((per_split + 63) / 64) * 64;
    return per_split == 0 ? 64 : per_split;
}

static int maxg_of(const Geom& g) { return g.G <= 1 ? 1 : (g.G <= 2 ? 2 : (g.G <= 4 ? 4 : 8)); }

int decode_logit_heads(const Geom& g) { return maxg_of(g); }

template <typename T, int EPL, int MAXG>
static void qk_valu(const Geom& g, const DevBuffers& bf, const SegList& sl, const void* q, const void* k, hipStream_t s)
{
    const dim3 grid(bf.dec_splits, g.Hkv, g.B), block(kDecThreads);
    hipLaunchKernelGGL((decode_qk_valu_kernel<T, EPL, MAXG>), grid, block, 0, s, g, sl, per_split_of(bf, sl.n_cached),
                       (const T*)q, (const T*)k, (const T*)bf.Kr, bf.rope, bf.logits, bf.part, bf.dec_splits);
}

template <typename T, int EPL, int MAXG>
static void pv_typed(const Geom& g, const DevBuffers& bf, const SegList& sl, hipStream_t s)
{
    const dim3 grid(bf.dec_splits, g.Hkv, g.B), block(kDecThreads);
    // the log-sum-exp of the step lives in the first B*Hq entries of the chunk scratch
    hipLaunchKernelGGL((decode_pv_kernel<T, EPL, MAXG>), grid, block, 0, s, g, sl, per_split_of(bf, sl.n_cached),
                       (const T*)bf.Vc, bf.logits, bf.part, bf.dec_splits, bf.opart, bf.mu, bf.lse);
}

#define CKV_G_SWITCH(fn, T, EPL, ...)                          \
    switch (maxg_of(g)) {                                      \
        case 1: fn<T, EPL, 1>(__VA_ARGS__); break;             \
        case 2: fn<T, EPL, 2>(__VA_ARGS__); break;             \
        case 4: fn<T, EPL, 4>(__VA_ARGS__); break;             \
        default: fn<T, EPL, 8>(__VA_ARGS__); break;            \
    }

#define CKV_DISPATCH(fn, ...)                                                                   \
    do {                                                                                        \
        const int epl = g.d / kLanesPerRow;                                                     \
        if (dtype == CASCADE_F32) {                                                             \
            if (epl == 8) { CKV_G_SWITCH(fn, float, 8, __VA_ARGS__) } else { CKV_G_SWITCH(fn, float, 4, __VA_ARGS__) } \
        } else {                                                                                \
            if (epl == 8) { CKV_G_SWITCH(fn, bf16_t, 8, __VA_ARGS__) } else { CKV_G_SWITCH(fn, bf16_t, 4, __VA_ARGS__) } \
        }                                                                                       \
    } while (0)

void launch_decode_qk(const Geom& g, int dtype, const DevBuffers& b, const SegList& sl, const void* q, const void* k,
                      hipStream_t s)
{
    if (dtype == CASCADE_BF16) {
        const dim3 grid(b.dec_splits, g.Hkv, g.B), block(kDecThreads);
        const int ps = per_split_of(b, sl.n_cached);
        const bool direct_only = b.opt_decode_qk_direct != 0;
        const int mg = maxg_of(g);
        const int rotations = 96 / mg < kMaxQueryRotations ? 96 / mg : kMaxQueryRotations;
        // the streaming kernel keeps every rotation of the queries in LDS
        const bool stream = !direct_only && sl.n_qvar <= rotations;
#define CKV_QK_MFMA(D, MG)                                                                                        \
    do {                                                                                                          \
        if (stream)                                                                                               \
            hipLaunchKernelGGL((decode_qk_stream_kernel<D, MG>), grid, block, 0, s, g, sl, ps, (const bf16_t*)q,    \
                               (const bf16_t*)k, (const bf16_t*)b.Kr, b.rope, b.logits, b.part, b.dec_splits);    \
        else                                                                                                      \
            hipLaunchKernelGGL((decode_qk_mfma_kernel<D, MG>), grid, block, 0, s, g, sl, ps, (const bf16_t*)q,      \
                               (const bf16_t*)k, (const bf16_t*)b.Kr, b.rope, b.logits, b.part, b.dec_splits);    \
    } while (0)
        if (g.d == 128) {
            if (mg == 1) CKV_QK_MFMA(128, 1); else if (mg == 2) CKV_QK_MFMA(128, 2); else if (mg == 4) CKV_QK_MFMA(128, 4); else CKV_QK_MFMA(128, 8);
        } else {
            if (mg == 1) CKV_QK_MFMA(64, 1); else if (mg == 2) CKV_QK_MFMA(64, 2); else if (mg == 4) CKV_QK_MFMA(64, 4); else CKV_QK_MFMA(64, 8);
        }
#undef CKV_QK_MFMA
        return;
    }
    CKV_DISPATCH(qk_valu, g, b, sl, q, k, s);
}

void launch_decode_pv(const Geom& g, int dtype, const DevBuffers& b, const SegList& sl, hipStream_t s)
{
    const bool valu_only = b.opt_decode_pv_valu != 0;
    if (dtype == CASCADE_BF16 && !valu_only) {
        const dim3 grid(b.dec_splits, g.Hkv, g.B), block(kDecThreads);
        const int ps = per_split_of(b, sl.n_cached);
#define CKV_PV_MFMA(D, MG)                                                                                 \
    hipLaunchKernelGGL((decode_pv_mfma_kernel<D, MG>), grid, block, 0, s, g, sl, ps, (const bf16_t*)b.Vc, b.logits, \
                       b.part, b.dec_splits, b.opart, b.mu, b.lse)
        const int mg = maxg_of(g);
        if (g.d == 128) {
            if (mg == 1) CKV_PV_MFMA(128, 1); else if (mg == 2) CKV_PV_MFMA(128, 2); else if (mg == 4) CKV_PV_MFMA(128, 4); else CKV_PV_MFMA(128, 8);
        } else {
            if (mg == 1) CKV_PV_MFMA(64, 1); else if (mg == 2) CKV_PV_MFMA(64, 2); else if (mg == 4) CKV_PV_MFMA(64, 4); else CKV_PV_MFMA(64, 8);
        }
#undef CKV_PV_MFMA
        return;
    }
    CKV_DISPATCH(pv_typed, g, b, sl, s);
}

void launch_decode_finish(const Geom& g, int dtype, const DevBuffers& b, const SegList& sl, const UpdatePlan& pl, int qstride,
                          const void* k, const void* v, void* out, hipStream_t s)
{
    const dim3 grid(g.Hkv, g.B), block(256);
    const UpdateBuffers upd = {b.rope, b.offers, b.winners, b.swaps, b.Kc, b.Kr, b.Vc, b.mu, b.ids, b.mu_chunk,
                               k, v, (long)g.Hkv * g.d, (long)g.Hkv * g.d};
    if (dtype == CASCADE_F32)
        hipLaunchKernelGGL(decode_finish_kernel<float>, grid, block, 0, s, g, pl, upd, sl.n_cached, b.dec_splits, qstride, maxg_of(g), b.opart,
                           b.logits, b.lse, (const float*)v, (float*)out, b.mu_chunk);
    else
        hipLaunchKernelGGL(decode_finish_kernel<bf16_t>, grid, block, 0, s, g, pl, upd, sl.n_cached, b.dec_splits, qstride, maxg_of(g), b.opart,
                           b.logits, b.lse, (const bf16_t*)v, (bf16_t*)out, b.mu_chunk);
}

bool decode_supported(const Geom& g) { return (g.d == 64 || g.d == 128) && g.G <= kMaxG; }

}  // namespace ckv
