// bf16 MFMA kernels of the strided prefill (Alg. 1, Fig. 4): chunk attention with online
// softmax (Eq. 2) and the exact EMA score sums (Section 3.1, coefficients of Alg. 3).
//
// MFMA used: v_mfma_f32_32x32x16_bf16, D[m][n] += sum_k A[m][k] B[k][n] with, for lane l,
//   A: row m = l%32, k = 8*(l/32) .. +7        B: column n = l%32, k = 8*(l/32) .. +7
//   D: column n = l%32, rows 8*(j/4) + 4*(l/32) + j%4 for accumulator register j = 0..15.
//
// Attention computes S^T = K Q^T (keys are rows, queries are columns), so one lane owns one
// query: row max and row sum are in-lane reductions plus one exchange with lane l^32, and the
// probabilities sit in the accumulators exactly as the B operand of O^T = V^T P^T needs them
// (the contraction index runs over keys in the accumulator's own order; the V^T tile in LDS is
// stored in that same order).
#include "launch.h"

namespace ckv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;

union Frag {
    bf16x8_t v;
    u32x4_t u;
};

__device__ inline uint32_t pack_bf16x2(float lo, float hi)
{
    // round to nearest even on both halves
    uint32_t a = __float_as_uint(lo), b = __float_as_uint(hi);
    a += 0x7FFFu + ((a >> 16) & 1u);
    b += 0x7FFFu + ((b >> 16) & 1u);
    return (a >> 16) | (b & 0xFFFF0000u);
}

constexpr int kAttnThreads = 256;
constexpr int kBM = 256;   // query rows per workgroup: 4 waves x 2 blocks of 32
constexpr int kBN = 64;    // keys per tile

template <int D>
__global__ __launch_bounds__(kAttnThreads) void attn_mfma_kernel(
    Geom g, SegList sl, int Q, const bf16_t* __restrict__ Qr, const bf16_t* __restrict__ Kr,
    const bf16_t* __restrict__ Vc, const bf16_t* __restrict__ Krc, const bf16_t* __restrict__ Vch,
    bf16_t* __restrict__ out, float* __restrict__ lse)
{
    constexpr int KS = D / 16;        // k-steps of S^T = K Q^T
    constexpr int DB = D / 32;        // 32-wide blocks of the head dimension in O^T
    constexpr int KSTR = D + 8;       // LDS row stride of the K tile (elements)
    constexpr int VSTR = kBN + 8;     // LDS row stride of the V^T tile (elements)
    __shared__ __attribute__((aligned(16))) bf16_t Ks[kBN * KSTR];
    __shared__ __attribute__((aligned(16))) bf16_t Vt[D * VSTR];

    const int BH = g.B * g.Hkv;
    const int bh = blockIdx.x % BH, tile = blockIdx.x / BH;   // consecutive workgroups: different KV heads
    const int b = bh / g.Hkv, hk = bh % g.Hkv;
    const int tid = threadIdx.x, wave = tid >> 6, l = tid & 63, l32 = l & 31, half = l >> 5;
    const int GQ = g.G * Q;

    // the two queries of this lane (one per 32-row block of the wave); rows are (head, token) pairs
    int qi[2], qh[2];
    bool qvalid[2];
    int wave_imax = 0, wave_imin = Q;
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const int r = tile * kBM + wave * 64 + qb * 32 + l32;
        qvalid[qb] = r < GQ;
        const int rc = min(r, GQ - 1);
        qh[qb] = hk * g.G + rc / Q;
        qi[qb] = rc % Q;
    }
    {
        const int r_lo = min(tile * kBM + wave * 64, GQ - 1), r_hi = min(tile * kBM + wave * 64 + 63, GQ - 1);
        if (r_lo / Q == r_hi / Q) { wave_imin = r_lo % Q; wave_imax = r_hi % Q; }
        else { wave_imin = 0; wave_imax = Q - 1; }
    }
    int wg_imax;
    {
        const int r_lo = min(tile * kBM, GQ - 1), r_hi = min(tile * kBM + kBM - 1, GQ - 1);
        wg_imax = (r_lo / Q == r_hi / Q) ? r_hi % Q : Q - 1;
    }

    f32x16_t o[DB][2];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int j = 0; j < 16; ++j) o[db][qb][j] = 0.f;
    float m[2] = {-INFINITY, -INFINITY}, lsum[2] = {0.f, 0.f};
    const float c2 = g.scale * 1.4426950408889634f;   // logits to the base-2 exponent

    Frag qf[2][KS];
    for (int si = 0; si < sl.n; ++si) {
        const Seg sg = sl.s[si];
        // this segment's rotated copy of the queries
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            const bf16_t* qrow = Qr + ((((size_t)sg.qvar * g.B + b) * g.Hq + qh[qb]) * Q + qi[qb]) * D + half * 8;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) qf[qb][ks].u = *reinterpret_cast<const u32x4_t*>(qrow + ks * 16);
        }
        const bf16_t* kbase = sg.chunk ? Krc + (size_t)bh * Q * D : Kr + ((size_t)bh * g.slots + sg.start) * D;
        const bf16_t* vbase = sg.chunk ? Vch + (size_t)bh * Q * D : Vc + ((size_t)bh * g.slots + sg.start) * D;
        const int len = sg.chunk ? min(sg.len, wg_imax + 1) : sg.len;

        for (int t0 = 0; t0 < len; t0 += kBN) {
            __syncthreads();   // the previous tile has been consumed
            // K tile: 64 rows of D elements, 16-byte pieces, row-major with padded stride
#pragma unroll
            for (int x = 0; x < (kBN * D / 8) / kAttnThreads; ++x) {
                const int p = tid + x * kAttnThreads;
                const int row = p / (D / 8), c8 = p % (D / 8);
                const int grow = min(t0 + row, sg.len - 1);
                const u32x4_t val = *reinterpret_cast<const u32x4_t*>(kbase + (size_t)grow * D + c8 * 8);
                *reinterpret_cast<u32x4_t*>(&Ks[row * KSTR + c8 * 8]) = val;
            }
            // V tile, transposed in registers: a thread takes 4 keys x 4 columns and writes, for
            // each column, its 4 keys as one 8-byte piece.  Inside every group of 16 keys the
            // 4-key pieces are stored in the order 0,2,1,3 (the accumulator order, see above).
#pragma unroll
            for (int x = 0; x < (kBN / 4) * (D / 4) / kAttnThreads; ++x) {
                const int p = tid + x * kAttnThreads;
                const int kq = p / (D / 4), dq = p % (D / 4);
                uint32_t lo[4], hi[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int grow = min(t0 + kq * 4 + r, sg.len - 1);
                    const uint2 u = *reinterpret_cast<const uint2*>(vbase + (size_t)grow * D + dq * 4);
                    lo[r] = u.x;
                    hi[r] = u.y;
                }
                const int sub = kq & 3, pos = ((sub & 1) << 1) | (sub >> 1);
                const int kcol = (kq >> 2) * 16 + pos * 4;
                uint2 w;
                w.x = (lo[0] & 0xFFFFu) | (lo[1] << 16);
                w.y = (lo[2] & 0xFFFFu) | (lo[3] << 16);
                *reinterpret_cast<uint2*>(&Vt[(dq * 4 + 0) * VSTR + kcol]) = w;
                w.x = (lo[0] >> 16) | (lo[1] & 0xFFFF0000u);
                w.y = (lo[2] >> 16) | (lo[3] & 0xFFFF0000u);
                *reinterpret_cast<uint2*>(&Vt[(dq * 4 + 1) * VSTR + kcol]) = w;
                w.x = (hi[0] & 0xFFFFu) | (hi[1] << 16);
                w.y = (hi[2] & 0xFFFFu) | (hi[3] << 16);
                *reinterpret_cast<uint2*>(&Vt[(dq * 4 + 2) * VSTR + kcol]) = w;
                w.x = (hi[0] >> 16) | (hi[1] & 0xFFFF0000u);
                w.y = (hi[2] >> 16) | (hi[3] & 0xFFFF0000u);
                *reinterpret_cast<uint2*>(&Vt[(dq * 4 + 3) * VSTR + kcol]) = w;
            }
            __syncthreads();
            if (sg.chunk && t0 > wave_imax) continue;   // every key of the tile lies after this wave's rows

            // S^T tile: [2 key blocks][2 query blocks]
            f32x16_t s[2][2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                    for (int j = 0; j < 16; ++j) s[kb][qb][j] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    Frag kf;
                    kf.u = *reinterpret_cast<const u32x4_t*>(&Ks[(kb * 32 + l32) * KSTR + ks * 16 + half * 8]);
#pragma unroll
                    for (int qb = 0; qb < 2; ++qb)
                        s[kb][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf.v, qf[qb][ks].v, s[kb][qb], 0, 0, 0);
                }
            }
            const bool need_mask = (t0 + kBN > sg.len) || (sg.chunk && t0 + kBN - 1 > wave_imin);
            Frag pf[2][2][2];   // [qb][kb][16-key half]
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                if (need_mask) {
                    const int lim = sg.chunk ? min(sg.len - 1, qi[qb]) : sg.len - 1;   // last visible key
#pragma unroll
                    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                        for (int j = 0; j < 16; ++j) {
                            const int kk = t0 + kb * 32 + (j >> 2) * 8 + half * 4 + (j & 3);
                            if (kk > lim) s[kb][qb][j] = -INFINITY;
                        }
                }
                float mt = -INFINITY;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int j = 0; j < 16; ++j) mt = fmaxf(mt, s[kb][qb][j]);
                mt = fmaxf(mt, __shfl_xor(mt, 32, 64));
                const float mn = fmaxf(m[qb], mt);
                const float alpha = exp2f((m[qb] - mn) * c2);
                const float mc = mn * c2;
                float ps = 0.f;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    float p[16];
#pragma unroll
                    for (int j = 0; j < 16; ++j) {
                        p[j] = exp2f(s[kb][qb][j] * c2 - mc);
                        ps += p[j];
                    }
#pragma unroll
                    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
                        for (int x = 0; x < 4; ++x)
                            pf[qb][kb][hf].u[x] = pack_bf16x2(p[hf * 8 + 2 * x], p[hf * 8 + 2 * x + 1]);
                }
                lsum[qb] = lsum[qb] * alpha + ps;
                m[qb] = mn;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int j = 0; j < 16; ++j) o[db][qb][j] *= alpha;
            }
            // O^T += V^T P^T
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int hf = 0; hf < 2; ++hf)
#pragma unroll
                    for (int db = 0; db < DB; ++db) {
                        Frag vf;
                        vf.u = *reinterpret_cast<const u32x4_t*>(&Vt[(db * 32 + l32) * VSTR + (kb * 2 + hf) * 16 + half * 8]);
#pragma unroll
                        for (int qb = 0; qb < 2; ++qb)
                            o[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf.v, pf[qb][kb][hf].v, o[db][qb], 0, 0, 0);
                    }
        }
    }

    // normalise and store: this lane owns query qb, columns 32*db + 8*(j/4) + 4*half + j%4
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const float lt = lsum[qb] + __shfl_xor(lsum[qb], 32, 64);
        if (!qvalid[qb]) continue;
        const float inv = 1.f / lt;
        bf16_t* orow = out + (((size_t)b * Q + qi[qb]) * g.Hq + qh[qb]) * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int jq = 0; jq < 4; ++jq) {
                uint2 w;
                w.x = pack_bf16x2(o[db][qb][jq * 4 + 0] * inv, o[db][qb][jq * 4 + 1] * inv);
                w.y = pack_bf16x2(o[db][qb][jq * 4 + 2] * inv, o[db][qb][jq * 4 + 3] * inv);
                *reinterpret_cast<uint2*>(orow + db * 32 + jq * 8 + half * 4) = w;
            }
        if (half == 0) lse[((size_t)b * g.Hq + qh[qb]) * Q + qi[qb]] = m[qb] * g.scale + logf(lt);
    }
}

void launch_attn_mfma(const Geom& g, const DevBuffers& b, const SegList& sl, int Q, int, void* out, hipStream_t s)
{
    const int tiles = (g.G * Q + kBM - 1) / kBM;
    const dim3 grid(tiles * g.B * g.Hkv), block(kAttnThreads);
    if (g.d == 128)
        hipLaunchKernelGGL(attn_mfma_kernel<128>, grid, block, 0, s, g, sl, Q, (const bf16_t*)b.Qr, (const bf16_t*)b.Kr,
                           (const bf16_t*)b.Vc, (const bf16_t*)b.Krc, (const bf16_t*)b.Vch, (bf16_t*)out, b.lse);
    else
        hipLaunchKernelGGL(attn_mfma_kernel<64>, grid, block, 0, s, g, sl, Q, (const bf16_t*)b.Qr, (const bf16_t*)b.Kr,
                           (const bf16_t*)b.Vc, (const bf16_t*)b.Krc, (const bf16_t*)b.Vch, (bf16_t*)out, b.lse);
}

// ------------------------------------------------------------------ exact score sums

// Key-stationary: a wave holds 32 keys as the B operand and runs the last `tail` query rows of
// every head of the group past them (S = Q K^T, one lane owns one key column).  With the stored
// log-sum-exp the probabilities are exact; each is weighted by its row's EMA coefficient and the
// column sums are an in-lane sum plus one exchange with lane l^32.
constexpr int kScoreKeys = 128;   // keys per workgroup (4 waves x 32)

template <int D>
__global__ __launch_bounds__(256) void score_mfma_kernel(
    Geom g, SegList sl, int Q, int qstride, int tail, float decay, const bf16_t* __restrict__ Qr,
    const bf16_t* __restrict__ Kr, const bf16_t* __restrict__ Krc, const float* __restrict__ lse,
    const float* __restrict__ wrow, float* __restrict__ mu, float* __restrict__ mu_chunk)
{
    constexpr int KS = D / 16;
    const int BH = g.B * g.Hkv;
    const int bh = blockIdx.x % BH;
    int tile = blockIdx.x / BH;
    const int b = bh / g.Hkv, hk = bh % g.Hkv;
    int si = 0;
    while (si < sl.n) {
        const int nt = (sl.s[si].len + kScoreKeys - 1) / kScoreKeys;
        if (tile < nt) break;
        tile -= nt;
        ++si;
    }
    if (si >= sl.n) return;
    const Seg sg = sl.s[si];
    const int tid = threadIdx.x, wave = tid >> 6, l = tid & 63, l32 = l & 31, half = l >> 5;
    const int kk = tile * kScoreKeys + wave * 32 + l32;      // key index inside the segment
    if (tile * kScoreKeys + wave * 32 >= sg.len) return;      // whole wave past the end
    const bool kvalid = kk < sg.len;
    const int kc = min(kk, sg.len - 1);
    const bf16_t* krow = sg.chunk ? Krc + ((size_t)bh * Q + kc) * D : Kr + ((size_t)bh * g.slots + sg.start + kc) * D;
    Frag kf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) kf[ks].u = *reinterpret_cast<const u32x4_t*>(krow + ks * 16 + half * 8);

    const int i_first = Q - tail;                       // first row that contributes
    const int n_rb = (tail + 31) / 32;
    const int i_start = Q - n_rb * 32;                  // may be negative: those rows are skipped
    // chunk keys are only seen by rows at or after them: skip row blocks entirely before the wave's keys
    const int wave_k0 = tile * kScoreKeys + wave * 32;
    float red = 0.f;
    for (int hh = 0; hh < g.G; ++hh) {
        const int h = hk * g.G + hh;
        const bf16_t* qbase = Qr + (((size_t)sg.qvar * g.B + b) * g.Hq + h) * (size_t)Q * D;
        const float* lrow = lse + ((size_t)b * g.Hq + h) * Q;
        float colsum = 0.f;
        for (int rb = 0; rb < n_rb; ++rb) {
            const int i0 = i_start + rb * 32;
            if (sg.chunk && i0 + 31 < wave_k0) continue;
            const int ia = min(max(i0 + l32, 0), Q - 1);
            const bf16_t* qrow = qbase + (size_t)ia * D + half * 8;
            f32x16_t s;
#pragma unroll
            for (int j = 0; j < 16; ++j) s[j] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                Frag qf;
                qf.u = *reinterpret_cast<const u32x4_t*>(qrow + ks * 16);
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf.v, kf[ks].v, s, 0, 0, 0);
            }
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const int i = i0 + (j >> 2) * 8 + half * 4 + (j & 3);
                const bool ok = i >= i_first && i >= 0 && (!sg.chunk || kk <= i);
                const int ic = min(max(i, 0), Q - 1);
                const float p = wrow[Q - 1 - ic] * __expf(s[j] * g.scale - lrow[ic]);
                colsum += ok ? p : 0.f;
            }
        }
        colsum += __shfl_xor(colsum, 32, 64);
        if (g.head_reduce == CASCADE_REDUCE_MAX) red = hh == 0 ? colsum : fmaxf(red, colsum);
        else red += colsum;
    }
    if (g.head_reduce == CASCADE_REDUCE_MEAN) red /= (float)g.G;
    if (half == 0 && kvalid) {
        if (sg.chunk) mu_chunk[(size_t)bh * qstride + kk] = red;
        else {
            float* p = mu + (size_t)bh * g.slots + sg.start + kk;
            *p = decay * *p + red;
        }
    }
}

void launch_score_mfma(const Geom& g, const DevBuffers& b, const SegList& sl, int Q, int max_chunk,
                       int tail_rows, float decay, hipStream_t s)
{
    int tiles = 0;
    for (int i = 0; i < sl.n; ++i) tiles += (sl.s[i].len + kScoreKeys - 1) / kScoreKeys;
    const dim3 grid(tiles * g.B * g.Hkv), block(256);
    if (g.d == 128)
        hipLaunchKernelGGL(score_mfma_kernel<128>, grid, block, 0, s, g, sl, Q, max_chunk, tail_rows, decay,
                           (const bf16_t*)b.Qr, (const bf16_t*)b.Kr, (const bf16_t*)b.Krc, b.lse, b.wrow, b.mu, b.mu_chunk);
    else
        hipLaunchKernelGGL(score_mfma_kernel<64>, grid, block, 0, s, g, sl, Q, max_chunk, tail_rows, decay,
                           (const bf16_t*)b.Qr, (const bf16_t*)b.Kr, (const bf16_t*)b.Krc, b.lse, b.wrow, b.mu, b.mu_chunk);
}

}  // namespace ckv
