// bf16 MFMA kernel of the exact EMA score sums of a chunk (Section 3.1, coefficients of Alg. 3).
//
// MFMA used: v_mfma_f32_32x32x16_bf16, D[m][n] += sum_k A[m][k] B[k][n] with, for lane l,
//   A: row m = l%32, k = 8*(l/32) .. +7        B: column n = l%32, k = 8*(l/32) .. +7
//   D: column n = l%32, rows 8*(j/4) + 4*(l/32) + j%4 for accumulator register j = 0..15.
#include <stdio.h>
#include <stdlib.h>

#include "mfma_util.h"

namespace ckv {

// ------------------------------------------------------------------ exact score sums

// Key-stationary: a wave keeps 64 keys (two 32-key blocks) in registers as the B operand and
// runs the last `tail` query rows of every head of the group past them (S = Q K^T, one lane owns
// one key column per block).  The rows of one head are staged through LDS in groups of 256 and
// shared by the four waves.  With the stored log-sum-exp the probabilities are exact:
// p = 2^(s - t[row]) (the queries carry the softmax scale and log2 e) with
// t = lse*log2(e) - log2(weight of the row), so a row that does not
// contribute has t = +inf.  Column sums are an in-lane sum plus one exchange with lane l^32;
// no atomics, so results are identical from run to run.
constexpr int kScoreThreads = 256;
constexpr int kScoreKeys = 256;    // keys per workgroup (4 waves x 2 blocks of 32)
constexpr int kScoreRows = 256;    // query rows staged per pass

template <int D>
__global__ __launch_bounds__(kScoreThreads, 2) void score_mfma_kernel(
    Geom g, SegList sl, int Q, int qstride, int tail, float decay, const bf16_t* __restrict__ Qr,
    const bf16_t* __restrict__ Kr, const bf16_t* __restrict__ Krc, const float* __restrict__ lse,
    const float* __restrict__ wrow, float* __restrict__ mu, float* __restrict__ mu_chunk)
{
    constexpr int KS = D / 16;
    constexpr int QSTR = D + 8;
    __shared__ __attribute__((aligned(16))) bf16_t Qs[kScoreRows * QSTR];
    __shared__ __attribute__((aligned(16))) float ts[kScoreRows];
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
    if (si >= sl.n) return;       // uniform for the workgroup
    const Seg sg = sl.s[si];
    const int tid = threadIdx.x, wave = tid >> 6, l = tid & 63, l32 = l & 31, half = l >> 5;
    const int wave_k0 = tile * kScoreKeys + wave * 64;       // first key of this wave inside the segment

    // this wave's keys as B operands (rows past the end of the segment repeat its last row)
    Frag kf[2][KS];
    int kk[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
        kk[kb] = wave_k0 + kb * 32 + l32;
        const int kc = min(kk[kb], sg.len - 1);
        const bf16_t* krow = sg.chunk ? Krc + ((size_t)bh * Q + kc) * D : Kr + ((size_t)bh * g.slots + sg.start + kc) * D;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) kf[kb][ks].u = *reinterpret_cast<const u32x4_t*>(krow + ks * 16 + half * 8);
    }

    const int i_first = Q - tail;                             // first row that contributes
    const int n_pass = (tail + kScoreRows - 1) / kScoreRows;
    float red[2] = {0.f, 0.f};
    for (int hh = 0; hh < g.G; ++hh) {
        const int h = hk * g.G + hh;
        const bf16_t* qbase = Qr + (((size_t)sg.qvar * g.B + b) * g.Hq + h) * (size_t)Q * D;
        const float* lrow = lse + ((size_t)b * g.Hq + h) * Q;
        float colsum[2] = {0.f, 0.f};
        for (int ps = 0; ps < n_pass; ++ps) {
            const int i_base = i_first + ps * kScoreRows;               // passes start at the first contributing row
            const int rows = min(kScoreRows, Q - i_base);               // the last pass may be short
            __syncthreads();                                            // the previous pass has been consumed
            // stage the rows of this pass (16-byte pieces) and their exponent offsets.  A full pass
            // issues all its loads before the first store; a short one (the last) stages only whole
            // blocks of 32 rows, rows past its end repeating the last row.
            if (rows == kScoreRows) {
                u32x4_t buf[kScoreRows * D / 8 / kScoreThreads];
#pragma unroll
                for (int x = 0; x < kScoreRows * D / 8 / kScoreThreads; ++x) {
                    const int p = tid + x * kScoreThreads;
                    buf[x] = *reinterpret_cast<const u32x4_t*>(qbase + (size_t)(i_base + p / (D / 8)) * D + (p % (D / 8)) * 8);
                }
#pragma unroll
                for (int x = 0; x < kScoreRows * D / 8 / kScoreThreads; ++x) {
                    const int p = tid + x * kScoreThreads;
                    *reinterpret_cast<u32x4_t*>(&Qs[(p / (D / 8)) * QSTR + (p % (D / 8)) * 8]) = buf[x];
                }
            } else {
                for (int p = tid; p < ((rows + 31) & ~31) * (D / 8); p += kScoreThreads) {
                    const int r = p / (D / 8), c8 = p % (D / 8);
                    *reinterpret_cast<u32x4_t*>(&Qs[r * QSTR + c8 * 8]) =
                        *reinterpret_cast<const u32x4_t*>(qbase + (size_t)min(i_base + r, Q - 1) * D + c8 * 8);
                }
            }
            {
                const int i = i_base + tid;                              // kScoreRows == kScoreThreads
                float t = INFINITY;
                if (i < Q) t = lrow[i] * 1.4426950408889634f - __log2f(wrow[Q - 1 - i]);
                ts[tid] = t;
            }
            __syncthreads();
            for (int rb = 0; rb < (rows + 31) / 32; ++rb) {
                const int i0 = i_base + rb * 32;
                if (sg.chunk && i0 + 31 < wave_k0) continue;             // chunk keys are seen by later rows only
                f32x16_t s[2];
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int j = 0; j < 16; ++j) s[kb][j] = 0.f;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    Frag qf;
                    qf.u = *reinterpret_cast<const u32x4_t*>(&Qs[(rb * 32 + l32) * QSTR + ks * 16 + half * 8]);
#pragma unroll
                    for (int kb = 0; kb < 2; ++kb)
                        s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf.v, kf[kb][ks].v, s[kb], 0, 0, 0);
                }
#pragma unroll
                for (int jq = 0; jq < 4; ++jq) {
                    const float4 t4 = *reinterpret_cast<const float4*>(&ts[rb * 32 + jq * 8 + half * 4]);
                    const float tt[4] = {t4.x, t4.y, t4.z, t4.w};
#pragma unroll
                    for (int x = 0; x < 4; ++x) {
                        const int i = i0 + jq * 8 + half * 4 + x;
#pragma unroll
                        for (int kb = 0; kb < 2; ++kb) {
                            const float p = __builtin_amdgcn_exp2f(s[kb][jq * 4 + x] - tt[x]);
                            colsum[kb] += (!sg.chunk || kk[kb] <= i) ? p : 0.f;
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            const float cs = colsum[kb] + __shfl_xor(colsum[kb], 32, 64);
            if (g.head_reduce == CASCADE_REDUCE_MAX) red[kb] = hh == 0 ? cs : fmaxf(red[kb], cs);
            else red[kb] += cs;
        }
    }
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
        float r = red[kb];
        if (g.head_reduce == CASCADE_REDUCE_MEAN) r /= (float)g.G;
        if (half == 0 && kk[kb] < sg.len) {
            if (sg.chunk) mu_chunk[(size_t)bh * qstride + kk[kb]] = r;
            else {
                float* p = mu + (size_t)bh * g.slots + sg.start + kk[kb];
                *p = decay * *p + r;
            }
        }
    }
}

void launch_score_mfma(const Geom& g, const DevBuffers& b, const SegList& sl, int Q, int max_chunk,
                       int tail_rows, float decay, hipStream_t s)
{
    int tiles = 0;
    for (int i = 0; i < sl.n; ++i) tiles += (sl.s[i].len + kScoreKeys - 1) / kScoreKeys;
    const dim3 grid(tiles * g.B * g.Hkv), block(kScoreThreads);
    if (g.d == 128)
        hipLaunchKernelGGL(score_mfma_kernel<128>, grid, block, 0, s, g, sl, Q, max_chunk, tail_rows, decay,
                           (const bf16_t*)b.Qr, (const bf16_t*)b.Kr, (const bf16_t*)b.Krc, b.lse, b.wrow, b.mu, b.mu_chunk);
    else
        hipLaunchKernelGGL(score_mfma_kernel<64>, grid, block, 0, s, g, sl, Q, max_chunk, tail_rows, decay,
                           (const bf16_t*)b.Qr, (const bf16_t*)b.Kr, (const bf16_t*)b.Krc, b.lse, b.wrow, b.mu, b.mu_chunk);
}

}  // namespace ckv
