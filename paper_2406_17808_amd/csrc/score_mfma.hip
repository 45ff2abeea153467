// bf16 MFMA kernel of the exact EMA score sums of a chunk (Section 3.1, coefficients of Alg. 3).
//
// MFMA used: v_mfma_f32_32x32x16_bf16, D[m][n] += sum_k A[m][k] B[k][n] with, for lane l,
//   A: row m = l%32, k = 8*(l/32) .. +7        B: column n = l%32, k = 8*(l/32) .. +7
//   D: column n = l%32, rows 8*(j/4) + 4*(l/32) + j%4 for accumulator register j = 0..15.
#include <stdio.h>
#include <stdlib.h>

#include "async_copy.h"
#include "mfma_util.h"

namespace ckv {

// ------------------------------------------------------------------ exact score sums

// Key-stationary: a wave keeps 64 keys (two 32-key blocks) in registers as the B operand and
// runs the last `tail` query rows of every head of the group past them (S = Q K^T, one lane owns
// one key column per block).  With the stored log-sum-exp the probabilities are exact:
// p = 2^(s - t[row]) (the queries carry the softmax scale and log2 e) with
// t = lse*log2(e) - log2(weight of the row).  Column sums are an in-lane sum plus one exchange
// with lane l^32; no atomics, so results are identical from run to run.
//
// The query rows reach LDS by asynchronous copies through a ring of three 64-row stages shared
// by the workgroup (one barrier per stage, the copies of the next two stages in flight while a
// stage is used; three workgroups per CU), running on across the heads of the group, so no wave
// waits for a staging round trip.  The exponent offsets come from a small table
// negt[head][row] = -t (-inf for rows that do not contribute, and for the padding behind the
// chunk), written by the attention kernel when it finishes a row; the accumulators start from
// it: a probability is then one v_exp_f32 of an accumulator.
constexpr int kScoreThreads = 256;
constexpr int kScoreKeysPerBlock = 128;   // keys per workgroup and key block of its waves (4 waves x 32)
constexpr int kStStages = 3;
constexpr int kStRows = kScorePadRows;

template <int D> struct ScoreSwz {   // permutation of the 16-byte pieces of a staged row
    __device__ static int of(int row) { return D == 128 ? (row & 15) : ((row >> 1) & 7); }
};

// NKB: 32-key blocks per wave.  Two halve the LDS reads per MFMA; one gives twice as many
// workgroups, for launches that would otherwise leave compute units without work.
template <int D, int NKB>
__global__ __launch_bounds__(kScoreThreads, 3) void score_stream_kernel(
    Geom g, SegList sl, int Q, int qstride, int tail, int qpad, float decay, const bf16_t* __restrict__ Qr,
    const bf16_t* __restrict__ Kr, const bf16_t* __restrict__ Krc, const float* __restrict__ negt,
    float* __restrict__ mu, float* __restrict__ mu_chunk)
{
    constexpr int KS = D / 16;
    constexpr int kScoreKeys = kScoreKeysPerBlock * NKB, kWaveKeys = 32 * NKB;
    constexpr int PPR = D / 8;                       // 16-byte pieces per row
    constexpr int RPI = 64 / PPR;                    // rows per copy instruction
    constexpr int kStageBytes = kStRows * D * 2;
    constexpr int NCW = kStageBytes / 1024 / 4;      // row copies per wave and stage
    constexpr int NOPS = NCW + 1;                    // vector memory operations per wave and stage
    __shared__ __attribute__((aligned(1024))) unsigned char ring[kStStages][kStageBytes];
    __shared__ __attribute__((aligned(256))) float tneg[kStStages][4][kStRows];   // every wave keeps its own copy
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
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), l = tid & 63, l32 = l & 31, half = l >> 5;
    const int wave_k0 = tile * kScoreKeys + wave * kWaveKeys;   // first key of this wave inside the segment

    // this wave's keys as B operands (rows past the end of the segment repeat its last row)
    Frag kf[NKB][KS];
    int kk[NKB];
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) {
        kk[kb] = wave_k0 + kb * 32 + l32;
        const int kc = min(kk[kb], sg.len - 1);
        const bf16_t* krow = sg.chunk ? Krc + ((size_t)bh * Q + kc) * D : Kr + ((size_t)bh * g.slots + sg.start + kc) * D;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) kf[kb][ks].u = *reinterpret_cast<const u32x4_t*>(krow + ks * 16 + half * 8);
    }
    // fragment reads of this lane: row block rb, step ks: row 32*rb + l32, piece 2*ks + half
    int a_off[2][KS];
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int row = 32 * rb + l32;
            a_off[rb][ks] = row * (D * 2) + (((2 * ks + half) ^ ScoreSwz<D>::of(row)) * 16);
        }

    const int i_first = Q - tail;                              // first row that contributes
    const int spp = (tail + kStRows - 1) / kStRows;            // stages per head
    const int T = g.G * spp;
    const uint32_t ring_lds = lds_address(&ring[0][0]), tneg_lds = lds_address(&tneg[0][0][0]);
    // the keys are in registers before the first copy is issued (a wait for them inside the loop
    // would also wait for every copy in flight)
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(kf[kb][ks].u));
    // what a lane copies of a stage: row x*RPI + l/PPR of the stage, one 16-byte piece (lane constants)
    uint32_t copy_off[NCW];
#pragma unroll
    for (int y = 0; y < NCW; ++y) {
        const int row = (wave * NCW + y) * RPI + l / PPR;
        copy_off[y] = (uint32_t)((row * PPR + ((l % PPR) ^ ScoreSwz<D>::of(row))) * 16);
    }
    int iss_hh = 0, iss_sp = 0;                                 // stage s, the next to issue, is stage iss_sp of head iss_hh
    auto issue = [&](int s) {
        const int i_base = i_first + iss_sp * kStRows;
        const int h = hk * g.G + iss_hh, slot = s % kStStages;
        if (++iss_sp == spp) { iss_sp = 0; ++iss_hh; }
        const bf16_t* qbase = Qr + (((size_t)sg.qvar * g.B + b) * g.Hq + h) * (size_t)Q * D;
        if (i_base + kStRows <= Q) {          // all rows of the stage exist: the lane offsets are constants
#pragma unroll
            for (int y = 0; y < NCW; ++y)
                async_copy_1k(qbase + (size_t)i_base * D, copy_off[y],
                              __builtin_amdgcn_readfirstlane(ring_lds + slot * kStageBytes + (wave * NCW + y) * 1024));
        } else {
#pragma unroll
            for (int y = 0; y < NCW; ++y) {
                const int x = wave * NCW + y;
                const int row = x * RPI + l / PPR;
                const int piece = (l % PPR) ^ ScoreSwz<D>::of(row);
                async_copy_1k(qbase, (uint32_t)((min(i_base + row, Q - 1) * PPR + piece) * 16),
                              __builtin_amdgcn_readfirstlane(ring_lds + slot * kStageBytes + x * 1024));
            }
        }
        async_copy_256(negt + ((size_t)b * g.Hq + h) * qpad + i_base, (uint32_t)(l * 4),
                       __builtin_amdgcn_readfirstlane(tneg_lds + (uint32_t)((slot * 4 + wave) * kStRows * 4)));
    };

    int issued = 0;
    for (; issued < kStStages - 1 && issued < T; ++issued) issue(issued);
    float red[NKB] = {}, colsum[NKB] = {};
    int hh = 0, sp = 0;                                         // stage s = stage sp of head hh
    for (int s = 0; s < T; ++s) {
        const int ahead = issued - s - 1;                       // stages issued after stage s
        static_assert(kStStages == 3 || kStStages == 4, "cases below");
        if (kStStages == 4 && ahead >= 2) wait_vm<2 * NOPS>();
        else if (ahead >= 1) wait_vm<NOPS>();
        else wait_vm<0>();
        wg_barrier();    // stage s is complete for every wave, and every wave has left stage s - 1
        if (issued < T) { issue(issued); ++issued; }            // into the slot of stage s - 1
        const int slot = s % kStStages;
        const int i_base = i_first + sp * kStRows;
        const int rows = min(kStRows, Q - i_base);
        const unsigned char* qs = &ring[slot][0];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
            const int i0 = i_base + rb * 32;
            if (rb * 32 >= rows) continue;
            if (sg.chunk && i0 + 31 < wave_k0) continue;        // chunk keys are seen by later rows only
            f32x16_t acc[NKB];
#pragma unroll
            for (int jq = 0; jq < 4; ++jq) {
                const float4 t4 = *reinterpret_cast<const float4*>(&tneg[slot][wave][rb * 32 + jq * 8 + half * 4]);
                acc[0][jq * 4 + 0] = t4.x; acc[0][jq * 4 + 1] = t4.y; acc[0][jq * 4 + 2] = t4.z; acc[0][jq * 4 + 3] = t4.w;
            }
            if (NKB == 2) acc[NKB - 1] = acc[0];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                Frag qf;
                qf.u = *reinterpret_cast<const u32x4_t*>(qs + a_off[rb][ks]);
#pragma unroll
                for (int kb = 0; kb < NKB; ++kb)
                    acc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf.v, kf[kb][ks].v, acc[kb], 0, 0, 0);
            }
            if (sg.chunk && i0 < wave_k0 + kWaveKeys - 1) {     // the diagonal crosses this block: mask
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    const int i = i0 + (j >> 2) * 8 + half * 4 + (j & 3);
#pragma unroll
                    for (int kb = 0; kb < NKB; ++kb) {
                        const float p = __builtin_amdgcn_exp2f(acc[kb][j]);
                        colsum[kb] += kk[kb] <= i ? p : 0.f;
                    }
                }
            } else {
#pragma unroll
                for (int j = 0; j < 16; ++j)
#pragma unroll
                    for (int kb = 0; kb < NKB; ++kb) colsum[kb] += __builtin_amdgcn_exp2f(acc[kb][j]);
            }
        }
        if (++sp == spp) {                                      // the head is finished
            sp = 0;
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb) {
                const float cs = colsum[kb] + __shfl_xor(colsum[kb], 32, 64);
                if (g.head_reduce == CASCADE_REDUCE_MAX) red[kb] = hh == 0 ? cs : fmaxf(red[kb], cs);
                else red[kb] += cs;
                colsum[kb] = 0.f;
            }
            ++hh;
        }
    }
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) {
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
    auto workgroups = [&](int keys) {
        int tiles = 0;
        for (int i = 0; i < sl.n; ++i) tiles += (sl.s[i].len + keys - 1) / keys;
        return tiles * g.B * g.Hkv;
    };
    // 256 keys per workgroup unless that leaves a good part of the 256 x 3 workgroup slots empty
    bool narrow = workgroups(2 * kScoreKeysPerBlock) < 600;
    if (b.opt_score_narrow >= 0) narrow = b.opt_score_narrow == 1;
    const dim3 grid(workgroups(narrow ? kScoreKeysPerBlock : 2 * kScoreKeysPerBlock)), block(kScoreThreads);
    const int qpad = max_chunk + kStRows;   // the attention launch left the offsets of this chunk's rows in b.negt
#define CKV_SCORE(D, NKB)                                                                                              \
    hipLaunchKernelGGL((score_stream_kernel<D, NKB>), grid, block, 0, s, g, sl, Q, max_chunk, tail_rows, qpad, decay,     \
                       (const bf16_t*)b.Qr, (const bf16_t*)b.Kr, (const bf16_t*)b.Krc, b.negt, b.mu, b.mu_chunk)
    if (g.d == 128) { if (narrow) CKV_SCORE(128, 1); else CKV_SCORE(128, 2); }
    else { if (narrow) CKV_SCORE(64, 1); else CKV_SCORE(64, 2); }
#undef CKV_SCORE
}

}  // namespace ckv
