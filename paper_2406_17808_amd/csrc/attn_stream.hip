// bf16 chunk attention of the strided prefill (Alg. 1, Fig. 4; online softmax of Eq. 2).
//
// kv_pack_kernel, once per chunk: the keys and values the chunk attends to (cache segments, then
// the chunk itself) are copied tile after tile (64 keys) in the order the attention kernel
// visits them; when the caller knows that a tile still holds what it held for the previous
// chunk, it leaves that tile out of the launch.  A packed tile is the exact LDS image the attention kernel wants: K with the
// 16-byte chunks of a row XOR-swizzled, V transposed (a row is one column of V with its 64 keys),
// so that the A operand of O^T = V^T P^T is a plain 16-byte LDS read.  The attention kernel then
// needs no segment logic for its loads.  The kernel also leaves the largest squared key norm of
// every tile in Knorm2: with |q| it bounds every logit of a row, and a wave whose rows are all
// bounded close to the maximum of their first tile does not track the maximum any further.
//
// attn_stream_kernel: a workgroup of eight waves owns 256 query rows, 32 per wave (one lane owns
// one query: the transposed formulation described in mfma_util.h).  Packed tiles go from global
// memory straight into LDS by asynchronous loads, four buffers deep.  Per tile a wave alternates
// between a matrix block (O^T += V^T P^T of tile t, then S^T = K Q^T of tile t+1: MFMAs and LDS
// reads only) and a vector block (mask, maximum, exponentials of tile t+1).  The two waves of a
// SIMD run these blocks in opposite phase, held there by two barriers per tile, so the matrix
// pipe and the vector ALU of the SIMD work at the same time.
//
// A chunk too short to give every compute unit a workgroup is split over the keys as well: up to
// eight workgroups share the tiles of one row block and write unnormalised partial results,
// which attn_merge_kernel combines (online-softmax merge of Eq. 2's sums).
#include <stdio.h>
#include <stdlib.h>

#include <type_traits>

#include "async_copy.h"
#include "mfma_util.h"

namespace ckv {

constexpr int kSWaves = 8;    // waves per workgroup: waves w and w+4 share a SIMD and run in opposite phase
constexpr int kSStages = 4;   // LDS buffers per operand

// LDS tiles have no padding and are filled by 1 KB asynchronous loads (every lane of a wave
// deposits its 16 bytes at consecutive LDS addresses).  Bank conflicts are avoided by an XOR
// swizzle of the 16-byte chunks of a row: chunk c of row r sits at position c ^ key(r).
// K tile: 64 keys x D, swizzled by choosing which chunk a lane fetches; read as one chunk per lane
// by 32 lanes on 32 rows (key: low bits of the row).
// V tile: D columns x 64 keys (8 chunks of 8 keys), already swizzled in the packed copy (key:
// bits 1..3 of the column, two rows span the 64 banks); chunk 2*g + h holds keys 16g + 4h + {0..3}
// and 16g + 8 + 4h + {0..3}, the order the probabilities of one lane have in the accumulators of S^T.
template <int D> struct Swz {
    static constexpr int CH = D / 8;                       // 16-byte chunks per K row
    __device__ static int key_k(int r) { return CH == 16 ? (r & 15) : ((r >> 1) & 7); }
};

constexpr int kPackThreads = 256;

// Tile n of the packed K and V copies of one (batch, KV head): 64 rows of a segment (rows past
// its end become zeros); K with its chunks swizzled, V transposed through LDS.
template <int D>
__global__ __launch_bounds__(kPackThreads) void kv_pack_kernel(Geom g, SegList sl, TileRuns runs, int Q, int tiles_per_bh,
                                                               const bf16_t* __restrict__ Kr, const bf16_t* __restrict__ Krc,
                                                               const bf16_t* __restrict__ Vc, const bf16_t* __restrict__ Vch,
                                                               bf16_t* __restrict__ Kt, bf16_t* __restrict__ Vt,
                                                               float* __restrict__ Knorm2)
{
    constexpr int STR = D + 8;   // LDS row stride in elements: 16-byte aligned rows
    __shared__ __attribute__((aligned(16))) bf16_t T[kBN * STR];
    __shared__ float wave_max[kPackThreads / 64];
    const int BH = g.B * g.Hkv;
    const int bh = blockIdx.x % BH, kth = blockIdx.x / BH;   // the kth tile of the runs
    int run = 0;
    while (run + 1 < runs.n && kth >= runs.ahead[run + 1]) ++run;
    const int n = runs.first[run] + (kth - runs.ahead[run]);
    int si = 0, first = 0;
    for (; si < sl.n; ++si) {
        const int nt = (sl.s[si].len + kBN - 1) / kBN;
        if (n < first + nt) break;
        first += nt;
    }
    if (si >= sl.n) return;   // cannot happen: the runs name tiles of the segment list
    const Seg sg = sl.s[si];
    const int t0 = (n - first) * kBN, rows = min(kBN, sg.len - t0);
    const size_t row0 = sg.chunk ? ((size_t)bh * Q + t0) : ((size_t)bh * g.slots + sg.start + t0);
    const bf16_t* src = (sg.chunk ? Vch : Vc) + row0 * D;
    const bf16_t* ksrc = (sg.chunk ? Krc : Kr) + row0 * D;
    bf16_t* kdst = Kt + ((size_t)bh * tiles_per_bh + n) * (kBN * D);
    const int tid = threadIdx.x;
    float norm2_max = 0.f;
#pragma unroll
    for (int p = tid; p < kBN * D / 8; p += kPackThreads) {
        const int r = p / (D / 8), c = p % (D / 8);
        u32x4_t v = {0u, 0u, 0u, 0u}, k = {0u, 0u, 0u, 0u};
        if (r < rows) {
            v = *reinterpret_cast<const u32x4_t*>(src + (size_t)r * D + c * 8);
            k = *reinterpret_cast<const u32x4_t*>(ksrc + (size_t)r * D + (c ^ Swz<D>::key_k(r)) * 8);
        }
        *reinterpret_cast<u32x4_t*>(&T[r * STR + c * 8]) = v;
        *reinterpret_cast<u32x4_t*>(kdst + (size_t)p * 8) = k;   // position c of row r holds chunk c ^ key
        // squared norm of the key row: the D/8 threads of a row are neighbours
        float ss = 0.f;
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const float lo = __uint_as_float(k[x] << 16), hi = __uint_as_float(k[x] & 0xFFFF0000u);
            ss += lo * lo + hi * hi;
        }
#pragma unroll
        for (int w = D / 16; w > 0; w >>= 1) ss += __shfl_xor(ss, w, D / 8);
        norm2_max = fmaxf(norm2_max, ss);
    }
    // the largest squared key norm of the tile (the attention kernel bounds its logits with it)
#pragma unroll
    for (int w = 32; w > 0; w >>= 1) norm2_max = fmaxf(norm2_max, __shfl_xor(norm2_max, w, 64));
    if ((tid & 63) == 0) wave_max[tid >> 6] = norm2_max;
    __syncthreads();
    if (tid == 0) {
        float m = wave_max[0];
#pragma unroll
        for (int w = 1; w < kPackThreads / 64; ++w) m = fmaxf(m, wave_max[w]);
        Knorm2[(size_t)bh * tiles_per_bh + n] = m;
    }
    bf16_t* dst = Vt + ((size_t)bh * tiles_per_bh + n) * (kBN * D);
#pragma unroll
    for (int p = tid; p < D * 8; p += kPackThreads) {
        const int d = p >> 3, c = (p & 7) ^ ((d >> 1) & 7);
        const int k0 = 16 * (c >> 1) + 4 * (c & 1);
        uint32_t w[4];
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const int ka = k0 + (x >> 1) * 8 + (x & 1) * 2;
            w[x] = (uint32_t)T[ka * STR + d] | ((uint32_t)T[(ka + 1) * STR + d] << 16);
        }
        const u32x4_t v = {w[0], w[1], w[2], w[3]};
        *reinterpret_cast<u32x4_t*>(dst + (size_t)p * 8) = v;
    }
}

// What the score kernel wants to know of a finished query row i with log-sum-exp L (base 2, of the
// scaled logits): its exponent offset negt = log2(weight of the row) - L, so that a probability
// times the row's EMA weight is 2^(s + negt) (Section 3.1; the weights are Alg. 3's); -inf for the
// rows before the last `tail`, which carry no weight, and for kScorePadRows rows of padding behind the chunk.
struct ScoreOffsets {
    const float* wrow;   // [max_chunk] weight of the row that has k rows after it
    float* negt;         // [B,Hq,qpad]
    int tail, qpad;
};

// Single-pass scores (Alg. 3): while a row block sweeps the keys it adds, per tile, the column sums
// over its queries of  C_EMA * S^ / (l + l * rho / gamma)  (S^ and l relative to the same running
// maximum, gamma tiles done including this one, rho tiles to go).  A workgroup owns a slice of
// `part`: [row block][tile][64 keys], written tile by tile with plain stores (no atomics: the sums
// are the same from run to run); single_pass_merge_kernel adds the row blocks up.
struct SinglePass {
    float* part;         // [B*Hkv][G][Q / 256][tiles_per_bh][64]
};

__device__ inline void write_score_offset(const ScoreOffsets& so, size_t head, int Q, int i, float lse2)
{
    float* row = so.negt + head * so.qpad;
    row[i] = i >= Q - so.tail ? __log2f(so.wrow[Q - 1 - i]) - lse2 : -INFINITY;
    for (int j = i + Q; j < Q + kScorePadRows; j += Q) row[j] = -INFINITY;   // the first rows between them cover the padding
}

// SPLIT: the tiles a row block visits are divided over n_split workgroups (for launches too small
// to fill the chip otherwise); each writes its unnormalised output, running maximum and row sum
// to part_o / part_ml, and attn_merge_kernel combines them.
// SP: single-pass scores (needs Q % 256 == 0 and no SPLIT: a row block is one head's 256 tokens; and
// every row of the chunk carrying EMA weight, so that every row block takes part).
template <int D, bool DBG, bool SPLIT, bool SP = false>
__global__ __launch_bounds__(kSWaves * 64, 1) void attn_stream_kernel(
    Geom g, SegList sl, int Q, int tiles_per_bh, const bf16_t* __restrict__ q, const float4* __restrict__ rope_t, int rope_rows, float qscale,
    const bf16_t* __restrict__ Kt, const bf16_t* __restrict__ Vt, bf16_t* __restrict__ out, float* __restrict__ lse,
    long long* dbg, int n_split, float* __restrict__ part_o, float* __restrict__ part_ml, const float* __restrict__ Knorm2,
    ScoreOffsets so, SinglePass sp)
{
    static_assert(!(SP && SPLIT), "single-pass scores are taken by unsplit launches only");
    constexpr int BM = kSWaves * 32;       // query rows per workgroup
    constexpr int KS = D / 16;             // k-steps of S^T = K Q^T
    constexpr int DB = D / 32;             // 32-wide blocks of the head dimension in O^T
    constexpr int CH = Swz<D>::CH;
    constexpr int TILE = kBN * D;          // elements per LDS tile
    constexpr int PW = CH / kSWaves;       // 1 KB copies per wave and tile (2 or 1)
    __shared__ __attribute__((aligned(1024))) bf16_t Ks[kSStages * TILE];
    __shared__ __attribute__((aligned(1024))) bf16_t Vs[kSStages * TILE];
    __shared__ float kn_wave[kSWaves];
    __shared__ float sp_sum[SP ? 2 : 1][SP ? kSWaves : 1][SP ? kBN : 1];   // per-wave column sums of the last two tiles
    __shared__ __attribute__((aligned(16))) float sp_w[SP ? kSWaves : 1][SP ? 32 : 4];   // the weights of a wave's 32 queries

    const int BH = g.B * g.Hkv;
    // consecutive workgroups: different KV heads; row blocks that see more of the chunk (longer loops) start first
    const int n_tiles = (int)(gridDim.x / BH) / (SPLIT ? n_split : 1);
    const int rest = (int)(blockIdx.x / BH);
    const int bh = blockIdx.x % BH, split = SPLIT ? rest % n_split : 0, tile = n_tiles - 1 - (SPLIT ? rest / n_split : rest);
    const int b = bh / g.Hkv, hk = bh % g.Hkv;
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), l = tid & 63, l32 = l & 31, half = l >> 5;
    const int GQ = g.G * Q;
    // second phase group (the waves that share a SIMD with waves 0..3): starts its matrix blocks one barrier later
    const bool late = wave >= kSWaves / 2;

    // the query of this lane; rows are (head, token) pairs
    const int r_row = tile * BM + wave * 32 + l32;
    const bool qvalid = r_row < GQ;
    const int rc = min(r_row, GQ - 1);
    const int qh = hk * g.G + rc / Q, qi = rc % Q;
    int wave_imax, wave_imin, wg_imax;
    {
        const int r_lo = min(tile * BM + wave * 32, GQ - 1), r_hi = min(tile * BM + wave * 32 + 31, GQ - 1);
        if (r_lo / Q == r_hi / Q) { wave_imin = r_lo % Q; wave_imax = r_hi % Q; }
        else { wave_imin = 0; wave_imax = Q - 1; }
        const int w_lo = min(tile * BM, GQ - 1), w_hi = min(tile * BM + BM - 1, GQ - 1);
        wg_imax = (w_lo / Q == w_hi / Q) ? w_hi % Q : Q - 1;
    }

    f32x16_t o[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int j = 0; j < 16; ++j) o[db][j] = 0.f;
    // The queries carry the softmax scale and log2(e): S^T holds base-2 exponents.  m_run is the
    // maximum the exponents are taken against; the accumulators of S^T start at -m_run (negm, all
    // sixteen registers the same value: a lane owns one query), so S^T comes out of the MFMAs
    // already relative to it.
    float m_run = 0.f;
    f32x16_t negm;
#pragma unroll
    for (int j = 0; j < 16; ++j) negm[j] = 0.f;
    float lsum = 0.f;   // this lane's part of the row sum
    bool seen = false;  // SPLIT: this row has seen a key
    bool bounded = false;   // see below: the per-tile maximum is not needed

    // The packed tiles are LDS images: every wave copies PW consecutive KB of each
    const uint32_t lds_k = lds_address(Ks) + (uint32_t)wave * PW * 1024u;
    const uint32_t lds_v = lds_address(Vs) + (uint32_t)wave * PW * 1024u;
    const bf16_t* kt_bh = Kt + (size_t)bh * tiles_per_bh * TILE + (size_t)wave * PW * 512;   // (SPLIT: moved to the first tile of the range below)
    const bf16_t* vt_bh = Vt + (size_t)bh * tiles_per_bh * TILE + (size_t)wave * PW * 512;
    auto copy_tile = [&](const bf16_t* src_bh, uint32_t lds, int n, int stage) {   // tile n of a packed copy
        const bf16_t* base = src_bh + (size_t)n * TILE;
        const uint32_t dst = lds + (uint32_t)stage * (TILE * 2);
#pragma unroll
        for (int x = 0; x < PW; ++x)
            async_copy_1k(base, (uint32_t)(x * 1024 + l * 16), __builtin_amdgcn_readfirstlane(dst + x * 1024u));
    };

    // LDS read addressing of this lane.  K fragment (key block kb, step ks): row kb*32 + l32,
    // chunk 2*ks + half.  V fragment (key group g16, column block db): row 32*db + l32, chunk
    // 2*g16 + half.
    const int kkey = Swz<D>::key_k(l32);   // same for row l32 + 32
    const int vkey = (l32 >> 1) & 7;       // same for rows l32 + 32, + 64, ...
    int koff[KS], voff[4];                 // element offsets inside a tile; kb and db add constants
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) koff[ks] = (l32 * CH + ((2 * ks + half) ^ kkey)) * 8;
#pragma unroll
    for (int g16 = 0; g16 < 4; ++g16) voff[g16] = (l32 * 8 + ((2 * g16 + half) ^ vkey)) * 8;

    // The query of this lane, rotated for one segment: the stored keys are rotated to their slot
    // index, so the query turns by (own cache index) - (cache index - slot index) of the segment,
    // sl.qrot0[variant] + qi.  The fragment of step ks holds elements 16 ks + 8 half .. + 7, whose
    // rotary partners (element + D/2) are the fragment of step ks + KS/2 of the same lane.  The
    // arithmetic is that of prep_kernel (scale first, then the rotation, then one rounding), which
    // writes the same values for the rows the score kernel reads.
    Frag qf[KS];
    float qn2 = 0.f;      // this lane's half of the squared norm of its (scaled) query, summed by the first load_q
    auto load_q = [&](const Seg& sg) {
        qn2 = 0.f;
        const bf16_t* qsrc = q + (((size_t)b * Q + qi) * g.Hq + qh) * D + half * 8;
        // (cos, sin) of this lane's 8 rotary pairs per step from the index-minor table: group ks * 8 + half * 4 + x
        const float4* cs = rope_t + ((size_t)half * 4 * rope_rows + (size_t)(sl.qrot0[sg.qvar] + qi));
        // All loads first (24 at D = 128), then the arithmetic: scheduled freely, the loads come in four or
        // five groups, each waiting for the one before.  (Measured: no difference; what a reload costs is
        // neither those round trips nor, much, the cache lines its loads touch: the index-minor table
        // below, 8 lines per load instead of 32, gains 2 % on a 16K cache and 0.7 % on a 64K cache.)
        u32x4_t lo[KS / 2], hi[KS / 2];
        float4 c4[KS / 2][4];      // (cos, sin) of 8 rotary pairs
#pragma unroll
        for (int ks = 0; ks < KS / 2; ++ks) {
            lo[ks] = *reinterpret_cast<const u32x4_t*>(qsrc + ks * 16);
            hi[ks] = *reinterpret_cast<const u32x4_t*>(qsrc + ks * 16 + D / 2);
#pragma unroll
            for (int x = 0; x < 4; ++x) c4[ks][x] = cs[(size_t)(ks * 8 + x) * rope_rows];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ks = 0; ks < KS / 2; ++ks) {
            float y0[8], y1[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint32_t wl = lo[ks][j >> 1], wh = hi[ks][j >> 1];
                const float x0 = __uint_as_float((j & 1) ? (wl & 0xFFFF0000u) : (wl << 16)) * qscale;
                const float x1 = __uint_as_float((j & 1) ? (wh & 0xFFFF0000u) : (wh << 16)) * qscale;
                const float cx = (j & 1) ? c4[ks][j >> 1].z : c4[ks][j >> 1].x, cy = (j & 1) ? c4[ks][j >> 1].w : c4[ks][j >> 1].y;
                y0[j] = rot_lo(x0, x1, cx, cy);
                y1[j] = rot_hi(x0, x1, cx, cy);
                qn2 += x0 * x0 + x1 * x1;
            }
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                qf[ks].u[x] = cvt_pk_bf16(y0[2 * x], y0[2 * x + 1]);
                qf[ks + KS / 2].u[x] = cvt_pk_bf16(y1[2 * x], y1[2 * x + 1]);
            }
        }
    };
    f32x16_t s[2];   // S^T of one tile: 2 key blocks of 32 keys
    Frag pf[4];      // its probabilities, 16 keys each: [key block][half]
    // S^T = K Q^T for the K tile at Kt
    auto qk_tile = [&](const bf16_t* Kt) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int j = 0; j < 16; ++j) s[kb][j] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                Frag kf;
                kf.u = *reinterpret_cast<const u32x4_t*>(Kt + koff[ks] + kb * (32 * D));
                s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf.v, qf[ks].v, s[kb], 0, 0, 0);
            }
    };
    // Single-pass scores: a row block is 256 tokens of one head (Q % 256 == 0).  cw: the weight of this
    // lane's row (Alg. 3's C_EMA).
    const int rbs_per_head = SP ? Q / BM : 1;
    const float cw = (SP && qvalid) ? so.wrow[Q - 1 - qi] : 0.f;
    float* sp_part = SP ? sp.part + ((size_t)bh * g.G * rbs_per_head + tile) * (size_t)tiles_per_bh * kBN : nullptr;
    float inv_steps = 0.f;               // 1 / tiles this row block visits, set once they are counted
    // Column sums over the 32 queries of this wave of  p * w  (w per query), for the 64 keys of a tile.
    // A lane owns a query, so the sum runs across lanes; the matrix pipe does the transposition: the
    // probabilities are already packed as an MFMA operand (pf, for O^T = V^T P^T); taken as the A operand
    // (rows: queries, contraction: 16 keys) against a 0/1 matrix that sends contraction index k to the
    // column of its key, two MFMAs per 32-key block leave P with the KEYS across the lanes and the
    // queries in the 16 accumulator registers (S^T is dead by now: its registers take the result).
    // What is left is an in-lane weighted sum (the weights of the wave's 32 queries go through LDS, 16 of
    // them per lane) and one exchange between the two lane halves, after which lane l holds the sum of
    // key l of the tile.  The probabilities enter rounded to bf16, as they do for the outputs.
    Frag bid[2];       // bid[hf][k][n] = 1 where column n is the key of contraction index k of pf[2 kb + hf]
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) {
        // element i of lane half h of pf[2 kb + hf] is key 16 hf + 8 (i / 4) + 4 h + i % 4 of the block
        const int np = l32 - 16 * hf;
        int i = -1;
        if (SP && np >= 0 && np < 16 && ((np >> 2) & 1) == half) i = 4 * (np >> 3) + (np & 3);
#pragma unroll
        for (int x = 0; x < 4; ++x) bid[hf].u[x] = (i >= 0 && (i >> 1) == x) ? ((i & 1) ? 0x3F800000u : 0x00003F80u) : 0u;
    }
    // The weights are set in the vector block that makes the probabilities of a tile (column_weights);
    // the four MFMAs and the weighted sums are part of the matrix block that multiplies those
    // probabilities with V (there the wave owns the matrix pipe, and the vector instructions fall into the
    // shadow of its MFMAs; in the vector block, which is as long as the matrix block without them, they cost
    // 1.28 against 1.04 ms on a 16K cache, with the four MFMAs queuing behind the other group's).
    auto column_weights = [&](int step) {
        const auto lp = __builtin_amdgcn_permlane32_swap(__float_as_uint(lsum), __float_as_uint(lsum), false, false);
        const float lt = __uint_as_float(lp[0]) + __uint_as_float(lp[1]);    // both halves of the row's keys
        // gamma / (gamma + rho) = step / NT; a row always sees a key of its first tile, so lt > 0
        const float w = cw * (float)step * inv_steps * __builtin_amdgcn_rcpf(lt);
        if (half == 0) sp_w[wave][l32] = w;
    };
    // The four waves of the late group add the eight waves' sums of tile t, 16 keys each, and store them.
    // Called in their vector block t: both groups have left their matrix block t (the barrier the caller
    // has passed), and the slot is written again in matrix block t + 2, two barriers later.  Lane l of wave
    // 4 + kq takes key 16 kq + l % 16 and the sums of waves 2 (l / 16) and 2 (l / 16) + 1; two lane exchanges
    // add the four pairs (in a fixed order: the result does not depend on timing).
    auto flush_column_sums = [&](int t, int kq) {
        const int key = 16 * kq + (l & 15), pair = l >> 4;
        float a = sp_sum[(t + 1) & 1][2 * pair][key] + sp_sum[(t + 1) & 1][2 * pair + 1][key];
        const auto r16 = __builtin_amdgcn_permlane16_swap(__float_as_uint(a), __float_as_uint(a), false, false);
        a = __uint_as_float(r16[0]) + __uint_as_float(r16[1]);       // rows 0+1 | 0+1 | 2+3 | 2+3
        const auto r32 = __builtin_amdgcn_permlane32_swap(__float_as_uint(a), __float_as_uint(a), false, false);
        a = __uint_as_float(r32[0]) + __uint_as_float(r32[1]);
        if (l < 16) counted_store_f32(sp_part, (uint32_t)((t * kBN + key) * 4), a);
    };
    // The vector block of one tile: mask the keys a query may not see (past the end of the
    // segment; later chunk tokens), take the row maximum of S^T (relative to m_run), raise m_run only
    // when that exceeds kRescaleLog2 (the probabilities then stay below 2^kRescaleLog2, and most
    // tiles skip the rescaling of O), and turn S^T into probabilities.  FIRST: S^T is absolute
    // and m_run not set yet (the first tile of a workgroup).
    auto softmax_tile = [&](const TileIter& it, bool first, auto interior, int step) {
        if (!decltype(interior)::value && ((it.t0 + kBN > it.sg.len) || (it.sg.chunk && it.t0 + kBN - 1 > wave_imin))) {
            const int lim = it.sg.chunk ? min(it.sg.len - 1, qi) : it.sg.len - 1;   // last visible key
            const int rel = lim - it.t0 - half * 4;   // accumulator j of block kb is key t0 + 4*half + (32 kb + 8 (j/4) + j%4)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    if (kb * 32 + (j >> 2) * 8 + (j & 3) > rel) s[kb][j] = -INFINITY;
                    // a few compares at a time: all 32 lane masks at once take 64 scalar registers, which
                    // pushes values that live across the loop out to vector lanes
                    if ((j & 3) == 3) __builtin_amdgcn_sched_barrier(0);
                }
        }
        if (!bounded || first) {   // bounded: no exponent of this workgroup can exceed m_run by more than 2^kBoundLog2
            float x = -INFINITY;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int j = 0; j < 16; ++j) x = fmaxf(x, s[kb][j]);
            const float mt = max_xor32(x);
            // SPLIT: a range may start with chunk tiles some rows do not see at all, so "first" is kept
            // per row: until a row has seen a key its m_run stays 0 and everything it holds is zero
            const bool fresh = SPLIT ? !seen : first;
            const bool grow = SPLIT ? (fresh ? mt > -INFINITY : mt > kRescaleLog2) : (first || mt > kRescaleLog2);
            if (SPLIT) seen = seen || mt > -INFINITY;
            if (__any(grow)) {
                const float delta = grow ? mt : 0.f;   // not SPLIT: every row sees a key of the first tile, finite there
                const float alpha = fresh ? 1.f : __builtin_amdgcn_exp2f(-delta);   // O and the row sum are still zero for a fresh row
                m_run += delta;
                lsum *= alpha;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int j = 0; j < 16; ++j) o[db][j] *= alpha;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int j = 0; j < 16; ++j) s[kb][j] -= delta;
#pragma unroll
                for (int j = 0; j < 16; ++j) negm[j] = -m_run;
            }
        }
#pragma unroll
        for (int qt = 0; qt < 4; ++qt) {
            const int kb = qt >> 1, hf = qt & 1;
#pragma unroll
            for (int x2 = 0; x2 < 4; ++x2) {
                const float p0 = __builtin_amdgcn_exp2f(s[kb][hf * 8 + 2 * x2]);
                const float p1 = __builtin_amdgcn_exp2f(s[kb][hf * 8 + 2 * x2 + 1]);
                pf[qt].u[x2] = cvt_pk_bf16(p0, p1);
                lsum += p0 + p1;   // plain adds: the dot-product instructions queue behind the MFMAs of the SIMD
            }
        }
        if (SP) column_weights(step);
    };
    auto wave_active = [&](const TileIter& it) { return !(it.sg.chunk && it.t0 > wave_imax); };

    // In iteration t, tile t is multiplied with V, tile t+1 with Q; the copies of V of tile t+2
    // and of K of tile t+3 are issued.  Only the softmax needs to know which segment a tile is from.
    int NT = 0;   // tiles this workgroup visits: chunk keys after its last row are never visible
    for (int i = 0; i < sl.n; ++i) NT += ((sl.s[i].chunk ? min(sl.s[i].len, wg_imax + 1) : sl.s[i].len) + kBN - 1) / kBN;
    if (SP) inv_steps = 1.f / (float)NT;
    int tile_first = 0;                  // SPLIT: first tile of this workgroup's range
    TileIter it1;
    it1.first(sl, wg_imax);
    if (!it1.valid(sl)) return;          // cannot happen: the chunk itself is always a segment
    // this lane's row of the partial results
    const size_t prow = ((((size_t)split * BH + bh) * n_tiles + tile) * BM) + wave * 32 + l32;
    if (SPLIT) {
        const int tb = (int)((long long)NT * split / n_split), te = (int)((long long)NT * (split + 1) / n_split);
        if (tb == te) {                  // nothing to do (uniform for the workgroup): an empty partial result
            if (half == 0) { part_ml[prow * 2] = 0.f; part_ml[prow * 2 + 1] = 0.f; }
            return;
        }
        for (int i = 0; i < tb; ++i) it1.next(sl, wg_imax);
        tile_first = tb;
        kt_bh += (size_t)tb * TILE;
        vt_bh += (size_t)tb * TILE;
        NT = te - tb;
    }

    // Copies.  Batch t is K of tile t+4 and V of tile t+3, each into the stage of the tile four
    // before it.  A wave issues its share of batch t at the start of its vector block t (those
    // tiles were last read in matrix block t-1, which both groups left before) and, before the
    // barrier that ends its iteration t, waits until only that batch is still in flight: its
    // share of batch t-1 has landed then.  The early group passes that barrier as 2t+2, the late
    // group as 2t+3, and the first read of batch t-1 (V of tile t+2, read ahead by the early
    // group) comes after barrier 2t+3.
    static_assert(kSStages == 4, "the copy schedule is written for four stages");
    auto issue = [&](int t) -> int {   // returns the number of copy instructions issued
        int n = 0;
        if (t + 4 < NT) { copy_tile(kt_bh, lds_k, t + 4, t & 3); n += PW; }
        if (t + 3 < NT) { copy_tile(vt_bh, lds_v, t + 3, (t + 3) & 3); n += PW; }
        return n;
    };
    auto publish = [&](int in_flight) {
        if (in_flight == 2 * PW) wait_vm<2 * PW>();
        else if (in_flight == PW) wait_vm<PW>();
        else wait_vm<0>();
    };
    // The 4*DB V fragments and 2*KS K fragments of a matrix block form one sequence; fragment i
    // is read kAhead MFMAs before MFMA i uses it (enough bytes in flight to cover the LDS latency
    // with one reading wave per SIMD), the first kAhead already before the preceding vector block.
    constexpr int kAhead = 8, NV = 4 * DB, NF = 4 * DB + 2 * KS;
    static_assert(kAhead <= NV, "the fragments read ahead of a matrix block are V fragments");
    auto read_frag = [&](const bf16_t* Vtile, const bf16_t* Ktile, int i) {
        Frag f;
        if (i < NV) f.u = *reinterpret_cast<const u32x4_t*>(Vtile + voff[i / DB] + (i % DB) * (32 * kBN));
        else f.u = *reinterpret_cast<const u32x4_t*>(Ktile + koff[(i - NV) / 2] + ((i - NV) % 2) * (32 * D));
        return f;
    };
    Frag fr[kAhead];

    // prologue: K of tiles 0..3, V of tiles 0..2; S^T and probabilities of tile 0
#pragma unroll
    for (int n = 0; n < 4; ++n)
        if (n < NT) copy_tile(kt_bh, lds_k, n, n);
#pragma unroll
    for (int n = 0; n < 3; ++n)
        if (n < NT) copy_tile(vt_bh, lds_v, n, n);
    load_q(it1.sg);
    int q_var = it1.sg.qvar;   // the rotation the query fragments hold (two segments may share one)
    // the largest squared key norm among the tiles of this workgroup
    float kn2 = 0.f;
    {
        const float* kn = Knorm2 + (size_t)bh * tiles_per_bh + (SPLIT ? tile_first : 0);
        for (int i = tid; i < NT; i += kSWaves * 64) kn2 = fmaxf(kn2, kn[i]);
#pragma unroll
        for (int w = 32; w > 0; w >>= 1) kn2 = fmaxf(kn2, __shfl_xor(kn2, w, 64));
        if (l == 0) kn_wave[wave] = kn2;
    }
    const float qnorm2 = qn2 + __shfl_xor(qn2, 32, 64);
    wait_vm<0>();
    __syncthreads();
#pragma unroll
    for (int w = 0; w < kSWaves; ++w) kn2 = fmaxf(kn2, kn_wave[w]);
    qk_tile(Ks);
    if (!SPLIT || wave_active(it1)) {
        softmax_tile(it1, true, std::false_type(), 1);    // not SPLIT: every wave sees the first tile
    } else {
#pragma unroll
        for (int qt = 0; qt < 4; ++qt)
#pragma unroll
            for (int x = 0; x < 4; ++x) pf[qt].u[x] = 0u;
#pragma unroll
        for (int j = 0; j < 16; ++j) negm[j] = 0.f;
    }
    // By Cauchy-Schwarz no exponent of this row exceeds |q| max|k| (the rotation keeps norms; 1 % for the
    // rounding of the rotated operands).  If that is within kBoundLog2 of the maximum of the first
    // tile for every row of the wave, probabilities stay below 2^kBoundLog2 whatever the later
    // tiles hold, m_run can stay where it is, and the per-tile maximum is skipped.
    if (!SPLIT) bounded = !__any(sqrtf(qnorm2 * kn2) * 1.01f > m_run + kBoundLog2);
    it1.next(sl, wg_imax);
    __syncthreads();      // barrier 0: every wave has read K of tile 0, its buffer may be refilled
#pragma unroll
    for (int i = 0; i < kAhead; ++i) fr[i] = read_frag(Vs, Ks, i);
    if (late) wg_barrier();     // barrier 1

    int n0 = 0;   // t
    long long tc[5] = {0, 0, 0, 0, 0}, tlast = 0;
    if (DBG) tlast = __builtin_readcyclecounter();
    auto lap = [&](int i) { if (DBG) { const long long now = __builtin_readcyclecounter(); tc[i] += now - tlast; tlast = now; } };
    // ---- matrix block of iteration t.  A wave that does not see tile t holds zero probabilities;
    // S^T of a tile this wave does not see (or that does not exist: stale buffer) is computed and
    // dropped.  The order of MFMAs and reads is pinned step by step.
    auto matrix_block = [&](int t) {
        __builtin_amdgcn_s_setprio(2);
        __builtin_amdgcn_sched_barrier(0);
        {
            const bf16_t* Vtile = Vs + (t & 3) * TILE;
            const bf16_t* Ktile = Ks + ((t + 1) & 3) * TILE;
            float4 w4[SP ? 4 : 1];
            float csum[2] = {0.f, 0.f};
            if (SP) {
                // S^T of tile t has become probabilities: its registers take P with the keys across the lanes
                // (accumulator j of this lane: query row 8 (j / 4) + 4 half + j % 4 of the wave)
                w4[0] = *reinterpret_cast<const float4*>(&sp_w[wave][4 * half]);    // the others follow two MFMAs ahead of their use
                const f32x16_t zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pf[0].v, bid[0].v, zero, 0, 0, 0);
                s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pf[2].v, bid[0].v, zero, 0, 0, 0);
                s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pf[1].v, bid[1].v, s[0], 0, 0, 0);
                s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pf[3].v, bid[1].v, s[1], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int i = 0; i < NF; ++i) {
                if (i < NV) o[i % DB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[i % kAhead].v, pf[i / DB].v, o[i % DB], 0, 0, 0);
                else s[(i - NV) % 2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[i % kAhead].v, qf[(i - NV) / 2].v, i - NV < 2 ? negm : s[(i - NV) % 2], 0, 0, 0);
                if (i + kAhead < NF) fr[i % kAhead] = read_frag(Vtile, Ktile, i + kAhead);
                // the weighted sums, in eight groups of four terms behind the first MFMAs (S^T is rewritten from MFMA NV on)
                constexpr int GPS = NV >= 16 ? 1 : 2, FIRST = NV >= 16 ? 4 : 3, LAST = FIRST + 8 / GPS;
                static_assert(LAST < NV, "the sums read S^T's registers before the next QK^T writes them");
                if (SP && i >= FIRST - 2 && i < LAST - 2 && (i - FIRST + 2) * GPS % 2 == 0 && ((i - FIRST + 2) * GPS) / 2 + 1 < 4)
                    w4[((i - FIRST + 2) * GPS) / 2 + 1] = *reinterpret_cast<const float4*>(&sp_w[wave][8 * (((i - FIRST + 2) * GPS) / 2 + 1) + 4 * half]);
                if (SP && i >= FIRST && i < LAST) {
#pragma unroll
                    for (int gq = (i - FIRST) * GPS; gq < (i - FIRST + 1) * GPS; ++gq) {
                        const int jq = gq >> 1, kb = gq & 1;
                        csum[kb] = __builtin_fmaf(s[kb][4 * jq + 0], w4[jq].x, csum[kb]);
                        csum[kb] = __builtin_fmaf(s[kb][4 * jq + 1], w4[jq].y, csum[kb]);
                        csum[kb] = __builtin_fmaf(s[kb][4 * jq + 2], w4[jq].z, csum[kb]);
                        csum[kb] = __builtin_fmaf(s[kb][4 * jq + 3], w4[jq].w, csum[kb]);
                    }
                }
                if (SP && i == LAST) {
                    // lower lanes keep key block 0, upper lanes key block 1, each adding the other half's queries
                    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(csum[0]), __float_as_uint(csum[1]), false, false);
                    sp_sum[(t + 1) & 1][wave][l] = __uint_as_float(r[0]) + __uint_as_float(r[1]);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // S^T is complete here: without this use the compiler may sink the last MFMAs (they touch no
        // memory) past the end of the block, below the barrier and into the vector block
        asm volatile("" : "+v"(s[0]), "+v"(s[1]));
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_setprio(0);
    };
    while (true) {
        // Steady state: as long as tile t+1 is a whole tile that every row of the wave sees completely,
        // with another tile of the same segment behind it and both copies of the batch ahead, an iteration
        // needs none of the tests below (visibility, masks, change of rotation, which copies to issue, how
        // many to wait for).  Waves may disagree on it: both loops pass the same barriers and issue the
        // same copies.
        if (q_var == it1.sg.qvar) {
            int k = min((it1.len - it1.t0 - 1) / kBN, NT - 4 - n0);
            if (it1.sg.chunk) k = min(k, (wave_imin + 1 - it1.t0) / kBN);   // chunk tiles every row of the wave sees whole
            for (; k > 0; --k) {
                lap(0);
                matrix_block(n0);
                lap(1);
                wg_barrier();
                lap(2);
                // measured orders of the three parts: exponentials, fragments, copies (this one) 3.329 ms;
                // fragments first 3.35; copies before the fragments 3.41
                softmax_tile(it1, false, std::true_type(), n0 + 2);
                if (SP && late) flush_column_sums(n0, wave - 4);
#pragma unroll
                for (int i = 0; i < kAhead; ++i) fr[i] = read_frag(Vs + ((n0 + 1) & 3) * TILE, Ks, i);
                copy_tile(kt_bh, lds_k, n0 + 4, n0 & 3);
                copy_tile(vt_bh, lds_v, n0 + 3, (n0 + 3) & 3);
                lap(3);
                wait_vm<2 * PW>();
                wg_barrier();
                lap(4);
                it1.t0 += kBN;
                ++n0;
            }
        }
        const bool has_next = n0 + 1 < NT;
        const bool act_next = has_next && wave_active(it1);
        if (act_next && q_var != it1.sg.qvar) {
            load_q(it1.sg);
            q_var = it1.sg.qvar;
            wait_vm<0>();   // here, so that no wait for these loads is placed among the MFMAs (it would also wait for the copies)
            // load_q holds all its loads in registers at once.  What can be had again for nothing is written after
            // it, and so is dead while it runs: the copies of -m_run (16 registers) and the fragments read ahead for
            // the coming matrix block (32; still in LDS).  Without this the reload spills.
#pragma unroll
            for (int j = 0; j < 16; ++j) negm[j] = -m_run;
#pragma unroll
            for (int i = 0; i < kAhead; ++i) fr[i] = read_frag(Vs + (n0 & 3) * TILE, Ks, i);
        }
        lap(0);
        matrix_block(n0);
        lap(1);
        if (!has_next) break;
        wg_barrier();     // barrier 2t+1 (early group), 2t+2 (late group)
        lap(2);
        // the first fragments of the next matrix block: V of tile t+1
#pragma unroll
        for (int i = 0; i < kAhead; ++i) fr[i] = read_frag(Vs + ((n0 + 1) & 3) * TILE, Ks, i);
        const int in_flight = issue(n0);   // here: a copy instruction can hold a wave up, and this block has time to spare
        // ---- vector block
        if (act_next) {
            softmax_tile(it1, false, std::false_type(), n0 + 2);
        } else {
#pragma unroll
            for (int qt = 0; qt < 4; ++qt)
#pragma unroll
                for (int x = 0; x < 4; ++x) pf[qt].u[x] = 0u;
        }
        if (SP && late) flush_column_sums(n0, wave - 4);
        lap(3);
        publish(in_flight);
        wg_barrier();     // barrier 2t+2 (early group), 2t+3 (late group)
        lap(4);
        it1.next(sl, wg_imax);
        ++n0;
    }
    if (!late) wg_barrier();   // the late group passed one barrier more
    if (SP) {
        wg_barrier();                            // every wave has left its last matrix block
        if (late) flush_column_sums(n0, wave - 4);    // the last tile
    }
    if (DBG && blockIdx.x == 100 && l == 0 && (wave == 0 || wave == 4)) {
#pragma unroll
        for (int i = 0; i < 5; ++i) dbg[(wave / 4) * 8 + i] = tc[i];
        dbg[(wave / 4) * 8 + 5] = n0 + 1;
    }
    // normalise and store: this lane owns one query, columns 32*db + 8*(j/4) + 4*half + j%4
    const float lt = lsum + __shfl_xor(lsum, 32, 64);
    if (SPLIT) {
        float* prow_o = part_o + prow * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int jq = 0; jq < 4; ++jq) {
                const float4 w = {o[db][jq * 4 + 0], o[db][jq * 4 + 1], o[db][jq * 4 + 2], o[db][jq * 4 + 3]};
                *reinterpret_cast<float4*>(prow_o + db * 32 + jq * 8 + half * 4) = w;
            }
        if (half == 0) { part_ml[prow * 2] = m_run; part_ml[prow * 2 + 1] = lt; }
        return;
    }
    if (qvalid) {
        const float inv = 1.f / lt;
        bf16_t* orow = out + (((size_t)b * Q + qi) * g.Hq + qh) * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int jq = 0; jq < 4; ++jq) {
                uint2 w;
                w.x = cvt_pk_bf16(o[db][jq * 4 + 0] * inv, o[db][jq * 4 + 1] * inv);
                w.y = cvt_pk_bf16(o[db][jq * 4 + 2] * inv, o[db][jq * 4 + 3] * inv);
                *reinterpret_cast<uint2*>(orow + db * 32 + jq * 8 + half * 4) = w;
            }
        if (half == 0) {
            lse[((size_t)b * g.Hq + qh) * Q + qi] = m_run * 0.6931471805599453f + logf(lt);
            write_score_offset(so, (size_t)b * g.Hq + qh, Q, qi, m_run + __log2f(lt));
        }
    }
}

// tiles of the packed V copy one (batch, KV head) needs for this segment list
static int packed_tiles(const SegList& sl)
{
    int n = 0;
    for (int i = 0; i < sl.n; ++i) n += (sl.s[i].len + kBN - 1) / kBN;
    return n;
}

int packed_tiles_of(const SegList& sl) { return packed_tiles(sl); }

// Tile n of a (batch, KV head) sits at tile index bh * b.vt_tiles + n of Kt, Vt and Knorm2: the
// stride is the capacity, so that tiles keep their place from one chunk to the next.
bool launch_kv_pack(const Geom& g, const DevBuffers& b, const SegList& sl, const TileRuns& runs, int Q, hipStream_t s)
{
    if (packed_tiles(sl) > b.vt_tiles) return false;   // the workspace was sized for every possible segment list
    if (runs.total == 0) return true;
    const dim3 grid(runs.total * g.B * g.Hkv), block(kPackThreads);
    if (g.d == 128)
        hipLaunchKernelGGL(kv_pack_kernel<128>, grid, block, 0, s, g, sl, runs, Q, b.vt_tiles, (const bf16_t*)b.Kr, (const bf16_t*)b.Krc,
                           (const bf16_t*)b.Vc, (const bf16_t*)b.Vch, (bf16_t*)b.Kt, (bf16_t*)b.Vt, b.knorm2);
    else
        hipLaunchKernelGGL(kv_pack_kernel<64>, grid, block, 0, s, g, sl, runs, Q, b.vt_tiles, (const bf16_t*)b.Kr, (const bf16_t*)b.Krc,
                           (const bf16_t*)b.Vc, (const bf16_t*)b.Vch, (bf16_t*)b.Kt, (bf16_t*)b.Vt, b.knorm2);
    return true;
}

// out = sum_s O_s 2^(m_s - M) / sum_s l_s 2^(m_s - M), M = max over the splits that saw a key;
// one workgroup of D threads per (KV head, query row of the group).
template <int D>
__global__ __launch_bounds__(D) void attn_merge_kernel(Geom g, int Q, int n_tiles, int n_split, int BM,
                                                       const float* __restrict__ part_o, const float* __restrict__ part_ml,
                                                       bf16_t* __restrict__ out, float* __restrict__ lse, ScoreOffsets so)
{
    const int BH = g.B * g.Hkv;
    const int bh = blockIdx.y, r = blockIdx.x;            // r = head-in-group * Q + token
    const int b = bh / g.Hkv, hk = bh % g.Hkv, qh = hk * g.G + r / Q, qi = r % Q;
    const int tile = r / BM, within = r % BM, e = threadIdx.x;
    float M = -INFINITY;
    for (int s = 0; s < n_split; ++s) {
        const size_t prow = (((size_t)s * BH + bh) * n_tiles + tile) * BM + within;
        if (part_ml[prow * 2 + 1] > 0.f) M = fmaxf(M, part_ml[prow * 2]);
    }
    float L = 0.f, acc = 0.f;
    for (int s = 0; s < n_split; ++s) {
        const size_t prow = (((size_t)s * BH + bh) * n_tiles + tile) * BM + within;
        const float ls = part_ml[prow * 2 + 1];
        if (ls > 0.f) {
            const float w = __builtin_amdgcn_exp2f(part_ml[prow * 2] - M);
            L += ls * w;
            acc += part_o[prow * D + e] * w;
        }
    }
    out[(((size_t)b * Q + qi) * g.Hq + qh) * D + e] = f32_to_bf16(acc / L);
    if (e == 0) {
        lse[((size_t)b * g.Hq + qh) * Q + qi] = M * 0.6931471805599453f + logf(L);
        write_score_offset(so, (size_t)b * g.Hq + qh, Q, qi, M + __log2f(L));
    }
}

// Single-pass scores, second half: per key, the row blocks' column sums added up in a fixed order,
// the query heads of the group reduced (max or mean), and the EMA step of Section 3.1 taken:
// cached rows mu <- decay * mu + increment, chunk tokens start at their increment.  One thread per
// key of a packed tile; a chunk tile was only visited by the row blocks that see it.
__global__ __launch_bounds__(kBN) void single_pass_merge_kernel(Geom g, SegList sl, int Q, int qstride, int tiles_per_bh, SinglePass sp,
                                                                float decay, float* __restrict__ mu, float* __restrict__ mu_chunk)
{
    const int n = blockIdx.x, bh = blockIdx.y, x = threadIdx.x;
    int si = 0, first = 0;
    for (; si < sl.n; ++si) {
        const int nt = (sl.s[si].len + kBN - 1) / kBN;
        if (n < first + nt) break;
        first += nt;
    }
    if (si >= sl.n) return;
    const Seg sg = sl.s[si];
    const int t0 = (n - first) * kBN, key = t0 + x;
    if (key >= sg.len) return;
    // row block r of a head covers tokens 256 r .. 256 r + 255 and visits the chunk's tiles up to its last token
    const int rbs = Q / 256, r_lo = sg.chunk ? t0 / 256 : 0;
    float red = 0.f;
    for (int hh = 0; hh < g.G; ++hh) {
        const float* p = sp.part + ((((size_t)bh * g.G + hh) * rbs) * (size_t)tiles_per_bh + n) * kBN + x;
        float v = 0.f;
        for (int r = r_lo; r < rbs; ++r) v += p[(size_t)r * tiles_per_bh * kBN];
        red = g.head_reduce == CASCADE_REDUCE_MAX ? (hh == 0 ? v : fmaxf(red, v)) : red + v;
    }
    if (g.head_reduce == CASCADE_REDUCE_MEAN) red /= (float)g.G;
    if (sg.chunk) mu_chunk[(size_t)bh * qstride + key] = red;
    else {
        float* m = mu + (size_t)bh * g.slots + sg.start + key;
        *m = decay * *m + red;
    }
}

// Workgroups per (row block, KV head) so that a small launch still fills the chip: none for 256
// workgroups or more.
int attn_splits(const Geom& g, int Q, int forced)
{
    constexpr int BM = kSWaves * 32;
    const int wgs = ((g.G * Q + BM - 1) / BM) * g.B * g.Hkv;
    int n = forced > 0 ? forced : 256 / wgs;
    if (n > 256 / wgs) n = 256 / wgs;       // the partial results are sized for 256 workgroups
    if (n > kMaxAttnSplits) n = kMaxAttnSplits;
    return n < 1 ? 1 : n;
}

// A chunk takes the single-pass scores when every one of its rows carries EMA weight (an EMA
// parameter close to 1, the paper's setting: otherwise the exact pass is short, and cheaper than
// column sums in every row block), its launch is not split over the keys, and its row blocks are
// whole heads' pieces (Q a multiple of 256); other chunks of such a context take the exact pass.
bool attn_single_pass_ok(const Geom& g, const DevBuffers& b, int Q, int tail_rows)
{
    return b.sp_part != nullptr && tail_rows >= Q && Q % (kSWaves * 32) == 0 && attn_splits(g, Q, b.opt_attn_splits) == 1;
}

void launch_single_pass_merge(const Geom& g, const DevBuffers& b, const SegList& sl, int Q, int max_chunk, float decay, hipStream_t s)
{
    const SinglePass sp = {b.sp_part};
    hipLaunchKernelGGL(single_pass_merge_kernel, dim3(packed_tiles(sl), g.B * g.Hkv), dim3(kBN), 0, s, g, sl, Q, max_chunk, b.vt_tiles, sp,
                       decay, b.mu, b.mu_chunk);
}

void launch_attn_stream(const Geom& g, const DevBuffers& b, const SegList& sl, int Q, const void* q, float qscale,
                        int tail_rows, int max_chunk, void* out, bool single_pass, hipStream_t s)
{
    const ScoreOffsets so = {b.wrow, b.negt, tail_rows, max_chunk + kScorePadRows};
    const SinglePass sp = {b.sp_part};
    const int tiles_per_bh = b.vt_tiles;   // stride between the packed streams of two (batch, KV head)
    constexpr int BM = kSWaves * 32;
    const int tiles = (g.G * Q + BM - 1) / BM;
    const int n_split = attn_splits(g, Q, b.opt_attn_splits);
    const dim3 grid(tiles * g.B * g.Hkv * n_split), block(kSWaves * 64);
    if (n_split > 1) {
        float* part_o = b.attn_part;
        float* part_ml = b.attn_part + (size_t)kAttnPartRows * g.d;
        if (g.d == 128) {
            hipLaunchKernelGGL((attn_stream_kernel<128, false, true>), grid, block, 0, s, g, sl, Q, tiles_per_bh, (const bf16_t*)q, (const float4*)b.rope_t, b.rope_rows, qscale,
                               (const bf16_t*)b.Kt, (const bf16_t*)b.Vt, (bf16_t*)out, b.lse, (long long*)nullptr, n_split, part_o, part_ml, b.knorm2, so, sp);
            hipLaunchKernelGGL(attn_merge_kernel<128>, dim3(g.G * Q, g.B * g.Hkv), dim3(128), 0, s, g, Q, tiles, n_split, BM,
                               part_o, part_ml, (bf16_t*)out, b.lse, so);
        } else {
            hipLaunchKernelGGL((attn_stream_kernel<64, false, true>), grid, block, 0, s, g, sl, Q, tiles_per_bh, (const bf16_t*)q, (const float4*)b.rope_t, b.rope_rows, qscale,
                               (const bf16_t*)b.Kt, (const bf16_t*)b.Vt, (bf16_t*)out, b.lse, (long long*)nullptr, n_split, part_o, part_ml, b.knorm2, so, sp);
            hipLaunchKernelGGL(attn_merge_kernel<64>, dim3(g.G * Q, g.B * g.Hkv), dim3(64), 0, s, g, Q, tiles, n_split, BM,
                               part_o, part_ml, (bf16_t*)out, b.lse, so);
        }
        return;
    }
#ifdef CASCADE_KV_ATTN_PHASE_TIMING   // development builds only: per-phase cycle counts of one workgroup
    if (g.d == 128) {
        long long* dbg = (long long*)b.logits;
        if (single_pass)
            hipLaunchKernelGGL((attn_stream_kernel<128, true, false, true>), grid, block, 0, s, g, sl, Q, tiles_per_bh, (const bf16_t*)q, (const float4*)b.rope_t, b.rope_rows, qscale,
                               (const bf16_t*)b.Kt, (const bf16_t*)b.Vt, (bf16_t*)out, b.lse, dbg, 1, (float*)nullptr, (float*)nullptr, b.knorm2, so, sp);
        else
            hipLaunchKernelGGL((attn_stream_kernel<128, true, false>), grid, block, 0, s, g, sl, Q, tiles_per_bh, (const bf16_t*)q, (const float4*)b.rope_t, b.rope_rows, qscale,
                               (const bf16_t*)b.Kt, (const bf16_t*)b.Vt, (bf16_t*)out, b.lse, dbg, 1, (float*)nullptr, (float*)nullptr, b.knorm2, so, sp);
        long long h[16];
        (void)hipStreamSynchronize(s);
        (void)hipMemcpy(h, dbg, sizeof(h), hipMemcpyDeviceToHost);
        for (int w = 0; w < 2; ++w)
            if (h[w * 8 + 5] > 0)
                printf("wave %d tiles %lld: top %lld mfma %lld wait1 %lld valu %lld wait2 %lld\n", w * 4, h[w * 8 + 5], h[w * 8 + 0] / h[w * 8 + 5],
                       h[w * 8 + 1] / h[w * 8 + 5], h[w * 8 + 2] / h[w * 8 + 5], h[w * 8 + 3] / h[w * 8 + 5], h[w * 8 + 4] / h[w * 8 + 5]);
        return;
    }
#endif
    if (single_pass) {      // (the caller has checked attn_single_pass_ok)
        if (g.d == 128)
            hipLaunchKernelGGL((attn_stream_kernel<128, false, false, true>), grid, block, 0, s, g, sl, Q, tiles_per_bh, (const bf16_t*)q, (const float4*)b.rope_t, b.rope_rows, qscale,
                               (const bf16_t*)b.Kt, (const bf16_t*)b.Vt, (bf16_t*)out, b.lse, (long long*)nullptr, 1, (float*)nullptr, (float*)nullptr, b.knorm2, so, sp);
        else
            hipLaunchKernelGGL((attn_stream_kernel<64, false, false, true>), grid, block, 0, s, g, sl, Q, tiles_per_bh, (const bf16_t*)q, (const float4*)b.rope_t, b.rope_rows, qscale,
                               (const bf16_t*)b.Kt, (const bf16_t*)b.Vt, (bf16_t*)out, b.lse, (long long*)nullptr, 1, (float*)nullptr, (float*)nullptr, b.knorm2, so, sp);
        return;
    }
    if (g.d == 128)
        hipLaunchKernelGGL((attn_stream_kernel<128, false, false>), grid, block, 0, s, g, sl, Q, tiles_per_bh, (const bf16_t*)q, (const float4*)b.rope_t, b.rope_rows, qscale,
                           (const bf16_t*)b.Kt, (const bf16_t*)b.Vt, (bf16_t*)out, b.lse, (long long*)nullptr, 1, (float*)nullptr, (float*)nullptr, b.knorm2, so, sp);
    else
        hipLaunchKernelGGL((attn_stream_kernel<64, false, false>), grid, block, 0, s, g, sl, Q, tiles_per_bh, (const bf16_t*)q, (const float4*)b.rope_t, b.rope_rows, qscale,
                           (const bf16_t*)b.Kt, (const bf16_t*)b.Vt, (bf16_t*)out, b.lse, (long long*)nullptr, 1, (float*)nullptr, (float*)nullptr, b.knorm2, so, sp);
}

}  // namespace ckv
