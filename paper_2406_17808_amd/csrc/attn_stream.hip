// bf16 chunk attention of the strided prefill (Alg. 1, Fig. 4; online softmax of Eq. 2).
//
// kv_pack_kernel, once per chunk: the keys and values the chunk attends to (cache segments, then
// the chunk itself) are copied tile after tile (64 keys) in the order the attention kernel
// visits them.  A packed tile is the exact LDS image the attention kernel wants: K with the
// 16-byte chunks of a row XOR-swizzled, V transposed (a row is one column of V with its 64 keys),
// so that the A operand of O^T = V^T P^T is a plain 16-byte LDS read.  The attention kernel then
// needs no segment logic for its loads.
//
// attn_stream_kernel: a workgroup of eight waves owns 256 query rows, 32 per wave (one lane owns
// one query: the transposed formulation described in mfma_util.h).  Packed tiles go from global
// memory straight into LDS by asynchronous loads, four buffers deep.  Per tile a wave alternates
// between a matrix block (O^T += V^T P^T of tile t, then S^T = K Q^T of tile t+1: MFMAs and LDS
// reads only) and a vector block (mask, maximum, exponentials of tile t+1).  The two waves of a
// SIMD run these blocks in opposite phase, held there by two barriers per tile, so the matrix
// pipe and the vector ALU of the SIMD work at the same time.
#include <stdio.h>
#include <stdlib.h>

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
__global__ __launch_bounds__(kPackThreads) void kv_pack_kernel(Geom g, SegList sl, int Q, int tiles_per_bh,
                                                               const bf16_t* __restrict__ Kr, const bf16_t* __restrict__ Krc,
                                                               const bf16_t* __restrict__ Vc, const bf16_t* __restrict__ Vch,
                                                               bf16_t* __restrict__ Kt, bf16_t* __restrict__ Vt)
{
    constexpr int STR = D + 8;   // LDS row stride in elements: 16-byte aligned rows
    __shared__ __attribute__((aligned(16))) bf16_t T[kBN * STR];
    const int BH = g.B * g.Hkv;
    const int bh = blockIdx.x % BH, n = blockIdx.x / BH;
    int si = 0, first = 0;
    for (; si < sl.n; ++si) {
        const int nt = (sl.s[si].len + kBN - 1) / kBN;
        if (n < first + nt) break;
        first += nt;
    }
    if (si >= sl.n) return;   // cannot happen: the grid has one workgroup per tile
    const Seg sg = sl.s[si];
    const int t0 = (n - first) * kBN, rows = min(kBN, sg.len - t0);
    const size_t row0 = sg.chunk ? ((size_t)bh * Q + t0) : ((size_t)bh * g.slots + sg.start + t0);
    const bf16_t* src = (sg.chunk ? Vch : Vc) + row0 * D;
    const bf16_t* ksrc = (sg.chunk ? Krc : Kr) + row0 * D;
    bf16_t* kdst = Kt + ((size_t)bh * tiles_per_bh + n) * (kBN * D);
    const int tid = threadIdx.x;
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
    }
    __syncthreads();
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

template <int D, bool DBG>
__global__ __launch_bounds__(kSWaves * 64, 1) void attn_stream_kernel(
    Geom g, SegList sl, int Q, int tiles_per_bh, const bf16_t* __restrict__ Qr, const bf16_t* __restrict__ Kt,
    const bf16_t* __restrict__ Vt, bf16_t* __restrict__ out, float* __restrict__ lse, long long* dbg)
{
    constexpr int BM = kSWaves * 32;       // query rows per workgroup
    constexpr int KS = D / 16;             // k-steps of S^T = K Q^T
    constexpr int DB = D / 32;             // 32-wide blocks of the head dimension in O^T
    constexpr int CH = Swz<D>::CH;
    constexpr int TILE = kBN * D;          // elements per LDS tile
    constexpr int PW = CH / kSWaves;       // 1 KB copies per wave and tile (2 or 1)
    __shared__ __attribute__((aligned(1024))) bf16_t Ks[kSStages * TILE];
    __shared__ __attribute__((aligned(1024))) bf16_t Vs[kSStages * TILE];

    const int BH = g.B * g.Hkv;
    // consecutive workgroups: different KV heads; row blocks that see more of the chunk (longer loops) start first
    const int bh = blockIdx.x % BH, tile = (int)(gridDim.x / BH) - 1 - (int)(blockIdx.x / BH);
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
    float lsum = 0.f;   // this lane's part of the row sum

    // The packed tiles are LDS images: every wave copies PW consecutive KB of each
    const uint32_t lds_k = lds_address(Ks) + (uint32_t)wave * PW * 1024u;
    const uint32_t lds_v = lds_address(Vs) + (uint32_t)wave * PW * 1024u;
    const bf16_t* kt_bh = Kt + (size_t)bh * tiles_per_bh * TILE + (size_t)wave * PW * 512;
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

    Frag qf[KS];
    auto load_q = [&](const Seg& sg) {   // this segment's rotated copy of the queries
        const bf16_t* qrow = Qr + ((((size_t)sg.qvar * g.B + b) * g.Hq + qh) * Q + qi) * D + half * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[ks].u = *reinterpret_cast<const u32x4_t*>(qrow + ks * 16);
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
    // The vector block of one tile: mask the keys a query may not see (past the end of the
    // segment; later chunk tokens), take the row maximum of S^T (relative to m_run), raise m_run only
    // when that exceeds kRescaleLog2 (the probabilities then stay below 2^kRescaleLog2, and most
    // tiles skip the rescaling of O), and turn S^T into probabilities.  FIRST: S^T is absolute
    // and m_run not set yet (the first tile of a workgroup).
    auto softmax_tile = [&](const TileIter& it, bool first) {
        if ((it.t0 + kBN > it.sg.len) || (it.sg.chunk && it.t0 + kBN - 1 > wave_imin)) {
            const int lim = it.sg.chunk ? min(it.sg.len - 1, qi) : it.sg.len - 1;   // last visible key
            const int rel = lim - it.t0 - half * 4;   // accumulator j of block kb is key t0 + 4*half + (32 kb + 8 (j/4) + j%4)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int j = 0; j < 16; ++j)
                    if (kb * 32 + (j >> 2) * 8 + (j & 3) > rel) s[kb][j] = -INFINITY;
        }
        float x = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int j = 0; j < 16; ++j) x = fmaxf(x, s[kb][j]);
        const float mt = max_xor32(x);
        const bool grow = first || mt > kRescaleLog2;
        if (__any(grow)) {
            const float delta = grow ? mt : 0.f;   // every row sees a key of the first tile: finite there
            const float alpha = first ? 1.f : __builtin_amdgcn_exp2f(-delta);   // O and the row sum are still zero on the first tile
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
    };
    auto wave_active = [&](const TileIter& it) { return !(it.sg.chunk && it.t0 > wave_imax); };

    // In iteration t, tile t is multiplied with V, tile t+1 with Q; the copies of V of tile t+2
    // and of K of tile t+3 are issued.  Only the softmax needs to know which segment a tile is from.
    int NT = 0;   // tiles this workgroup visits: chunk keys after its last row are never visible
    for (int i = 0; i < sl.n; ++i) NT += ((sl.s[i].chunk ? min(sl.s[i].len, wg_imax + 1) : sl.s[i].len) + kBN - 1) / kBN;
    TileIter it1;
    it1.first(sl, wg_imax);
    if (!it1.valid(sl)) return;          // cannot happen: the chunk itself is always a segment

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
    int q_seg = it1.si;
    wait_vm<0>();
    __syncthreads();
    qk_tile(Ks);
    softmax_tile(it1, true);    // every wave sees the first tile
    it1.next(sl, wg_imax);
    __syncthreads();      // barrier 0: every wave has read K of tile 0, its buffer may be refilled
#pragma unroll
    for (int i = 0; i < kAhead; ++i) fr[i] = read_frag(Vs, Ks, i);
    if (late) wg_barrier();     // barrier 1

    int n0 = 0;   // t
    long long tc[5] = {0, 0, 0, 0, 0}, tlast = 0;
    if (DBG) tlast = __builtin_readcyclecounter();
    auto lap = [&](int i) { if (DBG) { const long long now = __builtin_readcyclecounter(); tc[i] += now - tlast; tlast = now; } };
    while (true) {
        const bool has_next = n0 + 1 < NT;
        const bool act_next = has_next && wave_active(it1);
        if (act_next && q_seg != it1.si) {
            load_q(it1.sg);
            q_seg = it1.si;
            wait_vm<0>();   // here, so that no wait for these loads is placed among the MFMAs (it would also wait for the copies)
        }
        // ---- matrix block.  A wave that does not see tile t holds zero probabilities; S^T of a
        // tile this wave does not see (or that does not exist: stale buffer) is computed and
        // dropped.  The order of MFMAs and reads is pinned step by step.
        lap(0);
        __builtin_amdgcn_s_setprio(2);
        __builtin_amdgcn_sched_barrier(0);
        {
            const bf16_t* Vtile = Vs + (n0 & 3) * TILE;
            const bf16_t* Ktile = Ks + ((n0 + 1) & 3) * TILE;
#pragma unroll
            for (int i = 0; i < NF; ++i) {
                if (i < NV) o[i % DB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[i % kAhead].v, pf[i / DB].v, o[i % DB], 0, 0, 0);
                else s[(i - NV) % 2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[i % kAhead].v, qf[(i - NV) / 2].v, i - NV < 2 ? negm : s[(i - NV) % 2], 0, 0, 0);
                if (i + kAhead < NF) fr[i % kAhead] = read_frag(Vtile, Ktile, i + kAhead);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_setprio(0);
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
            softmax_tile(it1, false);
        } else {
#pragma unroll
            for (int qt = 0; qt < 4; ++qt)
#pragma unroll
                for (int x = 0; x < 4; ++x) pf[qt].u[x] = 0u;
        }
        lap(3);
        publish(in_flight);
        wg_barrier();     // barrier 2t+2 (early group), 2t+3 (late group)
        lap(4);
        it1.next(sl, wg_imax);
        ++n0;
    }
    if (!late) wg_barrier();   // the late group passed one barrier more
    if (DBG && blockIdx.x == 100 && l == 0 && (wave == 0 || wave == 4)) {
#pragma unroll
        for (int i = 0; i < 5; ++i) dbg[(wave / 4) * 8 + i] = tc[i];
        dbg[(wave / 4) * 8 + 5] = n0 + 1;
    }
    // normalise and store: this lane owns one query, columns 32*db + 8*(j/4) + 4*half + j%4
    const float lt = lsum + __shfl_xor(lsum, 32, 64);
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
        if (half == 0) lse[((size_t)b * g.Hq + qh) * Q + qi] = m_run * 0.6931471805599453f + logf(lt);
    }
}

// tiles of the packed V copy one (batch, KV head) needs for this segment list
static int packed_tiles(const SegList& sl)
{
    int n = 0;
    for (int i = 0; i < sl.n; ++i) n += (sl.s[i].len + kBN - 1) / kBN;
    return n;
}

bool launch_kv_pack(const Geom& g, const DevBuffers& b, const SegList& sl, int Q, hipStream_t s)
{
    const int tiles_per_bh = packed_tiles(sl);
    if (tiles_per_bh > b.vt_tiles) return false;   // the workspace was sized for every possible segment list
    const dim3 grid(tiles_per_bh * g.B * g.Hkv), block(kPackThreads);
    if (g.d == 128)
        hipLaunchKernelGGL(kv_pack_kernel<128>, grid, block, 0, s, g, sl, Q, tiles_per_bh, (const bf16_t*)b.Kr, (const bf16_t*)b.Krc,
                           (const bf16_t*)b.Vc, (const bf16_t*)b.Vch, (bf16_t*)b.Kt, (bf16_t*)b.Vt);
    else
        hipLaunchKernelGGL(kv_pack_kernel<64>, grid, block, 0, s, g, sl, Q, tiles_per_bh, (const bf16_t*)b.Kr, (const bf16_t*)b.Krc,
                           (const bf16_t*)b.Vc, (const bf16_t*)b.Vch, (bf16_t*)b.Kt, (bf16_t*)b.Vt);
    return true;
}

void launch_attn_stream(const Geom& g, const DevBuffers& b, const SegList& sl, int Q, void* out, hipStream_t s)
{
    const int tiles_per_bh = packed_tiles(sl);
    constexpr int BM = kSWaves * 32;
    const int tiles = (g.G * Q + BM - 1) / BM;
    const dim3 grid(tiles * g.B * g.Hkv), block(kSWaves * 64);
    static const char* dbg_env = getenv("CASCADE_KV_ATTN_DEBUG");
    if (dbg_env && g.d == 128) {   // phase timing of one workgroup (development aid)
        long long* dbg = (long long*)b.logits;
        hipLaunchKernelGGL((attn_stream_kernel<128, true>), grid, block, 0, s, g, sl, Q, tiles_per_bh, (const bf16_t*)b.Qr,
                           (const bf16_t*)b.Kt, (const bf16_t*)b.Vt, (bf16_t*)out, b.lse, dbg);
        long long h[16];
        (void)hipStreamSynchronize(s);
        (void)hipMemcpy(h, dbg, sizeof(h), hipMemcpyDeviceToHost);
        for (int w = 0; w < 2; ++w)
            if (h[w * 8 + 5] > 0)
                printf("wave %d tiles %lld: top %lld mfma %lld wait1 %lld valu %lld wait2 %lld\n", w * 4, h[w * 8 + 5], h[w * 8 + 0] / h[w * 8 + 5],
                       h[w * 8 + 1] / h[w * 8 + 5], h[w * 8 + 2] / h[w * 8 + 5], h[w * 8 + 3] / h[w * 8 + 5], h[w * 8 + 4] / h[w * 8 + 5]);
        return;
    }
    if (g.d == 128)
        hipLaunchKernelGGL((attn_stream_kernel<128, false>), grid, block, 0, s, g, sl, Q, tiles_per_bh, (const bf16_t*)b.Qr,
                           (const bf16_t*)b.Kt, (const bf16_t*)b.Vt, (bf16_t*)out, b.lse, (long long*)nullptr);
    else
        hipLaunchKernelGGL((attn_stream_kernel<64, false>), grid, block, 0, s, g, sl, Q, tiles_per_bh, (const bf16_t*)b.Qr,
                           (const bf16_t*)b.Kt, (const bf16_t*)b.Vt, (bf16_t*)out, b.lse, (long long*)nullptr);
}

}  // namespace ckv
