// Host-side structure of the cascade update and of the attention segments.
#include "structure.h"

#include <math.h>
#include <string.h>

#include <algorithm>

namespace ckv {

static thread_local std::string g_init_error;
void set_init_error(const std::string& msg) { g_init_error = msg; }
const char* init_error() { return g_init_error.c_str(); }

// ------------------------------------------------------------------ configuration

int check_config(const cascade_config* c, std::string& why)
{
    if (c->batch < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1) { why = "batch and head counts must be positive"; return CASCADE_E_INVALID_CONFIG; }
    if (c->n_q_heads % c->n_kv_heads) { why = "n_q_heads must be a multiple of n_kv_heads"; return CASCADE_E_INVALID_CONFIG; }
    if (c->dtype != CASCADE_F32 && c->dtype != CASCADE_BF16) { why = "dtype must be CASCADE_F32 or CASCADE_BF16"; return CASCADE_E_INVALID_CONFIG; }
    if (c->head_dim < 2 || c->head_dim % 2) { why = "head_dim must be even"; return CASCADE_E_INVALID_CONFIG; }
    if (c->n_sink < 0) { why = "n_sink must not be negative"; return CASCADE_E_INVALID_CONFIG; }
    if (c->n_cascades < 1 || c->n_cascades > CASCADE_MAX_CASCADES) { why = "n_cascades out of range"; return CASCADE_E_INVALID_CONFIG; }
    bool all_zero = true;
    for (int i = 0; i < c->n_cascades; ++i) {
        if (c->cascade_sizes[i] < 1) { why = "every cascade needs at least one slot"; return CASCADE_E_INVALID_CONFIG; }
        if (c->accept_period[i] < 0) { why = "accept_period must not be negative"; return CASCADE_E_INVALID_CONFIG; }
        if (c->accept_period[i] != 0) all_zero = false;
    }
    if (!all_zero) {
        if (c->accept_period[0] != 1) { why = "the first cascade must accept every token (accept_period[0] == 1)"; return CASCADE_E_INVALID_CONFIG; }
        for (int i = 0; i < c->n_cascades; ++i)
            if (c->accept_period[i] < 1) { why = "accept_period entries must be >= 1"; return CASCADE_E_INVALID_CONFIG; }
    }
    if (!(c->ema_beta >= 0.f && c->ema_beta < 1.f)) { why = "ema_beta must be in [0, 1)"; return CASCADE_E_INVALID_CONFIG; }
    if (!(c->rope_base > 0.f)) { why = "rope_base must be positive"; return CASCADE_E_INVALID_CONFIG; }
    if (c->softmax_scale < 0.f) { why = "softmax_scale must not be negative"; return CASCADE_E_INVALID_CONFIG; }
    if (c->max_chunk < 1) { why = "max_chunk must be >= 1"; return CASCADE_E_INVALID_CONFIG; }
    if (c->head_reduce != CASCADE_REDUCE_MAX && c->head_reduce != CASCADE_REDUCE_MEAN) { why = "unknown head_reduce"; return CASCADE_E_INVALID_CONFIG; }
    if (c->token_selection != 0 && c->token_selection != 1) { why = "token_selection must be 0 or 1"; return CASCADE_E_INVALID_CONFIG; }
    if (c->head_policy != CASCADE_HEADS_INDEPENDENT && c->head_policy != CASCADE_HEADS_HOMOGENEOUS) { why = "unknown head_policy"; return CASCADE_E_INVALID_CONFIG; }
    if (c->score_mode != CASCADE_SCORES_EXACT && c->score_mode != CASCADE_SCORES_SINGLE_PASS) { why = "unknown score_mode"; return CASCADE_E_INVALID_CONFIG; }
    if (c->score_mode == CASCADE_SCORES_SINGLE_PASS && c->dtype != CASCADE_BF16) { why = "single-pass scores need dtype CASCADE_BF16"; return CASCADE_E_UNSUPPORTED; }
    long slots = c->n_sink;
    for (int i = 0; i < c->n_cascades; ++i) slots += c->cascade_sizes[i];
    if (slots > (1L << 28)) { why = "cache too large"; return CASCADE_E_INVALID_CONFIG; }
    if (c->dtype == CASCADE_BF16 && c->head_dim != 64 && c->head_dim != 128) { why = "bf16 kernels cover head_dim 64 and 128"; return CASCADE_E_UNSUPPORTED; }
    if (c->dtype == CASCADE_F32 && c->head_dim > 256) { why = "fp32 kernels cover head_dim up to 256"; return CASCADE_E_UNSUPPORTED; }
    return CASCADE_OK;
}

void make_geom(const cascade_config* c, Geom& g)
{
    memset(&g, 0, sizeof(g));
    g.B = c->batch; g.Hq = c->n_q_heads; g.Hkv = c->n_kv_heads; g.G = g.Hq / g.Hkv; g.d = c->head_dim;
    g.n_sink = c->n_sink; g.N = c->n_cascades;
    bool all_zero = true;
    for (int i = 0; i < g.N; ++i) if (c->accept_period[i] != 0) all_zero = false;
    int slots = g.n_sink;
    for (int i = 0; i < g.N; ++i) {
        g.cap[i] = c->cascade_sizes[i];
        g.period[i] = all_zero ? (1 << i) : c->accept_period[i];
        slots += g.cap[i];
    }
    g.slots = slots;
    int base = g.n_sink;                       // physical order: sinks, last cascade, ..., first cascade
    for (int i = g.N - 1; i >= 0; --i) { g.base[i] = base; base += g.cap[i]; }
    g.token_selection = c->token_selection;
    g.head_reduce = c->head_reduce;
    g.head_policy = c->head_policy;
    g.beta = c->ema_beta;
    g.scale = c->softmax_scale > 0.f ? c->softmax_scale : (float)(1.0 / sqrt((double)g.d));
}


static int64_t gcd64(int64_t a, int64_t b)
{
    while (b) { int64_t r = a % b; a = b; b = r; }
    return a;
}

// Alg. 2 applied to Q tokens in order, scores aside.  The items offered to cascade c arrive
// at times tau_k = first + k*step (an arithmetic progression: cascade c-1 only evicts at its
// own accepting times once it is full).  Offer k is
//   APPEND  while the cascade is not full (accepting or eager add),
//   PUSH    when full and tau_k mod period == 0 (the oldest item moves on to cascade c+1),
//   SELECT  when full otherwise (competes with the newest item, one of the two is lost).
void plan_update(const Geom& g, HostState& st, int Q, UpdatePlan& plan)
{
    plan.Q = Q;
    plan.N = g.N;
    plan.sink_fill0 = st.sink_fill;
    plan.n_to_sink = std::min(Q, g.n_sink - st.sink_fill);
    plan.id0 = (int)st.n_seen;
    const int Qc = Q - plan.n_to_sink;

    int64_t first = st.t, step = 1;
    int M = Qc;
    for (int c = 0; c < g.N; ++c) {
        CascStep& cs = plan.c[c];
        const int cap = g.cap[c];
        const int64_t f = g.period[c];
        const bool full0 = st.count[c] == cap;
        cs.cap = cap;
        cs.base = g.base[c];
        cs.M = M;
        cs.A = std::min(M, cap - st.count[c]);
        cs.pstride = (int)(f / gcd64(step, f));
        // offers at accepting times are k = ka + i*pstride for the smallest such ka >= 0
        int ka = -1;
        for (int k = 0; k < cs.pstride && k < M; ++k)
            if ((first + (int64_t)k * step) % f == 0) { ka = k; break; }
        cs.kp0 = M;
        cs.P = 0;
        if (ka >= 0) {
            st.accepted[c] += (M - 1 - ka) / cs.pstride + 1;
            int k = ka;
            if (k < cs.A) k += ((cs.A - k + cs.pstride - 1) / cs.pstride) * cs.pstride;
            if (k < M) { cs.kp0 = k; cs.P = (M - 1 - k) / cs.pstride + 1; }
        }
        cs.J = cs.A + cs.P;
        cs.wpos0 = full0 ? st.xi[c] : st.count[c];
        cs.newest0 = full0 ? (st.xi[c] + cap - 1) % cap : 0;
        cs.pre = (full0 && M > 0 && cs.kp0 > 0) ? 1 : 0;

        st.discards[c] += M - cs.A - cs.P;              // every SELECT loses one item
        if (c == g.N - 1) st.discards[c] += cs.P;       // evicted from the last cascade
        st.count[c] += cs.A;
        if (st.count[c] == cap) st.xi[c] = (int)(((int64_t)(full0 ? st.xi[c] : 0) + cs.P) % cap);

        if (cs.P > 0) { first += (int64_t)cs.kp0 * step; step *= cs.pstride; }
        M = cs.P;
    }
    st.t += Qc;
    st.n_seen += Q;
    st.sink_fill += plan.n_to_sink;
}

// Cache order is sinks, last cascade oldest..newest, ..., first cascade (Section 3.1
// "Positional Encoding": the index inside the cache).  Stored keys are rotated to their
// physical slot index, so within a run where (cache index - slot index) is constant the
// queries need one rotation: by (own index) - (that constant).  The segments are listed in
// physical order (the wrapped part of a ring before its oldest part): attention does not care
// in which order it meets the keys, and a full cache then always reads front to back.  The
// wrapped part of a full ring is listed as [0, o) and [o, xi), o = xi mod 64, which fixes the
// place of every 64-row tile of the ring (see PackedLayout).
void build_segments(const Geom& g, const HostState& st, bool with_chunk, int Q, SegList& out)
{
    out.n = 0;
    out.n_qvar = 0;
    const int n = st.n_cached(g);
    out.n_cached = n;
    auto add = [&](int start, int len, int delta, int chunk) {
        if (len <= 0) return;
        const int rot0 = n - delta;
        int v = -1;
        for (int i = 0; i < out.n_qvar; ++i) if (out.qrot0[i] == rot0) v = i;
        if (v < 0) { v = out.n_qvar++; out.qrot0[v] = rot0; }
        Seg& s = out.s[out.n++];
        s.start = start; s.len = len; s.qvar = v; s.chunk = chunk;
    };
    add(0, st.sink_fill, 0, 0);
    int rank = st.sink_fill;                         // cache index of the oldest item of the cascade
    for (int c = g.N - 1; c >= 0; --c) {
        const int cnt = st.count[c], cap = g.cap[c], xi = st.xi[c], base = g.base[c];
        if (cnt < cap) {
            add(base, cnt, rank - base, 0);
        } else {
            const int o = xi % 64, wrapped = rank + (cap - xi) - base;
            add(base, o, wrapped, 0);                                 // wrapped part: ring [0, xi), in two pieces
            add(base + o, xi - o, wrapped, 0);
            add(base + xi, cap - xi, rank - (base + xi), 0);          // oldest part: ring [xi, cap)
        }
        rank += cnt;
    }
    if (with_chunk) add(0, Q, n, 1);                 // chunk key i is rotated to i and sits at n + i
}

void packed_layout(const Geom& g, const HostState& st, PackedLayout& out)
{
    out.full = st.sink_fill == g.n_sink;
    int tiles = (g.n_sink + 63) / 64;
    for (int c = g.N - 1; c >= 0; --c) {             // physical order: the last cascade first
        if (st.count[c] != g.cap[c]) out.full = false;
        const int o = st.xi[c] % 64;
        out.off[c] = o;
        out.tile0[c] = tiles;
        tiles += (o > 0 ? 1 : 0) + (g.cap[c] - o + 63) / 64;
    }
    out.cache_tiles = tiles;
}

bool same_offsets(const Geom& g, const PackedLayout& a, const PackedLayout& b)
{
    for (int c = 0; c < g.N; ++c) if (a.off[c] != b.off[c]) return false;
    return true;
}

static int tile_of_slot(const Geom& g, const PackedLayout& lay, int slot)
{
    if (slot < g.n_sink) return slot / 64;
    for (int c = 0; c < g.N; ++c) {
        const int r = slot - g.base[c];
        if (r < 0 || r >= g.cap[c]) continue;
        const int o = lay.off[c];
        return lay.tile0[c] + (r < o ? 0 : (o > 0 ? 1 : 0) + (r - o) / 64);
    }
    return -1;
}

int touched_slot_runs(const Geom& g, const UpdatePlan& pl, int* lo, int* hi)
{
    int n = 0;
    if (pl.n_to_sink > 0) { lo[n] = pl.sink_fill0; hi[n] = pl.sink_fill0 + pl.n_to_sink; ++n; }
    for (int c = 0; c < pl.N; ++c) {
        const CascStep& cs = pl.c[c];
        if (cs.M == 0) break;
        // ring positions wpos0 .. wpos0 + J - 1 are opened; before the first push the offers
        // compete with the item at newest0 = wpos0 - 1
        const int len = cs.J + cs.pre;
        if (len == 0) continue;
        if (len >= cs.cap) { lo[n] = cs.base; hi[n] = cs.base + cs.cap; ++n; continue; }
        const int start = cs.pre ? cs.newest0 : cs.wpos0;
        const int end = start + len;
        if (end <= cs.cap) { lo[n] = cs.base + start; hi[n] = cs.base + end; ++n; }
        else {
            lo[n] = cs.base + start; hi[n] = cs.base + cs.cap; ++n;
            lo[n] = cs.base; hi[n] = cs.base + end - cs.cap; ++n;
        }
    }
    return n;
}

bool add_tile_run(TileRuns& runs, int first, int count)
{
    if (count <= 0) return true;
    if (runs.n == kMaxTileRuns) return false;
    runs.first[runs.n] = first;
    runs.ahead[runs.n] = runs.total;
    runs.total += count;
    ++runs.n;
    return true;
}

bool add_touched_tiles(const Geom& g, const PackedLayout& layout, const UpdatePlan& pl, TileRuns& runs)
{
    int lo[kMaxTileRuns], hi[kMaxTileRuns];
    const int n = touched_slot_runs(g, pl, lo, hi);
    for (int i = 0; i < n; ++i) {                    // a run lies inside one ring: its tiles are consecutive
        const int t0 = tile_of_slot(g, layout, lo[i]), t1 = tile_of_slot(g, layout, hi[i] - 1);
        if (t0 < 0 || t1 < t0 || !add_tile_run(runs, t0, t1 - t0 + 1)) return false;
    }
    return true;
}

int slot_of_rank(const Geom& g, const HostState& st, int r)
{
    if (r < st.sink_fill) return r;
    r -= st.sink_fill;
    for (int c = g.N - 1; c >= 0; --c) {
        const int cnt = st.count[c];
        if (r < cnt) return g.base[c] + (cnt < g.cap[c] ? r : (st.xi[c] + r) % g.cap[c]);
        r -= cnt;
    }
    return -1;
}

}  // namespace ckv
