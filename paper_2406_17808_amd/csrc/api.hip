// Host side of the C ABI declared in include/cascade_kv.h: validation, workspace layout, the
// score-independent mirror of the cache structure, and the kernel sequence of every call.
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <string>
#include <vector>

#include "launch.h"
#include "plan_core.h"
#include "structure.h"

using namespace ckv;

struct cascade_ctx {
    cascade_config cfg;
    Geom g;
    HostState st;
    HostState st_prev;   // structure before the last call (for the diagnostic score snapshot)
    int last_tokens = 0;
    DevBuffers buf;
    int dtype;
    size_t elem;
    int max_chunk;
    int tail_k;          // rows of a chunk (counted from its end) that enter the score sums
    bool mfma;
    // bf16 path: Kt / Vt / Knorm2 belong to this context alone (not shared between layers), and, if
    // packed_valid, hold every cache tile where `packed` puts it, except those named by `stale`.
    // packed_reuse: tiles that are still valid are not packed again.
    bool packed_own = true;
    bool packed_reuse = true;
    bool packed_valid = false;
    PackedLayout packed;
    TileRuns stale;
    bool profiling = false;
    uint32_t prof_mask = ~0u;   // kernel families that get events while profiling
    bool is_static = false;   // one of the per-device contexts of cascade_init_static: never deleted
    bool poisoned = false;    // a launch of an earlier call failed: the device state is undefined
    bool last_single_pass = false;   // the last prefill call took the single-pass scores
    std::vector<std::pair<hipEvent_t, hipEvent_t>> prof[CASCADE_K_FAMILIES];
    std::string err;
};

// Brackets the launches of one kernel family with two events when profiling is on.
struct Timed {
    cascade_ctx* ctx;
    int fam;
    hipStream_t s;
    hipEvent_t stop = nullptr;
    Timed(cascade_ctx* c, int f, hipStream_t st) : ctx(c), fam(f), s(st)
    {
        if (!ctx->profiling || !(ctx->prof_mask >> fam & 1u)) return;
        hipEvent_t start;
        if (hipEventCreate(&start) != hipSuccess || hipEventCreate(&stop) != hipSuccess) { stop = nullptr; return; }
        (void)hipEventRecord(start, s);
        ctx->prof[fam].push_back({start, stop});
    }
    ~Timed() { if (stop) (void)hipEventRecord(stop, s); }
};

static int fail(cascade_ctx* ctx, int code, const std::string& msg)
{
    if (ctx) ctx->err = msg;
    else set_init_error(msg);
    return code;
}

static size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

static int decode_splits(const Geom& g)
{
    // enough workgroups to fill 256 compute units several times over, at least 256 rows each
    int s = (2048 + g.B * g.Hkv - 1) / (g.B * g.Hkv);
    const int max_s = (g.slots + 255) / 256;
    if (s > max_s) s = max_s;
    if (s < 1) s = 1;
    return s;
}

// Workspace layout in two regions: the state of one layer (the cache itself) and the buffers
// that live only inside one call (plus the two tables, which depend on the configuration
// alone), which several layers may share.  With null bases only the sizes are computed.
struct WorkspaceBytes {
    size_t state, shared;
};

static WorkspaceBytes carve(const cascade_config* c, const Geom& g, char* state_base, char* shared_base, DevBuffers* out)
{
    const size_t elem = c->dtype == CASCADE_BF16 ? 2 : 4;
    const size_t BH = (size_t)g.B * g.Hkv, BHq = (size_t)g.B * g.Hq;
    const size_t mc = (size_t)c->max_chunk;
    const int n_qvar_max = 2 * g.N + 2;
    const int splits = decode_splits(g);
    const int rope_rows = 2 * g.slots + c->max_chunk + 1;
    size_t off = 0;
    char* base = state_base;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return base ? (void*)(base + o) : (void*)nullptr; };
    DevBuffers b;
    memset(&b, 0, sizeof(b));
    b.Kc = take(BH * g.slots * g.d * elem);
    b.Kr = take(BH * g.slots * g.d * elem);
    b.Vc = take(BH * g.slots * g.d * elem);
    b.mu = (float*)take(BH * g.slots * 4);
    b.ids = (int32_t*)take(BH * g.slots * 4);
    b.swaps = (int32_t*)take(BH * g.N * 4);
    b.mu_snap = (float*)take(c->keep_update_scores ? BH * g.slots * 4 : 0);
    WorkspaceBytes bytes;
    bytes.state = off;
    off = 0;
    base = shared_base;
    b.rope = (float2*)take((size_t)rope_rows * (g.d / 2) * 8);
    b.wrow = (float*)take(mc * 4);
    b.Qr = take((size_t)n_qvar_max * BHq * mc * g.d * elem);
    b.Krc = take(BH * mc * g.d * elem);
    b.Vch = take(BH * mc * g.d * elem);
    // every segment list has at most kMaxSegments segments, each ending in one partly filled tile
    const bool mfma = c->dtype == CASCADE_BF16 && (g.d == 64 || g.d == 128);
    const int vt_tiles = mfma ? (g.slots + (int)mc) / 64 + kMaxSegments : 0;
    b.Kt = take(BH * (size_t)vt_tiles * 64 * g.d * elem);
    b.Vt = take(BH * (size_t)vt_tiles * 64 * g.d * elem);
    b.knorm2 = (float*)take(BH * (size_t)vt_tiles * 4);
    b.lse = (float*)take(BHq * mc * 4);
    b.mu_chunk = (float*)take(BH * mc * 4);
    b.negt = (float*)take(mfma ? BHq * (mc + 64) * 4 : 0);
    b.rope_t = (float2*)take(mfma ? (size_t)rope_rows * (g.d / 2) * 8 : 0);
    if (!mfma) b.rope_t = nullptr;
    b.attn_part = (float*)take(mfma ? (size_t)kAttnPartRows * (g.d + 2) * 4 : 0);
    const bool single_pass = mfma && c->score_mode == CASCADE_SCORES_SINGLE_PASS;
    b.sp_part = (float*)take(single_pass ? BH * (size_t)g.G * ((mc + 255) / 256) * (size_t)vt_tiles * 64 * 4 : 0);
    if (!single_pass) b.sp_part = nullptr;
    b.offers = (int32_t*)take(BH * 2 * mc * 4);
    b.winners = (int32_t*)take(BH * g.N * (mc + 1) * 4);
    const int move_stage_rows = (g.N + 1) * ((int)mc + 1);    // every cascade and the sinks: at most max_chunk + 1 entries each
    b.move_stage = take(g.d % 16 == 0 ? BH * (size_t)move_stage_rows * (2 * g.d * elem + 8) : 0);
    b.logits = (float*)take(BH * ((size_t)g.slots + 1) * (size_t)(g.G <= 8 ? decode_logit_heads(g) : g.G) * 4);
    b.part = (float*)take(BHq * splits * 2 * 4);
    b.opart = (float*)take(BHq * splits * g.d * 4);
    bytes.shared = off;
    b.rope_rows = rope_rows;
    b.dec_splits = splits;
    b.vt_tiles = vt_tiles;
    b.move_stage_rows = move_stage_rows;
    if (out) *out = b;
    return bytes;
}

extern "C" size_t cascade_workspace_bytes(const cascade_config* cfg)
{
    if (!cfg) return 0;
    std::string why;
    if (check_config(cfg, why) != CASCADE_OK) return 0;
    Geom g;
    make_geom(cfg, g);
    const WorkspaceBytes w = carve(cfg, g, nullptr, nullptr, nullptr);
    return w.state + w.shared;
}

extern "C" size_t cascade_layers_workspace_bytes(const cascade_config* cfg, int32_t n_layers)
{
    if (!cfg || n_layers < 1) return 0;
    std::string why;
    if (check_config(cfg, why) != CASCADE_OK) return 0;
    Geom g;
    make_geom(cfg, g);
    const WorkspaceBytes w = carve(cfg, g, nullptr, nullptr, nullptr);
    return w.state * (size_t)n_layers + w.shared;
}

static int hip_check(cascade_ctx* ctx, hipError_t e, const char* what)
{
    if (e == hipSuccess) return CASCADE_OK;
    return fail(ctx, CASCADE_E_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

// ------------------------------------------------------------------ init / destroy

// Host-side check of an initial state (may be null: empty cache); fills the host mirror.
static int check_init_state(const std::string& name, const Geom& g, const cascade_init_state* init_state, HostState& st, int& total)
{
    total = 0;
    if (!init_state) return CASCADE_OK;
    if (init_state->counts[0] < 0 || init_state->counts[0] > g.n_sink)
        return fail(nullptr, CASCADE_E_BAD_ARG, name + ": sink count exceeds n_sink");
    st.sink_fill = init_state->counts[0];
    total = st.sink_fill;
    for (int c = 0; c < g.N; ++c) {
        const int cnt = init_state->counts[1 + c];
        if (cnt < 0 || cnt > g.cap[c]) return fail(nullptr, CASCADE_E_BAD_ARG, name + ": a cascade count exceeds its capacity");
        st.count[c] = cnt;
        total += cnt;
    }
    if (init_state->t < 0 || init_state->n_seen < 0 || init_state->n_seen > 0x7FFFFFFF)
        return fail(nullptr, CASCADE_E_BAD_ARG, name + ": t / n_seen out of range");
    st.t = init_state->t;
    st.n_seen = init_state->n_seen;
    if (total > 0 && (!init_state->dev_k || !init_state->dev_v || !init_state->dev_mu || !init_state->dev_ids))
        return fail(nullptr, CASCADE_E_NULL_ARG, name + ": init_state with items needs k, v, mu and ids");
    return CASCADE_OK;
}

// One context over a state region and a shared region that the caller has already zeroed;
// `tables` says whether this call fills the tables of the shared region.  st / total come from
// check_init_state.
static int init_context(const char* who, const cascade_config* cfg, const Geom& g, char* state_base, char* shared_base,
                        bool tables, const cascade_init_state* init_state, const HostState& st, int total,
                        hipStream_t s, cascade_ctx** out_ctx, cascade_ctx* into = nullptr)
{
    const std::string name = who;
    cascade_ctx* ctx = into ? into : new cascade_ctx();   // into: a context that already exists and is reset by the caller
    ctx->cfg = *cfg;
    ctx->g = g;
    ctx->st = st;
    ctx->dtype = cfg->dtype;
    ctx->elem = cfg->dtype == CASCADE_BF16 ? 2 : 4;
    ctx->max_chunk = cfg->max_chunk;
    carve(cfg, g, state_base, shared_base, &ctx->buf);
    ctx->mfma = cfg->dtype == CASCADE_BF16;
    // development switches: the environment is read here and nowhere else
    if (const char* e = getenv("CASCADE_KV_SCALAR_ATTENTION")) if (e[0] == '1') ctx->mfma = false;
    if (const char* e = getenv("CASCADE_KV_PACK_REUSE")) ctx->packed_reuse = e[0] != '0';   // 0: pack every tile for every chunk
    ctx->buf.opt_attn_splits = 0;
    if (const char* e = getenv("CASCADE_KV_ATTN_SPLITS")) ctx->buf.opt_attn_splits = atoi(e);
    ctx->buf.opt_score_narrow = -1;
    if (const char* e = getenv("CASCADE_KV_SCORE_NARROW")) ctx->buf.opt_score_narrow = e[0] == '1' ? 1 : 0;
    ctx->buf.opt_decode_qk_direct = getenv("CASCADE_KV_DECODE_QK_DIRECT") != nullptr;
    ctx->buf.opt_decode_pv_valu = getenv("CASCADE_KV_DECODE_PV_VALU") != nullptr;
    ctx->buf.opt_update_staged = getenv("CASCADE_KV_UPDATE_STAGED") != nullptr;

    // rows of a chunk whose EMA weight beta^k has not dropped below the cut
    {
        const double beta = cfg->ema_beta;
        double eps = cfg->score_tail_eps == 0.f ? ldexp(1.0, -40) : (double)cfg->score_tail_eps;
        int k = cfg->max_chunk;
        if (eps > 0.0) {
            if (beta <= 0.0) k = 1;
            else {
                double kk = ceil(log(eps) / log(beta));
                if (kk < 1.0) kk = 1.0;
                if (kk < (double)k) k = (int)kk;
            }
        }
        ctx->tail_k = k;
    }

    const DevBuffers& b = ctx->buf;
    const size_t BH = (size_t)g.B * g.Hkv;
    launch_fill_i32(b.ids, BH * g.slots, -1, s);
    if (tables) {
        launch_rope_table(g, cfg->rope_base, b.rope, b.rope_t, b.rope_rows, s);
        launch_wrow_table(cfg->ema_beta, b.wrow, cfg->max_chunk, s);
    }
    if (init_state && total > 0)
        launch_load_state(g, ctx->dtype, b, init_state->dev_k, init_state->dev_v, init_state->dev_mu,
                          init_state->dev_ids, init_state->counts, total, s);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        const int rc = hip_check(nullptr, e, (name + ": launch").c_str());
        if (!into) delete ctx;
        return rc;
    }
    *out_ctx = ctx;
    return CASCADE_OK;
}

extern "C" int cascade_init(const cascade_config* cfg, void* dev_workspace, size_t workspace_bytes,
                            const cascade_init_state* init_state, void* stream, cascade_ctx** out_ctx)
{
    if (!cfg || !dev_workspace || !out_ctx) return fail(nullptr, CASCADE_E_NULL_ARG, "cascade_init: NULL argument");
    *out_ctx = nullptr;
    std::string why;
    int rc = check_config(cfg, why);
    if (rc != CASCADE_OK) return fail(nullptr, rc, "cascade_init: " + why);
    if (((uintptr_t)dev_workspace & 255) != 0) return fail(nullptr, CASCADE_E_BAD_ARG, "cascade_init: workspace must be 256-byte aligned");
    Geom g;
    make_geom(cfg, g);
    const WorkspaceBytes need = carve(cfg, g, nullptr, nullptr, nullptr);
    if (workspace_bytes < need.state + need.shared) return fail(nullptr, CASCADE_E_WORKSPACE_TOO_SMALL, "cascade_init: workspace too small");
    HostState st;
    int total = 0;
    rc = check_init_state("cascade_init", g, init_state, st, total);
    if (rc != CASCADE_OK) return rc;
    hipStream_t s = (hipStream_t)stream;
    // zero the cache (rows of empty slots are read, masked, by the attention tiles) and scratch
    // (by a fill kernel, not hipMemsetAsync: a caller may be capturing the stream into a graph)
    launch_fill_i32((int32_t*)dev_workspace, (need.state + need.shared) / 4, 0, s);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_check(nullptr, e, "cascade_init: clearing the workspace");
    char* base = (char*)dev_workspace;
    return init_context("cascade_init", cfg, g, base, base + need.state, true, init_state, st, total, s, out_ctx);
}

extern "C" int cascade_init_layers(const cascade_config* cfg, int32_t n_layers, void* dev_workspace, size_t workspace_bytes,
                                   const cascade_init_state* const* init_states, void* stream, cascade_ctx** out_ctxs)
{
    if (!cfg || !dev_workspace || !out_ctxs) return fail(nullptr, CASCADE_E_NULL_ARG, "cascade_init_layers: NULL argument");
    if (n_layers < 1) return fail(nullptr, CASCADE_E_BAD_ARG, "cascade_init_layers: n_layers must be at least 1");
    for (int i = 0; i < n_layers; ++i) out_ctxs[i] = nullptr;
    std::string why;
    int rc = check_config(cfg, why);
    if (rc != CASCADE_OK) return fail(nullptr, rc, "cascade_init_layers: " + why);
    if (((uintptr_t)dev_workspace & 255) != 0) return fail(nullptr, CASCADE_E_BAD_ARG, "cascade_init_layers: workspace must be 256-byte aligned");
    Geom g;
    make_geom(cfg, g);
    const WorkspaceBytes need = carve(cfg, g, nullptr, nullptr, nullptr);
    const size_t total = need.state * (size_t)n_layers + need.shared;
    if (workspace_bytes < total) return fail(nullptr, CASCADE_E_WORKSPACE_TOO_SMALL, "cascade_init_layers: workspace too small");
    std::vector<HostState> sts(n_layers);
    std::vector<int> totals(n_layers, 0);
    for (int i = 0; i < n_layers; ++i) {
        rc = check_init_state("cascade_init_layers", g, init_states ? init_states[i] : nullptr, sts[i], totals[i]);
        if (rc != CASCADE_OK) return rc;
    }
    hipStream_t s = (hipStream_t)stream;
    launch_fill_i32((int32_t*)dev_workspace, total / 4, 0, s);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_check(nullptr, e, "cascade_init_layers: clearing the workspace");
    char* base = (char*)dev_workspace;
    char* shared = base + need.state * (size_t)n_layers;
    for (int i = 0; i < n_layers; ++i) {
        rc = init_context("cascade_init_layers", cfg, g, base + need.state * (size_t)i, shared, i == 0,
                          init_states ? init_states[i] : nullptr, sts[i], totals[i], s, &out_ctxs[i]);
        if (rc != CASCADE_OK) {
            for (int j = 0; j < i; ++j) { cascade_destroy(out_ctxs[j]); out_ctxs[j] = nullptr; }
            return rc;
        }
        out_ctxs[i]->packed_own = n_layers == 1;   // layers pack into one shared copy, which the next layer overwrites
    }
    return CASCADE_OK;
}

static void drop_events(cascade_ctx* ctx)
{
    for (auto& fam : ctx->prof) {
        for (auto& ev : fam) { (void)hipEventDestroy(ev.first); (void)hipEventDestroy(ev.second); }
        fam.clear();
    }
}

extern "C" void cascade_destroy(cascade_ctx* ctx)
{
    if (!ctx) return;
    drop_events(ctx);
    if (ctx->is_static) return;   // lives as long as the library; the next cascade_init_static resets it
    delete ctx;
}

// ------------------------------------------------------------------ a context without a caller's workspace

// The workspace of cascade_init_static: one array per GPU, held from the moment the library is
// loaded on it until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; everything that touches the memory uses the address that call returns.
static __device__ __align__(256) unsigned char scratch[CASCADE_STATIC_WORKSPACE_BYTES];

// Keeps the array in the code object whatever the optimiser thinks of a variable no kernel names.
__global__ void static_workspace_anchor_kernel(unsigned char* out)
{
    if (out) *out = scratch[0];
}

constexpr int kMaxStaticDevices = 64;
static void* g_static_ptr[kMaxStaticDevices];          // device address of `scratch` on every device seen so far
static cascade_ctx* g_static_ctx[kMaxStaticDevices];   // the one static context of a device: created once, reused for ever

extern "C" int cascade_init_static(const cascade_config* cfg, const cascade_init_state* init_state, void* stream,
                                   cascade_ctx** out_ctx)
{
    if (!cfg || !out_ctx) return fail(nullptr, CASCADE_E_NULL_ARG, "cascade_init_static: NULL argument");
    *out_ctx = nullptr;
    std::string why;
    int rc = check_config(cfg, why);
    if (rc != CASCADE_OK) return fail(nullptr, rc, "cascade_init_static: " + why);
    Geom g;
    make_geom(cfg, g);
    const WorkspaceBytes need = carve(cfg, g, nullptr, nullptr, nullptr);
    if (need.state + need.shared > (size_t)CASCADE_STATIC_WORKSPACE_BYTES)
        return fail(nullptr, CASCADE_E_WORKSPACE_TOO_SMALL,
                    "cascade_init_static: this configuration needs " + std::to_string(need.state + need.shared) +
                        " bytes, the static workspace holds " + std::to_string((size_t)CASCADE_STATIC_WORKSPACE_BYTES));
    HostState st;
    int total = 0;
    rc = check_init_state("cascade_init_static", g, init_state, st, total);
    if (rc != CASCADE_OK) return rc;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_check(nullptr, e, "cascade_init_static: hipGetDevice");
    if (dev < 0 || dev >= kMaxStaticDevices) return fail(nullptr, CASCADE_E_UNSUPPORTED, "cascade_init_static: device index out of range");
    if (!g_static_ptr[dev]) {      // once per device, with that device current: every GPU has its own copy of the array
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return hip_check(nullptr, e != hipSuccess ? e : hipErrorInvalidSymbol, "cascade_init_static: hipGetSymbolAddress");
        g_static_ptr[dev] = p;
    }
    char* base = (char*)g_static_ptr[dev];
    if (!g_static_ctx[dev]) {      // the only host allocation, once per device; later calls reuse the object
        g_static_ctx[dev] = new cascade_ctx();
        g_static_ctx[dev]->is_static = true;
    }
    cascade_ctx* ctx = g_static_ctx[dev];
    drop_events(ctx);
    *ctx = cascade_ctx();          // forget whatever the previous static context of this device held
    ctx->is_static = true;
    hipStream_t s = (hipStream_t)stream;
    // the array keeps what the last context left: everything this one reads before writing starts from zero
    launch_fill_i32((int32_t*)base, (need.state + need.shared) / 4, 0, s);      // (a fill kernel: safe under a stream capture)
    e = hipGetLastError();
    if (e != hipSuccess) return hip_check(nullptr, e, "cascade_init_static: clearing the workspace");
    return init_context("cascade_init_static", cfg, g, base, base + need.state, true, init_state, st, total, s, out_ctx, ctx);
}

extern "C" int cascade_profile_begin_families(cascade_ctx* ctx, uint32_t family_mask)
{
    if (!ctx) return CASCADE_E_NULL_ARG;
    drop_events(ctx);
    ctx->profiling = true;
    ctx->prof_mask = family_mask;
    return CASCADE_OK;
}

extern "C" int cascade_profile_begin(cascade_ctx* ctx) { return cascade_profile_begin_families(ctx, ~0u); }

extern "C" int cascade_profile_end(cascade_ctx* ctx, cascade_profile* out)
{
    if (!ctx) return CASCADE_E_NULL_ARG;
    if (!out) return fail(ctx, CASCADE_E_NULL_ARG, "cascade_profile_end: NULL output");
    ctx->profiling = false;
    memset(out, 0, sizeof(*out));
    for (int f = 0; f < CASCADE_K_FAMILIES; ++f)
        for (auto& ev : ctx->prof[f]) {
            int rc = hip_check(ctx, hipEventSynchronize(ev.second), "cascade_profile_end: event");
            if (rc) { drop_events(ctx); return rc; }
            float ms = 0.f;
            rc = hip_check(ctx, hipEventElapsedTime(&ms, ev.first, ev.second), "cascade_profile_end: elapsed");
            if (rc) { drop_events(ctx); return rc; }
            out->ms[f] += ms;
            out->intervals[f] += 1;
        }
    drop_events(ctx);
    return CASCADE_OK;
}

extern "C" const char* cascade_last_error(const cascade_ctx* ctx) { return ctx ? ctx->err.c_str() : init_error(); }

// Diagnostics: keep the scores the coming insertion decisions are taken with.
static int snapshot_scores(cascade_ctx* ctx, int n_tokens, hipStream_t s)
{
    ctx->st_prev = ctx->st;
    ctx->last_tokens = n_tokens;
    if (!ctx->cfg.keep_update_scores) return CASCADE_OK;
    const size_t bytes = (size_t)ctx->g.B * ctx->g.Hkv * ctx->g.slots * 4;
    return hip_check(ctx, hipMemcpyAsync(ctx->buf.mu_snap, ctx->buf.mu, bytes, hipMemcpyDeviceToDevice, s),
                     "score snapshot");
}

// ------------------------------------------------------------------ prefill chunk

extern "C" int cascade_prefill_chunk(cascade_ctx* ctx, const void* dev_q, const void* dev_k, const void* dev_v,
                                     int32_t n_tokens, void* dev_out, void* stream)
{
    if (!ctx) return CASCADE_E_NULL_ARG;
    if (!dev_q || !dev_k || !dev_v || !dev_out) return fail(ctx, CASCADE_E_NULL_ARG, "cascade_prefill_chunk: NULL argument");
    if (n_tokens < 1 || n_tokens > ctx->max_chunk) return fail(ctx, CASCADE_E_BAD_ARG, "cascade_prefill_chunk: n_tokens out of range");
    if (ctx->st.n_seen + n_tokens > 0x7FFFFFFF) return fail(ctx, CASCADE_E_BAD_ARG, "cascade_prefill_chunk: token index overflow");
    if (ctx->poisoned) return fail(ctx, CASCADE_E_HIP, "cascade_prefill_chunk: an earlier call on this context failed to launch; the cache is undefined");
    const Geom& g = ctx->g;
    hipStream_t s = (hipStream_t)stream;
    const int Q = n_tokens;

    SegList sl;
    build_segments(g, ctx->st, true, Q, sl);
    bool packed_stable = false;   // the packed tiles of this call stay where they are for the next one
    PackedLayout lay;
    // the MFMA kernels take logits directly as base-2 exponents
    const float qscale = ctx->mfma ? g.scale * 1.4426950408889634f : 1.f;
    const int tail = Q < ctx->tail_k ? Q : ctx->tail_k;    // rows that carry weight in the score sums
    const bool single_pass = ctx->mfma && attn_single_pass_ok(g, ctx->buf, Q, tail);
    ctx->last_single_pass = single_pass;
    {
        Timed t(ctx, CASCADE_K_PREP, s);
        // bf16: the attention kernel rotates its queries itself; only the score kernel reads rotated copies
        // (single-pass scores: nobody reads rotated query copies)
        launch_prep(g, ctx->dtype, ctx->buf, sl, Q, qscale, ctx->mfma ? (single_pass ? Q : Q - tail) : 0, dev_q, dev_k, dev_v, s);
        if (ctx->mfma) {
            // The tiles of a full cache keep their place while the ring heads keep their offsets
            // inside a tile: then only the tiles the last update wrote, and the chunk's own, are
            // packed again.
            packed_layout(g, ctx->st, lay);
            const int chunk_tiles = (Q + 63) / 64;
            if (lay.full && packed_tiles_of(sl) != lay.cache_tiles + chunk_tiles)
                return fail(ctx, CASCADE_E_INTERNAL, "cascade_prefill_chunk: the segment list does not have the tiles of the packed layout");
            TileRuns runs;
            runs.n = 0; runs.total = 0;
            bool partial = ctx->packed_reuse && ctx->packed_own && lay.full && ctx->packed_valid && same_offsets(g, lay, ctx->packed);
            if (partial) {
                runs = ctx->stale;
                partial = add_tile_run(runs, lay.cache_tiles, chunk_tiles);
            }
            if (!partial) {
                runs.n = 0; runs.total = 0;
                add_tile_run(runs, 0, packed_tiles_of(sl));
            }
            ctx->packed_valid = false;   // until this call has gone through
            if (!launch_kv_pack(g, ctx->buf, sl, runs, Q, s))
                return fail(ctx, CASCADE_E_WORKSPACE_TOO_SMALL, "cascade_prefill_chunk: packed K/V buffers too small for this segment list");
            packed_stable = ctx->packed_own && lay.full;
        }
    }
    {
        Timed t(ctx, CASCADE_K_ATTENTION, s);
        if (ctx->mfma) launch_attn_stream(g, ctx->buf, sl, Q, dev_q, qscale, tail, ctx->max_chunk, dev_out, single_pass, s);
        else launch_attn_simple(g, ctx->dtype, ctx->buf, sl, Q, ctx->max_chunk, dev_out, s);
    }
    const float decay = (float)pow((double)g.beta, (double)Q);
    {
        Timed t(ctx, CASCADE_K_SCORES, s);
        if (single_pass) launch_single_pass_merge(g, ctx->buf, sl, Q, ctx->max_chunk, decay, s);
        else if (ctx->mfma) launch_score_mfma(g, ctx->buf, sl, Q, ctx->max_chunk, tail, decay, s);
        else launch_score_simple(g, ctx->dtype, ctx->buf, sl, Q, ctx->max_chunk, tail, decay, s);
        if (g.head_policy == CASCADE_HEADS_HOMOGENEOUS && g.Hkv > 1) launch_share_scores(g, ctx->buf, Q, ctx->max_chunk, s);
    }
    int rc = snapshot_scores(ctx, Q, s);
    if (rc) return rc;
    UpdatePlan pl;
    HostState st_next = ctx->st;      // the host mirror moves on only once every launch has been accepted
    plan_update(g, st_next, Q, pl);
    {
        Timed t(ctx, CASCADE_K_UPDATE, s);
        const bool direct = update_is_direct(g, ctx->buf, pl);
        if (!direct) launch_plan(g, ctx->buf, pl, ctx->max_chunk, s);
        launch_moves(g, ctx->dtype, ctx->buf, pl, ctx->max_chunk, dev_k, dev_v, g.Hkv * g.d, Q * g.Hkv * g.d, direct, s);
    }
    const int rc_launch = hip_check(ctx, hipGetLastError(), "cascade_prefill_chunk");
    if (rc_launch != CASCADE_OK) {    // some launches may have run: host and device no longer agree
        ctx->poisoned = true;
        return rc_launch;
    }
    ctx->st = st_next;
    if (packed_stable) {
        ctx->packed = lay;
        ctx->stale.n = 0; ctx->stale.total = 0;
        ctx->packed_valid = add_touched_tiles(g, lay, pl, ctx->stale);
    }
    return CASCADE_OK;
}

// ------------------------------------------------------------------ decode step

extern "C" int cascade_decode_step(cascade_ctx* ctx, const void* dev_q, const void* dev_k, const void* dev_v,
                                   void* dev_out, void* stream)
{
    if (!ctx) return CASCADE_E_NULL_ARG;
    if (!dev_q || !dev_k || !dev_v || !dev_out) return fail(ctx, CASCADE_E_NULL_ARG, "cascade_decode_step: NULL argument");
    const Geom& g = ctx->g;
    if (!decode_supported(g)) return fail(ctx, CASCADE_E_UNSUPPORTED, "cascade_decode_step: needs head_dim 64 or 128 and at most 8 query heads per KV head");
    if (ctx->st.n_seen + 1 > 0x7FFFFFFF) return fail(ctx, CASCADE_E_BAD_ARG, "cascade_decode_step: token index overflow");
    if (ctx->poisoned) return fail(ctx, CASCADE_E_HIP, "cascade_decode_step: an earlier call on this context failed to launch; the cache is undefined");
    hipStream_t s = (hipStream_t)stream;

    SegList sl;
    build_segments(g, ctx->st, false, 1, sl);
    ctx->packed_valid = false;   // the step writes cache rows the packed copies of the prefill path do not follow
    ctx->last_single_pass = false;
    {
        Timed t0(ctx, CASCADE_K_DECODE_QK, s);
        launch_decode_qk(g, ctx->dtype, ctx->buf, sl, dev_q, dev_k, s);
    }
    {
        Timed t1(ctx, CASCADE_K_DECODE_PV, s);
        launch_decode_pv(g, ctx->dtype, ctx->buf, sl, s);
        // homogeneous heads: the cached scores are shared here, the new token's inside decode_finish
        if (g.head_policy == CASCADE_HEADS_HOMOGENEOUS && g.Hkv > 1) launch_share_scores(g, ctx->buf, 0, ctx->max_chunk, s);
    }
    // the snapshot holds the cached scores after this step's EMA update and before the insertion
    int rc = snapshot_scores(ctx, 1, s);
    if (rc) return rc;
    UpdatePlan pl;
    HostState st_next = ctx->st;
    plan_update(g, st_next, 1, pl);
    {
        Timed t2(ctx, CASCADE_K_DECODE_FINISH, s);
        launch_decode_finish(g, ctx->dtype, ctx->buf, sl, pl, ctx->max_chunk, dev_k, dev_v, dev_out, s);
    }
    rc = hip_check(ctx, hipGetLastError(), "cascade_decode_step");
    if (rc != CASCADE_OK) { ctx->poisoned = true; return rc; }
    ctx->st = st_next;
    return CASCADE_OK;
}

// ------------------------------------------------------------------ read state

extern "C" int cascade_read_state(cascade_ctx* ctx, cascade_state_view* view, void* stream)
{
    if (!ctx) return CASCADE_E_NULL_ARG;
    if (!view) return fail(ctx, CASCADE_E_NULL_ARG, "cascade_read_state: NULL view");
    const Geom& g = ctx->g;
    const HostState& st = ctx->st;
    hipStream_t s = (hipStream_t)stream;
    int rc = hip_check(ctx, hipStreamSynchronize(s), "cascade_read_state: synchronize");
    if (rc) return rc;

    const size_t BH = (size_t)g.B * g.Hkv;
    const int n = st.n_cached(g);
    std::vector<int> slot(n);
    for (int r = 0; r < n; ++r) slot[r] = slot_of_rank(g, st, r);

    memset(view->counts, 0, sizeof(view->counts));
    memset(view->xi, 0, sizeof(view->xi));
    memset(view->accepted, 0, sizeof(view->accepted));
    memset(view->discards, 0, sizeof(view->discards));
    view->counts[0] = st.sink_fill;
    for (int c = 0; c < g.N; ++c) {
        view->counts[1 + c] = st.count[c];
        view->xi[c] = st.xi[c];
        view->accepted[c] = st.accepted[c];
        view->discards[c] = st.discards[c];
    }
    view->t = st.t;
    view->n_seen = st.n_seen;
    view->pre_count = ctx->st_prev.n_cached(g);
    view->last_tokens = ctx->last_tokens;
    view->last_single_pass = ctx->last_single_pass ? 1 : 0;

    if (ctx->cfg.keep_update_scores && view->host_pre_mu && ctx->last_tokens > 0) {
        std::vector<float> snap(BH * g.slots);
        rc = hip_check(ctx, hipMemcpy(snap.data(), ctx->buf.mu_snap, snap.size() * 4, hipMemcpyDeviceToHost), "cascade_read_state: copy score snapshot");
        if (rc) return rc;
        const int np = view->pre_count;
        for (int r = 0; r < np; ++r) {
            const int sl = slot_of_rank(g, ctx->st_prev, r);
            for (size_t bh = 0; bh < BH; ++bh) view->host_pre_mu[bh * g.slots + r] = snap[bh * g.slots + sl];
        }
    }
    if (ctx->cfg.keep_update_scores && view->host_chunk_mu && ctx->last_tokens > 0) {
        rc = hip_check(ctx, hipMemcpy(view->host_chunk_mu, ctx->buf.mu_chunk, BH * (size_t)ctx->max_chunk * 4, hipMemcpyDeviceToHost),
                       "cascade_read_state: copy chunk scores");
        if (rc) return rc;
    }

    if (view->host_ids || view->host_mu || view->host_slot) {
        std::vector<int32_t> ids(BH * g.slots);
        std::vector<float> mu(BH * g.slots);
        rc = hip_check(ctx, hipMemcpy(ids.data(), ctx->buf.ids, ids.size() * 4, hipMemcpyDeviceToHost), "cascade_read_state: copy ids");
        if (rc) return rc;
        rc = hip_check(ctx, hipMemcpy(mu.data(), ctx->buf.mu, mu.size() * 4, hipMemcpyDeviceToHost), "cascade_read_state: copy mu");
        if (rc) return rc;
        for (size_t bh = 0; bh < BH; ++bh)
            for (int r = 0; r < g.slots; ++r) {
                const size_t o = bh * g.slots + r;
                if (view->host_ids) view->host_ids[o] = r < n ? ids[bh * g.slots + slot[r]] : -1;
                if (view->host_mu) view->host_mu[o] = r < n ? mu[bh * g.slots + slot[r]] : 0.f;
                if (view->host_slot) view->host_slot[o] = r < n ? slot[r] : -1;
            }
    }
    if (view->host_swaps) {
        std::vector<int32_t> sw(BH * g.N);
        rc = hip_check(ctx, hipMemcpy(sw.data(), ctx->buf.swaps, sw.size() * 4, hipMemcpyDeviceToHost), "cascade_read_state: copy swaps");
        if (rc) return rc;
        for (size_t i = 0; i < sw.size(); ++i) view->host_swaps[i] = sw[i];
    }
    const size_t n_pairs = view->host_kv_pairs ? (size_t)(view->n_kv_pairs > 0 ? view->n_kv_pairs : 0) : BH;
    if (view->host_kv_pairs && (view->host_k || view->host_v))
        for (size_t i = 0; i < n_pairs; ++i)
            if (view->host_kv_pairs[i] < 0 || (size_t)view->host_kv_pairs[i] >= BH)
                return fail(ctx, CASCADE_E_BAD_ARG, "cascade_read_state: host_kv_pairs names a pair that does not exist");
    for (int which = 0; which < 2; ++which) {
        float* dst = which == 0 ? view->host_k : view->host_v;
        if (!dst) continue;
        const void* src = which == 0 ? ctx->buf.Kc : ctx->buf.Vc;
        std::vector<char> raw((size_t)g.slots * g.d * ctx->elem);
        for (size_t pi = 0; pi < n_pairs; ++pi) {
            const size_t bh = view->host_kv_pairs ? (size_t)view->host_kv_pairs[pi] : pi;
            rc = hip_check(ctx, hipMemcpy(raw.data(), (const char*)src + bh * raw.size(), raw.size(), hipMemcpyDeviceToHost),
                           "cascade_read_state: copy rows");
            if (rc) return rc;
            for (int r = 0; r < g.slots; ++r) {
                float* o = dst + (pi * g.slots + r) * g.d;
                if (r >= n) { memset(o, 0, sizeof(float) * g.d); continue; }
                if (ctx->dtype == CASCADE_BF16) {
                    const bf16_t* p = (const bf16_t*)raw.data() + (size_t)slot[r] * g.d;
                    for (int e = 0; e < g.d; ++e) o[e] = bf16_to_f32(p[e]);
                } else {
                    memcpy(o, (const float*)raw.data() + (size_t)slot[r] * g.d, sizeof(float) * g.d);
                }
            }
        }
    }
    return CASCADE_OK;
}
