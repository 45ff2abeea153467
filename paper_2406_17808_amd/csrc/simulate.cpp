// Host-only replay of the cascade update (no device is touched): cascade_simulate_structure of
// include/cascade_kv.h.  It runs the same segment / eviction routines as the device kernels
// (plan_core.h), one "thread" at a time, and checks every write against the slots the host
// predicts an update may touch.
#include <string.h>

#include <string>
#include <vector>

#include "plan_core.h"
#include "structure.h"

using namespace ckv;

static int fail(int code, const std::string& msg)
{
    set_init_error(msg);
    return code;
}

// Fill, ring heads and counters after feeding chunks of the given sizes to an empty cache; with
// scores also the membership.  Pure host arithmetic (no device is touched).  The membership is
// computed by the same segment / eviction routines the device kernels run (plan_core.h), one
// "thread" at a time.
extern "C" int cascade_simulate_structure(const cascade_config* cfg, const int32_t* chunk_sizes, int32_t n_chunks,
                                          const float* host_scores, cascade_state_view* view)
{
    if (!cfg || !view || (!chunk_sizes && n_chunks > 0)) return fail(CASCADE_E_NULL_ARG, "cascade_simulate_structure: NULL argument");
    std::string why;
    int rc = check_config(cfg, why);
    if (rc != CASCADE_OK) return fail(rc, "cascade_simulate_structure: " + why);
    Geom g;
    make_geom(cfg, g);
    HostState st;
    std::vector<float> mu;
    std::vector<int32_t> ids;
    std::vector<int64_t> swaps(g.N, 0);
    if (host_scores) { mu.assign(g.slots, 0.f); ids.assign(g.slots, -1); }
    size_t consumed = 0;
    for (int ci = 0; ci < n_chunks; ++ci) {
        const int Q = chunk_sizes[ci];
        if (Q < 1) return fail(CASCADE_E_BAD_ARG, "cascade_simulate_structure: chunk sizes must be >= 1");
        UpdatePlan pl;
        plan_update(g, st, Q, pl);
        if (!host_scores) continue;
        const float* muc = host_scores + consumed;
        consumed += Q;
        int run_lo[kMaxTileRuns], run_hi[kMaxTileRuns];
        const int n_runs = touched_slot_runs(g, pl, run_lo, run_hi);   // every write below must fall inside these
        std::vector<int32_t> off_a(Q + 1), off_b(Q + 1);
        std::vector<std::vector<int32_t>> W(g.N, std::vector<int32_t>(Q + 2, -1));
        int32_t *off_in = off_a.data(), *off_out = off_b.data();
        const bool direct = plan_is_direct(pl);
        for (int c = 0; c < g.N; ++c) {
            const CascStep& cs = pl.c[c];
            if (cs.M == 0) break;
            for (int sidx = 0; sidx < cs.J + cs.pre; ++sidx) {
                const int j = sidx - cs.pre;
                int sw;
                W[c][1 + j] = segment_winner(cs, c, j, g.slots, pl.n_to_sink, g.token_selection, off_in,
                                             mu.data(), muc, &sw);
                swaps[c] += sw;
                if (direct) {
                    // the device takes this update without the cascade-by-cascade hand-over: the offers
                    // named directly from the structure must be the ones handed over, segment by segment
                    int sw2;
                    const int w2 = segment_winner(cs, c, j, g.slots, pl.n_to_sink, g.token_selection, nullptr,
                                                  mu.data(), muc, &sw2, &pl);
                    if (w2 != W[c][1 + j] || sw2 != sw)
                        return fail(CASCADE_E_INTERNAL, "cascade_simulate_structure: direct and staged plans disagree");
                }
            }
            for (int i = 0; i < cs.P; ++i) off_out[i] = evicted_ref(cs, i, W[c].data());
            std::swap(off_in, off_out);
        }
        for (int c = g.N - 1; c >= -1; --c) {      // the last cascade first: sources are still intact
            int E, extra = 0;
            if (c < 0) E = pl.n_to_sink;
            else { if (pl.c[c].M == 0) continue; E = final_entries(pl.c[c], &extra); }
            for (int e = 0; e < E + extra; ++e) {
                int dst, ref;
                if (c < 0) { dst = pl.sink_fill0 + e; ref = g.slots + e; }
                else if (!final_entry(pl.c[c], e, E, W[c].data(), &dst, &ref)) continue;
                bool predicted = false;
                for (int r = 0; r < n_runs; ++r) predicted = predicted || (dst >= run_lo[r] && dst < run_hi[r]);
                if (!predicted) return fail(CASCADE_E_INTERNAL, "cascade_simulate_structure: a slot was written outside the predicted runs");
                if (ref < g.slots) { mu[dst] = mu[ref]; ids[dst] = ids[ref]; }
                else { mu[dst] = muc[ref - g.slots]; ids[dst] = pl.id0 + (ref - g.slots); }
            }
        }
    }
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
    view->pre_count = 0;
    view->last_tokens = 0;
    view->last_single_pass = 0;
    const int n = st.n_cached(g);
    for (int r = 0; r < g.slots; ++r) {
        const int sl = r < n ? slot_of_rank(g, st, r) : -1;
        if (view->host_slot) view->host_slot[r] = sl;
        if (host_scores && view->host_ids) view->host_ids[r] = sl >= 0 ? ids[sl] : -1;
        if (host_scores && view->host_mu) view->host_mu[r] = sl >= 0 ? mu[sl] : 0.f;
    }
    if (host_scores && view->host_swaps) for (int c = 0; c < g.N; ++c) view->host_swaps[c] = swaps[c];
    return CASCADE_OK;
}
