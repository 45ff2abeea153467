// Test infrastructure: the host logic of the library (structure.cpp, simulate.cpp, plan_core.h)
// and the C oracle's Alg. 2, built into ONE executable with AddressSanitizer and
// UndefinedBehaviorSanitizer, driven over seeded random geometries: the chunk-at-a-time replay of
// the update must give the membership, scores and swap counts of the oracle's token-by-token
// Alg. 2, and neither side may touch memory it does not own.  Exit code 0 = all cases agree.
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "../../include/cascade_kv.h"

extern "C" {
// the oracle's C interface (oracle/cascade_oracle.c)
typedef struct {
    int32_t n_q_heads, n_kv_heads, head_dim;
    int32_t n_sink, n_cascades;
    int32_t cascade_sizes[16];
    int64_t accept_period[16];
    double ema_beta, rope_base, softmax_scale;
    int32_t head_reduce, token_selection, head_policy;
} oracle_config;
typedef struct oracle_seq oracle_seq;
oracle_seq* oracle_create(const oracle_config* cfg);
void oracle_destroy(oracle_seq* S);
int oracle_insert_scored(oracle_seq* S, int g, double score);
int64_t oracle_count(const oracle_seq* S, int g);
int oracle_get_state(oracle_seq* S, int g, int64_t* ids, double* mu, int32_t* cascade_of, int64_t* counts, int64_t* stats, double* kv);
int oracle_chunk(oracle_seq* S, const float* q, const float* k, const float* v, int Q, double* out, int kv_lo, int kv_hi);
int64_t oracle_select_log(const oracle_seq* S, int g, int64_t* ids, double* mu, int64_t cap);
}

static uint64_t rng_state;
static uint32_t rnd(uint32_t n)   // splitmix64, value in [0, n)
{
    uint64_t z = (rng_state += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    z ^= z >> 31;
    return (uint32_t)(z % n);
}

static int one_case(int seed)
{
    rng_state = 0x1234567ull * (uint64_t)(seed + 1);
    cascade_config cfg;
    memset(&cfg, 0, sizeof(cfg));
    oracle_config oc;
    memset(&oc, 0, sizeof(oc));
    const int N = 1 + (int)rnd(5);
    cfg.batch = 1; cfg.n_q_heads = 1; cfg.n_kv_heads = 1; cfg.head_dim = 2; cfg.dtype = CASCADE_F32;
    cfg.n_sink = (int)rnd(4); cfg.n_cascades = N;
    cfg.ema_beta = 0.9f; cfg.rope_base = 10000.f; cfg.max_chunk = 64;
    cfg.token_selection = seed % 4 == 3 ? 0 : 1;
    oc.n_q_heads = oc.n_kv_heads = 1; oc.head_dim = 2; oc.n_sink = cfg.n_sink; oc.n_cascades = N;
    oc.ema_beta = 0.9; oc.rope_base = 10000.0; oc.token_selection = cfg.token_selection;
    int slots = cfg.n_sink;
    for (int c = 0; c < N; ++c) {
        cfg.cascade_sizes[c] = 1 + (int)rnd(seed % 5 == 0 ? 70 : 9);
        cfg.accept_period[c] = seed % 3 == 1 ? (c == 0 ? 1 : 1 + (int)rnd(5)) : 0;
        oc.cascade_sizes[c] = cfg.cascade_sizes[c];
        oc.accept_period[c] = seed % 3 == 1 ? cfg.accept_period[c] : (1 << c);
        slots += cfg.cascade_sizes[c];
    }
    oracle_seq* o = oracle_create(&oc);
    if (!o) { fprintf(stderr, "seed %d: oracle_create failed\n", seed); return 1; }
    std::vector<int32_t> chunks;
    std::vector<float> scores;
    std::vector<int32_t> ids(slots), slot(slots);
    std::vector<float> mu(slots);
    std::vector<int64_t> swaps(N), oids(slots), ocounts(1 + N), ostats(3 * N);
    std::vector<double> omu(slots);
    std::vector<int32_t> ocas(slots);
    int rc = 0;
    for (int step = 0; step < 25 && rc == 0; ++step) {
        const int Q = 1 + (int)rnd(49);
        chunks.push_back(Q);
        for (int i = 0; i < Q; ++i) {
            const float s = (float)rnd(6) / 8.0f;      // few distinct values: many ties
            scores.push_back(s);
            oracle_insert_scored(o, 0, (double)s);
        }
        cascade_state_view view;
        memset(&view, 0, sizeof(view));
        view.host_ids = ids.data(); view.host_mu = mu.data(); view.host_slot = slot.data(); view.host_swaps = swaps.data();
        const int e = cascade_simulate_structure(&cfg, chunks.data(), (int32_t)chunks.size(), scores.data(), &view);
        if (e != CASCADE_OK) { fprintf(stderr, "seed %d step %d: cascade_simulate_structure returned %d\n", seed, step, e); rc = 1; break; }
        const int64_t n = oracle_count(o, 0);
        oracle_get_state(o, 0, oids.data(), omu.data(), ocas.data(), ocounts.data(), ostats.data(), NULL);
        int total = 0;
        for (int c = 0; c <= N; ++c) {
            if (view.counts[c] != ocounts[c]) { fprintf(stderr, "seed %d step %d: count %d differs\n", seed, step, c); rc = 1; }
            total += view.counts[c];
        }
        if (total != n) rc = 1;
        for (int64_t r = 0; r < n && rc == 0; ++r)
            if (ids[r] != oids[r] || mu[r] != (float)omu[r]) { fprintf(stderr, "seed %d step %d: cache index %ld differs\n", seed, step, (long)r); rc = 1; }
        for (int c = 0; c < N && rc == 0; ++c)
            if (swaps[c] != ostats[3 * c + 1]) { fprintf(stderr, "seed %d step %d: swaps of cascade %d differ\n", seed, step, c); rc = 1; }
    }
    oracle_destroy(o);
    return rc;
}

// A few chunks through the oracle's attention path as well (its buffers are indexed by cache
// order, head and row: the sanitizers watch every one of those accesses).
static int oracle_attention_case()
{
    oracle_config oc;
    memset(&oc, 0, sizeof(oc));
    oc.n_q_heads = 4; oc.n_kv_heads = 2; oc.head_dim = 8; oc.n_sink = 2; oc.n_cascades = 3;
    for (int c = 0; c < 3; ++c) { oc.cascade_sizes[c] = 5; oc.accept_period[c] = 1 << c; }
    oc.ema_beta = 0.8; oc.rope_base = 50.0;
    for (int policy = 0; policy < 2; ++policy) {
        oc.head_policy = policy;
        oracle_seq* o = oracle_create(&oc);
        if (!o) return 1;
        rng_state = 99;
        for (int step = 0; step < 12; ++step) {
            const int Q = 1 + (int)rnd(7);
            std::vector<float> q((size_t)Q * 4 * 8), k((size_t)Q * 2 * 8), v((size_t)Q * 2 * 8);
            for (auto& x : q) x = (float)rnd(2000) / 1000.f - 1.f;
            for (auto& x : k) x = (float)rnd(2000) / 1000.f - 1.f;
            for (auto& x : v) x = (float)rnd(2000) / 1000.f - 1.f;
            std::vector<double> out((size_t)Q * 4 * 8);
            if (oracle_chunk(o, q.data(), k.data(), v.data(), Q, out.data(), 0, 2) != 0) { oracle_destroy(o); return 1; }
            for (double x : out) if (!(x == x)) { oracle_destroy(o); return 1; }
        }
        const int64_t nlog = oracle_select_log(o, 0, NULL, NULL, 0);
        std::vector<int64_t> lid(2 * (size_t)(nlog > 0 ? nlog : 1));
        std::vector<double> lmu(2 * (size_t)(nlog > 0 ? nlog : 1));
        oracle_select_log(o, 0, lid.data(), lmu.data(), nlog);
        oracle_destroy(o);
    }
    return 0;
}

int main(int argc, char** argv)
{
    const int n = argc > 1 ? atoi(argv[1]) : 40;
    int bad = 0;
    for (int seed = 0; seed < n; ++seed) bad += one_case(seed);
    bad += oracle_attention_case();
    printf("%d cases, %d failed\n", n + 1, bad);
    return bad ? 1 : 0;
}
