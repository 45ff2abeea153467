/*
 * CPU oracle for the cascading KV cache (arxiv 2406.17808).  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, token-by-token implementation of what the hot path computes, in
 * fp64, written from the paper.  It shares no code with the HIP path and is only
 * used by the tests, the smoke check and the CPU-baseline leg of the benchmark.
 *
 * What follows which passage:
 *   - attention of a query over (cache  U  own chunk up to itself): Eq. 2, the
 *     strided prefill of Alg. 1 (get -> layer -> update) and Fig. 4.
 *   - positional encoding by index inside the cache: Section 3.1 "Positional Encoding".
 *   - EMA of the attention each key receives: Section 3.1 "Token Selection";
 *     for a chunk every query row is one time step (the coefficients that
 *     Alg. 3 gives for the rows of a chunk are this recurrence unrolled).
 *   - the insertion of one item into sinks / cascades: Alg. 2.
 *   - GQA: one decision per KV head, query heads of a group reduced by max
 *     (or mean): Appendix "Head Policy and Head Reduction".  The same appendix's
 *     "homogeneous heads" (one decision shared by all heads) is the switch
 *     head_policy = 1: the head axis is reduced to ONE score per token, over all
 *     query heads, and every KV head takes its decisions with that score.
 *
 * Readings taken where the paper is silent:
 *   R1  a cascade with period f accepts when (t mod f) == 0, where t counts the
 *       tokens offered to the first cascade so far (sink insertions excluded).
 *   R2  the scores of a chunk are the exact softmax probabilities (final
 *       normaliser), not the running-normaliser extrapolation of Alg. 3.
 *   R3  per query head the chunk increment starts at 0 and follows
 *       d <- beta*d + (1-beta)*p row by row; heads are reduced on these
 *       increments; a cached item's score is multiplied by beta once per row
 *       and then receives the reduced increment; a new token starts at 0.
 *   R4  no eviction happens inside a chunk: every query sees the whole cache
 *       as it was before the chunk plus the causal part of its own chunk.
 *   R5  Alg. 2 is followed literally (discards start once the second cascade is
 *       full at a non-accepting step, not when the whole cache is full).
 *   R6  RoPE pairs (x_i, x_{i+d/2}), theta_i = base^(-2i/d), angle = pos*theta_i.
 *   R7  token selection replaces the newest item in place, strict '>' only.
 *   R8  (single-pass scores only, the *_single_pass entry points) Alg. 3 adds, while a program is
 *       still sweeping the keys, col_sum(S^ / (l + l*rho/gamma) * C_EMA): S^ = exp(S - m) and l the
 *       running normaliser after the current inner-loop step, gamma the steps completed including
 *       it, rho the steps remaining.  S^/l does not depend on the running maximum, so the added
 *       value is  C_EMA * (gamma / (gamma + rho)) * exp(S_ij) / sum of exp(S_ij') over the keys of
 *       the steps done so far.  Which step visits which key, and how many steps a program has, is
 *       the kernel's business (tile size, visiting order, rows per program): the caller passes both.
 *
 * Parity pins (tests/test_oracle_*.py): brute-force dense attention, the
 * sink + sliding-window special case (one cascade), the full causal attention
 * special case (nothing discarded yet), the positional-encoding example of
 * Section 3.1, a hand trace of Alg. 2, the acceptance rates and the span of
 * Eq. 4, the row-sum identity of the EMA increments, the comparison record of the
 * hand traces, and for homogeneous heads brute force over all query heads plus the
 * one-KV-head case where both policies coincide; for the single-pass scores (R8) a dense
 * formula over a random schedule, the exactness of the last step and of a one-step schedule.
 * R1 (phase of the
 * acceptance schedule) and the order of head reduction in R3 are fixed by these
 * readings only: parity unpinned by the paper for those two choices.
 *
 * The only memoisation is that a key's rotation at its cache index is computed
 * once per chunk instead of once per query; values are identical.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_MAX_CASCADES 16

typedef struct {
    int32_t n_q_heads, n_kv_heads, head_dim;
    int32_t n_sink, n_cascades;
    int32_t cascade_sizes[ORACLE_MAX_CASCADES];
    int64_t accept_period[ORACLE_MAX_CASCADES];
    double ema_beta, rope_base, softmax_scale;
    int32_t head_reduce;      /* 0 max, 1 mean */
    int32_t token_selection;  /* 1 as in the paper, 0: never replace */
    int32_t head_policy;      /* 0 independent KV heads (the paper's choice), 1 homogeneous */
} oracle_config;

typedef struct {
    int64_t id;   /* index of the token in the original sequence */
    double mu;    /* EMA of received attention */
    double *k;    /* un-rotated key, d values */
    double *v;
} item_t;

typedef struct {
    int cap, n;
    item_t *it;   /* it[0] oldest ... it[n-1] newest */
    int64_t accepted, swaps, discards;
} buf_t;

typedef struct {
    buf_t sink;
    buf_t casc[ORACLE_MAX_CASCADES];
    int64_t t;            /* tokens offered to the first cascade so far */
    int64_t n_seen;       /* tokens inserted so far (ids continue from here) */
    double *last_delta;   /* reduced chunk increments of the last chunk, cache order then chunk */
    int64_t last_delta_n;
    int64_t *discard_log; /* ids in the order they were discarded */
    int64_t n_discard_log, cap_discard_log;
    /* every token-selection comparison of Alg. 2 in the order it was taken: ids and scores of
       the incoming item and of the newest item of the cascade (a record, not arithmetic) */
    int64_t *select_ids;  /* [n][2] incoming, newest */
    double *select_mu;    /* [n][2] */
    int64_t n_select_log, cap_select_log;
} head_t;

typedef struct {
    oracle_config cfg;
    head_t *head;  /* n_kv_heads */
} oracle_seq;

/* ------------------------------------------------------------------ helpers */

static void item_free(item_t *x) { free(x->k); free(x->v); x->k = x->v = NULL; }

static void log_discard(head_t *H, int64_t id)
{
    if (H->n_discard_log == H->cap_discard_log) {
        H->cap_discard_log = H->cap_discard_log ? 2 * H->cap_discard_log : 1024;
        H->discard_log = (int64_t *)realloc(H->discard_log, sizeof(int64_t) * (size_t)H->cap_discard_log);
    }
    H->discard_log[H->n_discard_log++] = id;
}

static void log_select(head_t *H, int64_t id_in, double mu_in, int64_t id_newest, double mu_newest)
{
    if (H->n_select_log == H->cap_select_log) {
        H->cap_select_log = H->cap_select_log ? 2 * H->cap_select_log : 1024;
        H->select_ids = (int64_t *)realloc(H->select_ids, sizeof(int64_t) * 2 * (size_t)H->cap_select_log);
        H->select_mu = (double *)realloc(H->select_mu, sizeof(double) * 2 * (size_t)H->cap_select_log);
    }
    H->select_ids[2 * H->n_select_log] = id_in;
    H->select_ids[2 * H->n_select_log + 1] = id_newest;
    H->select_mu[2 * H->n_select_log] = mu_in;
    H->select_mu[2 * H->n_select_log + 1] = mu_newest;
    H->n_select_log++;
}

static void buf_append(buf_t *b, item_t x) { b->it[b->n++] = x; }

static item_t buf_pop_oldest(buf_t *b)
{
    item_t x = b->it[0];
    memmove(b->it, b->it + 1, sizeof(item_t) * (size_t)(b->n - 1));
    b->n--;
    return x;
}

/* Section 3.1 "Positional Encoding" with reading R6: rotate x (d values) to position pos. */
static void rope(const double *x, int d, double pos, double base, double *out)
{
    int half = d / 2;
    for (int i = 0; i < half; ++i) {
        double theta = pow(base, -2.0 * (double)i / (double)d);
        double a = pos * theta, c = cos(a), s = sin(a);
        out[i] = x[i] * c - x[i + half] * s;
        out[i + half] = x[i + half] * c + x[i] * s;
    }
}

/* ------------------------------------------------------------------ Alg. 2 */

/* Insert one item into the sinks / cascades of one KV head (Alg. 2, readings R1, R5, R7). */
static void cache_insert(const oracle_config *cfg, head_t *H, item_t x)
{
    if (H->sink.n < H->sink.cap) {          /* sinks are filled first and never evict */
        buf_append(&H->sink, x);
        return;
    }
    for (int c = 0; c < cfg->n_cascades; ++c) {
        buf_t *b = &H->casc[c];
        int accepting = (H->t % cfg->accept_period[c]) == 0;
        int full = (b->n == b->cap);
        if (accepting) {
            b->accepted++;
            if (!full) {
                buf_append(b, x);
                H->t++;
                return;
            }
            item_t old = buf_pop_oldest(b);
            buf_append(b, x);
            x = old;                         /* the evicted item is offered to the next cascade */
        } else {
            if (!full) {                     /* eager add */
                buf_append(b, x);
                H->t++;
                return;
            }
            item_t *newest = &b->it[b->n - 1];
            log_select(H, x.id, x.mu, newest->id, newest->mu);
            if (cfg->token_selection && x.mu > newest->mu) {
                log_discard(H, newest->id);
                item_free(newest);
                *newest = x;
                b->swaps++;
            } else {
                log_discard(H, x.id);
                item_free(&x);
            }
            b->discards++;
            H->t++;
            return;
        }
    }
    /* evicted from the last cascade */
    H->casc[cfg->n_cascades - 1].discards++;
    log_discard(H, x.id);
    item_free(&x);
    H->t++;
}

/* ------------------------------------------------------------------ life cycle */

oracle_seq *oracle_create(const oracle_config *cfg)
{
    if (!cfg || cfg->n_cascades < 1 || cfg->n_cascades > ORACLE_MAX_CASCADES) return NULL;
    if (cfg->head_dim % 2 || cfg->n_q_heads % cfg->n_kv_heads) return NULL;
    oracle_seq *S = (oracle_seq *)calloc(1, sizeof(oracle_seq));
    S->cfg = *cfg;
    if (S->cfg.softmax_scale == 0.0) S->cfg.softmax_scale = 1.0 / sqrt((double)cfg->head_dim);
    S->head = (head_t *)calloc((size_t)cfg->n_kv_heads, sizeof(head_t));
    for (int h = 0; h < cfg->n_kv_heads; ++h) {
        head_t *H = &S->head[h];
        H->sink.cap = cfg->n_sink;
        H->sink.it = (item_t *)calloc((size_t)(cfg->n_sink > 0 ? cfg->n_sink : 1), sizeof(item_t));
        for (int c = 0; c < cfg->n_cascades; ++c) {
            H->casc[c].cap = cfg->cascade_sizes[c];
            H->casc[c].it = (item_t *)calloc((size_t)cfg->cascade_sizes[c], sizeof(item_t));
        }
    }
    return S;
}

static void head_clear(const oracle_config *cfg, head_t *H)
{
    for (int i = 0; i < H->sink.n; ++i) item_free(&H->sink.it[i]);
    H->sink.n = 0;
    for (int c = 0; c < cfg->n_cascades; ++c) {
        for (int i = 0; i < H->casc[c].n; ++i) item_free(&H->casc[c].it[i]);
        H->casc[c].n = 0;
    }
}

void oracle_destroy(oracle_seq *S)
{
    if (!S) return;
    for (int h = 0; h < S->cfg.n_kv_heads; ++h) {
        head_t *H = &S->head[h];
        head_clear(&S->cfg, H);
        free(H->sink.it);
        for (int c = 0; c < S->cfg.n_cascades; ++c) free(H->casc[c].it);
        free(H->last_delta);
        free(H->discard_log);
        free(H->select_ids);
        free(H->select_mu);
    }
    free(S->head);
    free(S);
}

/* cache order: sinks, then the last cascade oldest to newest, ..., then the first cascade */
static int64_t head_order(const oracle_config *cfg, head_t *H, item_t **out)
{
    int64_t n = 0;
    for (int i = 0; i < H->sink.n; ++i) out[n++] = &H->sink.it[i];
    for (int c = cfg->n_cascades - 1; c >= 0; --c)
        for (int i = 0; i < H->casc[c].n; ++i) out[n++] = &H->casc[c].it[i];
    return n;
}

static int64_t head_count(const oracle_config *cfg, const head_t *H)
{
    int64_t n = H->sink.n;
    for (int c = 0; c < cfg->n_cascades; ++c) n += H->casc[c].n;
    return n;
}

/* ------------------------------------------------------------------ one chunk */

/*
 * Attention of the query rows [row_lo, row_hi) of a chunk of Q tokens for KV head g, against the
 * cache as it is plus the chunk's own keys up to each row (Eq. 2, Fig. 4), and the EMA recurrence
 * over exactly those rows, started at 0 before row_lo and reduced over the query heads of the
 * group.  With row_lo = 0 and row_hi = Q this is the whole chunk.  The state is not modified.
 * out [Q][Hq][d]: only the evaluated rows and the heads of g are written.
 * delta [n + Q]: reduced increments in cache order, then chunk tokens.
 */
/*
 * step_of_key (may be NULL: exact scores) [n + Q]: inner-loop step, counted from 1, at which the
 * program visits each key (cache order, then the chunk's keys); steps_of_row [G][Q]: number of
 * inner-loop steps of the program that holds query row (head of the group, chunk row).  With them
 * the increments are Alg. 3's single-pass values (reading R8) instead of the exact probabilities;
 * the outputs are the exact attention either way.
 */
static void eval_rows_scheduled(const oracle_seq *S, int g, const float *q, const float *k, const float *v,
                                int Q, int row_lo, int row_hi, const int32_t *step_of_key, const int32_t *steps_of_row,
                                double *out, double *delta)
{
    const oracle_config *cfg = &S->cfg;
    head_t *H = &S->head[g];
    const int d = cfg->head_dim, Hq = cfg->n_q_heads, Hkv = cfg->n_kv_heads;
    const int G = Hq / Hkv;
    const double beta = cfg->ema_beta;

    int64_t cap_total = cfg->n_sink;
    for (int c = 0; c < cfg->n_cascades; ++c) cap_total += cfg->cascade_sizes[c];
    item_t **order = (item_t **)malloc(sizeof(item_t *) * (size_t)(cap_total + 1));
    const int64_t n = head_order(cfg, H, order);
    const int64_t nk = n + Q;

    /* keys rotated at their index in the cache; chunk token i sits at index n + i */
    double *kr = (double *)malloc(sizeof(double) * (size_t)nk * (size_t)d);
    double *vv = (double *)malloc(sizeof(double) * (size_t)nk * (size_t)d);
    double *tmp = (double *)malloc(sizeof(double) * (size_t)d);
    for (int64_t j = 0; j < n; ++j) {
        rope(order[j]->k, d, (double)j, cfg->rope_base, kr + j * d);
        memcpy(vv + j * d, order[j]->v, sizeof(double) * (size_t)d);
    }
    for (int i = 0; i < row_hi; ++i) {
        const float *ki = k + ((size_t)i * Hkv + g) * d, *vi = v + ((size_t)i * Hkv + g) * d;
        for (int e = 0; e < d; ++e) { tmp[e] = ki[e]; vv[(n + i) * d + e] = vi[e]; }
        rope(tmp, d, (double)(n + i), cfg->rope_base, kr + (n + i) * d);
    }

    double *delta_h = (double *)malloc(sizeof(double) * (size_t)nk);   /* one query head */
    double *p = (double *)malloc(sizeof(double) * (size_t)nk);
    double *qr = (double *)malloc(sizeof(double) * (size_t)d);

    for (int hh = 0; hh < G; ++hh) {
        const int h = g * G + hh;
        for (int64_t j = 0; j < nk; ++j) delta_h[j] = 0.0;
        for (int i = row_lo; i < row_hi; ++i) {
            const float *qi = q + ((size_t)i * Hq + h) * d;
            for (int e = 0; e < d; ++e) tmp[e] = qi[e];
            rope(tmp, d, (double)(n + i), cfg->rope_base, qr);
            const int64_t vis = n + i + 1;              /* cache and own chunk up to itself */
            double mx = -INFINITY;
            for (int64_t j = 0; j < vis; ++j) {
                double s = 0.0;
                const double *kj = kr + j * d;
                for (int e = 0; e < d; ++e) s += qr[e] * kj[e];
                s *= cfg->softmax_scale;
                p[j] = s;
                if (s > mx) mx = s;
            }
            double sum = 0.0;
            for (int64_t j = 0; j < vis; ++j) { p[j] = exp(p[j] - mx); sum += p[j]; }
            double *o = out + ((size_t)i * Hq + h) * d;
            for (int e = 0; e < d; ++e) o[e] = 0.0;
            for (int64_t j = 0; j < vis; ++j) {
                p[j] /= sum;
                const double *vj = vv + j * d;
                for (int e = 0; e < d; ++e) o[e] += p[j] * vj[e];
            }
            if (step_of_key) {
                /* Alg. 3: what the sweep adds for key j at its step gamma = step_of_key[j], with the
                   normaliser as it stands after that step and rho = T - gamma steps to go */
                const int T = steps_of_row[(size_t)hh * Q + i];
                double *l_after = (double *)calloc((size_t)T + 1, sizeof(double));
                for (int64_t j = 0; j < vis; ++j) l_after[step_of_key[j]] += p[j] * sum;   /* S^ = exp(S - m) again */
                for (int t = 1; t <= T; ++t) l_after[t] += l_after[t - 1];
                for (int64_t j = 0; j < vis; ++j) {
                    const double gamma = (double)step_of_key[j], rho = (double)T - gamma;
                    const double l = l_after[step_of_key[j]];
                    p[j] = (p[j] * sum) / (l + l * rho / gamma);
                }
                free(l_after);
            }
            /* one EMA time step per query row; keys this row cannot see receive 0 */
            for (int64_t j = 0; j < nk; ++j) delta_h[j] = beta * delta_h[j] + (1.0 - beta) * (j < vis ? p[j] : 0.0);
        }
        for (int64_t j = 0; j < nk; ++j) {
            if (hh == 0) delta[j] = delta_h[j];
            else if (cfg->head_reduce == 0) delta[j] = delta_h[j] > delta[j] ? delta_h[j] : delta[j];
            else delta[j] += delta_h[j];
        }
    }
    if (cfg->head_reduce == 1) for (int64_t j = 0; j < nk; ++j) delta[j] /= (double)G;
    free(order); free(kr); free(vv); free(tmp); free(delta_h); free(p); free(qr);
}

static void eval_rows(const oracle_seq *S, int g, const float *q, const float *k, const float *v,
                      int Q, int row_lo, int row_hi, double *out, double *delta)
{
    eval_rows_scheduled(S, g, q, k, v, Q, row_lo, row_hi, NULL, NULL, out, delta);
}

/* The reduced increments of the whole chunk for KV head g (not applied yet). */
static double *chunk_increments(oracle_seq *S, int g, const float *q, const float *k, const float *v,
                                int Q, const int32_t *step_of_key, const int32_t *steps_of_row, double *out)
{
    const int64_t n = head_count(&S->cfg, &S->head[g]);
    double *delta = (double *)malloc(sizeof(double) * (size_t)(n + Q));
    eval_rows_scheduled(S, g, q, k, v, Q, 0, Q, step_of_key, steps_of_row, out, delta);
    return delta;
}

/* The EMA update of the cached items of KV head g with the increments delta (ownership of
 * delta passes to the head), then the insertion of the chunk's tokens. */
static void chunk_apply(oracle_seq *S, int g, const float *k, const float *v, int Q, double *delta)
{
    const oracle_config *cfg = &S->cfg;
    head_t *H = &S->head[g];
    const int d = cfg->head_dim, Hkv = cfg->n_kv_heads;
    const double beta = cfg->ema_beta;
    const int64_t n = head_count(cfg, H);

    /* cached items decay once per row of the chunk, then receive the reduced increment */
    int64_t cap_total = cfg->n_sink;
    for (int c = 0; c < cfg->n_cascades; ++c) cap_total += cfg->cascade_sizes[c];
    item_t **order = (item_t **)malloc(sizeof(item_t *) * (size_t)(cap_total + 1));
    head_order(cfg, H, order);
    for (int64_t j = 0; j < n; ++j) {
        double mu = order[j]->mu;
        for (int i = 0; i < Q; ++i) mu *= beta;
        order[j]->mu = mu + delta[j];
    }
    free(order);
    free(H->last_delta);
    H->last_delta = delta;
    H->last_delta_n = n + Q;

    /* the chunk's tokens enter the cache in order with their frozen scores (Alg. 1, Alg. 2) */
    for (int i = 0; i < Q; ++i) {
        item_t x;
        x.id = H->n_seen++;
        x.mu = delta[n + i];
        x.k = (double *)malloc(sizeof(double) * (size_t)d);
        x.v = (double *)malloc(sizeof(double) * (size_t)d);
        const float *ki = k + ((size_t)i * Hkv + g) * d, *vi = v + ((size_t)i * Hkv + g) * d;
        for (int e = 0; e < d; ++e) { x.k[e] = ki[e]; x.v[e] = vi[e]; }
        cache_insert(cfg, H, x);
    }
}

/*
 * One chunk of Q tokens for the KV heads [kv_lo, kv_hi).
 * q [Q][Hq][d], k and v [Q][Hkv][d] float32 (un-rotated), out [Q][Hq][d] float64
 * (only the query heads of the selected KV heads are written).
 * A decode step is a chunk of one token.
 * Homogeneous heads (Appendix "Head Policy and Head Reduction") need all KV heads at once:
 * the increments are reduced over ALL query heads (the max of the per-group maxima; the mean of
 * the per-group means, the groups being equally large), every KV head then updates and inserts
 * with that one vector, so all KV heads hold the same tokens at all times.
 */
static int chunk_scheduled(oracle_seq *S, const float *q, const float *k, const float *v, int Q,
                           double *out, int kv_lo, int kv_hi, const int32_t *step_of_key, const int32_t *steps_of_row)
{
    if (!S || !q || !k || !v || !out || Q < 1) return -1;
    if (kv_lo < 0 || kv_hi > S->cfg.n_kv_heads || kv_lo >= kv_hi) return -1;
    const int Hkv = S->cfg.n_kv_heads;
    if (S->cfg.head_policy == 1 && (kv_lo != 0 || kv_hi != Hkv)) return -1;
    double **delta = (double **)calloc((size_t)Hkv, sizeof(double *));
#pragma omp parallel for schedule(dynamic, 1)
    for (int g = kv_lo; g < kv_hi; ++g) delta[g] = chunk_increments(S, g, q, k, v, Q, step_of_key, steps_of_row, out);
    if (S->cfg.head_policy == 1) {
        const int64_t nk = head_count(&S->cfg, &S->head[0]) + Q;   /* the same for every head */
        for (int64_t j = 0; j < nk; ++j) {
            double r = delta[0][j];
            for (int g = 1; g < Hkv; ++g) {
                if (S->cfg.head_reduce == 0) r = delta[g][j] > r ? delta[g][j] : r;
                else r += delta[g][j];
            }
            if (S->cfg.head_reduce == 1) r /= (double)Hkv;
            for (int g = 0; g < Hkv; ++g) delta[g][j] = r;
        }
    }
#pragma omp parallel for schedule(dynamic, 1)
    for (int g = kv_lo; g < kv_hi; ++g) chunk_apply(S, g, k, v, Q, delta[g]);
    free(delta);
    return 0;
}

int oracle_chunk(oracle_seq *S, const float *q, const float *k, const float *v, int Q,
                 double *out, int kv_lo, int kv_hi)
{
    return chunk_scheduled(S, q, k, v, Q, out, kv_lo, kv_hi, NULL, NULL);
}

/*
 * The same chunk with Alg. 3's single-pass scores (reading R8) in place of the exact ones.  The
 * schedule must be the same for all selected KV heads (they hold equally many items):
 * step_of_key [count + Q], steps_of_row [G][Q]; steps are counted from 1 and never exceed the
 * row's number of steps for a key the row can see.
 */
int oracle_chunk_single_pass(oracle_seq *S, const float *q, const float *k, const float *v, int Q,
                             double *out, int kv_lo, int kv_hi, const int32_t *step_of_key, const int32_t *steps_of_row)
{
    if (!step_of_key || !steps_of_row) return -1;
    return chunk_scheduled(S, q, k, v, Q, out, kv_lo, kv_hi, step_of_key, steps_of_row);
}

int oracle_eval_rows_single_pass(const oracle_seq *S, int g, const float *q, const float *k, const float *v, int Q,
                                 int row_lo, int row_hi, const int32_t *step_of_key, const int32_t *steps_of_row,
                                 double *out, double *delta)
{
    if (!S || !q || !k || !v || !out || !delta || !step_of_key || !steps_of_row) return -1;
    if (g < 0 || g >= S->cfg.n_kv_heads || row_lo < 0 || row_hi > Q || row_lo >= row_hi) return -1;
    eval_rows_scheduled(S, g, q, k, v, Q, row_lo, row_hi, step_of_key, steps_of_row, out, delta);
    return 0;
}

/*
 * Rows [row_lo, row_hi) of a chunk only, for KV head g, without touching the cache: their
 * outputs and the EMA increments those rows alone produce (see eval_rows).  Lets a test check
 * sampled rows of a chunk that is too long to evaluate whole.  delta holds count(g) + Q values.
 */
int oracle_eval_rows(const oracle_seq *S, int g, const float *q, const float *k, const float *v, int Q,
                     int row_lo, int row_hi, double *out, double *delta)
{
    if (!S || !q || !k || !v || !out || !delta) return -1;
    if (g < 0 || g >= S->cfg.n_kv_heads || row_lo < 0 || row_hi > Q || row_lo >= row_hi) return -1;
    eval_rows(S, g, q, k, v, Q, row_lo, row_hi, out, delta);
    return 0;
}

/* Insert one item with a given score into KV head g (Alg. 2 alone, for tests of the policy). */
int oracle_insert_scored(oracle_seq *S, int g, double score)
{
    if (!S || g < 0 || g >= S->cfg.n_kv_heads) return -1;
    head_t *H = &S->head[g];
    const int d = S->cfg.head_dim;
    item_t x;
    x.id = H->n_seen++;
    x.mu = score;
    x.k = (double *)calloc((size_t)d, sizeof(double));
    x.v = (double *)calloc((size_t)d, sizeof(double));
    cache_insert(&S->cfg, H, x);
    return 0;
}

/* ------------------------------------------------------------------ state access */

int64_t oracle_count(const oracle_seq *S, int g) { return head_count(&S->cfg, &S->head[g]); }
int64_t oracle_t(const oracle_seq *S, int g) { return S->head[g].t; }
int64_t oracle_n_seen(const oracle_seq *S, int g) { return S->head[g].n_seen; }

/*
 * State of KV head g in cache order.  ids/mu/cascade_of [count]; cascade_of is 0 for a
 * sink and c (1-based) for cascade c.  counts [1 + n_cascades] = sink fill, cascade fills.
 * stats [3 * n_cascades] = accepted, swaps, discards per cascade.  kv (may be NULL)
 * receives K then V, each [count][d].
 */
int oracle_get_state(oracle_seq *S, int g, int64_t *ids, double *mu, int32_t *cascade_of,
                     int64_t *counts, int64_t *stats, double *kv)
{
    const oracle_config *cfg = &S->cfg;
    head_t *H = &S->head[g];
    const int d = cfg->head_dim;
    int64_t n = 0, total = head_count(cfg, H);
    for (int i = 0; i < H->sink.n; ++i, ++n) {
        ids[n] = H->sink.it[i].id; mu[n] = H->sink.it[i].mu; cascade_of[n] = 0;
        if (kv) { memcpy(kv + n * d, H->sink.it[i].k, sizeof(double) * (size_t)d);
                  memcpy(kv + (total + n) * d, H->sink.it[i].v, sizeof(double) * (size_t)d); }
    }
    for (int c = cfg->n_cascades - 1; c >= 0; --c)
        for (int i = 0; i < H->casc[c].n; ++i, ++n) {
            ids[n] = H->casc[c].it[i].id; mu[n] = H->casc[c].it[i].mu; cascade_of[n] = c + 1;
            if (kv) { memcpy(kv + n * d, H->casc[c].it[i].k, sizeof(double) * (size_t)d);
                      memcpy(kv + (total + n) * d, H->casc[c].it[i].v, sizeof(double) * (size_t)d); }
        }
    counts[0] = H->sink.n;
    for (int c = 0; c < cfg->n_cascades; ++c) {
        counts[1 + c] = H->casc[c].n;
        stats[3 * c + 0] = H->casc[c].accepted;
        stats[3 * c + 1] = H->casc[c].swaps;
        stats[3 * c + 2] = H->casc[c].discards;
    }
    return 0;
}

/*
 * Replace the state of KV head g.  Rows are in cache order: counts[0] sinks, then
 * counts[n_cascades] items of the last cascade oldest to newest, ..., then counts[1]
 * items of the first cascade.  k, v are [count][d] float32.
 */
int oracle_set_state(oracle_seq *S, int g, const int64_t *ids, const double *mu, const int64_t *counts,
                     const float *k, const float *v, int64_t t, int64_t n_seen)
{
    const oracle_config *cfg = &S->cfg;
    head_t *H = &S->head[g];
    const int d = cfg->head_dim;
    if (counts[0] > cfg->n_sink) return -1;
    for (int c = 0; c < cfg->n_cascades; ++c) if (counts[1 + c] > cfg->cascade_sizes[c]) return -1;
    head_clear(cfg, H);
    int64_t r = 0;
    for (int part = 0; part <= cfg->n_cascades; ++part) {
        buf_t *b = part == 0 ? &H->sink : &H->casc[cfg->n_cascades - part];
        int64_t cnt = part == 0 ? counts[0] : counts[1 + cfg->n_cascades - part];
        for (int64_t i = 0; i < cnt; ++i, ++r) {
            item_t x;
            x.id = ids[r]; x.mu = mu[r];
            x.k = (double *)malloc(sizeof(double) * (size_t)d);
            x.v = (double *)malloc(sizeof(double) * (size_t)d);
            for (int e = 0; e < d; ++e) { x.k[e] = k[r * d + e]; x.v[e] = v[r * d + e]; }
            buf_append(b, x);
        }
    }
    H->t = t;
    H->n_seen = n_seen;
    return 0;
}

int64_t oracle_last_delta(const oracle_seq *S, int g, double *out, int64_t cap)
{
    const head_t *H = &S->head[g];
    int64_t n = H->last_delta_n < cap ? H->last_delta_n : cap;
    if (out) memcpy(out, H->last_delta, sizeof(double) * (size_t)n);
    return H->last_delta_n;
}

/* The selection comparisons taken so far (see head_t); returns their number.  ids and mu
 * receive [min(n, cap)][2] values: incoming item, newest item. */
int64_t oracle_select_log(const oracle_seq *S, int g, int64_t *ids, double *mu, int64_t cap)
{
    const head_t *H = &S->head[g];
    int64_t n = H->n_select_log < cap ? H->n_select_log : cap;
    if (ids && n > 0) memcpy(ids, H->select_ids, sizeof(int64_t) * 2 * (size_t)n);
    if (mu && n > 0) memcpy(mu, H->select_mu, sizeof(double) * 2 * (size_t)n);
    return H->n_select_log;
}

void oracle_clear_logs(oracle_seq *S, int g)
{
    S->head[g].n_select_log = 0;
    S->head[g].n_discard_log = 0;
}

int64_t oracle_discard_log(const oracle_seq *S, int g, int64_t *out, int64_t cap)
{
    const head_t *H = &S->head[g];
    int64_t n = H->n_discard_log < cap ? H->n_discard_log : cap;
    if (out) memcpy(out, H->discard_log, sizeof(int64_t) * (size_t)n);
    return H->n_discard_log;
}
