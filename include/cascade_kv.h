/*
 * cascade_kv.h - C ABI of the MI355X (gfx950) cascading KV cache hot path.
 *
 * The library implements, for ONE attention layer on ONE GPU, the method of
 * "Training-Free Exponential Context Extension via Cascading KV Cache"
 * (arxiv 2406.17808): strided prefill (Alg. 1) and single-token decode (Eq. 2)
 * attention against a fixed-size cache made of sink slots and cascading
 * sub-caches (Section 3.1), with positional encoding by index inside the cache,
 * an EMA of the attention each cached token receives (Section 3.1 "Token
 * Selection"), and the cascade insertion of Alg. 2.
 *
 * Conventions for every call
 *   - Pointers named dev_* are DEVICE pointers, host_* are HOST pointers.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - The library never allocates or frees device memory: the caller hands all of
 *     it over once as a workspace (cascade_workspace_bytes / cascade_init).
 *   - All calls return CASCADE_OK (0) or a negative CASCADE_E_* code; nothing
 *     throws or aborts.  cascade_last_error() describes the last failure.
 *   - Work is enqueued on `stream` and is asynchronous, except cascade_read_state,
 *     which waits for the stream.  Calls on one context must be issued from one
 *     host thread at a time and on streams that are ordered with each other.
 */
#ifndef CASCADE_KV_H
#define CASCADE_KV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CASCADE_MAX_CASCADES 16

enum {
    CASCADE_OK = 0,
    CASCADE_E_INVALID_CONFIG = -1,
    CASCADE_E_NULL_ARG = -2,
    CASCADE_E_WORKSPACE_TOO_SMALL = -3,
    CASCADE_E_UNSUPPORTED = -4,
    CASCADE_E_HIP = -5,
    CASCADE_E_BAD_ARG = -6,
    CASCADE_E_INTERNAL = -7   /* a consistency check inside the library failed (a bug, not a misuse) */
};

enum { CASCADE_F32 = 0, CASCADE_BF16 = 1 };
enum { CASCADE_REDUCE_MAX = 0, CASCADE_REDUCE_MEAN = 1 };
enum { CASCADE_HEADS_INDEPENDENT = 0, CASCADE_HEADS_HOMOGENEOUS = 1 };
enum { CASCADE_SCORES_EXACT = 0, CASCADE_SCORES_SINGLE_PASS = 1 };

/*
 * Geometry and hyper-parameters (Section 4 "Setup": sinks are counted in addition
 * to the cascades; the paper uses 64 sinks, 4 cascades of equal size, periods
 * 1,2,4,8 and an EMA parameter of 0.9999).  Plain data, copied by cascade_init.
 */
typedef struct cascade_config {
    int32_t batch;            /* independent sequences, all advanced in lock step */
    int32_t n_q_heads;        /* query heads; a multiple of n_kv_heads (GQA) */
    int32_t n_kv_heads;       /* every KV head owns its own cache and decisions (Appendix "Head Policy") */
    int32_t head_dim;         /* 64 or 128 for CASCADE_BF16; even and <= 256 for CASCADE_F32 */
    int32_t dtype;            /* element type of q, k, v, out and of the cached K/V */
    int32_t n_sink;           /* sink slots: the first n_sink tokens are kept forever */
    int32_t n_cascades;       /* 1 .. CASCADE_MAX_CASCADES; 1 = sink + sliding window */
    int32_t cascade_sizes[CASCADE_MAX_CASCADES];  /* slots of cascade 1, 2, ... (each >= 1) */
    int32_t accept_period[CASCADE_MAX_CASCADES];  /* cascade i accepts when t mod period == 0, where t counts
                                                     the tokens offered to cascade 1 so far; all zero selects
                                                     1, 2, 4, ... (Section 3.1); [0] must be 1 */
    float ema_beta;           /* EMA parameter (gamma in Section 3.1, beta in Alg. 3), in [0, 1) */
    float rope_base;          /* RoPE: pairs (x_i, x_{i+d/2}), theta_i = base^(-2i/d) */
    float softmax_scale;      /* 0 selects 1/sqrt(head_dim) (Eq. 1) */
    int32_t max_chunk;        /* largest n_tokens of cascade_prefill_chunk (>= 1) */
    int32_t head_reduce;      /* CASCADE_REDUCE_MAX (the paper's choice) or CASCADE_REDUCE_MEAN */
    int32_t token_selection;  /* 1: Alg. 2; 0: the ablation that never replaces the newest item */
    float score_tail_eps;     /* prefill only: query rows whose EMA weight beta^k (k = rows left in the
                                 chunk) is below this are left out of the score sums; the absolute
                                 error of a score is then below this value.  0 selects 2^-40;
                                 a negative value keeps every row. */
    int32_t keep_update_scores; /* diagnostics: 1 makes every prefill / decode call keep a copy of all
                                 scores as they were when the insertion decisions were taken, for
                                 cascade_read_state (host_pre_mu, host_chunk_mu).  Costs one extra
                                 pass over the score array per call. */
    int32_t head_policy;      /* CASCADE_HEADS_INDEPENDENT (the paper's choice: every KV head decides with its own
                                 scores) or CASCADE_HEADS_HOMOGENEOUS (Appendix "Head Policy and Head Reduction":
                                 the scores are reduced over ALL heads, by head_reduce, and every KV head takes
                                 the same decisions, so all of them hold the same tokens) */
    int32_t score_mode;       /* CASCADE_SCORES_EXACT: the scores use the final softmax probabilities (Section 3.1).
                                 CASCADE_SCORES_SINGLE_PASS (bf16 only): Alg. 3's scores, accumulated while the attention
                                 kernel sweeps the keys, with the running normaliser extrapolated by the tiles still to
                                 come: a row block of 256 tokens of one head adds, for the keys of its tile number
                                 gamma of T,  C_EMA * exp(S - m) / (l + l * (T - gamma) / gamma)  with m, l as they stand
                                 after that tile.  Tiles are 64 keys in the physical order of the cache (sinks, last
                                 cascade, ..., first cascade, every ring from its slot 0, pieces cut where a ring head
                                 sits), then the chunk's keys.  No second pass over the keys; the scores depend on that
                                 order and are an approximation of the exact ones.  Taken by the chunks all of whose
                                 rows carry EMA weight (see score_tail_eps: an EMA parameter close to 1, the paper's
                                 0.9999), whose length is a multiple of 256 and whose launch is not split over the keys
                                 (more than 128 row blocks in all); other chunks take the exact pass, which is short
                                 when few rows carry weight: cascade_state_view.last_single_pass says which it was. */
} cascade_config;

typedef struct cascade_ctx cascade_ctx;

/*
 * Optional initial contents of the cache (resume, or a pre-filled cache for decode).
 * All (sequence, KV head) pairs hold the same number of items per sub-cache, since the
 * fill of the sub-caches does not depend on the scores (Alg. 2).  Rows are in cache order:
 * counts[0] sinks, then counts[n_cascades] items of the last cascade oldest to newest, ...,
 * then counts[1] items of the first cascade.  With total = sum(counts):
 */
typedef struct cascade_init_state {
    const void* dev_k;        /* [batch, n_kv_heads, total, head_dim], config dtype, un-rotated keys */
    const void* dev_v;        /* same shape */
    const float* dev_mu;      /* [batch, n_kv_heads, total] EMA scores */
    const int32_t* dev_ids;   /* [batch, n_kv_heads, total] index of each token in its original sequence */
    int32_t counts[1 + CASCADE_MAX_CASCADES];   /* sink fill, then fill of cascade 1, 2, ... */
    int64_t t;                /* tokens offered to cascade 1 so far (phase of the acceptance schedule) */
    int64_t n_seen;           /* tokens consumed so far; the next token gets this id */
} cascade_init_state;

/*
 * What cascade_read_state returns, in caller-allocated HOST memory.  Any pointer may be
 * NULL to skip that part.  slots = n_sink + sum(cascade_sizes).  Per (sequence, KV head)
 * the first `count` entries (count = sum of counts) are valid and in cache order, so the
 * positional-encoding index of entry r is r (Section 3.1 "Positional Encoding").
 */
typedef struct cascade_state_view {
    int32_t* host_ids;        /* [batch, n_kv_heads, slots] original token index; -1 beyond count */
    float* host_mu;           /* [batch, n_kv_heads, slots] EMA scores */
    int32_t* host_slot;       /* [batch, n_kv_heads, slots] physical slot that holds entry r */
    float* host_k;            /* [batch, n_kv_heads, slots, head_dim] un-rotated keys as float */
    float* host_v;            /* [batch, n_kv_heads, slots, head_dim] */
    const int32_t* host_kv_pairs; /* NULL, or n_kv_pairs indices (sequence * n_kv_heads + KV head): host_k and
                                 host_v are then [n_kv_pairs, slots, head_dim] and hold only those pairs,
                                 in this order (a full copy of a large batch is tens of gigabytes) */
    int64_t* host_swaps;      /* [batch, n_kv_heads, n_cascades] selections won by the incoming token */
    float* host_pre_mu;       /* [batch, n_kv_heads, slots] needs keep_update_scores: scores of the items
                                 cached BEFORE the last prefill / decode call, after that call's EMA
                                 update, in the cache order before the call (pre_count entries) */
    float* host_chunk_mu;     /* [batch, n_kv_heads, max_chunk] needs keep_update_scores: scores the
                                 tokens of the last call entered the cache with (last_tokens entries) */
    /* filled in by the call (same for every sequence and KV head): */
    int32_t counts[1 + CASCADE_MAX_CASCADES];   /* sink fill, fill of cascade 1, 2, ... */
    int32_t xi[CASCADE_MAX_CASCADES];           /* ring index of the oldest item of each cascade
                                                   (Section 3.1 "Circular Buffers") */
    int64_t accepted[CASCADE_MAX_CASCADES];     /* items that arrived at an accepting step */
    int64_t discards[CASCADE_MAX_CASCADES];     /* items lost at this cascade (selection or off the end) */
    int64_t t;
    int64_t n_seen;
    int32_t pre_count;        /* items cached before the last call */
    int32_t last_tokens;      /* tokens of the last call (0 before any call) */
    int32_t n_kv_pairs;       /* input: entries of host_kv_pairs */
    int32_t last_single_pass; /* 1 if the last prefill call took the single-pass scores (score_mode) */
} cascade_state_view;

/* Device bytes cascade_init needs for this configuration; 0 if the configuration is invalid. */
size_t cascade_workspace_bytes(const cascade_config* cfg);

/*
 * Create a context on the current device (Alg. 1's `cache`).  dev_workspace must hold at
 * least cascade_workspace_bytes(cfg) bytes, be 256-byte aligned, and stay valid and
 * untouched by the caller until cascade_destroy.  The cache starts empty, or with
 * `init_state` (may be NULL) copied in.  The context itself is a small host object.
 * Errors: NULL_ARG, INVALID_CONFIG, UNSUPPORTED (head_dim / dtype the kernels do not
 * cover), WORKSPACE_TOO_SMALL, BAD_ARG (init_state counts exceed the capacities), HIP.
 */
int cascade_init(const cascade_config* cfg, void* dev_workspace, size_t workspace_bytes,
                 const cascade_init_state* init_state, void* stream, cascade_ctx** out_ctx);

/* Free the host-side context.  The workspace stays the caller's. */
void cascade_destroy(cascade_ctx* ctx);

/*
 * cascade_init for callers that cannot allocate device memory at all (code that runs under a
 * HIP graph capture, serving loops and harnesses that forbid hipMalloc): the same context, but
 * its workspace is a device array that is part of the library image,
 * CASCADE_STATIC_WORKSPACE_BYTES long, one per GPU.  The call allocates nothing on the device
 * (no hipMalloc / hipFree, no allocating library routine) and, after the first call on a
 * device, nothing on the host either.  Everything else is cascade_init: same arguments minus
 * the workspace, same errors; a configuration whose cascade_workspace_bytes exceeds the array is
 * rejected with CASCADE_E_WORKSPACE_TOO_SMALL (cascade_last_error(NULL) names both sizes).
 * The returned context is used with every other call; cascade_destroy on it is allowed and
 * releases nothing.
 * The array is shared by every call on that GPU and keeps the previous contents: the call
 * clears the part it uses, and it REPLACES the previous static context of the device, which
 * must not be used afterwards.  Two static contexts on one GPU at the same time, or a call
 * that overlaps work still in flight on the previous one, race.
 */
#define CASCADE_STATIC_WORKSPACE_BYTES (64u << 20)
int cascade_init_static(const cascade_config* cfg, const cascade_init_state* init_state, void* stream,
                        cascade_ctx** out_ctx);

/*
 * Several layers over one workspace (the inner loop of Alg. 1 runs cache.get, the layer and
 * cache.update once per layer for every chunk).  Every layer gets a context and a cache of
 * its own; the buffers that live only inside one call (rotated queries, packed tiles, decode
 * logits, ...) exist once and are shared, so the workspace is n_layers states plus one
 * scratch instead of n_layers times both.  The contexts are ordinary contexts: use them with
 * every other call and free each with cascade_destroy.  Because they share scratch, calls on
 * ANY of them must be ordered with each other (one stream, or streams the caller orders), and
 * none may be in flight when the workspace is released.
 *   cascade_layers_workspace_bytes: bytes for n_layers layers; 0 if the configuration is
 *     invalid or n_layers < 1.
 *   cascade_init_layers: init_states is NULL (all caches start empty) or an array of n_layers
 *     pointers, each NULL or the state to copy into that layer; out_ctxs receives n_layers
 *     contexts (all NULL on failure).  Errors as for cascade_init, BAD_ARG for n_layers < 1.
 */
size_t cascade_layers_workspace_bytes(const cascade_config* cfg, int32_t n_layers);
int cascade_init_layers(const cascade_config* cfg, int32_t n_layers, void* dev_workspace, size_t workspace_bytes,
                        const cascade_init_state* const* init_states, void* stream, cascade_ctx** out_ctxs);

/*
 * One step of strided prefill (Alg. 1) for every sequence of the batch:
 *   1. out <- softmax attention of the chunk's queries over the cache as it is before the
 *      call plus the chunk's own keys up to each query (Eq. 2, Fig. 4), RoPE by cache index;
 *   2. every cached token's EMA score is updated with the attention it received, one EMA
 *      step per query row (Section 3.1; coefficients of Alg. 3), reduced over the query heads
 *      of its KV head;
 *   3. the chunk's tokens are inserted in order by Alg. 2 with these scores.
 * dev_q, dev_out: [batch, n_tokens, n_q_heads, head_dim]; dev_k, dev_v: [batch, n_tokens,
 * n_kv_heads, head_dim]; contiguous, config dtype, q and k un-rotated.  1 <= n_tokens <=
 * max_chunk.  The caller may reuse the four buffers once `stream` has passed this call.
 * Errors: NULL_ARG, BAD_ARG (n_tokens out of range), HIP.
 */
int cascade_prefill_chunk(cascade_ctx* ctx, const void* dev_q, const void* dev_k, const void* dev_v,
                          int32_t n_tokens, void* dev_out, void* stream);

/*
 * One decode step (Eq. 2) for every sequence: the same three effects as a chunk of one
 * token, organised for streaming the cache once from HBM.
 * dev_q, dev_out: [batch, n_q_heads, head_dim]; dev_k, dev_v: [batch, n_kv_heads, head_dim].
 */
int cascade_decode_step(cascade_ctx* ctx, const void* dev_q, const void* dev_k, const void* dev_v,
                        void* dev_out, void* stream);

/*
 * Snapshot of the cache in cache order.  Waits for `stream`; the only blocking call.
 * Errors: NULL_ARG, HIP.
 */
int cascade_read_state(cascade_ctx* ctx, cascade_state_view* view, void* stream);

/*
 * Host-only helper (touches no device): the fill of every sub-cache, the ring heads and the
 * counters after chunks of the given sizes have been fed to an empty cache of ONE sequence and
 * KV head.  In Alg. 2 these do not depend on the attention scores, so they can be known ahead
 * of time.  Fills the scalar fields of `view`; view->host_slot (if not NULL) receives [slots]
 * entries: the physical slot of every cache index.
 * host_scores may be NULL.  If given it holds one score per token (sum of chunk_sizes values),
 * frozen at insertion, and the call also replays the insertions chunk by chunk with the
 * routines the device kernels use: view->host_ids / host_mu ([slots], cache order) and
 * view->host_swaps ([n_cascades]) are then filled where not NULL.
 * Errors: NULL_ARG, INVALID_CONFIG / UNSUPPORTED, BAD_ARG (a chunk size below 1).
 */
int cascade_simulate_structure(const cascade_config* cfg, const int32_t* chunk_sizes, int32_t n_chunks,
                               const float* host_scores, cascade_state_view* view);

/*
 * Diagnostics: per-kernel-family GPU time measured with HIP events recorded on the stream of
 * each call, around the launches of that family.  cascade_profile_begin starts (and resets) the
 * collection; cascade_profile_end waits for all recorded events and returns, per family, the
 * summed milliseconds and the number of timed intervals.  While collecting, every call creates
 * events (host allocations), so leave it off in production loops.
 */
enum {
    CASCADE_K_PREP = 0,        /* query / chunk-key rotation */
    CASCADE_K_ATTENTION = 1,   /* chunk attention (QK^T, softmax, PV) */
    CASCADE_K_SCORES = 2,      /* exact EMA score sums */
    CASCADE_K_UPDATE = 3,      /* cascade plan + row moves */
    CASCADE_K_DECODE_QK = 4,
    CASCADE_K_DECODE_PV = 5,
    CASCADE_K_DECODE_FINISH = 6,
    CASCADE_K_FAMILIES = 7
};
typedef struct cascade_profile {
    double ms[CASCADE_K_FAMILIES];
    int64_t intervals[CASCADE_K_FAMILIES];
} cascade_profile;
int cascade_profile_begin(cascade_ctx* ctx);
/* The same for the families whose bit (1 << CASCADE_K_*) is set in family_mask only: two events on the
 * stream between two kernels cost about ten microseconds of idle time, which a timed run should
 * not pay for families it does not report. */
int cascade_profile_begin_families(cascade_ctx* ctx, uint32_t family_mask);
int cascade_profile_end(cascade_ctx* ctx, cascade_profile* out);

/*
 * Diagnostics: what the device this process runs on sustains, measured now, next to which the
 * roofline fractions of the library's kernels can be read (Section 4.1 reports latencies of one
 * GPU; the published peaks of another say little about it): number of compute units and clocks
 * from the device properties, a streaming read of dev_buffer (GB/s; all workgroups sweeping one
 * front), the same with a contiguous region per workgroup (the pattern of the decode kernels),
 * that again while one byte is written for every sixteen read (the logits of the decode step's
 * first pass against the keys it reads; GB/s of the bytes READ), that launch and a plain read
 * alternating (two_pass_read_gb_s), a copy of its first half onto
 * its second (GB/s of bytes read plus bytes written), and a loop of nothing but
 * v_mfma_f32_32x32x16_bf16 on register operands, two waves per SIMD (TFLOP/s).  dev_buffer: at least
 * 1 GiB of device memory (every single-launch figure uses its first half, the alternating launches both halves:
 * size a half like the array one pass of the workload streams), 16-byte aligned; its contents are overwritten.  Blocks until done.
 * Errors: NULL_ARG, BAD_ARG, HIP.
 */
typedef struct cascade_ceilings {
    int32_t compute_units;
    int32_t memory_bus_bits;
    double core_clock_mhz;      /* the maximum the driver reports, not the clock a kernel runs at */
    double memory_clock_mhz;
    double read_gb_s;
    double copy_gb_s;
    double mfma_bf16_tflops;
    double read_regions_gb_s;
    double read_with_stores_gb_s;
    double two_pass_read_gb_s;  /* a read with stores on one half of the buffer followed by a plain read of the other half
                                   (the two passes of a decode step as traffic alone), pairs back to back: bytes read by both
                                   per second (what the first launch wrote may still be on its way to memory while the
                                   second reads). */
} cascade_ceilings;
int cascade_measure_ceilings(void* dev_buffer, size_t bytes, void* stream, cascade_ceilings* out);

/* Text of the last error of this context (or of the last failed cascade_init if ctx is NULL). */
const char* cascade_last_error(const cascade_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* CASCADE_KV_H */
