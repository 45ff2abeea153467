// Launchers of the HIP kernels (one per kernel family), called by the host API.
#pragma once

#include "internal.h"

namespace ckv {

// A split attention launch has at most 256 workgroups of 256 rows.
constexpr int kAttnPartRows = 256 * 256;
constexpr int kMaxAttnSplits = 8;

// Device memory of one context, carved out of the caller's workspace.
struct DevBuffers {
    // cache
    void* Kc;        // [B,Hkv,slots,d] un-rotated keys
    void* Kr;        // [B,Hkv,slots,d] keys rotated to their physical slot index
    void* Vc;        // [B,Hkv,slots,d]
    float* mu;       // [B,Hkv,slots] EMA scores
    int32_t* ids;    // [B,Hkv,slots] original token index, -1 = empty
    int32_t* swaps;  // [B,Hkv,N]
    float* mu_snap;  // [B,Hkv,slots] diagnostics: scores when the last insertion decisions were taken
    // tables
    float2* rope;    // [rope_rows, d/2] (cos, sin) of index * theta_i
    float2* rope_t;  // bf16 MFMA path: the same, [d/4, rope_rows, 2] (index-minor: see rope_table_kernel)
    float* wrow;     // [max_chunk] beta^k (1 - beta): EMA weight of the row that has k rows after it
    // per-call scratch
    void* Qr;        // [n_qvar_max, B, Hq, max_chunk, d] rotated query copies (bf16 MFMA path: times scale * log2 e)
    void* Krc;       // [B,Hkv,max_chunk,d] chunk keys rotated to their chunk index
    void* Vch;       // [B,Hkv,max_chunk,d] chunk values, head-major
    void* Kt;        // [B,Hkv,vt_tiles,64,d] bf16 MFMA path: rotated keys of cache and chunk, tile by tile
    void* Vt;        // [B,Hkv,vt_tiles,d,64] the same for V, every tile transposed
    float* knorm2;   // [B,Hkv,vt_tiles] largest squared key norm of every packed tile
    float* lse;      // [B,Hq,max_chunk] log-sum-exp of every query row (natural log, scaled logits)
    float* mu_chunk; // [B,Hkv,max_chunk] scores of the chunk's tokens
    float* attn_part;// [kAttnPartRows, d + 2] bf16 MFMA path: partial outputs, maxima and row sums of a split attention launch
    float* negt;     // [B,Hq,max_chunk+64] bf16 MFMA path: exponent offsets of the score sums (-inf: row does not contribute)
    float* sp_part;  // [B,Hkv,G,max_chunk/256,vt_tiles,64] single-pass scores only (else null): column sums per row block
    int32_t* offers; // [B,Hkv,2,max_chunk]
    int32_t* winners;// [B,Hkv,N,max_chunk+1]
    void* move_stage;// [B,Hkv,move_stage_rows] x (K row, V row, score, id): sources of the update's moves, gathered before any is overwritten
    int move_stage_rows;
    // decode scratch
    float* logits;   // [B,Hkv,slots+1,decode_logit_heads]
    float* part;     // [B,Hq,dec_splits,2] (max, sum) of every split
    float* opart;    // [B,Hq,dec_splits,d]
    int rope_rows;
    int dec_splits;
    int vt_tiles;    // capacity of Kt and Vt per (batch, KV head)
    // development switches (tests, A/B timing), read from the environment ONCE, when the context is
    // created; no launch looks at the environment
    int opt_attn_splits;       // CASCADE_KV_ATTN_SPLITS: workgroups per row block of a small attention launch; 0 = automatic
    int opt_score_narrow;      // CASCADE_KV_SCORE_NARROW: 0 / 1 force the 64- / 32-key form of the score kernel; -1 = automatic
    int opt_decode_qk_direct;  // CASCADE_KV_DECODE_QK_DIRECT: bf16 decode logits by the register-load kernel
    int opt_decode_pv_valu;    // CASCADE_KV_DECODE_PV_VALU: bf16 decode outputs by the VALU kernel
    int opt_update_staged;     // CASCADE_KV_UPDATE_STAGED: always plan the update cascade by cascade (plan_kernel)
};

// tables
void launch_rope_table(const Geom& g, float base, float2* rope, float2* rope_t, int rows, hipStream_t s);
void launch_wrow_table(float beta, float* wrow, int n, hipStream_t s);

// cache maintenance
void launch_fill_i32(int32_t* p, size_t n, int32_t value, hipStream_t s);
void launch_load_state(const Geom& g, int dtype, const DevBuffers& b, const void* k, const void* v,
                       const float* mu, const int32_t* ids, const int* counts, int total, hipStream_t s);
// q_first_row: the rotated query copies are written for chunk rows q_first_row .. Q-1 only
void launch_prep(const Geom& g, int dtype, const DevBuffers& b, const SegList& sl, int Q, float qscale, int q_first_row,
                 const void* q, const void* k, const void* v, hipStream_t s);
// homogeneous heads: the scores of the cached rows (and of n_new new tokens) reduced over the KV heads and shared
void launch_share_scores(const Geom& g, const DevBuffers& b, int n_new, int max_chunk, hipStream_t s);
void launch_plan(const Geom& g, const DevBuffers& b, const UpdatePlan& pl, int max_chunk, hipStream_t s);
// update_is_direct: the update needs no launch_plan (every segment can be decided on its own, by the
// first launch of launch_moves); pass its result as `direct`
bool update_is_direct(const Geom& g, const DevBuffers& b, const UpdatePlan& pl);
void launch_moves(const Geom& g, int dtype, const DevBuffers& b, const UpdatePlan& pl, int max_chunk,
                  const void* k, const void* v, int k_token_stride, int k_batch_stride, bool direct, hipStream_t s);

// attention, generic (any dtype / head_dim): scalar arithmetic
void launch_attn_simple(const Geom& g, int dtype, const DevBuffers& b, const SegList& sl, int Q,
                        int max_chunk, void* out, hipStream_t s);
void launch_score_simple(const Geom& g, int dtype, const DevBuffers& b, const SegList& sl, int Q,
                         int max_chunk, int tail_rows, float decay, hipStream_t s);

// attention, bf16 MFMA (head_dim 64 or 128).  launch_kv_pack copies the keys and values of the
// segment list into Kt / Vt, tile by tile (tile n = rows 64n .. 64n+63 of the concatenated
// segments), for the tiles named by `runs` only (false if Kt / Vt do not hold that many tiles);
// launch_attn_stream reads only those copies, and the caller's queries (q: [B,Q,Hq,d], rotated on the fly).
int packed_tiles_of(const SegList& sl);
bool launch_kv_pack(const Geom& g, const DevBuffers& b, const SegList& sl, const TileRuns& runs, int Q, hipStream_t s);
// It also leaves the exponent offsets of the last tail_rows rows in b.negt for launch_score_mfma.
// single_pass (only if attn_single_pass_ok): the kernel also leaves the column sums of Alg. 3's single-pass
// scores in b.sp_part, which launch_single_pass_merge turns into the scores (instead of launch_score_mfma).
bool attn_single_pass_ok(const Geom& g, const DevBuffers& b, int Q, int tail_rows);
void launch_attn_stream(const Geom& g, const DevBuffers& b, const SegList& sl, int Q, const void* q, float qscale,
                        int tail_rows, int max_chunk, void* out, bool single_pass, hipStream_t s);
void launch_single_pass_merge(const Geom& g, const DevBuffers& b, const SegList& sl, int Q, int max_chunk, float decay, hipStream_t s);
void launch_score_mfma(const Geom& g, const DevBuffers& b, const SegList& sl, int Q, int max_chunk,
                       int tail_rows, float decay, hipStream_t s);

// decode
void launch_decode_qk(const Geom& g, int dtype, const DevBuffers& b, const SegList& sl,
                      const void* q, const void* k, hipStream_t s);
void launch_decode_pv(const Geom& g, int dtype, const DevBuffers& b, const SegList& sl, hipStream_t s);
// merges the split outputs into `out`, gives the new token its score and inserts it (plan and moves of `pl`, one token)
void launch_decode_finish(const Geom& g, int dtype, const DevBuffers& b, const SegList& sl, const UpdatePlan& pl, int qstride,
                          const void* k, const void* v, void* out, hipStream_t s);
bool decode_supported(const Geom& g);
int decode_logit_heads(const Geom& g);   // heads per row of the logits buffer (group size rounded up to 1, 2, 4, 8)

}  // namespace ckv
