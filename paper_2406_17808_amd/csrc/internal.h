// Internal declarations shared by the host API and the HIP kernels of the cascading KV cache.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/cascade_kv.h"

namespace ckv {

constexpr int kMaxCascades = CASCADE_MAX_CASCADES;
constexpr int kMaxQueryRotations = 2 * CASCADE_MAX_CASCADES + 2;   // sinks, two runs per ring, the chunk
constexpr int kMaxSegments = 3 * CASCADE_MAX_CASCADES + 2;         // a run may be listed in two pieces

// ------------------------------------------------------------------ element types
typedef uint16_t bf16_t;   // raw bfloat16 bits

__host__ __device__ inline float bf16_to_f32(bf16_t x)
{
    union { uint32_t u; float f; } c;
    c.u = (uint32_t)x << 16;
    return c.f;
}

__host__ __device__ inline bf16_t f32_to_bf16(float f)   // round to nearest even
{
    union { uint32_t u; float f; } c;
    c.f = f;
    uint32_t lsb = (c.u >> 16) & 1u;
    c.u += 0x7FFFu + lsb;
    return (bf16_t)(c.u >> 16);
}

// One rotary pair (x0, x1) turned by the angle whose cosine and sine are c and s, with the
// roundings spelled out: one rounded product, then one fused multiply-add.  Every kernel that
// rotates a key or a query that will be rounded to bf16 goes through here, so that all of them, and
// a reference that wants to reproduce those bf16 values bit for bit, round alike whatever the
// compiler would have contracted.
__host__ __device__ inline float rot_lo(float x0, float x1, float c, float s) { return __builtin_fmaf(x0, c, -(x1 * s)); }
__host__ __device__ inline float rot_hi(float x0, float x1, float c, float s) { return __builtin_fmaf(x1, c, x0 * s); }

template <typename T> struct Elem;
template <> struct Elem<float> {
    __host__ __device__ static float load(const float* p) { return *p; }
    __host__ __device__ static void store(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
    __host__ __device__ static float load(const bf16_t* p) { return bf16_to_f32(*p); }
    __host__ __device__ static void store(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

// ------------------------------------------------------------------ geometry (constant per context)
// Physical slot layout per (sequence, KV head): [sinks | last cascade | ... | first cascade].
struct Geom {
    int B, Hq, Hkv, G, d;
    int n_sink, N, slots;
    int cap[kMaxCascades];     // cascade c (0-based; 0 = first cascade)
    int base[kMaxCascades];    // first physical slot of cascade c
    int period[kMaxCascades];
    int token_selection, head_reduce, head_policy;
    float beta, scale;
};

// ------------------------------------------------------------------ attention segments
// A run of physical rows whose positional index differs from the stored rotation anchor by
// one constant, so a single rotation of the queries serves the whole run.
struct Seg {
    int start;    // first physical slot (cache) or first chunk index (chunk segment)
    int len;
    int qvar;     // which rotated copy of the queries to use
    int chunk;    // 1: the chunk's own keys (causal), 0: cached rows
};

struct SegList {
    int n;                 // segments
    int n_qvar;            // rotated query copies
    int n_cached;          // cached rows before the chunk = positional index of chunk token 0
    int qrot0[kMaxQueryRotations];   // rotation index of chunk row 0 for query copy v (row i uses qrot0 + i)
    Seg s[kMaxSegments];
};

// ------------------------------------------------------------------ structure of one cache update
// The fill, the ring heads and the acceptance times of Alg. 2 do not depend on the scores,
// so the host knows for every cascade which offers append, push (evict) or compete.
struct CascStep {
    int cap, base;
    int M;          // items offered to this cascade during the update, in order
    int A;          // the first A offers are appended (cascade not yet full)
    int kp0;        // first offer index >= A that arrives at an accepting time (>= M if none)
    int pstride;    // offer-index distance between accepting times
    int P;          // pushes: offers kp0 + i*pstride, i < P, each evicts the oldest item
    int J;          // slots opened = A + P
    int wpos0;      // ring position written by the first open
    int pre;        // 1: the cascade is full at the start and offers [0, kp0) compete with its newest item
    int newest0;    // ring position of the newest item at the start (meaningful when pre)
};

struct UpdatePlan {
    int Q;           // tokens of the chunk
    int n_to_sink;   // the first n_to_sink tokens go to sink slots sink_fill0 ...
    int sink_fill0;
    int N;
    int id0;         // original index of chunk token 0
    CascStep c[kMaxCascades];
};

// A few runs of 64-row tiles (of the packed K / V copies the bf16 attention kernel reads).
constexpr int kMaxTileRuns = 2 * CASCADE_MAX_CASCADES + 2;   // sinks, two per ring, the chunk
struct TileRuns {
    int n;                       // runs
    int total;                   // tiles in all runs
    int first[kMaxTileRuns];     // first tile of run i
    int ahead[kMaxTileRuns];     // tiles in the runs before run i
};

// scratch index space of the update: refs < slots name a physical slot, refs >= slots a chunk token
}  // namespace ckv
