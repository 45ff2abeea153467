// The score-dependent part of the cascade update (Alg. 2 applied to a whole chunk), written
// once for the device kernels and for the host-side simulation.
//
// An item is named by a ref: a physical slot (< slots) or slots + chunk index.  Within one
// cascade the offers of an update fall into segments: every slot that is opened (an append
// or a push) is followed by the offers that compete for it until the next slot opens.  The
// winner of a segment is its first maximum: Alg. 2 replaces the newest item only on a
// strictly higher score.
#pragma once

#include "internal.h"

namespace ckv {

__host__ __device__ inline float ref_score(int ref, int slots, const float* mu, const float* mu_chunk)
{
    return ref < slots ? mu[ref] : mu_chunk[ref - slots];
}

// ref of offer k of cascade c (cascade 0 is offered the chunk's tokens that did not go to sinks)
__host__ __device__ inline int offer_ref(int c, int k, int slots, int n_to_sink, const int32_t* off_in)
{
    return c == 0 ? slots + n_to_sink + k : off_in[k];
}

// When no cascade has a slot written twice in one update (J <= cap for every cascade: the usual
// case, a chunk no longer than any ring), and none overwrites the slot whose holder the first
// offers compete for, the item a push evicts is simply what its ring position held before the
// update: the offers of cascade c can be named without knowing any winner of cascade c - 1, and the
// segments of ALL cascades can be decided at the same time.
__host__ __device__ inline bool plan_is_direct(const UpdatePlan& pl)
{
    for (int c = 0; c < pl.N; ++c) {
        if (pl.c[c].M == 0) break;
        if (pl.c[c].J > pl.c[c].cap || (pl.c[c].J == pl.c[c].cap && pl.c[c].pre)) return false;
    }
    return true;
}

// ref of offer k of cascade c under plan_is_direct: push k of cascade c - 1 evicts ring position wpos0 + A + k
__host__ __device__ inline int offer_ref_direct(const UpdatePlan& pl, int c, int k, int slots)
{
    if (c == 0) return slots + pl.n_to_sink + k;
    const CascStep& prev = pl.c[c - 1];
    return prev.base + (prev.wpos0 + prev.A + k) % prev.cap;
}

// Winner of segment j of cascade c (j = -1: the item that was newest before the update and the
// offers that compete with it before any slot opens).  *swaps receives the replacements.
// off_in == nullptr: the offers are named directly (plan_is_direct), `pl` must be given.
__host__ __device__ inline int segment_winner(const CascStep& cs, int c, int j, int slots, int n_to_sink,
                                              int token_selection, const int32_t* off_in,
                                              const float* mu, const float* mu_chunk, int* swaps,
                                              const UpdatePlan* pl = nullptr)
{
    int best, kb, ke;
    if (j < 0) {
        best = cs.base + cs.newest0;
        kb = 0;
        ke = cs.kp0 < cs.M ? cs.kp0 : cs.M;
    } else {
        const int kh = j < cs.A ? j : cs.kp0 + (j - cs.A) * cs.pstride;
        best = off_in ? offer_ref(c, kh, slots, n_to_sink, off_in) : offer_ref_direct(*pl, c, kh, slots);
        kb = kh + 1;
        if (j + 1 < cs.A) ke = kb;                                   // the next offer is appended too
        else if (j + 1 == cs.A) ke = cs.kp0 < cs.M ? cs.kp0 : cs.M;  // last append: until the first push
        else ke = kh + cs.pstride < cs.M ? kh + cs.pstride : cs.M;   // push: until the next push
    }
    int n_swaps = 0;
    if (token_selection) {
        float bs = ref_score(best, slots, mu, mu_chunk);
        for (int k = kb; k < ke; ++k) {
            const int r = off_in ? offer_ref(c, k, slots, n_to_sink, off_in) : offer_ref_direct(*pl, c, k, slots);
            const float s = ref_score(r, slots, mu, mu_chunk);
            if (s > bs) { best = r; bs = s; ++n_swaps; }
        }
    }
    *swaps = n_swaps;
    return best;
}

// The item evicted by push i of the cascade: what its ring position held before the write.
// W[0] is the winner of segment -1, W[1 + j] that of segment j.
__host__ __device__ inline int evicted_ref(const CascStep& cs, int i, const int32_t* W)
{
    const int j = cs.A + i;
    const int p = (cs.wpos0 + j) % cs.cap;
    if (j >= cs.cap) return W[1 + j - cs.cap];       // written earlier in this same update
    if (cs.pre && p == cs.newest0) return W[0];
    return cs.base + p;
}

// Final content of the cascade: entry e < E is the e-th of the last E slots opened, entry E
// (if present) the item that was newest before the update.  Returns false if nothing moves.
__host__ __device__ inline bool final_entry(const CascStep& cs, int e, int E, const int32_t* W, int* dst, int* ref)
{
    if (e < E) {
        const int j = cs.J - E + e;
        *dst = cs.base + (cs.wpos0 + j) % cs.cap;
        *ref = W[1 + j];
        return true;
    }
    *dst = cs.base + cs.newest0;
    *ref = W[0];
    return *ref != *dst;
}

__host__ __device__ inline int final_entries(const CascStep& cs, int* extra)
{
    const int E = cs.J < cs.cap ? cs.J : cs.cap;
    *extra = (cs.pre && cs.J < cs.cap) ? 1 : 0;
    return E;
}

}  // namespace ckv
