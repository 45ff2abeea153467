// Plan and moves of a small update (a decode step: one token) by one workgroup per (sequence,
// KV head), called at the end of a kernel that workgroup runs anyway: it takes the decisions of
// plan_kernel (the routines of plan_core.h) and then writes the final content of every touched
// slot itself, the last cascade first (destinations of cascade c take their sources from earlier
// cascades or from the new tokens only, so every source is still intact when it is read), with
// a barrier between cascades.  All threads of the workgroup must call it.
#pragma once

#include "internal.h"
#include "plan_core.h"

namespace ckv {

struct UpdateBuffers {
    const float2* rope;
    int32_t *offers, *winners, *swaps;
    void *Kc, *Kr, *Vc;
    float* mu;
    int32_t* ids;
    const float* mu_chunk;
    const void *k_in, *v_in;       // the new tokens: [B, tokens, Hkv, d]
    long tok_stride, batch_stride;
};

template <typename T>
__device__ inline void small_update(const Geom& g, const UpdatePlan& pl, int qstride, const UpdateBuffers& u, int b, int h)
{
    const int bh = b * g.Hkv + h;
    const float2* rope = u.rope;
    int32_t *offers = u.offers, *winners = u.winners, *swaps = u.swaps;
    T *Kc = (T*)u.Kc, *Kr = (T*)u.Kr, *Vc = (T*)u.Vc;
    float* mu = u.mu;
    int32_t* ids = u.ids;
    const float* mu_chunk = u.mu_chunk;
    const T *k_in = (const T*)u.k_in, *v_in = (const T*)u.v_in;
    const long tok_stride = u.tok_stride, batch_stride = u.batch_stride;
    const float* mub = mu + (size_t)bh * g.slots;
    const float* muc = mu_chunk + (size_t)bh * qstride;
    int32_t* off_in = offers + (size_t)bh * 2 * qstride;
    int32_t* off_out = off_in + qstride;
    for (int c = 0; c < pl.N; ++c) {
        const CascStep cs = pl.c[c];
        if (cs.M == 0) break;
        int32_t* W = winners + ((size_t)bh * pl.N + c) * (qstride + 1);
        const int nseg = cs.J + cs.pre;
        int my_swaps = 0;
        for (int sidx = threadIdx.x; sidx < nseg; sidx += blockDim.x) {
            const int j = sidx - cs.pre;
            int sw;
            W[1 + j] = segment_winner(cs, c, j, g.slots, pl.n_to_sink, g.token_selection, off_in, mub, muc, &sw);
            my_swaps += sw;
        }
        if (my_swaps) atomicAdd(&swaps[bh * pl.N + c], my_swaps);
        __syncthreads();
        for (int i = threadIdx.x; i < cs.P; i += blockDim.x) off_out[i] = evicted_ref(cs, i, W);
        __syncthreads();
        int32_t* tmp = off_in; off_in = off_out; off_out = tmp;
    }
    const int half = g.d / 2;
    for (int c = pl.N - 1; c >= -1; --c) {
        int E, extra = 0;
        if (c < 0) E = pl.n_to_sink;
        else { if (pl.c[c].M == 0) continue; E = final_entries(pl.c[c], &extra); }
        for (int e = 0; e < E + extra; ++e) {
            int dst, ref;
            if (c < 0) { dst = pl.sink_fill0 + e; ref = g.slots + e; }
            else {
                const int32_t* W = winners + ((size_t)bh * pl.N + c) * (qstride + 1);
                if (!final_entry(pl.c[c], e, E, W, &dst, &ref)) continue;
            }
            const size_t drow = ((size_t)bh * g.slots + dst) * g.d;
            const T *ks, *vs;
            float score;
            int id;
            if (ref < g.slots) {
                const size_t srow = ((size_t)bh * g.slots + ref) * g.d;
                ks = Kc + srow; vs = Vc + srow;
                score = mu[(size_t)bh * g.slots + ref];
                id = ids[(size_t)bh * g.slots + ref];
            } else {
                const int i = ref - g.slots;
                const size_t srow = (size_t)b * batch_stride + (size_t)i * tok_stride + (size_t)h * g.d;
                ks = k_in + srow; vs = v_in + srow;
                score = mu_chunk[(size_t)bh * qstride + i];
                id = pl.id0 + i;
            }
            for (int p = threadIdx.x; p < half; p += blockDim.x) {
                const float x0 = Elem<T>::load(ks + p), x1 = Elem<T>::load(ks + p + half);
                const float2 cs2 = rope[(size_t)dst * half + p];
                Elem<T>::store(Kc + drow + p, x0);
                Elem<T>::store(Kc + drow + p + half, x1);
                Elem<T>::store(Kr + drow + p, rot_lo(x0, x1, cs2.x, cs2.y));
                Elem<T>::store(Kr + drow + p + half, rot_hi(x0, x1, cs2.x, cs2.y));
                Vc[drow + p] = vs[p];
                Vc[drow + p + half] = vs[p + half];
            }
            if (threadIdx.x == 0) {
                mu[(size_t)bh * g.slots + dst] = score;
                ids[(size_t)bh * g.slots + dst] = id;
            }
        }
        __syncthreads();   // the rows of this cascade are written before an earlier cascade's slots are overwritten
    }
}

}  // namespace ckv
