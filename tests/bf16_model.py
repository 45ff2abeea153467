"""A dense numpy reference of one chunk of bf16 attention WITH the rounding points of the bf16
contract, for one (sequence, KV head).  Test infrastructure; shares no code with the HIP library
or with the oracle.

The oracle computes in ideal arithmetic (fp64).  The bf16 path rounds at exactly two places
(everything else is fp32 or wider):
  1. the MFMA operands of QK^T: the query, scaled by softmax_scale * log2(e) and rotated, and the
     key, rotated, are rounded to bf16.  Only the DIFFERENCE of the two rotation angles matters to
     the exact product, but the rounding acts on the rotated vectors, so the anchors matter here:
     a cached key is stored rotated to the index of the physical slot it sits in, a chunk key to
     its index inside the chunk, and the query turns by whatever makes the difference equal
     (query cache index) - (key cache index)  (Section 3.1 "Positional Encoding");
  2. the probabilities, rounded to bf16 as the MFMA operand of PV; the normaliser is the sum of
     the unrounded probabilities.
With both switched off this is plain softmax attention at cache-index positions (Eq. 2), which a
CPU test pins against the oracle; with both on, the difference between the library and this
model is what is left after the contract roundings are accounted for: the rounding of the output
itself to bf16 (relative 2^-9 per element) and the power-of-two phase at which a probability is
rounded (the kernel rounds 2^(s - m) for a running maximum m that is not the final one).
"""
import numpy as np

LOG2E = 1.4426950408889634


def to_bf16(x):
    """Round float32 values to the nearest bfloat16, ties to even (result as float32)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32).astype(np.uint64)
    lsb = (bits >> np.uint64(16)) & np.uint64(1)
    bits = (bits + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
    return bits.astype(np.uint32).view(np.float32).reshape(x.shape)


def _table(index, d, base):
    """(cos, sin) of index * base^(-2i/d), evaluated in fp64 and stored as float32."""
    theta = np.float64(base) ** (-2.0 * np.arange(d // 2) / d)
    a = np.asarray(index, dtype=np.float64)[..., None] * theta
    return np.cos(a).astype(np.float32), np.sin(a).astype(np.float32)


def _rotate_f32(x, index, d, base):
    """Pairs (x_i, x_{i+d/2}) rotated by index * theta_i in float32 arithmetic with the roundings of
    the bf16 contract: lo = fma(x0, c, -(x1 * s)), hi = fma(x1, c, x0 * s): one product rounded to
    float32, then a fused multiply-add (the exact product of two float32 values fits a float64; the
    sum is rounded to float64 and then to float32, which differs from a single rounding only in
    ties of probability 2^-29)."""
    half = d // 2
    c, s = _table(index, d, base)
    x = np.asarray(x, dtype=np.float32)
    x0, x1 = x[..., :half], x[..., half:]
    t_lo = (x1 * s).astype(np.float32).astype(np.float64)
    t_hi = (x0 * s).astype(np.float32).astype(np.float64)
    lo = (x0.astype(np.float64) * c.astype(np.float64) - t_lo).astype(np.float32)
    hi = (x1.astype(np.float64) * c.astype(np.float64) + t_hi).astype(np.float32)
    return np.concatenate([lo, hi], axis=-1)


def chunk_reference(q, k_chunk, v_chunk, k_cache, v_cache, slot, rows, rope_base, softmax_scale=0.0,
                    round_operands=True, round_probabilities=True, ema_beta=None):
    """q [Q,G,d] (the query heads of this KV head), k_chunk, v_chunk [Q,d], k_cache, v_cache [n,d]
    in cache order, slot [n] the physical slot of every cached row; all bf16-valued float arrays.
    rows: chunk rows to evaluate.  Returns out [len(rows), G, d] float64 and, if ema_beta is given,
    the EMA increments [G, n + Q] those rows produce: sum over the rows of beta^(Q-1-i) (1-beta) P[i, :]
    (Section 3.1; the coefficients of Alg. 3)."""
    Q, G, d = q.shape
    n = k_cache.shape[0]
    rows = np.asarray(rows, dtype=np.int64)
    scale = np.float32(softmax_scale if softmax_scale > 0 else 1.0 / np.sqrt(d)) * np.float32(LOG2E)
    rnd = to_bf16 if round_operands else (lambda x: np.asarray(x, dtype=np.float32))
    # keys at their anchors
    kc = rnd(_rotate_f32(k_cache, slot, d, rope_base)) if n else np.zeros((0, d), np.float32)
    kq = rnd(_rotate_f32(k_chunk, np.arange(Q), d, rope_base))
    vals = np.concatenate([v_cache, v_chunk]).astype(np.float64)
    out = np.zeros((len(rows), G, d))
    delta = np.zeros((G, n + Q)) if ema_beta is not None else None
    # cached key j sits at cache index j with anchor slot[j]: the query at cache index n + i turns by
    # n + i - (j - slot[j]); rows that share (j - slot[j]) share a rotation
    shift = (np.arange(n) - np.asarray(slot, dtype=np.int64)) if n else np.zeros(0, np.int64)
    groups = []
    for sh in np.unique(shift):
        idx = np.nonzero(shift == sh)[0]
        groups.append((int(sh), idx, kc[idx].astype(np.float64).T))
    kq_t = kq.astype(np.float64).T
    for r, i in enumerate(rows):
        qs = (np.asarray(q[i], dtype=np.float32) * scale).astype(np.float32)      # scale first, then the rotation
        logits = np.full((G, n + Q), -np.inf)
        for sh, idx, kt in groups:
            qr = rnd(_rotate_f32(qs, np.full(G, n + i - sh), d, rope_base)).astype(np.float64)
            logits[:, idx] = qr @ kt
        qr = rnd(_rotate_f32(qs, np.full(G, i), d, rope_base)).astype(np.float64)
        logits[:, n:n + i + 1] = qr @ kq_t[:, :i + 1]
        m = logits.max(axis=1, keepdims=True)
        p = np.exp2(logits - m)
        l = p.sum(axis=1, keepdims=True)
        pv = to_bf16(p.astype(np.float32)).astype(np.float64) if round_probabilities else p
        out[r] = (pv @ vals) / l
        if delta is not None:
            delta += ema_beta ** (Q - 1 - i) * (1.0 - ema_beta) * (p / l)
    return out, delta
