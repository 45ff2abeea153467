"""Seeded synthetic workloads for the cascading KV cache hot path.

This module only describes shapes and draws random numbers.  It holds none of
the method's arithmetic (no attention, no RoPE, no cache policy), so that both
the HIP path and the CPU oracle can be fed the same bits from it without
sharing any code of the method itself.

The workloads stand in for the paper's latency experiment (a single
attention layer at Llama-3.1-8B head geometry streaming a long prompt,
Section 4.1; ``prefill_paper_16k`` has that experiment's own cache size, stride
and EMA decay; ``prefill_passkey_*`` and ``prefill_longbench_8k`` have the cache
geometries of the passkey and long-context-understanding experiments) and, for
the planted key of ``prefill_1m``, for the passkey experiment (Section 4.4); no
dataset or trained weight is involved.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, Optional, Tuple

import numpy as np


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str                 # "f32" or "bf16"
    n_sink: int
    cascade_sizes: Tuple[int, ...]
    seq_len: int               # prefill tokens (decode: number of decode steps)
    chunk: int                 # prefill chunk (stride); 1 for decode
    ema_beta: float
    rope_base: float
    input_scale: float         # multiplies the N(0,1) draws of q, k and v
    planted_key: bool = False
    decode: bool = False

    @property
    def n_cascades(self) -> int:
        return len(self.cascade_sizes)

    @property
    def n_slots(self) -> int:
        return self.n_sink + sum(self.cascade_sizes)

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def n_chunks(self) -> int:
        return (self.seq_len + self.chunk - 1) // self.chunk


# The synthetic configurations.  Cascade totals exclude the sink slots
# (the paper counts sinks in addition to the cache size, Section 4 "Setup").
WORKLOADS: Dict[str, Workload] = {
    "tiny_f32": Workload(
        name="tiny_f32", batch=1, n_q_heads=1, n_kv_heads=1, head_dim=64, dtype="f32",
        n_sink=4, cascade_sizes=(64, 64, 64, 64), seq_len=2048, chunk=32,
        ema_beta=0.9, rope_base=10000.0, input_scale=1.0),
    "prefill_32k": Workload(
        name="prefill_32k", batch=1, n_q_heads=32, n_kv_heads=8, head_dim=128, dtype="bf16",
        n_sink=64, cascade_sizes=(1024,) * 4, seq_len=32768, chunk=1024,
        ema_beta=0.9, rope_base=500000.0, input_scale=1.0 / math.sqrt(128.0)),
    "prefill_131k": Workload(
        name="prefill_131k", batch=1, n_q_heads=32, n_kv_heads=8, head_dim=128, dtype="bf16",
        n_sink=64, cascade_sizes=(2048,) * 8, seq_len=131072, chunk=2048,
        ema_beta=0.9, rope_base=500000.0, input_scale=1.0),
    "prefill_1m": Workload(
        name="prefill_1m", batch=1, n_q_heads=32, n_kv_heads=8, head_dim=128, dtype="bf16",
        n_sink=64, cascade_sizes=(16384,) * 4, seq_len=1048576, chunk=4096,
        ema_beta=0.9, rope_base=500000.0, input_scale=1.0, planted_key=True),
    # the geometry of the paper's own latency figure (Section 4.1, Appendix "latency"): 16K cache,
    # stride 4096, EMA decay 0.9999 (every query row of a chunk carries weight in the scores)
    "prefill_paper_16k": Workload(
        name="prefill_paper_16k", batch=1, n_q_heads=32, n_kv_heads=8, head_dim=128, dtype="bf16",
        n_sink=64, cascade_sizes=(4096,) * 4, seq_len=1048576, chunk=4096,
        ema_beta=0.9999, rope_base=500000.0, input_scale=1.0),
    # the geometries of the paper's other experiments (all with its EMA decay 0.9999):
    # passkey retrieval (Section 4.4): 8 cascades, caches of 32K and 65K, stride 4096
    "prefill_passkey_32k": Workload(
        name="prefill_passkey_32k", batch=1, n_q_heads=32, n_kv_heads=8, head_dim=128, dtype="bf16",
        n_sink=64, cascade_sizes=(4096,) * 8, seq_len=1048576, chunk=4096,
        ema_beta=0.9999, rope_base=500000.0, input_scale=1.0),
    "prefill_passkey_65k": Workload(
        name="prefill_passkey_65k", batch=1, n_q_heads=32, n_kv_heads=8, head_dim=128, dtype="bf16",
        n_sink=64, cascade_sizes=(8192,) * 8, seq_len=1048576, chunk=4096,
        ema_beta=0.9999, rope_base=500000.0, input_scale=1.0),
    # long-context understanding (Section 4.3): cache 2^floor(log2(L/4)) for a prompt of L tokens,
    # stride 512; L = 40000 gives an 8192-slot cache and a last chunk of 64 tokens
    "prefill_longbench_8k": Workload(
        name="prefill_longbench_8k", batch=1, n_q_heads=32, n_kv_heads=8, head_dim=128, dtype="bf16",
        n_sink=64, cascade_sizes=(2048,) * 4, seq_len=40000, chunk=512,
        ema_beta=0.9999, rope_base=500000.0, input_scale=1.0),
    "decode_b32": Workload(
        name="decode_b32", batch=32, n_q_heads=32, n_kv_heads=8, head_dim=128, dtype="bf16",
        n_sink=64, cascade_sizes=(16384,) * 4, seq_len=1024, chunk=1,
        ema_beta=0.9, rope_base=500000.0, input_scale=1.0, decode=True),
}

_TENSOR_IDS = {"q": 0, "k": 1, "v": 2, "state_k": 3, "state_v": 4, "state_mu": 5, "plant": 6}


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); result is float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32).astype(np.uint64)
    lsb = (bits >> np.uint64(16)) & np.uint64(1)
    bits = (bits + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
    return bits.astype(np.uint32).view(np.float32).reshape(x.shape)


def _rng(seed: int, wl: Workload, index: int, tensor: str) -> np.random.Generator:
    # a stable digest of the workload name (hash() of str is salted per process)
    stable = 0
    for ch in wl.name.encode():
        stable = (stable * 131 + ch) % (1 << 31)
    key = (np.uint64(seed) << np.uint64(32)) ^ np.uint64(stable)
    counter = [np.uint64(index), np.uint64(_TENSOR_IDS[tensor]), np.uint64(0), np.uint64(0)]
    return np.random.Generator(np.random.Philox(key=key, counter=counter))


def _normal(seed: int, wl: Workload, index: int, tensor: str, shape) -> np.ndarray:
    x = _rng(seed, wl, index, tensor).standard_normal(size=shape, dtype=np.float32)
    x *= np.float32(wl.input_scale)
    if wl.dtype == "bf16":
        x = round_to_bf16(x)
    return x


def planted_key_spec(wl: Workload, seed: int) -> Optional[dict]:
    """Where the planted key of a workload sits and which direction it uses.

    The direction ``u`` lives only in the lowest-frequency rotary pairs (the
    last 8 of the d/2 half-split pairs), where the rotation angle between the
    key's and the final queries' cache positions stays small, so a pre-rotation
    alignment survives positional encoding.  ``w`` is a second unit vector in
    the same pairs, orthogonal to ``u``.
    """
    if not wl.planted_key:
        return None
    g = _rng(seed, wl, 0, "plant")
    span = sum(wl.cascade_sizes[i] << i for i in range(wl.n_cascades))
    lo = wl.seq_len - (3 * span) // 4
    hi = wl.seq_len - wl.cascade_sizes[0] - wl.chunk
    pos = int(g.integers(lo, hi))
    d, half = wl.head_dim, wl.head_dim // 2
    comp = np.concatenate([np.arange(half - 8, half), np.arange(d - 8, d)])
    a = g.standard_normal(16)
    b = g.standard_normal(16)
    a /= np.linalg.norm(a)
    b -= a * (a @ b)
    b /= np.linalg.norm(b)
    u = np.zeros(d)
    w = np.zeros(d)
    u[comp] = a
    w[comp] = b
    return {"position": pos, "u": u, "w": w, "cosine": 0.9, "norm_factor": 4.0,
            "query_gain": 1.0, "last_queries": 64}


def chunk_inputs(wl: Workload, seed: int, chunk_index: int, n_tokens: Optional[int] = None):
    """q [B,n,Hq,d], k [B,n,Hkv,d], v [B,n,Hkv,d] of one prefill chunk as float32.

    For a bf16 workload every value is already rounded to bfloat16, so a
    float32 -> bfloat16 conversion of these arrays is exact.
    """
    start = chunk_index * wl.chunk
    n = min(wl.chunk, wl.seq_len - start) if n_tokens is None else n_tokens
    q = _normal(seed, wl, chunk_index, "q", (wl.batch, wl.chunk, wl.n_q_heads, wl.head_dim))[:, :n]
    k = _normal(seed, wl, chunk_index, "k", (wl.batch, wl.chunk, wl.n_kv_heads, wl.head_dim))[:, :n]
    v = _normal(seed, wl, chunk_index, "v", (wl.batch, wl.chunk, wl.n_kv_heads, wl.head_dim))[:, :n]
    spec = planted_key_spec(wl, seed)
    if spec is not None:
        d = wl.head_dim
        p = spec["position"]
        if start <= p < start + n:
            c = spec["cosine"]
            kk = spec["norm_factor"] * math.sqrt(d) * (c * spec["u"] + math.sqrt(1.0 - c * c) * spec["w"])
            k = k.copy()
            k[:, p - start, :, :] = round_to_bf16(kk.astype(np.float32))
        first_q = wl.seq_len - spec["last_queries"]
        lo, hi = max(first_q, start), min(wl.seq_len, start + n)
        if lo < hi:
            q = q.copy()
            add = (spec["query_gain"] * math.sqrt(d) * spec["u"]).astype(np.float32)
            q[:, lo - start:hi - start] = round_to_bf16(q[:, lo - start:hi - start] + add)
    return np.ascontiguousarray(q), np.ascontiguousarray(k), np.ascontiguousarray(v)


def decode_inputs(wl: Workload, seed: int, step: int):
    """q [B,Hq,d], k [B,Hkv,d], v [B,Hkv,d] of one decode step as float32."""
    q = _normal(seed, wl, step, "q", (wl.batch, wl.n_q_heads, wl.head_dim))
    k = _normal(seed, wl, step, "k", (wl.batch, wl.n_kv_heads, wl.head_dim))
    v = _normal(seed, wl, step, "v", (wl.batch, wl.n_kv_heads, wl.head_dim))
    return q, k, v


def prefilled_state(wl: Workload, seed: int, seq: int, kv_head: int, n_prior_tokens: Optional[int] = None):
    """A full cache for one (sequence, KV head): K, V [slots,d], mu [slots], ids [slots].

    Rows are in cache order (sinks, then the last cascade oldest to newest, ...,
    then the first cascade).  K and V are N(0,1) draws, scores are U(0,1), and
    the token ids are the sinks followed by the most recent ``slots - n_sink``
    positions of a stream of ``n_prior_tokens`` tokens, which keeps them
    strictly increasing along the cache order.
    """
    slots = wl.n_slots
    idx = seq * wl.n_kv_heads + kv_head
    k = _normal(seed, wl, idx, "state_k", (slots, wl.head_dim))
    v = _normal(seed, wl, idx, "state_v", (slots, wl.head_dim))
    mu = _rng(seed, wl, idx, "state_mu").random(size=slots, dtype=np.float32)
    total = 4 * slots if n_prior_tokens is None else n_prior_tokens
    ids = np.concatenate([np.arange(wl.n_sink), np.arange(total - (slots - wl.n_sink), total)]).astype(np.int64)
    return k, v, mu, ids


def chunk_inputs_torch(wl: Workload, seed: int, chunk_index: int, device, n_tokens: Optional[int] = None):
    """The same recipe as chunk_inputs, drawn on the device by torch's seeded generator (for the
    long workloads, where drawing on the host would dominate a run).  Returns q, k, v tensors
    in the workload's dtype.  The bits differ from chunk_inputs; whoever needs both sides to see
    the same values copies these tensors to the host."""
    import torch
    start = chunk_index * wl.chunk
    n = min(wl.chunk, wl.seq_len - start) if n_tokens is None else n_tokens
    gen = torch.Generator(device=device)
    stable = 0
    for ch in wl.name.encode():
        stable = (stable * 131 + ch) % (1 << 31)
    gen.manual_seed((seed << 40) ^ (stable << 8) ^ (chunk_index * 2654435761 % (1 << 40)))
    dt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32

    def draw(heads):
        x = torch.randn((wl.batch, wl.chunk, heads, wl.head_dim), generator=gen, device=device, dtype=torch.float32)
        return (x * wl.input_scale)[:, :n].to(dt).contiguous()

    q, k, v = draw(wl.n_q_heads), draw(wl.n_kv_heads), draw(wl.n_kv_heads)
    spec = planted_key_spec(wl, seed)
    if spec is not None:
        d = wl.head_dim
        p = spec["position"]
        if start <= p < start + n:
            c = spec["cosine"]
            kk = spec["norm_factor"] * math.sqrt(d) * (c * spec["u"] + math.sqrt(1.0 - c * c) * spec["w"])
            k[:, p - start, :, :] = torch.from_numpy(kk.astype(np.float32)).to(device).to(dt)
        first_q = wl.seq_len - spec["last_queries"]
        lo, hi = max(first_q, start), min(wl.seq_len, start + n)
        if lo < hi:
            add = torch.from_numpy((spec["query_gain"] * math.sqrt(d) * spec["u"]).astype(np.float32)).to(device)
            q[:, lo - start:hi - start] = (q[:, lo - start:hi - start].float() + add).to(dt)
    return q, k, v
