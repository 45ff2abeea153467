"""ctypes binding of libcascade_kv.so (the C ABI of include/cascade_kv.h).

Argument marshalling only: every step of the path runs in the HIP kernels of the library.
PyTorch is used by callers for device memory and streams; this module only passes raw
pointers.  If the library has not been built, loading fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

from .build import library_path

CASCADE_MAX_CASCADES = 16
CASCADE_OK = 0
CASCADE_E_INVALID_CONFIG = -1
CASCADE_E_NULL_ARG = -2
CASCADE_E_WORKSPACE_TOO_SMALL = -3
CASCADE_E_UNSUPPORTED = -4
CASCADE_E_HIP = -5
CASCADE_E_BAD_ARG = -6
CASCADE_E_INTERNAL = -7
CASCADE_F32 = 0
CASCADE_BF16 = 1
CASCADE_REDUCE_MAX = 0
CASCADE_REDUCE_MEAN = 1
CASCADE_HEADS_INDEPENDENT = 0
CASCADE_HEADS_HOMOGENEOUS = 1
CASCADE_SCORES_EXACT = 0
CASCADE_SCORES_SINGLE_PASS = 1

EXPORTED_SYMBOLS = [
    "cascade_workspace_bytes", "cascade_init", "cascade_destroy", "cascade_prefill_chunk",
    "cascade_decode_step", "cascade_read_state", "cascade_simulate_structure", "cascade_last_error",
    "cascade_profile_begin", "cascade_profile_end", "cascade_layers_workspace_bytes", "cascade_init_layers",
    "cascade_init_static", "cascade_measure_ceilings", "cascade_profile_begin_families",
]
CASCADE_STATIC_WORKSPACE_BYTES = 64 << 20

CASCADE_K_FAMILIES = 7
KERNEL_FAMILIES = ["prep", "attention", "scores", "update", "decode_qk", "decode_pv", "decode_finish"]


class CascadeError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"cascade_kv error {code}: {message}")
        self.code = code


class cascade_config(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("dtype", ctypes.c_int32), ("n_sink", ctypes.c_int32),
        ("n_cascades", ctypes.c_int32),
        ("cascade_sizes", ctypes.c_int32 * CASCADE_MAX_CASCADES),
        ("accept_period", ctypes.c_int32 * CASCADE_MAX_CASCADES),
        ("ema_beta", ctypes.c_float), ("rope_base", ctypes.c_float), ("softmax_scale", ctypes.c_float),
        ("max_chunk", ctypes.c_int32), ("head_reduce", ctypes.c_int32), ("token_selection", ctypes.c_int32),
        ("score_tail_eps", ctypes.c_float), ("keep_update_scores", ctypes.c_int32),
        ("head_policy", ctypes.c_int32), ("score_mode", ctypes.c_int32),
    ]


class cascade_init_state(ctypes.Structure):
    _fields_ = [
        ("dev_k", ctypes.c_void_p), ("dev_v", ctypes.c_void_p), ("dev_mu", ctypes.c_void_p),
        ("dev_ids", ctypes.c_void_p),
        ("counts", ctypes.c_int32 * (1 + CASCADE_MAX_CASCADES)),
        ("t", ctypes.c_int64), ("n_seen", ctypes.c_int64),
    ]


class cascade_state_view(ctypes.Structure):
    _fields_ = [
        ("host_ids", ctypes.c_void_p), ("host_mu", ctypes.c_void_p), ("host_slot", ctypes.c_void_p),
        ("host_k", ctypes.c_void_p), ("host_v", ctypes.c_void_p),
        ("host_kv_pairs", ctypes.c_void_p),
        ("host_swaps", ctypes.c_void_p),
        ("host_pre_mu", ctypes.c_void_p), ("host_chunk_mu", ctypes.c_void_p),
        ("counts", ctypes.c_int32 * (1 + CASCADE_MAX_CASCADES)),
        ("xi", ctypes.c_int32 * CASCADE_MAX_CASCADES),
        ("accepted", ctypes.c_int64 * CASCADE_MAX_CASCADES),
        ("discards", ctypes.c_int64 * CASCADE_MAX_CASCADES),
        ("t", ctypes.c_int64), ("n_seen", ctypes.c_int64),
        ("pre_count", ctypes.c_int32), ("last_tokens", ctypes.c_int32), ("n_kv_pairs", ctypes.c_int32),
        ("last_single_pass", ctypes.c_int32),
    ]


class cascade_ceilings(ctypes.Structure):
    _fields_ = [("compute_units", ctypes.c_int32), ("memory_bus_bits", ctypes.c_int32),
                ("core_clock_mhz", ctypes.c_double), ("memory_clock_mhz", ctypes.c_double),
                ("read_gb_s", ctypes.c_double), ("copy_gb_s", ctypes.c_double), ("mfma_bf16_tflops", ctypes.c_double),
                ("read_regions_gb_s", ctypes.c_double), ("read_with_stores_gb_s", ctypes.c_double),
                ("two_pass_read_gb_s", ctypes.c_double)]


class cascade_profile(ctypes.Structure):
    _fields_ = [("ms", ctypes.c_double * CASCADE_K_FAMILIES), ("intervals", ctypes.c_int64 * CASCADE_K_FAMILIES)]


_LIB = None


def load_library():
    """Load libcascade_kv.so; raises if it has not been built (there is no fallback)."""
    global _LIB
    if _LIB is None:
        path = library_path()
        if not os.path.exists(path):
            raise RuntimeError(f"{path} is missing: build it first (python -m paper_2406_17808_amd.build)")
        L = ctypes.CDLL(path)
        P = ctypes.c_void_p
        L.cascade_workspace_bytes.restype = ctypes.c_size_t
        L.cascade_workspace_bytes.argtypes = [ctypes.POINTER(cascade_config)]
        L.cascade_init.restype = ctypes.c_int
        L.cascade_init.argtypes = [ctypes.POINTER(cascade_config), P, ctypes.c_size_t,
                                   ctypes.POINTER(cascade_init_state), P, ctypes.POINTER(P)]
        L.cascade_layers_workspace_bytes.restype = ctypes.c_size_t
        L.cascade_layers_workspace_bytes.argtypes = [ctypes.POINTER(cascade_config), ctypes.c_int32]
        L.cascade_init_layers.restype = ctypes.c_int
        L.cascade_init_layers.argtypes = [ctypes.POINTER(cascade_config), ctypes.c_int32, P, ctypes.c_size_t, P, P, P]
        L.cascade_init_static.restype = ctypes.c_int
        L.cascade_init_static.argtypes = [ctypes.POINTER(cascade_config), ctypes.POINTER(cascade_init_state), P, ctypes.POINTER(P)]
        L.cascade_destroy.restype = None
        L.cascade_destroy.argtypes = [P]
        L.cascade_prefill_chunk.restype = ctypes.c_int
        L.cascade_prefill_chunk.argtypes = [P, P, P, P, ctypes.c_int32, P, P]
        L.cascade_decode_step.restype = ctypes.c_int
        L.cascade_decode_step.argtypes = [P, P, P, P, P, P]
        L.cascade_read_state.restype = ctypes.c_int
        L.cascade_read_state.argtypes = [P, ctypes.POINTER(cascade_state_view), P]
        L.cascade_simulate_structure.restype = ctypes.c_int
        L.cascade_simulate_structure.argtypes = [ctypes.POINTER(cascade_config), P, ctypes.c_int32, P,
                                                 ctypes.POINTER(cascade_state_view)]
        L.cascade_profile_begin.restype = ctypes.c_int
        L.cascade_profile_begin.argtypes = [P]
        L.cascade_profile_begin_families.restype = ctypes.c_int
        L.cascade_profile_begin_families.argtypes = [P, ctypes.c_uint32]
        L.cascade_profile_end.restype = ctypes.c_int
        L.cascade_profile_end.argtypes = [P, ctypes.POINTER(cascade_profile)]
        L.cascade_measure_ceilings.restype = ctypes.c_int
        L.cascade_measure_ceilings.argtypes = [P, ctypes.c_size_t, P, ctypes.POINTER(cascade_ceilings)]
        L.cascade_last_error.restype = ctypes.c_char_p
        L.cascade_last_error.argtypes = [P]
        _LIB = L
    return _LIB


def make_config(batch: int, n_q_heads: int, n_kv_heads: int, head_dim: int, dtype: int, n_sink: int,
                cascade_sizes: Sequence[int], ema_beta: float, rope_base: float, max_chunk: int,
                accept_period: Optional[Sequence[int]] = None, softmax_scale: float = 0.0,
                head_reduce: int = CASCADE_REDUCE_MAX, token_selection: int = 1,
                score_tail_eps: float = 0.0, keep_update_scores: int = 0,
                head_policy: int = CASCADE_HEADS_INDEPENDENT, score_mode: int = CASCADE_SCORES_EXACT) -> cascade_config:
    c = cascade_config()
    c.batch, c.n_q_heads, c.n_kv_heads, c.head_dim, c.dtype = batch, n_q_heads, n_kv_heads, head_dim, dtype
    c.n_sink, c.n_cascades = n_sink, len(cascade_sizes)
    for i, s in enumerate(cascade_sizes[:CASCADE_MAX_CASCADES]):
        c.cascade_sizes[i] = int(s)
    if accept_period is not None:
        for i, p in enumerate(accept_period[:CASCADE_MAX_CASCADES]):
            c.accept_period[i] = int(p)
    c.ema_beta, c.rope_base, c.softmax_scale = ema_beta, rope_base, softmax_scale
    c.max_chunk, c.head_reduce, c.token_selection = max_chunk, head_reduce, token_selection
    c.score_tail_eps = score_tail_eps
    c.keep_update_scores = keep_update_scores
    c.head_policy, c.score_mode = head_policy, score_mode
    return c


def _check(rc: int, ctx) -> None:
    if rc != CASCADE_OK:
        msg = load_library().cascade_last_error(ctx)
        raise CascadeError(rc, msg.decode() if msg else "")


def cascade_workspace_bytes(cfg: cascade_config) -> int:
    return int(load_library().cascade_workspace_bytes(ctypes.byref(cfg)))


def cascade_init(cfg: cascade_config, dev_workspace: int, workspace_bytes: int,
                 init_state: Optional[cascade_init_state] = None, stream: int = 0) -> ctypes.c_void_p:
    ctx = ctypes.c_void_p()
    rc = load_library().cascade_init(ctypes.byref(cfg), dev_workspace, workspace_bytes,
                                     ctypes.byref(init_state) if init_state is not None else None,
                                     stream, ctypes.byref(ctx))
    _check(rc, None)
    return ctx


def cascade_init_static(cfg: cascade_config, init_state: Optional[cascade_init_state] = None, stream: int = 0) -> ctypes.c_void_p:
    """A context whose workspace is the library's own static device array (no device allocation)."""
    ctx = ctypes.c_void_p()
    rc = load_library().cascade_init_static(ctypes.byref(cfg), ctypes.byref(init_state) if init_state is not None else None,
                                            stream, ctypes.byref(ctx))
    _check(rc, None)
    return ctx


def cascade_layers_workspace_bytes(cfg: cascade_config, n_layers: int) -> int:
    return int(load_library().cascade_layers_workspace_bytes(ctypes.byref(cfg), n_layers))


def cascade_init_layers(cfg: cascade_config, n_layers: int, dev_workspace: int, workspace_bytes: int,
                        init_states: Optional[Sequence[Optional[cascade_init_state]]] = None, stream: int = 0):
    """n_layers contexts that share the per-call scratch of one workspace; returns them as a list."""
    n = max(int(n_layers), 0)
    ctxs = (ctypes.c_void_p * max(n, 1))()
    states = None
    if init_states is not None:
        assert len(init_states) == n
        states = (ctypes.c_void_p * max(n, 1))()
        for i, st in enumerate(init_states):
            states[i] = ctypes.cast(ctypes.pointer(st), ctypes.c_void_p).value if st is not None else None
    rc = load_library().cascade_init_layers(ctypes.byref(cfg), n_layers, dev_workspace, workspace_bytes,
                                            states, stream, ctxs)
    _check(rc, None)
    return [ctypes.c_void_p(ctxs[i]) for i in range(n)]


def cascade_destroy(ctx) -> None:
    load_library().cascade_destroy(ctx)


def cascade_prefill_chunk(ctx, dev_q: int, dev_k: int, dev_v: int, n_tokens: int, dev_out: int, stream: int = 0) -> None:
    _check(load_library().cascade_prefill_chunk(ctx, dev_q, dev_k, dev_v, n_tokens, dev_out, stream), ctx)


def cascade_decode_step(ctx, dev_q: int, dev_k: int, dev_v: int, dev_out: int, stream: int = 0) -> None:
    _check(load_library().cascade_decode_step(ctx, dev_q, dev_k, dev_v, dev_out, stream), ctx)


def cascade_profile_begin(ctx, families=None) -> None:
    """families: names from KERNEL_FAMILIES to put events around (None: all of them)."""
    if families is None:
        _check(load_library().cascade_profile_begin(ctx), ctx)
    else:
        mask = sum(1 << KERNEL_FAMILIES.index(f) for f in families)
        _check(load_library().cascade_profile_begin_families(ctx, mask), ctx)


def cascade_profile_end(ctx) -> dict:
    """{family: (milliseconds, intervals)} of the kernels launched since cascade_profile_begin."""
    p = cascade_profile()
    _check(load_library().cascade_profile_end(ctx, ctypes.byref(p)), ctx)
    return {name: (float(p.ms[i]), int(p.intervals[i])) for i, name in enumerate(KERNEL_FAMILIES)}


def cascade_measure_ceilings(dev_buffer: int, nbytes: int, stream: int = 0) -> dict:
    """Measured ceilings of the current device (see include/cascade_kv.h) as a dict."""
    c = cascade_ceilings()
    _check(load_library().cascade_measure_ceilings(dev_buffer, nbytes, stream, ctypes.byref(c)), None)
    return {name: getattr(c, name) for name, _ in cascade_ceilings._fields_}


class StateArrays:
    """Host arrays of a cascade_read_state call (cache order; see include/cascade_kv.h)."""

    def __init__(self, view: cascade_state_view, n_cascades: int, ids, mu, slot, k, v, swaps):
        self.counts = np.array(view.counts[:1 + n_cascades], dtype=np.int64)
        self.xi = np.array(view.xi[:n_cascades], dtype=np.int64)
        self.accepted = np.array(view.accepted[:n_cascades], dtype=np.int64)
        self.discards = np.array(view.discards[:n_cascades], dtype=np.int64)
        self.t, self.n_seen = int(view.t), int(view.n_seen)
        self.count = int(self.counts.sum())
        self.ids, self.mu, self.slot, self.k, self.v, self.swaps = ids, mu, slot, k, v, swaps
        self.pre_count, self.last_tokens = int(view.pre_count), int(view.last_tokens)
        self.last_single_pass = bool(view.last_single_pass)
        self.pre_mu = self.chunk_mu = None


class PairRows:
    """K or V rows of selected (sequence, KV head) pairs, indexed like the full [B, Hkv, slots, d] array."""

    def __init__(self, pairs, rows: np.ndarray):
        self.index = {tuple(p): i for i, p in enumerate(pairs)}
        self.rows = rows

    def __getitem__(self, key):
        b, g = key[0], key[1]
        return self.rows[(self.index[(int(b), int(g))],) + tuple(key[2:])]


def cascade_read_state(ctx, cfg: cascade_config, with_kv: bool = False, stream: int = 0, kv_pairs=None) -> StateArrays:
    """kv_pairs: with_kv for these (sequence, KV head) pairs only (k and v are then PairRows)."""
    B, H, N, d = cfg.batch, cfg.n_kv_heads, cfg.n_cascades, cfg.head_dim
    slots = cfg.n_sink + sum(cfg.cascade_sizes[i] for i in range(N))
    ids = np.empty((B, H, slots), dtype=np.int32)
    mu = np.empty((B, H, slots), dtype=np.float32)
    slot = np.empty((B, H, slots), dtype=np.int32)
    swaps = np.empty((B, H, N), dtype=np.int64)
    view = cascade_state_view()
    pair_idx = None
    if with_kv and kv_pairs is not None:
        pair_idx = np.ascontiguousarray([b * H + g for b, g in kv_pairs], dtype=np.int32)
        view.host_kv_pairs, view.n_kv_pairs = pair_idx.ctypes.data, len(pair_idx)
        k = np.empty((len(pair_idx), slots, d), dtype=np.float32)
        v = np.empty((len(pair_idx), slots, d), dtype=np.float32)
    else:
        k = np.empty((B, H, slots, d), dtype=np.float32) if with_kv else None
        v = np.empty((B, H, slots, d), dtype=np.float32) if with_kv else None
    view.host_ids, view.host_mu, view.host_slot = ids.ctypes.data, mu.ctypes.data, slot.ctypes.data
    view.host_swaps = swaps.ctypes.data
    view.host_k = k.ctypes.data if with_kv else None
    view.host_v = v.ctypes.data if with_kv else None
    pre_mu = chunk_mu = None
    if cfg.keep_update_scores:
        pre_mu = np.zeros((B, H, slots), dtype=np.float32)
        chunk_mu = np.zeros((B, H, cfg.max_chunk), dtype=np.float32)
        view.host_pre_mu, view.host_chunk_mu = pre_mu.ctypes.data, chunk_mu.ctypes.data
    _check(load_library().cascade_read_state(ctx, ctypes.byref(view), stream), ctx)
    if pair_idx is not None:
        k, v = PairRows(kv_pairs, k), PairRows(kv_pairs, v)
    out = StateArrays(view, N, ids, mu, slot, k, v, swaps)
    out.pre_mu, out.chunk_mu = pre_mu, chunk_mu
    return out


def cascade_simulate_structure(cfg: cascade_config, chunk_sizes: Sequence[int],
                               scores: Optional[Sequence[float]] = None) -> StateArrays:
    N = cfg.n_cascades
    slots = cfg.n_sink + sum(cfg.cascade_sizes[i] for i in range(N))
    sizes = np.ascontiguousarray(chunk_sizes, dtype=np.int32)
    slot = np.empty(max(slots, 1), dtype=np.int32)
    view = cascade_state_view()
    view.host_slot = slot.ctypes.data
    ids = mu = swaps = sc = None
    if scores is not None:
        sc = np.ascontiguousarray(scores, dtype=np.float32)
        assert len(sc) == int(sizes.sum())
        ids = np.empty(max(slots, 1), dtype=np.int32)
        mu = np.empty(max(slots, 1), dtype=np.float32)
        swaps = np.zeros(N, dtype=np.int64)
        view.host_ids, view.host_mu, view.host_swaps = ids.ctypes.data, mu.ctypes.data, swaps.ctypes.data
    rc = load_library().cascade_simulate_structure(ctypes.byref(cfg), sizes.ctypes.data, len(sizes),
                                                   None if sc is None else sc.ctypes.data, ctypes.byref(view))
    _check(rc, None)
    return StateArrays(view, N, None if ids is None else ids[:slots], None if mu is None else mu[:slots],
                       slot[:slots], None, None, swaps)
