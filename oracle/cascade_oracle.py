"""ctypes wrapper around the C oracle (``cascade_oracle.c``).  Test infrastructure only.

Argument marshalling only: every computation happens in the C file.
"""
from __future__ import annotations

import ctypes
import dataclasses
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_MAX_CASCADES = 16
_LIB = None


def oracle_library_path() -> str:
    return os.path.join(_HERE, "liboracle.so")


def build_oracle(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP across KV heads only)."""
    src = os.path.join(_HERE, "cascade_oracle.c")
    out = oracle_library_path()
    if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
                               "-Wall", "-Wextra", "-o", out, src, "-lm"])
    return out


class _CConfig(ctypes.Structure):
    _fields_ = [
        ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
        ("n_sink", ctypes.c_int32), ("n_cascades", ctypes.c_int32),
        ("cascade_sizes", ctypes.c_int32 * _MAX_CASCADES),
        ("accept_period", ctypes.c_int64 * _MAX_CASCADES),
        ("ema_beta", ctypes.c_double), ("rope_base", ctypes.c_double), ("softmax_scale", ctypes.c_double),
        ("head_reduce", ctypes.c_int32), ("token_selection", ctypes.c_int32), ("head_policy", ctypes.c_int32),
    ]


def _lib():
    global _LIB
    if _LIB is None:
        L = ctypes.CDLL(build_oracle())
        P = ctypes.c_void_p
        L.oracle_create.restype = P
        L.oracle_create.argtypes = [ctypes.POINTER(_CConfig)]
        L.oracle_destroy.argtypes = [P]
        L.oracle_chunk.restype = ctypes.c_int
        L.oracle_chunk.argtypes = [P, P, P, P, ctypes.c_int, P, ctypes.c_int, ctypes.c_int]
        L.oracle_eval_rows.restype = ctypes.c_int
        L.oracle_eval_rows.argtypes = [P, ctypes.c_int, P, P, P, ctypes.c_int, ctypes.c_int, ctypes.c_int, P, P]
        L.oracle_chunk_single_pass.restype = ctypes.c_int
        L.oracle_chunk_single_pass.argtypes = [P, P, P, P, ctypes.c_int, P, ctypes.c_int, ctypes.c_int, P, P]
        L.oracle_eval_rows_single_pass.restype = ctypes.c_int
        L.oracle_eval_rows_single_pass.argtypes = [P, ctypes.c_int, P, P, P, ctypes.c_int, ctypes.c_int, ctypes.c_int, P, P, P, P]
        L.oracle_insert_scored.restype = ctypes.c_int
        L.oracle_insert_scored.argtypes = [P, ctypes.c_int, ctypes.c_double]
        for name in ("oracle_count", "oracle_t", "oracle_n_seen"):
            getattr(L, name).restype = ctypes.c_int64
            getattr(L, name).argtypes = [P, ctypes.c_int]
        L.oracle_get_state.restype = ctypes.c_int
        L.oracle_get_state.argtypes = [P, ctypes.c_int, P, P, P, P, P, P]
        L.oracle_set_state.restype = ctypes.c_int
        L.oracle_set_state.argtypes = [P, ctypes.c_int, P, P, P, P, P, ctypes.c_int64, ctypes.c_int64]
        L.oracle_last_delta.restype = ctypes.c_int64
        L.oracle_last_delta.argtypes = [P, ctypes.c_int, P, ctypes.c_int64]
        L.oracle_discard_log.restype = ctypes.c_int64
        L.oracle_discard_log.argtypes = [P, ctypes.c_int, P, ctypes.c_int64]
        L.oracle_select_log.restype = ctypes.c_int64
        L.oracle_select_log.argtypes = [P, ctypes.c_int, P, P, ctypes.c_int64]
        L.oracle_clear_logs.restype = None
        L.oracle_clear_logs.argtypes = [P, ctypes.c_int]
        _LIB = L
    return _LIB


@dataclasses.dataclass
class OracleConfig:
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    n_sink: int
    cascade_sizes: Sequence[int]
    ema_beta: float
    rope_base: float
    accept_period: Optional[Sequence[int]] = None   # default 2**i for cascade i (0-based)
    softmax_scale: float = 0.0                      # 0 -> 1/sqrt(head_dim)
    head_reduce: int = 0                            # 0 max, 1 mean
    token_selection: int = 1
    head_policy: int = 0                            # 0 independent KV heads, 1 homogeneous

    def periods(self):
        if self.accept_period is not None:
            return list(self.accept_period)
        return [1 << i for i in range(len(self.cascade_sizes))]


@dataclasses.dataclass
class HeadState:
    ids: np.ndarray          # [count] int64, cache order
    mu: np.ndarray           # [count] float64
    cascade_of: np.ndarray   # [count] int32: 0 sink, c for cascade c (1-based)
    counts: np.ndarray       # [1 + N]: sink fill, cascade fills
    stats: np.ndarray        # [N, 3]: accepted, swaps, discards
    t: int
    n_seen: int
    k: Optional[np.ndarray] = None   # [count, d] float64
    v: Optional[np.ndarray] = None

    @property
    def pos(self) -> np.ndarray:
        """Positional-encoding index of every cached token: its index in the cache."""
        return np.arange(len(self.ids), dtype=np.int64)


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


class OracleSeq:
    """The oracle's cache and attention for ONE sequence (all its KV heads)."""

    def __init__(self, cfg: OracleConfig):
        self.cfg = cfg
        c = _CConfig()
        c.n_q_heads, c.n_kv_heads, c.head_dim = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
        c.n_sink, c.n_cascades = cfg.n_sink, len(cfg.cascade_sizes)
        for i, s in enumerate(cfg.cascade_sizes):
            c.cascade_sizes[i] = int(s)
        for i, p in enumerate(cfg.periods()):
            c.accept_period[i] = int(p)
        c.ema_beta, c.rope_base, c.softmax_scale = cfg.ema_beta, cfg.rope_base, cfg.softmax_scale
        c.head_reduce, c.token_selection, c.head_policy = cfg.head_reduce, cfg.token_selection, cfg.head_policy
        self._h = _lib().oracle_create(ctypes.byref(c))
        if not self._h:
            raise ValueError("oracle_create rejected the configuration")

    def close(self):
        if self._h:
            _lib().oracle_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- the path ---------------------------------------------------------
    def _schedule(self, schedule, n: int, Q: int):
        """schedule = (step_of_key [n + Q], steps_of_row [G, Q]) of Alg. 3's single-pass scores."""
        G = self.cfg.n_q_heads // self.cfg.n_kv_heads
        step_of_key = np.ascontiguousarray(schedule[0], dtype=np.int32)
        steps_of_row = np.ascontiguousarray(schedule[1], dtype=np.int32)
        assert step_of_key.shape == (n + Q,) and steps_of_row.shape == (G, Q), (step_of_key.shape, steps_of_row.shape)
        assert step_of_key.min() >= 1 and steps_of_row.min() >= 1
        return step_of_key, steps_of_row

    def chunk(self, q: np.ndarray, k: np.ndarray, v: np.ndarray,
              kv_heads: Optional[Tuple[int, int]] = None, schedule=None) -> np.ndarray:
        """q [Q,Hq,d], k, v [Q,Hkv,d] -> out [Q,Hq,d] float64, then the chunk enters the cache.
        schedule: None for exact scores, else the visiting schedule of Alg. 3's single-pass scores."""
        cfg = self.cfg
        q = np.ascontiguousarray(q, dtype=np.float32)
        k = np.ascontiguousarray(k, dtype=np.float32)
        v = np.ascontiguousarray(v, dtype=np.float32)
        Q = q.shape[0]
        assert q.shape == (Q, cfg.n_q_heads, cfg.head_dim), q.shape
        assert k.shape == (Q, cfg.n_kv_heads, cfg.head_dim) and v.shape == k.shape
        lo, hi = kv_heads if kv_heads is not None else (0, cfg.n_kv_heads)
        out = np.zeros((Q, cfg.n_q_heads, cfg.head_dim), dtype=np.float64)
        if schedule is None:
            rc = _lib().oracle_chunk(self._h, _ptr(q), _ptr(k), _ptr(v), Q, _ptr(out), lo, hi)
        else:
            sk, sr = self._schedule(schedule, self.count(lo), Q)
            rc = _lib().oracle_chunk_single_pass(self._h, _ptr(q), _ptr(k), _ptr(v), Q, _ptr(out), lo, hi, _ptr(sk), _ptr(sr))
        if rc != 0:
            raise RuntimeError("oracle_chunk failed")
        return out

    def eval_rows(self, kv_head: int, q: np.ndarray, k: np.ndarray, v: np.ndarray, row_lo: int, row_hi: int, schedule=None):
        """Rows [row_lo, row_hi) of the chunk (q, k, v) for one KV head, cache untouched.
        Returns (out [Q,Hq,d] with only those rows and that head group written,
        delta [count + Q]: the EMA increments those rows alone produce)."""
        cfg = self.cfg
        q = np.ascontiguousarray(q, dtype=np.float32)
        k = np.ascontiguousarray(k, dtype=np.float32)
        v = np.ascontiguousarray(v, dtype=np.float32)
        Q = q.shape[0]
        assert q.shape == (Q, cfg.n_q_heads, cfg.head_dim) and k.shape == (Q, cfg.n_kv_heads, cfg.head_dim)
        out = np.zeros((Q, cfg.n_q_heads, cfg.head_dim), dtype=np.float64)
        delta = np.zeros(self.count(kv_head) + Q, dtype=np.float64)
        if schedule is None:
            rc = _lib().oracle_eval_rows(self._h, kv_head, _ptr(q), _ptr(k), _ptr(v), Q, row_lo, row_hi, _ptr(out), _ptr(delta))
        else:
            sk, sr = self._schedule(schedule, self.count(kv_head), Q)
            rc = _lib().oracle_eval_rows_single_pass(self._h, kv_head, _ptr(q), _ptr(k), _ptr(v), Q, row_lo, row_hi,
                                                     _ptr(sk), _ptr(sr), _ptr(out), _ptr(delta))
        if rc != 0:
            raise RuntimeError("oracle_eval_rows failed")
        return out, delta

    def decode(self, q: np.ndarray, k: np.ndarray, v: np.ndarray, kv_heads=None) -> np.ndarray:
        """One decode step: q [Hq,d], k, v [Hkv,d] -> out [Hq,d]."""
        return self.chunk(q[None], k[None], v[None], kv_heads)[0]

    def insert_scored(self, kv_head: int, score: float) -> None:
        """Alg. 2 alone: insert the next token id with a given, frozen score."""
        if _lib().oracle_insert_scored(self._h, kv_head, float(score)) != 0:
            raise RuntimeError("oracle_insert_scored failed")

    # -- state ------------------------------------------------------------
    def count(self, kv_head: int) -> int:
        return int(_lib().oracle_count(self._h, kv_head))

    def state(self, kv_head: int, with_kv: bool = False) -> HeadState:
        cfg = self.cfg
        n = self.count(kv_head)
        N = len(cfg.cascade_sizes)
        ids = np.zeros(n, dtype=np.int64)
        mu = np.zeros(n, dtype=np.float64)
        cas = np.zeros(n, dtype=np.int32)
        counts = np.zeros(1 + N, dtype=np.int64)
        stats = np.zeros(3 * N, dtype=np.int64)
        kv = np.zeros((2, n, cfg.head_dim), dtype=np.float64) if with_kv else None
        _lib().oracle_get_state(self._h, kv_head, _ptr(ids), _ptr(mu), _ptr(cas), _ptr(counts), _ptr(stats), _ptr(kv))
        return HeadState(ids, mu, cas, counts, stats.reshape(N, 3),
                         int(_lib().oracle_t(self._h, kv_head)), int(_lib().oracle_n_seen(self._h, kv_head)),
                         None if kv is None else kv[0], None if kv is None else kv[1])

    def set_state(self, kv_head: int, ids, mu, counts, k, v, t: int, n_seen: int) -> None:
        ids = np.ascontiguousarray(ids, dtype=np.int64)
        mu = np.ascontiguousarray(mu, dtype=np.float64)
        counts = np.ascontiguousarray(counts, dtype=np.int64)
        k = np.ascontiguousarray(k, dtype=np.float32)
        v = np.ascontiguousarray(v, dtype=np.float32)
        n = int(counts.sum())
        assert len(counts) == 1 + len(self.cfg.cascade_sizes)
        assert ids.shape == (n,) and mu.shape == (n,) and k.shape == (n, self.cfg.head_dim) and v.shape == k.shape
        rc = _lib().oracle_set_state(self._h, kv_head, _ptr(ids), _ptr(mu), _ptr(counts), _ptr(k), _ptr(v),
                                     int(t), int(n_seen))
        if rc != 0:
            raise ValueError("oracle_set_state rejected the state")

    def last_delta(self, kv_head: int) -> np.ndarray:
        """Reduced EMA increments of the last chunk: cache order (before the chunk), then chunk tokens."""
        n = int(_lib().oracle_last_delta(self._h, kv_head, None, 0))
        out = np.zeros(n, dtype=np.float64)
        _lib().oracle_last_delta(self._h, kv_head, _ptr(out), n)
        return out

    def select_log(self, kv_head: int):
        """Every token-selection comparison of Alg. 2 so far (or since clear_logs), in order:
        (ids [n,2], mu [n,2]) of the incoming item and of the newest item of the cascade."""
        n = int(_lib().oracle_select_log(self._h, kv_head, None, None, 0))
        ids = np.zeros((max(n, 1), 2), dtype=np.int64)
        mu = np.zeros((max(n, 1), 2), dtype=np.float64)
        _lib().oracle_select_log(self._h, kv_head, _ptr(ids), _ptr(mu), n)
        return ids[:n], mu[:n]

    def clear_logs(self, kv_head: int) -> None:
        _lib().oracle_clear_logs(self._h, kv_head)

    def discard_log(self, kv_head: int) -> np.ndarray:
        n = int(_lib().oracle_discard_log(self._h, kv_head, None, 0))
        out = np.zeros(max(n, 1), dtype=np.int64)
        _lib().oracle_discard_log(self._h, kv_head, _ptr(out), n)
        return out[:n]
