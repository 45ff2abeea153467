"""Shared machinery of the GPU parity tests: drive the HIP library and the CPU oracle with the
same inputs and compare, element by element.

How parity is decomposed (per chunk or decode step, per sequence and KV head):
  outputs   relative L2 error of every (token, query head) row against the oracle;
  scores    the EMA scores the insertion decisions are taken with (diagnostic snapshot of the
            library) against the oracle's, relative error;
  decisions Alg. 2 replayed by the oracle WITH THE LIBRARY'S OWN SCORES must reproduce the
            library's cache membership and carried scores exactly (integer work: bit-exact);
  drift     membership against the oracle running on its own scores; positions that differ are
            counted and reported (they can only come from score gaps inside float noise).
In "one step ahead" mode the oracle is re-loaded with the library's state after every compared
step, so one noise-level flip does not contaminate later comparisons.
"""
from __future__ import annotations

import dataclasses
from typing import List, Optional

import numpy as np
import torch

from oracle import OracleConfig, OracleSeq
from paper_2406_17808_amd import binding as B
from paper_2406_17808_amd.cache import CascadeKVCache


def periods_of(cfg: B.cascade_config):
    N = cfg.n_cascades
    p = [cfg.accept_period[i] for i in range(N)]
    return None if all(x == 0 for x in p) else p


def oracle_config_of(cfg: B.cascade_config) -> OracleConfig:
    N = cfg.n_cascades
    return OracleConfig(n_q_heads=cfg.n_q_heads, n_kv_heads=cfg.n_kv_heads, head_dim=cfg.head_dim,
                        n_sink=cfg.n_sink, cascade_sizes=[cfg.cascade_sizes[i] for i in range(N)],
                        ema_beta=float(np.float32(cfg.ema_beta)), rope_base=float(np.float32(cfg.rope_base)),
                        accept_period=periods_of(cfg), softmax_scale=float(cfg.softmax_scale),
                        head_reduce=cfg.head_reduce, token_selection=cfg.token_selection)


def policy_oracle(cfg: B.cascade_config) -> OracleSeq:
    N = cfg.n_cascades
    return OracleSeq(OracleConfig(1, 1, 2, cfg.n_sink, [cfg.cascade_sizes[i] for i in range(N)], 0.9, 10.0,
                                  accept_period=periods_of(cfg), token_selection=cfg.token_selection))


def to_device(x: np.ndarray, cfg: B.cascade_config, device="cuda:0") -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(x)).to(device)
    return t.to(torch.bfloat16) if cfg.dtype == B.CASCADE_BF16 else t


@dataclasses.dataclass
class StepReport:
    out_err: float = 0.0          # max over rows of ||gpu - ref|| / ||ref||
    score_err: float = 0.0        # max relative error of the decision scores
    drift: int = 0                # cache positions whose id differs from the free oracle's
    compared: int = 0             # cache positions compared
    replay_exact: bool = True


def gpu_decision_scores(st, b, g, npre, n_tok) -> np.ndarray:
    """Scores the library took its insertion decisions with: items cached before the call (cache
    order before the call), then the call's tokens."""
    return np.concatenate([st.pre_mu[b, g, :npre], st.chunk_mu[b, g, :n_tok]]).astype(np.float64)


def replay_is_exact(cfg: B.cascade_config, prev, st, b, g, mu_gpu) -> bool:
    """Alg. 2 replayed by the oracle with the library's own scores, from the library's state
    before the call (`prev`), must give the library's state after it (`st`) bit for bit."""
    npre = prev.count
    pol = policy_oracle(cfg)
    zeros = np.zeros((npre, 2), dtype=np.float32)
    pol.set_state(0, prev.ids[b, g, :npre].astype(np.int64), mu_gpu[:npre], prev.counts, zeros, zeros,
                  prev.t, prev.n_seen)
    for s in mu_gpu[npre:]:
        pol.insert_scored(0, float(s))
    ps = pol.state(0)
    cnt = st.count
    ok = (ps.ids.tolist() == st.ids[b, g, :cnt].tolist()
          and np.array_equal(ps.mu.astype(np.float32), st.mu[b, g, :cnt])
          and ps.counts.tolist() == st.counts.tolist() and ps.t == st.t and ps.n_seen == st.n_seen)
    pol.close()
    return bool(ok)


def row_errors(out, ref, heads) -> float:
    """max over rows of ||out - ref|| / ||ref|| for the given query heads; out, ref [rows, Hq, d]."""
    num = np.linalg.norm(out[:, heads] - ref[:, heads], axis=-1)
    den = np.linalg.norm(ref[:, heads], axis=-1)
    return float((num / np.maximum(den, 1e-30)).max())


class ParityRun:
    """One library context and one oracle per compared sequence, advanced together."""

    def __init__(self, cfg: B.cascade_config, one_step_ahead: bool, kv_heads: Optional[List[int]] = None,
                 init_state: Optional[B.cascade_init_state] = None, device="cuda:0", seqs: Optional[List[int]] = None,
                 gpu: Optional[CascadeKVCache] = None):
        assert cfg.keep_update_scores == 1
        self.cfg = cfg
        self.gpu = gpu if gpu is not None else CascadeKVCache(cfg, device, init_state)   # gpu: an existing context
        self.ocfg = oracle_config_of(cfg)
        self.seqs = list(range(cfg.batch)) if seqs is None else seqs
        self.oracles = {b: OracleSeq(self.ocfg) for b in self.seqs}
        self.one_step = one_step_ahead
        self.heads = list(range(cfg.n_kv_heads)) if kv_heads is None else kv_heads
        self.G = cfg.n_q_heads // cfg.n_kv_heads
        self.reports: List[StepReport] = []
        self.prev = self.gpu.read_state()           # library state before the next call
        self.device = device

    # -- oracle <- library ---------------------------------------------------
    def sync_oracle_from_gpu(self, st=None):
        st = st if st is not None else self.gpu.read_state(with_kv=True)
        n = st.count
        for b, o in self.oracles.items():
            for g in self.heads:
                o.set_state(g, st.ids[b, g, :n].astype(np.int64), st.mu[b, g, :n].astype(np.float64), st.counts,
                            st.k[b, g, :n], st.v[b, g, :n], st.t, st.n_seen)
        self.prev = st

    def advance_gpu_only(self, dq, dk, dv, decode: bool = False):
        """A step that is not compared (device tensors); the oracle falls behind until the next sync."""
        if decode:
            self.gpu.decode_step(dq, dk, dv)
        else:
            self.gpu.prefill_chunk(dq, dk, dv)

    # -- one compared step -----------------------------------------------------
    def step(self, q: np.ndarray, k: np.ndarray, v: np.ndarray, decode: bool = False) -> StepReport:
        """q [B,n,Hq,d], k, v [B,n,Hkv,d] float32 (bf16-valued for a bf16 context); decode: n == 1."""
        cfg = self.cfg
        n_tok = q.shape[1]
        dq, dk, dv = to_device(q, cfg, self.device), to_device(k, cfg, self.device), to_device(v, cfg, self.device)
        if decode:
            out = self.gpu.decode_step(dq[:, 0].contiguous(), dk[:, 0].contiguous(), dv[:, 0].contiguous())[:, None]
        else:
            out = self.gpu.prefill_chunk(dq, dk, dv)
        st = self.gpu.read_state(with_kv=self.one_step)
        out = out.float().cpu().numpy()
        rep = StepReport()
        beta = float(np.float32(cfg.ema_beta))
        for b, o in self.oracles.items():
            pre = {g: o.state(g) for g in self.heads}
            hs = (min(self.heads), max(self.heads) + 1)
            ref = o.chunk(q[b], k[b], v[b], kv_heads=hs)
            for g in self.heads:
                hq = slice(g * self.G, (g + 1) * self.G)
                rep.out_err = max(rep.out_err, row_errors(out[b], ref, hq))
                # scores the decisions are taken with
                delta = o.last_delta(g)
                npre = len(pre[g].ids)
                assert st.pre_count == npre and st.last_tokens == n_tok
                mu_ref = np.concatenate([pre[g].mu * beta ** n_tok + delta[:npre], delta[npre:]])
                mu_gpu = gpu_decision_scores(st, b, g, npre, n_tok)
                rel = np.abs(mu_gpu - mu_ref) / np.maximum(np.abs(mu_ref), 1e-12)
                rep.score_err = max(rep.score_err, float(rel.max()))
                # decisions: Alg. 2 replayed with the library's scores
                rep.replay_exact &= replay_is_exact(cfg, self.prev, st, b, g, mu_gpu)
                # drift against the oracle on its own scores
                post = o.state(g)
                cnt = st.count
                rep.compared += cnt
                if post.counts.tolist() != st.counts.tolist():
                    rep.drift += cnt
                else:
                    rep.drift += int((post.ids != st.ids[b, g, :cnt]).sum())
        if self.one_step:
            self.sync_oracle_from_gpu(st)
        else:
            self.prev = st
        self.reports.append(rep)
        return rep

    def close(self):
        self.gpu.close()
        for o in self.oracles.values():
            o.close()
