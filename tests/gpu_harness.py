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
  rows      the K and V rows the library holds for every cached token must be, bit for bit, the
            rows that were fed for that token (Alg. 2 moves keys and values with their token);
            checked against the inputs themselves before the library's state is ever handed to the
            oracle, so a move that copied a wrong row cannot be adopted by the oracle;
  flips     where the membership differs from the free oracle's, the two records of selection
            comparisons (the oracle's on its own scores, the replay's on the library's scores; the
            k-th comparison happens at the same step and cascade in both, since the structure of
            Alg. 2 does not depend on the scores) are compared one by one: a comparison between
            the same two tokens that came out differently is a flip and must be noise-level by
            the oracle's own scores, |mu_a - mu_b| <= tau * max(mu_a, mu_b); one with other
            participants is downstream of an earlier flip and is only counted.
In "one step ahead" mode the oracle is re-loaded with the library's state after every compared
step, so one noise-level flip does not contaminate later comparisons.
"""
from __future__ import annotations

import dataclasses
import threading
from typing import List, Optional

import numpy as np
import torch

from oracle import OracleConfig, OracleSeq
from paper_2406_17808_amd import binding as B
from paper_2406_17808_amd.cache import CascadeKVCache


# A comparison can come out differently on the two sides only if the two scores differ by less
# than the two score errors together.  Scores agree to about 2^-7 (bf16: operand rounding of the
# rotated q and k) or 2^-14 (fp32) relative, hence twice that.
TAU = {B.CASCADE_BF16: 2.0 ** -6, B.CASCADE_F32: 2.0 ** -13}


class FedRows:
    """Every K / V row handed to one context, retrievable by (sequence, KV head, token id)."""

    def __init__(self):
        self._init = None      # (ids [n] sorted, k [B,Hkv,n,d], v) of an initial state
        self._chunks = []      # (first id, k [B,n,Hkv,d], v)
        self._regen = None

    def add_initial(self, ids, k, v):
        """ids [n] increasing; k, v: anything indexable as [b, g] -> [n, d] (rows in the order of ids)."""
        self._init = (np.asarray(ids, dtype=np.int64), k, v)

    def add(self, first_id: int, k: np.ndarray, v: np.ndarray):
        self._chunks.append((int(first_id), np.asarray(k, dtype=np.float32), np.asarray(v, dtype=np.float32)))

    def regenerate_with(self, fn, chunk: int):
        """For streams too long to keep: fn(chunk index) -> (k, v) [B,n,Hkv,d] of that chunk of `chunk` tokens."""
        self._regen = (fn, int(chunk))

    def rows(self, b: int, g: int, ids: np.ndarray):
        ids = np.asarray(ids, dtype=np.int64)
        d = None
        out_k = out_v = None
        found = np.zeros(len(ids), dtype=bool)

        def put(sel, kk, vv):
            nonlocal out_k, out_v
            if out_k is None:
                out_k = np.zeros((len(ids), kk.shape[-1]), dtype=np.float32)
                out_v = np.zeros_like(out_k)
            out_k[sel], out_v[sel] = kk, vv
            found[sel] = True

        if self._init is not None:
            iids, ik, iv = self._init
            pos = np.searchsorted(iids, ids)
            ok = (pos < len(iids)) & (iids[np.minimum(pos, len(iids) - 1)] == ids)
            if ok.any():
                put(ok, np.asarray(ik[b, g][pos[ok]], dtype=np.float32), np.asarray(iv[b, g][pos[ok]], dtype=np.float32))
        for first, k, v in self._chunks:
            sel = (ids >= first) & (ids < first + k.shape[1]) & ~found
            if sel.any():
                put(sel, k[b, ids[sel] - first, g], v[b, ids[sel] - first, g])
        if self._regen is not None and not found.all():
            fn, chunk = self._regen
            for c in np.unique(ids[~found] // chunk):
                k, v = fn(int(c))
                sel = (ids // chunk == c) & ~found
                put(sel, k[b, ids[sel] - c * chunk, g], v[b, ids[sel] - c * chunk, g])
        assert found.all(), f"token ids never fed: {ids[~found][:8]}"
        return out_k, out_v


def check_cached_rows(st, b: int, g: int, fed: FedRows) -> None:
    """The library's K / V rows of (b, g) against the rows fed for the same token ids, bit for bit."""
    n = st.count
    ids = st.ids[b, g, :n]
    k, v = fed.rows(b, g, ids)
    for name, got, want in (("K", st.k[b, g, :n], k), ("V", st.v[b, g, :n], v)):
        bad = np.nonzero((got.view(np.uint32) != want.view(np.uint32)).any(axis=1))[0]
        assert len(bad) == 0, (f"sequence {b} KV head {g}: {len(bad)} cached {name} rows differ from the rows fed for "
                               f"their tokens; first at cache index {int(bad[0])} (token {int(ids[bad[0]])})")


def classify_flips(ref_log, gpu_log, token_selection: int, tau: float):
    """ref_log, gpu_log: (ids [n,2], mu [n,2]) selection comparisons of the oracle on its own scores
    and of the replay on the library's scores.  Returns (noise-level flips, mismatches, downstream)."""
    (ri, rm), (gi, gm) = ref_log, gpu_log
    assert len(ri) == len(gi), "the number of selection comparisons does not depend on the scores"
    noise = mismatch = downstream = 0
    for k in range(len(ri)):
        if ri[k, 0] != gi[k, 0] or ri[k, 1] != gi[k, 1]:
            downstream += 1
            continue
        won_ref = bool(token_selection) and rm[k, 0] > rm[k, 1]
        won_gpu = bool(token_selection) and gm[k, 0] > gm[k, 1]
        if won_ref == won_gpu:
            continue
        gap = abs(rm[k, 0] - rm[k, 1])
        if gap <= tau * max(abs(rm[k, 0]), abs(rm[k, 1])):
            noise += 1
        else:
            mismatch += 1
    return noise, mismatch, downstream


def visiting_schedule(cfg: B.cascade_config, st, Q: int):
    """The order in which the library's chunk attention visits the keys, as the single-pass scores
    of Alg. 3 need it (an input of the oracle's *_single_pass calls), written from the documented
    layout: the cache is swept in PHYSICAL order (sinks, then the last cascade ... the first cascade,
    every ring from its slot 0; a full ring is cut at xi mod 64 and at its head xi), every piece in
    tiles of 64 keys, then the chunk's own keys; a row block is 256 tokens of one head and visits
    the chunk's tiles up to its last token.  st: the library's state before the chunk.
    Returns step_of_key [n + Q] (cache order, then chunk; counted from 1) and steps_of_row [G, Q]."""
    N = cfg.n_cascades
    sizes = [cfg.cascade_sizes[i] for i in range(N)]
    bases, base = [0] * N, cfg.n_sink
    for c in range(N - 1, -1, -1):
        bases[c] = base
        base += sizes[c]
    pieces = [(0, int(st.counts[0]))]
    for c in range(N - 1, -1, -1):
        cnt, cap, xi = int(st.counts[1 + c]), sizes[c], int(st.xi[c])
        if cnt < cap:
            pieces.append((bases[c], cnt))
        else:
            o = xi % 64
            pieces += [(bases[c], o), (bases[c] + o, xi - o), (bases[c] + xi, cap - xi)]
    step_of_slot = np.zeros(cfg.n_sink + sum(sizes), dtype=np.int32)
    tiles = 0
    for start, length in pieces:
        if length <= 0:
            continue
        step_of_slot[start:start + length] = tiles + np.arange(length) // 64 + 1
        tiles += (length + 63) // 64
    n = st.count
    step_of_key = np.concatenate([step_of_slot[st.slot[0, 0, :n]], tiles + np.arange(Q) // 64 + 1]).astype(np.int32)
    assert step_of_key.min() >= 1
    G = cfg.n_q_heads // cfg.n_kv_heads
    last_token = (np.arange(Q) // 256 + 1) * 256
    steps_of_row = np.broadcast_to(tiles + (np.minimum(Q, last_token) + 63) // 64, (G, Q)).astype(np.int32)
    return step_of_key, steps_of_row


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
                        head_reduce=cfg.head_reduce, token_selection=cfg.token_selection,
                        head_policy=getattr(cfg, "head_policy", 0))


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
    flips_noise: int = 0          # selection comparisons that came out differently inside the noise of the scores
    flips_mismatch: int = 0       # ... and outside it: a failure
    flips_downstream: int = 0     # comparisons with other participants than the oracle's (after an earlier flip)
    model_out_err: float = 0.0    # bf16 only, on request: outputs / scores against the numpy model that rounds
    model_score_err: float = 0.0  # where the bf16 contract rounds (bf16_model.py)
    single_pass: bool = False     # the call took Alg. 3's single-pass scores (and the oracle was given the schedule)
    diverged_from_exact: int = 0  # single pass, on request: cache positions that differ from the EXACT-score oracle's


def gpu_decision_scores(st, b, g, npre, n_tok) -> np.ndarray:
    """Scores the library took its insertion decisions with: items cached before the call (cache
    order before the call), then the call's tokens."""
    return np.concatenate([st.pre_mu[b, g, :npre], st.chunk_mu[b, g, :n_tok]]).astype(np.float64)


def replay_is_exact(cfg: B.cascade_config, prev, st, b, g, mu_gpu, log_out: Optional[list] = None,
                    state_out: Optional[list] = None) -> bool:
    """Alg. 2 replayed by the oracle with the library's own scores, from the library's state
    before the call (`prev`), must give the library's state after it (`st`) bit for bit.
    log_out (a list) receives the replay's record of selection comparisons, state_out the replay's
    state after the call."""
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
    if log_out is not None:
        log_out.append(pol.select_log(0))
    if state_out is not None:
        state_out.append(ps)
    pol.close()
    return bool(ok)


def compare_decisions(cfg: B.cascade_config, rep: StepReport, o: OracleSeq, g: int, prev, st, b: int, mu_gpu,
                      same_start: bool, tau: Optional[float] = None) -> None:
    """Decisions of one (sequence, KV head) after the oracle has taken the same step: the exact
    replay, the drift against the oracle's own membership, and the flips (only where both sides
    started the step from the same membership: `same_start`)."""
    log = []
    rep.replay_exact &= replay_is_exact(cfg, prev, st, b, g, mu_gpu, log)
    post = o.state(g)
    cnt = st.count
    rep.compared += cnt
    if post.counts.tolist() != st.counts.tolist():
        rep.drift += cnt
    else:
        rep.drift += int((post.ids != st.ids[b, g, :cnt]).sum())
    if same_start:
        noise, mismatch, downstream = classify_flips(o.select_log(g), log[0], cfg.token_selection,
                                                     TAU[cfg.dtype] if tau is None else tau)
        rep.flips_noise += noise
        rep.flips_mismatch += mismatch
        rep.flips_downstream += downstream


def row_errors(out, ref, heads) -> float:
    """max over rows of ||out - ref|| / ||ref|| for the given query heads; out, ref [rows, Hq, d]."""
    num = np.linalg.norm(out[:, heads] - ref[:, heads], axis=-1)
    den = np.linalg.norm(ref[:, heads], axis=-1)
    return float((num / np.maximum(den, 1e-30)).max())


class ParityRun:
    """One library context and one oracle per compared sequence, advanced together."""

    def __init__(self, cfg: B.cascade_config, one_step_ahead: bool, kv_heads: Optional[List[int]] = None,
                 init_state: Optional[B.cascade_init_state] = None, device="cuda:0", seqs: Optional[List[int]] = None,
                 gpu: Optional[CascadeKVCache] = None, tau: Optional[float] = None):
        assert cfg.keep_update_scores == 1
        self.cfg = cfg
        self.tau = tau
        self.fed = FedRows()
        self.gpu = gpu if gpu is not None else CascadeKVCache(cfg, device, init_state)   # gpu: an existing context
        self.ocfg = oracle_config_of(cfg)
        self.seqs = list(range(cfg.batch)) if seqs is None else seqs
        self.oracles = {b: OracleSeq(self.ocfg) for b in self.seqs}
        self.one_step = one_step_ahead
        self.heads = list(range(cfg.n_kv_heads)) if kv_heads is None else kv_heads
        self.G = cfg.n_q_heads // cfg.n_kv_heads
        self.reports: List[StepReport] = []
        self.prev = self.gpu.read_state()           # library state before the next call
        self._n_seen = self.prev.n_seen             # id of the next token fed
        self.device = device

    def prev_n_seen(self) -> int:
        return self._n_seen

    # -- oracle <- library ---------------------------------------------------
    def read_state(self):
        """The library's state with the K / V rows of the compared (sequence, KV head) pairs."""
        return self.gpu.read_state(with_kv=True, kv_pairs=[(b, g) for b in self.seqs for g in self.heads])

    def check_rows(self, st) -> None:
        for b in self.seqs:
            for g in self.heads:
                check_cached_rows(st, b, g, self.fed)

    def sync_oracle_from_gpu(self, st=None):
        st = st if st is not None else self.read_state()
        self.check_rows(st)        # before the oracle adopts anything: the rows are the ones that were fed
        n = st.count
        for b, o in self.oracles.items():
            for g in self.heads:
                o.set_state(g, st.ids[b, g, :n].astype(np.int64), st.mu[b, g, :n].astype(np.float64), st.counts,
                            st.k[b, g, :n], st.v[b, g, :n], st.t, st.n_seen)
        self.prev = st

    def advance_gpu_only(self, dq, dk, dv, decode: bool = False, record: bool = True):
        """A step that is not compared (device tensors); the oracle falls behind until the next sync.
        record=False: the caller has given self.fed another way to find the rows of this step."""
        if record:
            hk, hv = dk.float().cpu().numpy(), dv.float().cpu().numpy()
            self.fed.add(self.prev_n_seen(), hk[:, None] if decode else hk, hv[:, None] if decode else hv)
        self._n_seen += 1 if decode else dq.shape[1]
        if decode:
            self.gpu.decode_step(dq, dk, dv)
        else:
            self.gpu.prefill_chunk(dq, dk, dv)

    # -- one compared step -----------------------------------------------------
    def step(self, q: np.ndarray, k: np.ndarray, v: np.ndarray, decode: bool = False, threaded: bool = False,
             with_model: bool = False, exact_twin: bool = False) -> StepReport:
        """q [B,n,Hq,d], k, v [B,n,Hkv,d] float32 (bf16-valued for a bf16 context); decode: n == 1.
        threaded: the oracle evaluates only the compared KV heads, each on a thread of its own.
        with_model (prefill, bf16, one step ahead): also compare with the bf16 rounding model.
        exact_twin (single-pass scores, one step ahead): a second oracle takes the same step from the
        same state with the EXACT scores; the positions where the library's cache then differs from
        its cache are counted (how far the approximation moves the membership)."""
        cfg = self.cfg
        n_tok = q.shape[1]
        dq, dk, dv = to_device(q, cfg, self.device), to_device(k, cfg, self.device), to_device(v, cfg, self.device)
        self.fed.add(self._n_seen, k, v)
        self._n_seen += n_tok
        if decode:
            out = self.gpu.decode_step(dq[:, 0].contiguous(), dk[:, 0].contiguous(), dv[:, 0].contiguous())[:, None]
        else:
            out = self.gpu.prefill_chunk(dq, dk, dv)
        st = self.read_state()
        self.check_rows(st)
        out = out.float().cpu().numpy()
        rep = StepReport()
        beta = float(np.float32(cfg.ema_beta))
        rep.single_pass = bool(st.last_single_pass)
        schedule = visiting_schedule(cfg, self.prev, n_tok) if rep.single_pass else None
        for b, o in self.oracles.items():
            pre = {g: o.state(g) for g in self.heads}
            for g in range(cfg.n_kv_heads):
                o.clear_logs(g)
            twin = None
            if exact_twin and rep.single_pass:
                assert self.one_step
                twin = OracleSeq(self.ocfg)
                for g in self.heads:
                    full = o.state(g, with_kv=True)
                    twin.set_state(g, full.ids, full.mu, full.counts, full.k, full.v, full.t, full.n_seen)
            refs = {}
            if threaded and self.ocfg.head_policy == 0:
                def work(g, o=o, b=b):
                    refs[g] = o.chunk(q[b], k[b], v[b], kv_heads=(g, g + 1), schedule=schedule)
                    if twin is not None:
                        twin.chunk(q[b], k[b], v[b], kv_heads=(g, g + 1))
                threads = [threading.Thread(target=work, args=(g,)) for g in self.heads]
                [t.start() for t in threads]
                [t.join() for t in threads]
            else:
                hs = (0, cfg.n_kv_heads) if self.ocfg.head_policy == 1 else (min(self.heads), max(self.heads) + 1)
                ref = o.chunk(q[b], k[b], v[b], kv_heads=hs, schedule=schedule)
                refs = {g: ref for g in self.heads}
                if twin is not None:
                    twin.chunk(q[b], k[b], v[b], kv_heads=hs)
            for g in self.heads:
                hq = slice(g * self.G, (g + 1) * self.G)
                rep.out_err = max(rep.out_err, row_errors(out[b], refs[g], hq))
                # scores the decisions are taken with
                delta = o.last_delta(g)
                npre = len(pre[g].ids)
                assert st.pre_count == npre and st.last_tokens == n_tok
                mu_ref = np.concatenate([pre[g].mu * beta ** n_tok + delta[:npre], delta[npre:]])
                mu_gpu = gpu_decision_scores(st, b, g, npre, n_tok)
                rel = np.abs(mu_gpu - mu_ref) / np.maximum(np.abs(mu_ref), 1e-12)
                rep.score_err = max(rep.score_err, float(rel.max()))
                # decisions: Alg. 2 replayed with the library's scores; drift and flips against the
                # oracle on its own scores
                same_start = pre[g].ids.tolist() == self.prev.ids[b, g, :npre].tolist()
                compare_decisions(cfg, rep, o, g, self.prev, st, b, mu_gpu, same_start, self.tau)
                if twin is not None:
                    rep.diverged_from_exact += int((twin.state(g).ids != st.ids[b, g, :st.count]).sum())
                if with_model:
                    from bf16_model import chunk_reference
                    assert self.one_step and not decode and cfg.dtype == B.CASCADE_BF16 and cfg.head_reduce == 0
                    pk = self.prev.k[b, g, :npre] if npre else np.zeros((0, cfg.head_dim), np.float32)
                    pv = self.prev.v[b, g, :npre] if npre else np.zeros((0, cfg.head_dim), np.float32)
                    mo, md = chunk_reference(q[b][:, hq], k[b][:, g], v[b][:, g], pk, pv, self.prev.slot[b, g, :npre],
                                             np.arange(n_tok), float(np.float32(cfg.rope_base)), float(cfg.softmax_scale),
                                             ema_beta=beta)
                    num = np.linalg.norm(out[b][:, hq] - mo, axis=-1)
                    rep.model_out_err = max(rep.model_out_err, float((num / np.linalg.norm(mo, axis=-1)).max()))
                    mu_model = np.concatenate([pre[g].mu * beta ** n_tok, np.zeros(n_tok)]) + md.max(axis=0)
                    relm = np.abs(mu_gpu - mu_model) / np.maximum(np.abs(mu_model), 1e-12)
                    rep.model_score_err = max(rep.model_score_err, float(relm[mu_model > 1e-30].max()))
            if twin is not None:
                twin.close()
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
