"""Pins of the oracle's attention, positional encoding and EMA scores.

The checks below are dense numpy formulas (matrix softmax, RoPE written as a complex
multiplication) applied to special cases where the method has a textbook definition:
full causal attention, sink + sliding window, and brute force over the cache membership.
"""
import numpy as np
import pytest

from oracle import OracleConfig, OracleSeq


def rope_complex(x, pos, base):
    """RoPE on the last axis of x at integer positions pos (broadcast over leading axes):
    the pair (x_i, x_{i+d/2}) is the complex number x_i + 1j*x_{i+d/2}, multiplied by
    exp(1j * pos * base**(-2i/d))."""
    d = x.shape[-1]
    half = d // 2
    z = x[..., :half] + 1j * x[..., half:]
    theta = base ** (-2.0 * np.arange(half) / d)
    z = z * np.exp(1j * np.asarray(pos, dtype=np.float64)[..., None] * theta)
    return np.concatenate([z.real, z.imag], axis=-1)


def dense_attention(q, qpos, keys, kpos, vals, visible, base, scale):
    """q [m,d] at qpos [m]; keys/vals [n,d] at kpos [n]; visible [m,n] bool -> (out [m,d], P [m,n])."""
    s = rope_complex(q, qpos, base) @ rope_complex(keys, kpos, base).T * scale
    s = np.where(visible, s, -np.inf)
    s = s - s.max(axis=1, keepdims=True)
    p = np.exp(s)
    p /= p.sum(axis=1, keepdims=True)
    return p @ vals, p


def _rand(rng, *shape):
    return rng.standard_normal(shape).astype(np.float32)


def test_full_causal_attention_before_any_discard(oracle_mod):
    """While nothing has been discarded the cache order is the original order and the PE index
    is the original index (Section 3.1), so the outputs are ordinary causal attention (Eq. 1)."""
    rng = np.random.default_rng(10)
    Hq, Hkv, d, S, Q = 4, 2, 16, 48, 8
    cfg = OracleConfig(n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, n_sink=4, cascade_sizes=[24, 24],
                       ema_beta=0.9, rope_base=10000.0)
    o = OracleSeq(cfg)
    q, k, v = _rand(rng, S, Hq, d), _rand(rng, S, Hkv, d), _rand(rng, S, Hkv, d)
    outs = np.concatenate([o.chunk(q[s:s + Q], k[s:s + Q], v[s:s + Q]) for s in range(0, S, Q)])
    assert len(o.discard_log(0)) == 0
    pos = np.arange(S)
    causal = pos[:, None] >= pos[None, :]
    for h in range(Hq):
        g = h // (Hq // Hkv)
        ref, _ = dense_attention(q[:, h].astype(np.float64), pos, k[:, g].astype(np.float64), pos,
                                 v[:, g].astype(np.float64), causal, 10000.0, d ** -0.5)
        np.testing.assert_allclose(outs[:, h], ref, rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("Q", [1, 5])
def test_one_cascade_equals_streaming_llm(oracle_mod, Q):
    """One cascade that accepts everything = sink cache (Section 3.1): each chunk attends to the
    first alpha tokens plus the last |C| tokens before the chunk (Eq. 3), with PE = cache index,
    plus its own causal part (Fig. 4)."""
    rng = np.random.default_rng(11)
    H, d, S, alpha, C = 2, 8, 60, 3, 9
    cfg = OracleConfig(n_q_heads=H, n_kv_heads=H, head_dim=d, n_sink=alpha, cascade_sizes=[C],
                       ema_beta=0.5, rope_base=100.0)
    o = OracleSeq(cfg)
    q, k, v = _rand(rng, S, H, d), _rand(rng, S, H, d), _rand(rng, S, H, d)
    for s in range(0, S, Q):
        out = o.chunk(q[s:s + Q], k[s:s + Q], v[s:s + Q])
        cached = list(range(min(s, alpha))) + list(range(max(alpha, s - C), s))
        members = np.array(cached + list(range(s, s + Q)))
        n = len(cached)
        kpos = np.arange(len(members))
        vis = np.concatenate([np.ones((Q, n), bool), np.tril(np.ones((Q, Q), bool))], axis=1)
        for h in range(H):
            ref, _ = dense_attention(q[s:s + Q, h].astype(np.float64), n + np.arange(Q),
                                     k[members, h].astype(np.float64), kpos,
                                     v[members, h].astype(np.float64), vis, 100.0, d ** -0.5)
            np.testing.assert_allclose(out[:, h], ref, rtol=1e-10, atol=1e-12)


def test_brute_force_over_membership_and_ema(oracle_mod):
    """Brute force: for every chunk take the membership the policy produced, build the dense
    masked attention over those tokens at PE = cache index (Eq. 2, Section 3.1), and check
    outputs, the EMA increments (Section 3.1 "Token Selection": one step per query row, so
    row i of a chunk of Q weighs beta^(Q-1-i)(1-beta), the coefficients of Alg. 3), the max
    reduction over the query heads of a group (Appendix "Head Policy"), and the updated scores."""
    rng = np.random.default_rng(12)
    Hq, Hkv, d, S, Q, beta, base = 4, 2, 8, 96, 6, 0.8, 50.0
    G = Hq // Hkv
    cfg = OracleConfig(n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, n_sink=2, cascade_sizes=[4, 4, 4],
                       ema_beta=beta, rope_base=base)
    o = OracleSeq(cfg)
    q, k, v = _rand(rng, S, Hq, d), _rand(rng, S, Hkv, d), _rand(rng, S, Hkv, d)
    w = beta ** (Q - 1 - np.arange(Q)) * (1 - beta)
    for s in range(0, S, Q):
        before = [o.state(g) for g in range(Hkv)]
        out = o.chunk(q[s:s + Q], k[s:s + Q], v[s:s + Q])
        for g in range(Hkv):
            cached = before[g].ids
            n = len(cached)
            members = np.concatenate([cached, np.arange(s, s + Q)])
            vis = np.concatenate([np.ones((Q, n), bool), np.tril(np.ones((Q, Q), bool))], axis=1)
            deltas = []
            for hh in range(G):
                h = g * G + hh
                ref, P = dense_attention(q[s:s + Q, h].astype(np.float64), n + np.arange(Q),
                                         k[members, g].astype(np.float64), np.arange(n + Q),
                                         v[members, g].astype(np.float64), vis, base, d ** -0.5)
                np.testing.assert_allclose(out[:, h], ref, rtol=1e-10, atol=1e-12)
                dh = w @ P
                # every row of P sums to one, so the increments of one head sum to 1 - beta^Q
                assert abs(dh.sum() - (1 - beta ** Q)) < 1e-12
                deltas.append(dh)
            delta = np.max(deltas, axis=0)
            np.testing.assert_allclose(o.last_delta(g), delta, rtol=1e-10, atol=1e-15)
            # scores after the chunk, for every token that is still cached
            after = o.state(g)
            mu_expect = {int(i): beta ** Q * m + dl for i, m, dl in zip(cached, before[g].mu, delta[:n])}
            mu_expect.update({s + i: delta[n + i] for i in range(Q)})
            for i, m in zip(after.ids, after.mu):
                assert abs(m - mu_expect[int(i)]) <= 1e-12 * max(1.0, abs(m)), (s, g, i)
    assert sum(len(o.discard_log(g)) for g in range(Hkv)) > 50


@pytest.mark.parametrize("reduce", [0, 1])
def test_homogeneous_heads_brute_force(oracle_mod, reduce):
    """Homogeneous heads (Appendix "Head Policy and Head Reduction"): the head axis of the
    attention is reduced to ONE score per token, so every KV head takes the same decisions and
    holds the same tokens.  Brute force as above, with the increments reduced over all query
    heads (dense attention per head against that head's own keys of the common membership)."""
    rng = np.random.default_rng(15)
    Hq, Hkv, d, S, Q, beta, base = 6, 3, 8, 72, 6, 0.8, 50.0
    G = Hq // Hkv
    cfg = OracleConfig(n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, n_sink=2, cascade_sizes=[4, 4, 4],
                       ema_beta=beta, rope_base=base, head_reduce=reduce, head_policy=1)
    o = OracleSeq(cfg)
    q, k, v = _rand(rng, S, Hq, d), _rand(rng, S, Hkv, d), _rand(rng, S, Hkv, d)
    w = beta ** (Q - 1 - np.arange(Q)) * (1 - beta)
    for s in range(0, S, Q):
        before = [o.state(g) for g in range(Hkv)]
        for g in range(1, Hkv):      # one membership, one score vector
            assert before[g].ids.tolist() == before[0].ids.tolist()
            assert before[g].mu.tolist() == before[0].mu.tolist()
        out = o.chunk(q[s:s + Q], k[s:s + Q], v[s:s + Q])
        cached = before[0].ids
        n = len(cached)
        members = np.concatenate([cached, np.arange(s, s + Q)])
        vis = np.concatenate([np.ones((Q, n), bool), np.tril(np.ones((Q, Q), bool))], axis=1)
        deltas = []
        for h in range(Hq):
            g = h // G
            ref, P = dense_attention(q[s:s + Q, h].astype(np.float64), n + np.arange(Q),
                                     k[members, g].astype(np.float64), np.arange(n + Q),
                                     v[members, g].astype(np.float64), vis, base, d ** -0.5)
            np.testing.assert_allclose(out[:, h], ref, rtol=1e-10, atol=1e-12)
            deltas.append(w @ P)
        delta = np.max(deltas, axis=0) if reduce == 0 else np.mean(deltas, axis=0)
        for g in range(Hkv):
            np.testing.assert_allclose(o.last_delta(g), delta, rtol=1e-10, atol=1e-15)
    assert len(o.discard_log(0)) > 30
    # a subset of the KV heads cannot be advanced alone under this policy
    with pytest.raises(RuntimeError):
        o.chunk(q[:Q], k[:Q], v[:Q], kv_heads=(0, 1))


def test_homogeneous_equals_independent_for_one_kv_head(oracle_mod):
    rng = np.random.default_rng(16)
    Hq, d, Q = 4, 8, 5
    q, k, v = _rand(rng, 40, Hq, d), _rand(rng, 40, 1, d), _rand(rng, 40, 1, d)
    states = []
    for policy in (0, 1):
        o = OracleSeq(OracleConfig(n_q_heads=Hq, n_kv_heads=1, head_dim=d, n_sink=1, cascade_sizes=[3, 3],
                                   ema_beta=0.7, rope_base=10.0, head_policy=policy))
        outs = [o.chunk(q[s:s + Q], k[s:s + Q], v[s:s + Q]) for s in range(0, 40, Q)]
        states.append((np.concatenate(outs), o.state(0)))
    assert np.array_equal(states[0][0], states[1][0])
    assert states[0][1].ids.tolist() == states[1][1].ids.tolist() and states[0][1].mu.tolist() == states[1][1].mu.tolist()


def _single_pass_dense(q, qpos, keys, kpos, vis, base, scale, step_of_key, T):
    """Alg. 3 written densely: while the sweep stands at step t the normaliser holds the keys of the
    steps 1..t, and what is added for a key of step t is exp(S) / (l_t + l_t * (T - t) / t)."""
    s = rope_complex(q, qpos, base) @ rope_complex(keys, kpos, base).T * scale
    e = np.where(vis, np.exp(s - np.where(vis, s, -np.inf).max(axis=1, keepdims=True)), 0.0)
    out = np.zeros_like(e)
    for t in range(1, T + 1):
        done = step_of_key <= t
        l_t = e[:, done].sum(axis=1)
        now = step_of_key == t
        out[:, now] = e[:, now] / (l_t + l_t * (T - t) / t)[:, None]
    return out


def test_single_pass_scores_brute_force(oracle_mod):
    """Alg. 3's single-pass scores (the running normaliser extrapolated by the steps still to go)
    against a dense formula, for a random assignment of keys to inner-loop steps; the outputs stay the
    exact attention.  Keys of the last step get their exact probability, a single step gives the exact
    scores throughout, and every single-pass value is at least (step / steps) times the exact one."""
    rng = np.random.default_rng(21)
    Hq, Hkv, d, Q, beta, base = 4, 2, 8, 6, 0.8, 50.0
    G = Hq // Hkv
    cfg = OracleConfig(n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, n_sink=2, cascade_sizes=[5, 5],
                       ema_beta=beta, rope_base=base)
    o = OracleSeq(cfg)
    q0, k0, v0 = _rand(rng, 30, Hq, d), _rand(rng, 30, Hkv, d), _rand(rng, 30, Hkv, d)
    for s in range(0, 30, Q):
        o.chunk(q0[s:s + Q], k0[s:s + Q], v0[s:s + Q])
    q, k, v = _rand(rng, Q, Hq, d), _rand(rng, Q, Hkv, d), _rand(rng, Q, Hkv, d)
    w = beta ** (Q - 1 - np.arange(Q)) * (1 - beta)
    for g in range(Hkv):
        st = o.state(g, with_kv=True)
        n = len(st.ids)
        T = 5
        # any schedule: the steps of the cached keys in random order, the chunk's keys in the last two steps
        step_of_key = np.concatenate([rng.integers(1, 4, size=n), np.where(np.arange(Q) < 3, 4, 5)]).astype(np.int32)
        steps_of_row = np.full((G, Q), T, dtype=np.int32)
        exact_out, exact_delta = o.eval_rows(g, q, k, v, 0, Q)
        out, delta = o.eval_rows(g, q, k, v, 0, Q, schedule=(step_of_key, steps_of_row))
        assert np.array_equal(out, exact_out)                    # the attention itself is not approximated
        keys = np.concatenate([st.k, k[:, g].astype(np.float64)])
        vis = np.concatenate([np.ones((Q, n), bool), np.tril(np.ones((Q, Q), bool))], axis=1)
        per_head, per_head_exact = [], []
        for hh in range(G):
            qq = q[:, g * G + hh].astype(np.float64)
            ph = _single_pass_dense(qq, n + np.arange(Q), keys, np.arange(n + Q), vis, base, d ** -0.5, step_of_key, T)
            _, P = dense_attention(qq, n + np.arange(Q), keys, np.arange(n + Q), np.concatenate([st.v, v[:, g].astype(np.float64)]),
                                   vis, base, d ** -0.5)
            last = step_of_key == T
            np.testing.assert_allclose(ph[:, last], P[:, last], rtol=1e-12, atol=1e-300)   # rho = 0: exact
            assert (ph >= P * (step_of_key / T)[None, :] * (1 - 1e-12)).all()
            per_head.append(w @ ph)
            per_head_exact.append(w @ P)
        np.testing.assert_allclose(delta, np.max(per_head, axis=0), rtol=1e-10, atol=1e-300)
        np.testing.assert_allclose(exact_delta, np.max(per_head_exact, axis=0), rtol=1e-10, atol=1e-300)
        assert np.abs(delta - exact_delta).max() > 1e-3           # and it is a different quantity
        # one step: nothing is extrapolated
        one = (np.ones(n + Q, dtype=np.int32), np.ones((G, Q), dtype=np.int32))
        _, delta_one = o.eval_rows(g, q, k, v, 0, Q, schedule=one)
        np.testing.assert_allclose(delta_one, exact_delta, rtol=1e-12, atol=1e-300)
    # the whole chunk with a schedule: the cached scores are updated with the single-pass increments
    g = 0
    before = o.state(g)
    n = len(before.ids)
    sched = (np.concatenate([np.full(n, 1), np.full(Q, 2)]).astype(np.int32), np.full((G, Q), 2, dtype=np.int32))
    _, d_sp = o.eval_rows(g, q, k, v, 0, Q, schedule=sched)
    o.chunk(q, k, v, kv_heads=(g, g + 1), schedule=sched)
    np.testing.assert_array_equal(o.last_delta(g), d_sp)
    after = o.state(g)
    expect = {int(i): beta ** Q * m + dl for i, m, dl in zip(before.ids, before.mu, d_sp[:n])}
    for i, m in zip(after.ids, after.mu):
        if int(i) in expect:
            assert abs(m - expect[int(i)]) <= 1e-12 * max(1.0, abs(m))


def test_mean_head_reduction(oracle_mod):
    """The mean reduction over the query heads of a group (Appendix "Head Policy")."""
    rng = np.random.default_rng(13)
    Hq, Hkv, d, Q, beta = 3, 1, 4, 5, 0.7
    cfg = OracleConfig(n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, n_sink=1, cascade_sizes=[8],
                       ema_beta=beta, rope_base=10.0, head_reduce=1)
    o = OracleSeq(cfg)
    q, k, v = _rand(rng, Q, Hq, d), _rand(rng, Q, Hkv, d), _rand(rng, Q, Hkv, d)
    o.chunk(q, k, v)
    w = beta ** (Q - 1 - np.arange(Q)) * (1 - beta)
    vis = np.tril(np.ones((Q, Q), bool))
    deltas = [w @ dense_attention(q[:, h].astype(np.float64), np.arange(Q), k[:, 0].astype(np.float64),
                                  np.arange(Q), v[:, 0].astype(np.float64), vis, 10.0, 0.5)[1] for h in range(Hq)]
    np.testing.assert_allclose(o.last_delta(0), np.mean(deltas, axis=0), rtol=1e-10)


def test_decode_step_is_single_row_ema(oracle_mod):
    """A decode step (Eq. 2) is a chunk of one: mu <- gamma*mu + (1-gamma)*s (Section 3.1)."""
    rng = np.random.default_rng(14)
    H, d, beta = 1, 4, 0.6
    cfg = OracleConfig(n_q_heads=H, n_kv_heads=H, head_dim=d, n_sink=1, cascade_sizes=[16],
                       ema_beta=beta, rope_base=10.0)
    o = OracleSeq(cfg)
    mu = {}
    ks, vs = [], []
    for t in range(10):
        q, k, v = _rand(rng, H, d), _rand(rng, H, d), _rand(rng, H, d)
        ks.append(k[0]); vs.append(v[0])
        out = o.decode(q, k, v)
        K, V = np.array(ks, dtype=np.float64), np.array(vs, dtype=np.float64)
        ref, P = dense_attention(q.astype(np.float64), np.array([t]), K, np.arange(t + 1), V,
                                 np.ones((1, t + 1), bool), 10.0, 0.5)
        np.testing.assert_allclose(out, ref, rtol=1e-10, atol=1e-12)
        for j in range(t + 1):
            mu[j] = beta * mu.get(j, 0.0) + (1 - beta) * P[0, j]
        st = o.state(0)
        np.testing.assert_allclose(st.mu, [mu[int(i)] for i in st.ids], rtol=1e-12)


def test_rope_relative_shift(oracle_mod):
    """RoPE scores depend on position differences only: adding sink tokens in front that get
    (numerically) no attention shifts every index and must leave the outputs unchanged."""
    rng = np.random.default_rng(15)
    H, d, S = 1, 8, 12
    q, k, v = _rand(rng, S, H, d), _rand(rng, S, H, d), _rand(rng, S, H, d)
    base = OracleConfig(n_q_heads=H, n_kv_heads=H, head_dim=d, n_sink=0, cascade_sizes=[64],
                        ema_beta=0.9, rope_base=1000.0)
    o1 = OracleSeq(base)
    ref = o1.chunk(q, k, v)
    # the same stream behind 5 leading tokens with zero keys (logit 0) and zero values: the
    # real tokens keep their mutual logits, and the mass the zero keys take is known densely.
    o2 = OracleSeq(base)
    lead = 5
    zk = np.zeros((lead, H, d), np.float32)
    o2.chunk(_rand(rng, lead, H, d), zk, zk)
    out = o2.chunk(q, k, v)
    pos = np.arange(S)
    _, P = dense_attention(q[:, 0].astype(np.float64), lead + pos,
                           np.concatenate([zk[:, 0], k[:, 0]]).astype(np.float64), np.arange(lead + S),
                           np.concatenate([zk[:, 0], v[:, 0]]).astype(np.float64),
                           np.concatenate([np.ones((S, lead), bool), np.tril(np.ones((S, S), bool))], axis=1),
                           1000.0, d ** -0.5)
    keep = P[:, lead:].sum(axis=1, keepdims=True)     # mass left on the real tokens
    np.testing.assert_allclose(out[:, 0], ref[:, 0] * keep, rtol=1e-9, atol=1e-12)


def test_row_range_evaluation_matches_whole_chunk(oracle_mod):
    """oracle.eval_rows over all rows reproduces the chunk's outputs and increments; over a tail
    of rows it gives the dense formula restricted to those rows (weights beta^(Q-1-i)(1-beta))."""
    rng = np.random.default_rng(16)
    Hq, Hkv, d, Q, beta, base = 4, 2, 8, 12, 0.7, 100.0
    cfg = OracleConfig(n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, n_sink=2, cascade_sizes=[5, 5],
                       ema_beta=beta, rope_base=base)
    o = OracleSeq(cfg)
    for _ in range(3):
        o.chunk(_rand(rng, Q, Hq, d), _rand(rng, Q, Hkv, d), _rand(rng, Q, Hkv, d))
    q, k, v = _rand(rng, Q, Hq, d), _rand(rng, Q, Hkv, d), _rand(rng, Q, Hkv, d)
    g = 1
    before = o.state(g, with_kv=True)
    full_out, full_delta = o.eval_rows(g, q, k, v, 0, Q)
    tail_out, tail_delta = o.eval_rows(g, q, k, v, Q - 4, Q)
    assert o.state(g).ids.tolist() == before.ids.tolist()          # the cache is untouched
    n = len(before.ids)
    keys = np.concatenate([before.k, k[:, g].astype(np.float64)])
    vals = np.concatenate([before.v, v[:, g].astype(np.float64)])
    vis = np.concatenate([np.ones((Q, n), bool), np.tril(np.ones((Q, Q), bool))], axis=1)
    w = beta ** (Q - 1 - np.arange(Q)) * (1 - beta)
    d_full, d_tail = [], []
    for hh in range(Hq // Hkv):
        h = g * (Hq // Hkv) + hh
        ref, P = dense_attention(q[:, h].astype(np.float64), n + np.arange(Q), keys, np.arange(n + Q), vals, vis,
                                 base, d ** -0.5)
        np.testing.assert_allclose(full_out[:, h], ref, rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(tail_out[Q - 4:, h], ref[Q - 4:], rtol=1e-10, atol=1e-12)
        d_full.append(w @ P)
        d_tail.append(w[Q - 4:] @ P[Q - 4:])
    np.testing.assert_allclose(full_delta, np.max(d_full, axis=0), rtol=1e-10, atol=1e-15)
    np.testing.assert_allclose(tail_delta, np.max(d_tail, axis=0), rtol=1e-10, atol=1e-15)
    out = o.chunk(q, k, v, kv_heads=(g, g + 1))
    np.testing.assert_array_equal(out[:, 2:], full_out[:, 2:])
    np.testing.assert_array_equal(o.last_delta(g), full_delta)
