"""Pins of the oracle's cache policy (Alg. 2) against what the paper and arithmetic fix.

None of these retypes the oracle's code: they use hand-worked traces, the
sliding-window special case, counting arguments and the span formula of Eq. 4.
"""
import os

import numpy as np
import pytest

from oracle import OracleConfig, OracleSeq

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "alg2_hand_traces.txt")


def _policy_only(n_sink, sizes, periods=None, token_selection=1):
    return OracleSeq(OracleConfig(n_q_heads=1, n_kv_heads=1, head_dim=2, n_sink=n_sink, cascade_sizes=sizes,
                                  ema_beta=0.9, rope_base=10000.0, accept_period=periods,
                                  token_selection=token_selection))


def _traces():
    out = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = [p.strip() for p in line.split(";")]
            ints = lambda s: [int(x) for x in s.split(",") if x != ""]
            out.append((int(parts[0]), ints(parts[1]), ints(parts[2]),
                        [float(x) for x in parts[3].split(",")], ints(parts[4]), ints(parts[5])))
    return out


@pytest.mark.parametrize("trace", _traces())
def test_alg2_hand_trace(oracle_mod, trace):
    """Alg. 2, traced by hand (tests/golden/alg2_hand_traces.txt)."""
    n_sink, sizes, periods, scores, final, discards = trace
    o = _policy_only(n_sink, sizes, periods)
    for s in scores:
        o.insert_scored(0, s)
    st = o.state(0)
    assert st.ids.tolist() == final
    assert o.discard_log(0).tolist() == discards
    # Section 3.1 "Positional Encoding": index inside the cache
    assert st.pos.tolist() == list(range(len(final)))


def test_select_log_of_the_hand_traces(oracle_mod):
    """The record of token-selection comparisons (which pair, which scores, in which order)
    against the same two hand traces (tests/golden/alg2_select_log.txt)."""
    expect = {}
    with open(os.path.join(os.path.dirname(GOLDEN), "alg2_select_log.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = [p.strip() for p in line.split(";")]
            pairs = [[int(x) for x in p.split(">")] for p in parts[1].split(",")]
            mus = [[float(x) for x in p.split(",")] for p in parts[2:]]
            expect[parts[0]] = (pairs, mus)
    for name, trace in zip("AB", _traces()):
        n_sink, sizes, periods, scores, _, _ = trace
        o = _policy_only(n_sink, sizes, periods)
        for s in scores:
            o.insert_scored(0, s)
        ids, mu = o.select_log(0)
        assert ids.tolist() == expect[name][0]
        assert mu.tolist() == expect[name][1]
        o.clear_logs(0)
        assert len(o.select_log(0)[0]) == 0 and len(o.discard_log(0)) == 0


def test_one_cascade_is_sink_plus_sliding_window(oracle_mod):
    """Section 3.1: with one cascade that accepts everything the cache is StreamingLLM's
    (Eq. 3 plus the sink rule): the first alpha tokens and the most recent |C| tokens."""
    rng = np.random.default_rng(0)
    o = _policy_only(3, [7])
    for t in range(60):
        o.insert_scored(0, rng.random())
        ids = o.state(0).ids.tolist()
        n = t + 1
        expect = list(range(min(n, 3))) + list(range(max(3, n - 7), n))
        assert ids == expect, (t, ids, expect)


def test_first_discard_position(oracle_mod):
    """With 4 sinks and 4 cascades of 64 the first token is lost while inserting token 133:
    cascade 1 fills with tokens 4..67, its evictions fill cascade 2 eagerly until t=127, the
    eviction at t=128 is accepted (and passed on), the one at t=129 meets a full cascade 2
    at a non-accepting step (Alg. 2, token-selection branch)."""
    o = _policy_only(4, [64] * 4)
    rng = np.random.default_rng(1)
    for tok in range(133):
        o.insert_scored(0, rng.random())
        assert len(o.discard_log(0)) == 0, tok
    assert o.count(0) == 133
    o.insert_scored(0, rng.random())
    assert len(o.discard_log(0)) == 1
    assert o.count(0) == 133


def test_invariants_random_scores(oracle_mod):
    """Structure that holds for any scores: ids increase along the cache order, cascade 1 is
    exactly the last |C_1| tokens, every token is either cached or discarded exactly once,
    and cascade i (sizes even, periods 2^(i-1)) holds one token from each of a run of
    consecutive aligned blocks of 2^(i-1) tokens (the acceptance schedule of Section 3.1)."""
    n_sink, sizes = 4, [16, 16, 16, 16]
    o = _policy_only(n_sink, sizes)
    rng = np.random.default_rng(2)
    T = 1500
    for tok in range(T):
        o.insert_scored(0, rng.random())
    st = o.state(0)
    ids = st.ids
    assert np.all(np.diff(ids) > 0)
    assert ids[st.cascade_of == 1].tolist() == list(range(T - 16, T))
    assert ids[st.cascade_of == 0].tolist() == [0, 1, 2, 3]
    lost = o.discard_log(0)
    assert len(set(lost.tolist())) == len(lost)
    assert sorted(lost.tolist() + ids.tolist()) == list(range(T))
    for c in (2, 3, 4):
        blocks = (ids[st.cascade_of == c] - n_sink) >> (c - 1)
        assert np.all(np.diff(blocks) == 1), (c, blocks)
    # all cascades are full by now
    assert st.counts.tolist() == [4, 16, 16, 16, 16]


def test_acceptance_rates_and_span(oracle_mod):
    """Cascade 2 takes every 2nd, cascade 3 every 4th iteration (Section 3.1), so the age of
    the oldest token of cascade i approaches the partial sums of Eq. 4, sum_j 2^(j-1)|C_j|."""
    n_sink, size, N = 2, 32, 4
    o = _policy_only(n_sink, [size] * N, token_selection=0)
    T = 4000
    for tok in range(T):
        o.insert_scored(0, 0.0)
    st = o.state(0)
    partial = 0
    for c in range(1, N + 1):
        partial += size << (c - 1)
        oldest_age = T - int(st.ids[st.cascade_of == c][0])
        assert partial - (1 << (c - 1)) <= oldest_age <= partial, (c, oldest_age, partial)
    # accepted[c] counts arrivals at accepting steps: all T - n_sink for cascade 1
    t_total = T - n_sink
    assert st.stats[0, 0] == t_total
    # cascade 2 is offered a token on every step after cascade 1 is full and accepts on even t
    offered2 = t_total - size
    assert abs(int(st.stats[1, 0]) - offered2 // 2) <= 1
    # Eq. 4 for 8 cascades: window sparsity 1 - |C|/S~ = 1 - 8/255 > 96 %
    span8 = sum(size << i for i in range(8))
    assert 1.0 - (8 * size) / span8 > 0.96


def test_selection_off_never_swaps(oracle_mod):
    """The ablation without token selection always drops the incoming token (Section 4.7)."""
    o = _policy_only(1, [4, 4], token_selection=0)
    rng = np.random.default_rng(3)
    for tok in range(200):
        o.insert_scored(0, rng.random())
    st = o.state(0)
    assert st.stats[:, 1].sum() == 0
    # cascade 2 then holds the tokens that arrived at even t, i.e. every other eviction
    c2 = st.ids[st.cascade_of == 2]
    assert np.all(np.diff(c2) == 2)


def test_selection_keeps_higher_score(oracle_mod):
    """Two cascades of one slot, no sinks: token j leaves cascade 1 at t = j + 1 and cascade 2
    accepts at even t, so odd tokens are accepted and the even token after each is a challenger
    that only wins with a strictly higher score (Alg. 2, token-selection branch)."""
    rng = np.random.default_rng(4)
    for n_tokens in range(4, 40):
        scores = rng.integers(0, 4, size=n_tokens).astype(float)   # many ties
        o = _policy_only(0, [1, 1])
        for s in scores:
            o.insert_scored(0, s)
        st = o.state(0)
        held = int(st.ids[st.cascade_of == 2][0])
        last_evicted = n_tokens - 2            # the newest token sits in cascade 1
        if last_evicted % 2 == 1:              # accepted unconditionally at even t
            assert held == last_evicted
        else:                                  # challenger of the token accepted just before
            a = last_evicted - 1
            assert held == (last_evicted if scores[last_evicted] > scores[a] else a)


def test_set_state_roundtrip_and_pe_example(oracle_mod):
    """Section 3.1 example: a cache holding original indices [0,1,3,5,7,8] gets PE [0..5]."""
    o = _policy_only(2, [2, 2])
    ids = np.array([0, 1, 3, 5, 7, 8])
    k = np.zeros((6, 2), dtype=np.float32)
    o.set_state(0, ids, np.linspace(0.1, 0.6, 6), [2, 2, 2], k, k, t=7, n_seen=9)
    st = o.state(0)
    assert st.ids.tolist() == [0, 1, 3, 5, 7, 8]
    assert st.cascade_of.tolist() == [0, 0, 2, 2, 1, 1]
    assert st.pos.tolist() == [0, 1, 2, 3, 4, 5]
    assert st.t == 7 and st.n_seen == 9
