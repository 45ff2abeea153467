"""CPU tests of the parity machinery itself: the bf16 rounding model against the oracle, the
checker of cached K / V rows against a planted wrong row, and the classification of selection
comparisons that come out differently on two score vectors."""
import types

import numpy as np
import pytest

from bf16_model import chunk_reference, to_bf16
from oracle import OracleConfig, OracleSeq


def _bf16_rand(rng, *shape):
    return to_bf16(rng.standard_normal(shape).astype(np.float32))


@pytest.mark.parametrize("d,G", [(64, 2), (128, 4)])
def test_rounding_model_is_the_oracle_without_roundings(oracle_mod, d, G):
    """With both roundings off the model is softmax attention at cache-index positions and the EMA
    increments of Section 3.1: it must agree with the oracle to fp32 rotation accuracy, whatever
    anchors the cached keys are rotated to (only angle differences enter); with the roundings on it
    stays within the bf16 tolerance of the oracle and differs from it by more than fp32 noise."""
    rng = np.random.default_rng(3)
    n0, Q, beta, base = 70, 24, 0.9, 10000.0
    cfg = OracleConfig(n_q_heads=G, n_kv_heads=1, head_dim=d, n_sink=4, cascade_sizes=[40, 40],
                       ema_beta=beta, rope_base=base)
    o = OracleSeq(cfg)
    o.chunk(_bf16_rand(rng, n0, G, d), _bf16_rand(rng, n0, 1, d), _bf16_rand(rng, n0, 1, d))
    st = o.state(0, with_kv=True)
    n = len(st.ids)
    q, k, v = _bf16_rand(rng, Q, G, d), _bf16_rand(rng, Q, 1, d), _bf16_rand(rng, Q, 1, d)
    ref, delta_ref = o.eval_rows(0, q, k, v, 0, Q)
    rows = np.arange(Q)
    slot = rng.permutation(200)[:n]          # anchors unrelated to the cache index
    kc, vc = st.k.astype(np.float32), st.v.astype(np.float32)
    out, delta = chunk_reference(q, k[:, 0], v[:, 0], kc, vc, slot, rows, base, round_operands=False,
                                 round_probabilities=False, ema_beta=beta)
    err = np.linalg.norm(out - ref, axis=-1) / np.linalg.norm(ref, axis=-1)
    assert err.max() < 2e-5, err.max()
    np.testing.assert_allclose(delta.max(axis=0), delta_ref, rtol=2e-4, atol=1e-12)
    out_r, delta_r = chunk_reference(q, k[:, 0], v[:, 0], kc, vc, slot, rows, base, ema_beta=beta)
    err_r = np.linalg.norm(out_r - ref, axis=-1) / np.linalg.norm(ref, axis=-1)
    assert 1e-4 < err_r.max() < 2e-2, err_r.max()
    rel = np.abs(delta_r.max(axis=0) - delta_ref) / np.maximum(delta_ref, 1e-12)
    assert 1e-4 < rel[delta_ref > 1e-9].max() < 6e-2
    o.close()


def _fake_state(ids, k, v):
    n = len(ids)
    return types.SimpleNamespace(count=n, ids=ids[None, None].astype(np.int32), k=k[None, None], v=v[None, None])


def test_row_checker_catches_one_wrong_row():
    """The checker compares every cached K / V row with the row that was fed for the same token:
    a state whose ids are right but one of whose rows is another token's must fail, as must a
    single flipped mantissa bit."""
    from gpu_harness import FedRows, check_cached_rows
    rng = np.random.default_rng(5)
    fed = FedRows()
    k0, v0 = _bf16_rand(rng, 1, 40, 1, 16), _bf16_rand(rng, 1, 40, 1, 16)
    k1, v1 = _bf16_rand(rng, 1, 25, 1, 16), _bf16_rand(rng, 1, 25, 1, 16)
    fed.add(0, k0, v0)
    fed.add(40, k1, v1)
    ids = np.array([0, 1, 7, 12, 39, 40, 41, 64])
    allk, allv = np.concatenate([k0, k1], axis=1)[0, :, 0], np.concatenate([v0, v1], axis=1)[0, :, 0]
    good = _fake_state(ids, allk[ids].copy(), allv[ids].copy())
    check_cached_rows(good, 0, 0, fed)
    bad = _fake_state(ids, allk[ids].copy(), allv[ids].copy())
    bad.k[0, 0, 3] = allk[13]                  # the right id with the neighbouring token's key
    with pytest.raises(AssertionError, match="cached K rows differ"):
        check_cached_rows(bad, 0, 0, fed)
    bad = _fake_state(ids, allk[ids].copy(), allv[ids].copy())
    bad.v[0, 0, 6].view(np.uint32)[5] ^= 1 << 16   # one bf16 mantissa bit of one element
    with pytest.raises(AssertionError, match="cached V rows differ"):
        check_cached_rows(bad, 0, 0, fed)
    # rows of an initial state and of a stream that is drawn again on demand
    fed2 = FedRows()
    init_ids = np.array([3, 5, 100, 101])
    fed2.add_initial(init_ids, {(0, 0): allk[:4]}, {(0, 0): allv[:4]})
    fed2.regenerate_with(lambda c: (k1[:, :5] + c, v1[:, :5] + c), 5)
    kk, vv = fed2.rows(0, 0, np.array([100, 3, 7, 21]))
    assert np.array_equal(kk[0], allk[2]) and np.array_equal(kk[1], allk[0])
    assert np.array_equal(kk[2], k1[0, 2, 0] + 1) and np.array_equal(vv[3], v1[0, 1, 0] + 4)


def test_flip_classification():
    """Same participants, different outcome: noise-level only if the oracle's own scores are within
    tau of each other; other participants: downstream of an earlier flip."""
    from gpu_harness import classify_flips
    ids = np.array([[5, 4], [7, 6], [9, 8], [11, 10]])
    ref = (ids, np.array([[0.500, 0.501], [0.3, 0.9], [0.20, 0.10], [0.4, 0.4]]))
    same = (ids, np.array([[0.499, 0.502], [0.31, 0.88], [0.21, 0.11], [0.4, 0.4]]))
    assert classify_flips(ref, same, 1, 2.0 ** -6) == (0, 0, 0)
    close = (ids, np.array([[0.502, 0.501], [0.3, 0.9], [0.20, 0.10], [0.4, 0.4]]))      # 5 beats 4 by a hair
    assert classify_flips(ref, close, 1, 2.0 ** -6) == (1, 0, 0)
    wide = (ids, np.array([[0.500, 0.501], [0.3, 0.9], [0.05, 0.10], [0.4, 0.4]]))       # 9 loses against 8: gap 0.1
    assert classify_flips(ref, wide, 1, 2.0 ** -6) == (0, 1, 0)
    other = (np.array([[5, 4], [7, 5], [9, 8], [11, 10]]), ref[1])                       # after 5 replaced 4
    assert classify_flips(ref, other, 1, 2.0 ** -6) == (0, 0, 1)
    assert classify_flips(ref, wide, 0, 2.0 ** -6) == (0, 0, 0)                          # nothing is ever replaced


@pytest.mark.parametrize("seed", range(6))
def test_visiting_schedule_covers_every_key_once(seed):
    """The visiting schedule handed to the single-pass oracle, built from the documented layout on the
    structure the library's host replay reports: tiles of at most 64 keys, numbered without gaps,
    the keys of one tile contiguous in physical order, the chunk's tiles after the cache's."""
    from gpu_harness import visiting_schedule
    from paper_2406_17808_amd import binding as B
    rng = np.random.default_rng(300 + seed)
    N = int(rng.integers(1, 5))
    sizes = [int(rng.integers(1, 6)) * 50 for _ in range(N)]
    cfg = B.make_config(batch=1, n_q_heads=4, n_kv_heads=2, head_dim=64, dtype=B.CASCADE_BF16, n_sink=int(rng.integers(0, 70)),
                        cascade_sizes=sizes, ema_beta=0.9, rope_base=10000.0, max_chunk=512)
    chunks = [int(x) for x in rng.integers(1, 400, size=int(rng.integers(1, 12)))]
    st = B.cascade_simulate_structure(cfg, chunks)
    st.slot = st.slot[None, None]
    Q = 512
    step_of_key, steps_of_row = visiting_schedule(cfg, st, Q)
    n = st.count
    assert step_of_key.shape == (n + Q,) and steps_of_row.shape == (2, Q)
    cache_tiles = int(step_of_key[:n].max()) if n else 0
    assert sorted(set(step_of_key[:n].tolist())) == list(range(1, cache_tiles + 1))
    slot = st.slot[0, 0, :n]
    for t in range(1, cache_tiles + 1):
        members = np.sort(slot[step_of_key[:n] == t])
        assert 1 <= len(members) <= 64 and members[-1] - members[0] == len(members) - 1      # one run of physical slots
    assert step_of_key[n:].tolist() == [cache_tiles + j // 64 + 1 for j in range(Q)]
    assert steps_of_row[0, 0] == cache_tiles + 4 and steps_of_row[1, 511] == cache_tiles + 8
