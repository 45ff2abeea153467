"""CPU-only tests of the C-ABI library: it loads, exports what the header declares, rejects bad
arguments before touching a device, and its host-side structure logic agrees with Alg. 2."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import OracleConfig, OracleSeq
from paper_2406_17808_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.library_path()):
        from paper_2406_17808_amd.build import build_library
        build_library()
    return B.load_library()


def _cfg(**kw):
    base = dict(batch=1, n_q_heads=4, n_kv_heads=2, head_dim=64, dtype=B.CASCADE_F32, n_sink=4,
                cascade_sizes=[8, 8, 8], ema_beta=0.9, rope_base=10000.0, max_chunk=16)
    base.update(kw)
    return B.make_config(**base)


def test_library_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "cascade_kv.h")).read()
    declared = set(re.findall(r"\b(cascade_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTED_SYMBOLS)
    for name in declared:
        assert hasattr(lib, name), name


def test_struct_layouts_match_header(lib):
    # sizes follow from the field lists of include/cascade_kv.h
    assert ctypes.sizeof(B.cascade_config) == 7 * 4 + 16 * 4 * 2 + 3 * 4 + 3 * 4 + 4 + 4 + 2 * 4
    assert ctypes.sizeof(B.cascade_init_state) == 4 * 8 + 17 * 4 + 4 + 2 * 8
    assert ctypes.sizeof(B.cascade_state_view) == 9 * 8 + 17 * 4 + 16 * 4 + 4 + 2 * 16 * 8 + 2 * 8 + 4 * 4
    assert ctypes.sizeof(B.cascade_ceilings) == 2 * 4 + 8 * 8


@pytest.mark.parametrize("kw,code", [
    (dict(batch=0), B.CASCADE_E_INVALID_CONFIG),
    (dict(n_q_heads=3), B.CASCADE_E_INVALID_CONFIG),
    (dict(head_dim=63), B.CASCADE_E_INVALID_CONFIG),
    (dict(cascade_sizes=[]), B.CASCADE_E_INVALID_CONFIG),
    (dict(cascade_sizes=[4, 0]), B.CASCADE_E_INVALID_CONFIG),
    (dict(accept_period=[2, 4, 8]), B.CASCADE_E_INVALID_CONFIG),
    (dict(ema_beta=1.0), B.CASCADE_E_INVALID_CONFIG),
    (dict(max_chunk=0), B.CASCADE_E_INVALID_CONFIG),
    (dict(head_reduce=7), B.CASCADE_E_INVALID_CONFIG),
    (dict(dtype=B.CASCADE_BF16, head_dim=96), B.CASCADE_E_UNSUPPORTED),
    (dict(head_dim=512), B.CASCADE_E_UNSUPPORTED),
])
def test_invalid_configs_are_rejected_on_the_host(lib, kw, code):
    cfg = _cfg(**kw)
    assert B.cascade_workspace_bytes(cfg) == 0
    with pytest.raises(B.CascadeError) as e:
        B.cascade_init(cfg, 256, 1 << 30)
    assert e.value.code == code
    assert len(str(e.value)) > 20


def test_init_argument_errors(lib):
    cfg = _cfg()
    need = B.cascade_workspace_bytes(cfg)
    assert need > 0
    with pytest.raises(B.CascadeError) as e:
        B.cascade_init(cfg, 0, need)
    assert e.value.code == B.CASCADE_E_NULL_ARG
    with pytest.raises(B.CascadeError) as e:
        B.cascade_init(cfg, 4096, need - 1)
    assert e.value.code == B.CASCADE_E_WORKSPACE_TOO_SMALL
    with pytest.raises(B.CascadeError) as e:
        B.cascade_init(cfg, 4096 + 8, need)
    assert e.value.code == B.CASCADE_E_BAD_ARG
    st = B.cascade_init_state()
    st.counts[0] = 5          # more sinks than n_sink
    with pytest.raises(B.CascadeError) as e:
        B.cascade_init(cfg, 4096, need, st)
    assert e.value.code == B.CASCADE_E_BAD_ARG
    assert lib.cascade_prefill_chunk(None, 1, 1, 1, 1, 1, None) == B.CASCADE_E_NULL_ARG
    assert lib.cascade_decode_step(None, 1, 1, 1, 1, None) == B.CASCADE_E_NULL_ARG
    assert lib.cascade_read_state(None, None, None) == B.CASCADE_E_NULL_ARG


def test_layers_share_one_scratch(lib):
    """n layers need n states and one scratch: the size is affine in n, one layer is the plain
    workspace, and a large cache costs little more than its three row arrays per extra layer."""
    cfg = _cfg()
    one = B.cascade_workspace_bytes(cfg)
    sizes = [B.cascade_layers_workspace_bytes(cfg, n) for n in (1, 2, 3, 7)]
    assert sizes[0] == one
    state = sizes[1] - sizes[0]
    assert 0 < state < one
    assert sizes[2] == one + 2 * state and sizes[3] == one + 6 * state
    assert B.cascade_layers_workspace_bytes(cfg, 0) == 0
    assert B.cascade_layers_workspace_bytes(_cfg(batch=0), 2) == 0
    huge = _cfg(dtype=B.CASCADE_BF16, head_dim=128, n_q_heads=32, n_kv_heads=8, n_sink=64,
                cascade_sizes=[16384] * 4, max_chunk=1)
    rows = 8 * 65600 * 128 * 2
    per_layer = B.cascade_layers_workspace_bytes(huge, 5) - B.cascade_layers_workspace_bytes(huge, 4)
    assert 3 * rows < per_layer < 3.1 * rows
    # argument errors
    with pytest.raises(B.CascadeError) as e:
        B.cascade_init_layers(cfg, 0, 4096, 1 << 30)
    assert e.value.code == B.CASCADE_E_BAD_ARG
    with pytest.raises(B.CascadeError) as e:
        B.cascade_init_layers(cfg, 2, 4096, sizes[1] - 1)
    assert e.value.code == B.CASCADE_E_WORKSPACE_TOO_SMALL
    with pytest.raises(B.CascadeError) as e:
        B.cascade_init_layers(cfg, 2, 0, sizes[1])
    assert e.value.code == B.CASCADE_E_NULL_ARG
    with pytest.raises(B.CascadeError) as e:
        B.cascade_init_layers(_cfg(ema_beta=1.0), 2, 4096, 1 << 30)
    assert e.value.code == B.CASCADE_E_INVALID_CONFIG


def test_workspace_grows_with_the_cache(lib):
    small = B.cascade_workspace_bytes(_cfg())
    big = B.cascade_workspace_bytes(_cfg(cascade_sizes=[64, 64, 64]))
    assert big > small
    # five row arrays (K, rotated K, V, and the per-chunk packed copies of rotated K and V of the
    # bf16 MFMA path) dominate a large cache; the two layouts of the rotation table (2 x slots rows of
    # d/2 (cos, sin) pairs each) come to one more
    huge = _cfg(dtype=B.CASCADE_BF16, head_dim=128, n_q_heads=32, n_kv_heads=8, n_sink=64,
                cascade_sizes=[16384] * 4, max_chunk=1)
    rows = 8 * 65600 * 128 * 2
    assert 5 * rows < B.cascade_workspace_bytes(huge) < 7 * rows


@pytest.mark.parametrize("seed", range(6))
def test_structure_matches_alg2(lib, oracle_mod, seed):
    """Fill, acceptance counters and discards computed by the host for whole chunks equal those of
    the oracle inserting the same tokens one at a time (Alg. 2)."""
    rng = np.random.default_rng(100 + seed)
    N = int(rng.integers(1, 6))
    sizes = [int(x) for x in rng.integers(1, 12, size=N)]
    n_sink = int(rng.integers(0, 5))
    periods = None
    if seed % 2:
        periods = [1] + [int(x) for x in rng.integers(1, 7, size=N - 1)]
    chunks = [int(x) for x in rng.integers(1, 40, size=30)]
    cfg = _cfg(n_sink=n_sink, cascade_sizes=sizes, accept_period=periods, max_chunk=64)
    o = OracleSeq(OracleConfig(1, 1, 2, n_sink, sizes, 0.9, 10000.0, accept_period=periods))
    for upto in range(1, len(chunks) + 1):
        for _ in range(chunks[upto - 1]):
            o.insert_scored(0, rng.random())
        st = o.state(0)
        sim = B.cascade_simulate_structure(cfg, chunks[:upto])
        assert sim.counts.tolist() == st.counts.tolist()
        assert sim.t == st.t and sim.n_seen == st.n_seen
        assert sim.accepted.tolist() == st.stats[:, 0].tolist()
        assert sim.discards.tolist() == st.stats[:, 2].tolist()
        # the slot map is a bijection onto distinct slots inside the right regions
        slot = sim.slot[:sim.count]
        assert len(set(slot.tolist())) == sim.count
        assert slot[:sim.counts[0]].tolist() == list(range(sim.counts[0]))


def test_ring_heads_follow_the_circular_buffer_rule(lib):
    """xi advances by one per eviction, modulo the cascade size (Section 3.1 "Circular Buffers")."""
    cfg = _cfg(n_sink=2, cascade_sizes=[5, 3], max_chunk=64)
    for total in range(1, 60):
        sim = B.cascade_simulate_structure(cfg, [1] * total)
        offered1 = max(0, total - 2)
        pushes1 = max(0, offered1 - 5)
        assert sim.xi[0] == pushes1 % 5
        # cascade 2 is offered one item per push of cascade 1, fills eagerly, then pushes at even t
        one_by_one = B.cascade_simulate_structure(cfg, [total])
        assert one_by_one.xi.tolist() == sim.xi.tolist()
        assert one_by_one.counts.tolist() == sim.counts.tolist()


@pytest.mark.parametrize("seed", range(12))
def test_chunked_update_equals_token_by_token_alg2(lib, oracle_mod, seed):
    """The chunk-at-a-time update (segments, winners, evictions; the routines the device kernels
    run) yields the membership, scores and swap counts of Alg. 2 applied one token at a time."""
    rng = np.random.default_rng(200 + seed)
    N = int(rng.integers(1, 6))
    sizes = [int(x) for x in rng.integers(1, 10, size=N)]
    n_sink = int(rng.integers(0, 4))
    periods = None
    if seed % 3 == 1:
        periods = [1] + [int(x) for x in rng.integers(1, 6, size=N - 1)]
    sel = 0 if seed % 4 == 3 else 1
    chunks = [int(x) for x in rng.integers(1, 50, size=25)]
    total = sum(chunks)
    # few distinct values: many ties, which must keep the resident item
    scores = (rng.integers(0, 6, size=total) / 8.0).astype(np.float32)
    cfg = _cfg(n_sink=n_sink, cascade_sizes=sizes, accept_period=periods, max_chunk=64, token_selection=sel)
    o = OracleSeq(OracleConfig(1, 1, 2, n_sink, sizes, 0.9, 10000.0, accept_period=periods, token_selection=sel))
    done = 0
    for upto in range(1, len(chunks) + 1):
        for s in scores[done:done + chunks[upto - 1]]:
            o.insert_scored(0, float(s))
        done += chunks[upto - 1]
        st = o.state(0)
        sim = B.cascade_simulate_structure(cfg, chunks[:upto], scores[:done])
        assert sim.ids[:sim.count].tolist() == st.ids.tolist(), (seed, upto)
        np.testing.assert_array_equal(sim.mu[:sim.count], st.mu.astype(np.float32))
        assert sim.swaps.tolist() == st.stats[:, 1].tolist()


@pytest.mark.parametrize("seed", range(8))
def test_update_writes_stay_in_predicted_runs(lib, seed):
    """The prefill path re-packs only the K/V tiles an update may have written, which it predicts
    from the structure alone (ring positions opened, plus the resident item the first offers compete
    with).  The host replay checks every write against that prediction and fails with
    CASCADE_E_INTERNAL otherwise; here on tile-sized rings, chunks that wrap them, and many ties."""
    rng = np.random.default_rng(900 + seed)
    N = int(rng.integers(1, 5))
    sizes = [int(x) * 64 for x in rng.integers(1, 4, size=N)]
    n_sink = int(rng.choice([0, 3, 64]))
    periods = None if seed % 2 == 0 else [1] + [int(x) for x in rng.integers(1, 5, size=N - 1)]
    chunks = [int(x) for x in rng.choice([1, 5, 63, 64, 65, 128, 200, 256], size=30)]
    scores = (rng.integers(0, 5, size=sum(chunks)) / 4.0).astype(np.float32)
    cfg = _cfg(n_sink=n_sink, cascade_sizes=sizes, accept_period=periods, max_chunk=256, token_selection=1 - seed % 4 // 3)
    sim = B.cascade_simulate_structure(cfg, chunks, scores)   # raises on any error code
    assert sim.count == min(sum(chunks), n_sink + sum(sizes)) or sim.count <= n_sink + sum(sizes)
