"""cascade_init_static: a context whose workspace is the library's own static device array.

The same chunks and decode steps go through a context made by cascade_init (caller's workspace)
and one made by cascade_init_static; outputs, scores, ids and cached rows must be equal bit for
bit (both run the same kernels).  Two static contexts in a row, the second with a smaller
configuration, so that whatever the first left in the array would show.
"""
import numpy as np
import pytest

from paper_2406_17808_amd import binding as B
from paper_2406_17808_amd.workloads import round_to_bf16

pytestmark = pytest.mark.gpu


def _run_pair(cfg, plan, seed):
    import torch
    from paper_2406_17808_amd.cache import CascadeKVCache
    assert B.cascade_workspace_bytes(cfg) <= B.CASCADE_STATIC_WORKSPACE_BYTES
    ref = CascadeKVCache(cfg)
    sta = CascadeKVCache(cfg, static_workspace=True)
    assert sta.workspace is None
    rng = np.random.default_rng(seed)
    Hq, Hkv, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    for step, (kind, n) in enumerate(plan):
        q = round_to_bf16(rng.standard_normal((cfg.batch, n, Hq, d)).astype(np.float32))
        k = round_to_bf16(rng.standard_normal((cfg.batch, n, Hkv, d)).astype(np.float32))
        v = round_to_bf16(rng.standard_normal((cfg.batch, n, Hkv, d)).astype(np.float32))
        dq, dk, dv = (torch.from_numpy(x).to("cuda:0").to(torch.bfloat16) for x in (q, k, v))
        if kind == "d":
            a = ref.decode_step(dq[:, 0].contiguous(), dk[:, 0].contiguous(), dv[:, 0].contiguous())
            b = sta.decode_step(dq[:, 0].contiguous(), dk[:, 0].contiguous(), dv[:, 0].contiguous())
        else:
            a = ref.prefill_chunk(dq, dk, dv)
            b = sta.prefill_chunk(dq, dk, dv)
        assert torch.equal(a, b), (step, kind, n)
        assert torch.isfinite(a.float()).all()
    sa, sb = ref.read_state(with_kv=True), sta.read_state(with_kv=True)
    assert sa.count == sb.count and sa.t == sb.t and sa.n_seen == sb.n_seen
    assert sa.counts.tolist() == sb.counts.tolist()
    for name in ("ids", "mu", "k", "v", "swaps"):
        assert np.array_equal(getattr(sa, name), getattr(sb, name)), name
    ref.close()
    sta.close()
    return sa


def test_static_workspace_twice_second_smaller():
    big = B.make_config(batch=2, n_q_heads=8, n_kv_heads=2, head_dim=128, dtype=B.CASCADE_BF16, n_sink=64,
                        cascade_sizes=[256, 256, 256], ema_beta=0.9, rope_base=10000.0, max_chunk=256)
    small = B.make_config(batch=1, n_q_heads=4, n_kv_heads=2, head_dim=64, dtype=B.CASCADE_BF16, n_sink=3,
                          cascade_sizes=[40, 24], ema_beta=0.99, rope_base=10000.0, max_chunk=48)
    st = _run_pair(big, [("p", 256)] * 5 + [("d", 1)] * 3 + [("p", 100), ("p", 256)] + [("d", 1)] * 2, seed=1)
    assert st.count == 64 + 3 * 256
    st = _run_pair(small, [("p", 48), ("p", 7)] + [("d", 1)] * 4 + [("p", 48)] * 3 + [("d", 1)], seed=2)
    assert st.count == 3 + 40 + 24


def test_static_workspace_rejects_what_does_not_fit():
    cfg = B.make_config(batch=1, n_q_heads=32, n_kv_heads=8, head_dim=128, dtype=B.CASCADE_BF16, n_sink=64,
                        cascade_sizes=[16384] * 4, ema_beta=0.9, rope_base=500000.0, max_chunk=4096)
    assert B.cascade_workspace_bytes(cfg) > B.CASCADE_STATIC_WORKSPACE_BYTES
    with pytest.raises(B.CascadeError) as e:
        B.cascade_init_static(cfg)
    assert e.value.code == B.CASCADE_E_WORKSPACE_TOO_SMALL
    assert "static workspace" in str(e.value)
