"""Run-to-run identity: the kernels use no atomics on floating-point data and reduce in a fixed
order, so the same inputs must give the same bits.  This is also the race detector of the hand
counted waits (s_waitcnt vmcnt(N)) and the fence-less barriers of the streaming kernels: a copy
read before it has landed, or a buffer refilled before it was read, shows as a difference."""
import numpy as np
import pytest

from paper_2406_17808_amd import binding as B
from paper_2406_17808_amd.workloads import WORKLOADS, chunk_inputs_torch

pytestmark = pytest.mark.gpu


def _one_run(wl, cfg, n_chunks, n_decode, outs):
    import torch
    from paper_2406_17808_amd.cache import CascadeKVCache
    cache = CascadeKVCache(cfg)
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(4242)
    for c in range(n_chunks):
        q, k, v = chunk_inputs_torch(wl, 0, c, "cuda:0")
        outs.append(cache.prefill_chunk(q, k, v).clone())
    d = wl.head_dim
    for _ in range(n_decode):
        q = torch.randn((wl.batch, wl.n_q_heads, d), generator=gen, device="cuda:0").to(torch.bfloat16)
        k = torch.randn((wl.batch, wl.n_kv_heads, d), generator=gen, device="cuda:0").to(torch.bfloat16)
        v = torch.randn((wl.batch, wl.n_kv_heads, d), generator=gen, device="cuda:0").to(torch.bfloat16)
        outs.append(cache.decode_step(q, k, v).clone())
    st = cache.read_state(with_kv=True)
    cache.close()
    return st


@pytest.mark.parametrize("name,n_chunks,mode", [("prefill_32k", 32, "exact"), ("prefill_paper_16k", 6, "exact"),
                                                ("prefill_paper_16k", 6, "single_pass")])
def test_two_runs_give_the_same_bits(name, n_chunks, mode):
    """prefill_32k whole (split attention launches, the narrow score kernel) and six chunks of the
    paper's 16K geometry (unsplit attention, every row in the score sums: by the exact pass, and by the
    column sums inside the attention kernel, whose partial sums meet in LDS and in a per-row-block
    array), each followed by eight decode steps, twice from fresh contexts: every output, score, id
    and cached row bit-equal."""
    import torch
    from paper_2406_17808_amd.cache import config_of
    wl = WORKLOADS[name]
    cfg = config_of(wl, score_mode=B.CASCADE_SCORES_SINGLE_PASS if mode == "single_pass" else B.CASCADE_SCORES_EXACT)
    outs_a, outs_b = [], []
    a = _one_run(wl, cfg, n_chunks, 8, outs_a)
    b = _one_run(wl, cfg, n_chunks, 8, outs_b)
    for i, (x, y) in enumerate(zip(outs_a, outs_b)):
        assert torch.equal(x, y), f"{name}: output of call {i} differs between two runs"
    assert a.counts.tolist() == b.counts.tolist() and a.t == b.t and a.n_seen == b.n_seen
    for field in ("ids", "mu", "k", "v", "swaps"):
        x, y = getattr(a, field), getattr(b, field)
        same = np.array_equal(x.view(np.uint32) if x.dtype == np.float32 else x, y.view(np.uint32) if y.dtype == np.float32 else y)
        assert same, f"{name}: {field} differs between two runs"
