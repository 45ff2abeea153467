"""GPU parity on small configurations: every output row, every decision score and every cache
membership is compared with the CPU oracle (see gpu_harness.py for how parity is decomposed)."""
import numpy as np
import pytest

from paper_2406_17808_amd import binding as B
from paper_2406_17808_amd.workloads import WORKLOADS, chunk_inputs, round_to_bf16

pytestmark = pytest.mark.gpu


def _inputs(rng, cfg, n, scale=1.0):
    shape_q = (cfg.batch, n, cfg.n_q_heads, cfg.head_dim)
    shape_k = (cfg.batch, n, cfg.n_kv_heads, cfg.head_dim)
    q, k, v = (rng.standard_normal(s).astype(np.float32) * np.float32(scale) for s in (shape_q, shape_k, shape_k))
    if cfg.dtype == B.CASCADE_BF16:
        q, k, v = round_to_bf16(q), round_to_bf16(k), round_to_bf16(v)
    return q, k, v


def _tolerances(cfg):
    # outputs: the bar of the benchmark spec; scores: same arithmetic, same bar with headroom for
    # sums of few terms (bf16: operand rounding of rotated q and k, 2^-9 each, over d terms)
    return (2e-2, 6e-2) if cfg.dtype == B.CASCADE_BF16 else (1e-5, 5e-5)


def test_tiny_f32_free_running(oracle_mod):
    """The fp32 configuration: 2048 tokens, 4 sinks + 4 x 64 slots, chunks of 32, free running.
    Membership must equal the oracle's after every chunk (bit-exact), outputs within 1e-5."""
    from gpu_harness import ParityRun
    from paper_2406_17808_amd.cache import config_of
    wl = WORKLOADS["tiny_f32"]
    cfg = config_of(wl, keep_update_scores=1)
    run = ParityRun(cfg, one_step_ahead=False)
    worst_out = worst_score = 0.0
    for c in range(wl.n_chunks):
        q, k, v = chunk_inputs(wl, 0, c)
        rep = run.step(q, k, v)
        assert rep.replay_exact, c
        assert rep.drift == 0, (c, rep)
        worst_out, worst_score = max(worst_out, rep.out_err), max(worst_score, rep.score_err)
    print(f"tiny_f32: max out err {worst_out:.3e}, max score err {worst_score:.3e}")
    assert worst_out <= 1e-5
    assert worst_score <= 5e-5
    st = run.gpu.read_state()
    assert st.counts.tolist() == [4, 64, 64, 64, 64] and st.n_seen == 2048
    run.close()


@pytest.mark.parametrize("case", [
    dict(name="bf16_d128_ragged", dtype=B.CASCADE_BF16, d=128, Hq=8, Hkv=2, batch=1, n_sink=5,
         sizes=[48, 40, 36], chunks=[1, 7, 64, 100, 33, 128, 128, 2, 90, 128, 128, 77, 128, 128, 128], max_chunk=128),
    dict(name="bf16_d64_batch2", dtype=B.CASCADE_BF16, d=64, Hq=4, Hkv=4, batch=2, n_sink=3,
         sizes=[70, 70], chunks=[50, 50, 50, 50, 50, 13, 96, 96, 96, 96], max_chunk=96),
    dict(name="bf16_chunk_larger_than_cache", dtype=B.CASCADE_BF16, d=128, Hq=4, Hkv=1, batch=1, n_sink=4,
         sizes=[8, 8, 8], chunks=[300, 300, 17, 300], max_chunk=300),
    dict(name="bf16_big_tiles", dtype=B.CASCADE_BF16, d=128, Hq=8, Hkv=2, batch=1, n_sink=64,
         sizes=[256, 256, 256, 256], chunks=[512] * 8, max_chunk=512),
    dict(name="bf16_all_rows_in_scores", dtype=B.CASCADE_BF16, d=128, Hq=8, Hkv=2, batch=1, n_sink=4,
         sizes=[64, 64], chunks=[300] * 4, max_chunk=300, beta=0.99, score_tail_eps=-1.0, score_narrow=0),
    # keys grow along every chunk, so the running maximum of a row keeps rising by more than the
    # kernel's rescaling threshold.  bf16 operand rounding is relative: with logits of magnitude
    # ~20 the exponents are off by ~20 * 2^-8, hence the wider tolerance of this case against the
    # oracle's ideal arithmetic.  That the excess is this operand rounding and nothing else is
    # checked against the numpy model that rounds where the bf16 contract does ("model": the bounds
    # on outputs and scores against it: what is left in an output is its own rounding to bf16 and
    # the rounding of the probabilities at another power-of-two phase; the scores agree to fp32
    # accuracy).
    dict(name="bf16_rising_logits", dtype=B.CASCADE_BF16, d=64, Hq=4, Hkv=2, batch=1, n_sink=4,
         sizes=[96, 96, 96], chunks=[256] * 6, max_chunk=256, input_scale=1.5, key_ramp=2.0, tol_out=0.1, tol_score=0.3,
         model=(2.0 ** -7, 2.0 ** -12)),
    dict(name="f32_periods_mean", dtype=B.CASCADE_F32, d=32, Hq=4, Hkv=2, batch=2, n_sink=2,
         sizes=[9, 5, 7], chunks=[20, 3, 20, 20, 1, 20, 20, 20], max_chunk=20, periods=[1, 3, 2],
         head_reduce=B.CASCADE_REDUCE_MEAN),
    dict(name="f32_no_selection_one_cascade", dtype=B.CASCADE_F32, d=64, Hq=2, Hkv=2, batch=1, n_sink=4,
         sizes=[24], chunks=[10] * 8, max_chunk=10, token_selection=0),
    dict(name="f32_all_rows_in_scores", dtype=B.CASCADE_F32, d=64, Hq=2, Hkv=1, batch=1, n_sink=2,
         sizes=[16, 16], chunks=[40] * 5, max_chunk=40, beta=0.999, score_tail_eps=-1.0),
    # the same launch shapes with the attention kept in one workgroup per row block (small
    # launches are otherwise split over the keys), and with an odd number of splits
    dict(name="bf16_d128_ragged_unsplit", dtype=B.CASCADE_BF16, d=128, Hq=8, Hkv=2, batch=1, n_sink=5,
         sizes=[48, 40, 36], chunks=[1, 7, 64, 100, 33, 128, 128, 2, 90, 128, 128, 77, 128, 128, 128], max_chunk=128,
         attn_splits=1, score_narrow=0),
    dict(name="bf16_big_tiles_unsplit", dtype=B.CASCADE_BF16, d=128, Hq=8, Hkv=2, batch=1, n_sink=64,
         sizes=[256, 256, 256, 256], chunks=[512] * 8, max_chunk=512, attn_splits=1, score_narrow=0),
    dict(name="bf16_big_tiles_three_splits", dtype=B.CASCADE_BF16, d=128, Hq=8, Hkv=2, batch=1, n_sink=64,
         sizes=[256, 256, 256, 256], chunks=[512] * 8, max_chunk=512, attn_splits=3),
    dict(name="bf16_rising_logits_unsplit", dtype=B.CASCADE_BF16, d=64, Hq=4, Hkv=2, batch=1, n_sink=4,
         sizes=[96, 96, 96], chunks=[256] * 6, max_chunk=256, input_scale=1.5, key_ramp=2.0, tol_out=0.1, tol_score=0.3,
         attn_splits=1, model=(2.0 ** -7, 2.0 ** -12)),
    # an ordinary case against the same model, for scale
    dict(name="bf16_big_tiles_model", dtype=B.CASCADE_BF16, d=128, Hq=8, Hkv=2, batch=1, n_sink=64,
         sizes=[256, 256, 256, 256], chunks=[512] * 4, max_chunk=512, model=(2.0 ** -7, 2.0 ** -12)),
    # one slowly rotating RoPE pair carries 32 in every query and 64 in the marked keys, which lifts
    # their logits by about 2^8 / sqrt(d) x 2^3 x log2(e) (far more than an fp32 exponent holds)
    # over the keys without it: the running maximum has to follow, whatever a launch concluded
    # from the key norms.  "after_sinks" marks every token but the first four (the step comes at
    # the second tile of every workgroup), "chunk_tail" the last 64 tokens of a chunk (it comes at
    # the last tile first and then wherever those tokens land in the cache).  With a RoPE base of
    # 1e6 that pair turns by less than 1e-3 rad over the cache, so the lift is the same for every
    # marked key up to ~1e-4 and bf16 operand rounding does not enter.  In "chunk_tail" most tokens
    # end with a score below 2^-200, zero in fp32 and not in the oracle's fp64: their order, and so
    # the free-running membership, is not comparable there (the replayed decisions still are).
    dict(name="bf16_logit_step_after_sinks_unsplit", dtype=B.CASCADE_BF16, d=128, Hq=4, Hkv=2, batch=1, n_sink=4,
         sizes=[96, 96, 96], chunks=[256] * 5, max_chunk=256, logit_step="after_sinks", rope_base=1e6, attn_splits=1),
    dict(name="bf16_logit_step_chunk_tail_unsplit", dtype=B.CASCADE_BF16, d=128, Hq=4, Hkv=2, batch=1, n_sink=4,
         sizes=[96, 96, 96], chunks=[256] * 5, max_chunk=256, logit_step="chunk_tail", rope_base=1e6, attn_splits=1, compare_membership=False),
    # rings of whole tiles, all full after a few chunks: the packed K/V tiles then keep their place
    # from chunk to chunk and only the ones the last update wrote are packed again, as long as every
    # ring head keeps its offset inside a tile.  Chunks of 128 and 100 change the offset of the
    # third ring's head, and of all heads (everything is packed once, then tiles are kept again).
    dict(name="bf16_tile_aligned_rings", dtype=B.CASCADE_BF16, d=128, Hq=4, Hkv=2, batch=1, n_sink=64,
         sizes=[128, 128, 128], chunks=[256] * 6 + [128] + [256] * 2 + [128] + [256] * 4 + [100] + [256] * 2, max_chunk=256, pack_reuse=1),
    dict(name="bf16_tile_aligned_rings_d64_unsplit", dtype=B.CASCADE_BF16, d=64, Hq=8, Hkv=2, batch=2, n_sink=64,
         sizes=[256, 128], chunks=[256] * 4 + [64] * 3 + [192] + [256] * 3, max_chunk=256, attn_splits=1, pack_reuse=1),
    dict(name="bf16_logit_step_chunk_tail_d64", dtype=B.CASCADE_BF16, d=64, Hq=4, Hkv=2, batch=1, n_sink=4,
         sizes=[96, 96, 96], chunks=[256] * 5, max_chunk=256, logit_step="chunk_tail", rope_base=1e6, compare_membership=False),
], ids=lambda c: c["name"])
def test_prefill_one_step_ahead(oracle_mod, case, monkeypatch):
    from gpu_harness import ParityRun
    if "attn_splits" in case:
        monkeypatch.setenv("CASCADE_KV_ATTN_SPLITS", str(case["attn_splits"]))
    if "score_narrow" in case:   # 0: the score kernel keeps 64 keys per wave however small the launch
        monkeypatch.setenv("CASCADE_KV_SCORE_NARROW", str(case["score_narrow"]))
    if "pack_reuse" in case:   # 0: every tile is packed for every chunk
        monkeypatch.setenv("CASCADE_KV_PACK_REUSE", str(case["pack_reuse"]))
    cfg = B.make_config(batch=case["batch"], n_q_heads=case["Hq"], n_kv_heads=case["Hkv"], head_dim=case["d"],
                        dtype=case["dtype"], n_sink=case["n_sink"], cascade_sizes=case["sizes"],
                        ema_beta=case.get("beta", 0.9), rope_base=case.get("rope_base", 10000.0), max_chunk=case["max_chunk"],
                        accept_period=case.get("periods"), head_reduce=case.get("head_reduce", 0),
                        token_selection=case.get("token_selection", 1),
                        score_tail_eps=case.get("score_tail_eps", 0.0), keep_update_scores=1)
    tol_out, tol_score = _tolerances(cfg)
    tol_out, tol_score = case.get("tol_out", tol_out), case.get("tol_score", tol_score)
    rng = np.random.default_rng(7)
    # a comparison may flip where two scores are as close as the score tolerance of the case allows
    run = ParityRun(cfg, one_step_ahead=True, tau=case.get("tol_score"))
    drift = compared = seen = flips = 0
    worst_out = worst_score = worst_model_out = worst_model_score = 0.0
    for i, n in enumerate(case["chunks"]):
        q, k, v = _inputs(rng, cfg, n, case.get("input_scale", 1.0))
        if "key_ramp" in case:
            ramp = (1.0 + case["key_ramp"] * np.arange(n, dtype=np.float32) / n)[None, :, None, None]
            k = round_to_bf16(k * ramp) if cfg.dtype == B.CASCADE_BF16 else k * ramp
        if "logit_step" in case:
            lo, hi = cfg.head_dim // 2 - 1, cfg.head_dim - 1   # the pair with the smallest RoPE frequency
            marked = np.arange(n) >= n - 64 if case["logit_step"] == "chunk_tail" else np.arange(n) + seen >= 4
            q[..., lo], q[..., hi] = 32.0, 0.0
            k[..., lo], k[..., hi] = np.where(marked, 64.0, 0.0).astype(np.float32)[None, :, None], 0.0
        seen += n
        rep = run.step(q, k, v, with_model="model" in case)
        assert rep.replay_exact, (case["name"], i)
        # membership may only differ from the free oracle through comparisons whose two scores are
        # inside float noise of each other by the oracle's own account
        if case.get("compare_membership", True):
            assert rep.flips_mismatch == 0, (case["name"], i, rep)
        worst_out, worst_score = max(worst_out, rep.out_err), max(worst_score, rep.score_err)
        worst_model_out, worst_model_score = max(worst_model_out, rep.model_out_err), max(worst_model_score, rep.model_score_err)
        drift += rep.drift
        compared += rep.compared
        flips += rep.flips_noise
    print(f"{case['name']}: out {worst_out:.3e} score {worst_score:.3e} drift {drift}/{compared} noise-level flips {flips}"
          + (f" model: out {worst_model_out:.3e} score {worst_model_score:.3e}" if "model" in case else ""))
    assert worst_out <= tol_out
    assert worst_score <= tol_score
    if "model" in case:
        assert worst_model_out <= case["model"][0] and worst_model_score <= case["model"][1]
    if cfg.dtype == B.CASCADE_F32 and case.get("compare_membership", True):
        assert drift == 0, (drift, compared)
    run.close()


@pytest.mark.parametrize("seed", list(range(10)))
def test_kept_tiles_random_rings(oracle_mod, seed, monkeypatch):
    """Rings of whole tiles with random sizes, sink counts that are and are not multiples of a
    tile, chunks that keep every ring head at its offset inside a tile, chunks that do not, and
    decode steps in between: the packed K/V tiles are kept from chunk to chunk whenever the heads
    allow it, and every step is compared with the oracle."""
    from gpu_harness import ParityRun
    monkeypatch.setenv("CASCADE_KV_PACK_REUSE", "1")
    rng = np.random.default_rng(5000 + seed)
    N = int(rng.integers(1, 4))
    sizes = [int(rng.integers(1, 5)) * 64 for _ in range(N)]
    n_sink = int(rng.choice([0, 5, 64, 70]))
    d, hkv, G = int(rng.choice([64, 128])), int(rng.choice([1, 2])), int(rng.choice([1, 2, 4]))
    unit = 64 * 2 ** (N - 1)      # the last cascade then receives a multiple of 64 tokens per chunk
    cfg = B.make_config(batch=1, n_q_heads=hkv * G, n_kv_heads=hkv, head_dim=d, dtype=B.CASCADE_BF16, n_sink=n_sink,
                        cascade_sizes=sizes, ema_beta=float(rng.choice([0.9, 0.99])), rope_base=10000.0,
                        max_chunk=4 * unit, keep_update_scores=1)
    tol_out, tol_score = _tolerances(cfg)
    run = ParityRun(cfg, one_step_ahead=True)
    plan = []
    for _ in range(14):
        r = rng.random()
        if r < 0.7:
            plan.append(("p", int(rng.integers(1, 5)) * unit))
        elif r < 0.85:
            plan.append(("p", int(rng.integers(1, 4 * unit + 1))))
        else:
            plan += [("d", 1)] * int(rng.integers(1, 4))
    for i, (kind, n) in enumerate(plan):
        q, k, v = _inputs(rng, cfg, n)
        rep = run.step(q, k, v, decode=(kind == "d"))
        assert rep.replay_exact, (seed, i, kind, n)
        assert rep.out_err <= tol_out and rep.score_err <= tol_score, (seed, i, kind, n, rep)
    run.close()


def test_sixteen_cascades(oracle_mod):
    """The largest number of sub-caches the configuration allows: once all rings are full the
    segment list holds three pieces per ring (50 segments, 34 query rotations); a decode step then
    has more rotations than its streaming kernel keeps in LDS and takes the register-load kernel."""
    from gpu_harness import ParityRun
    cfg = B.make_config(batch=1, n_q_heads=4, n_kv_heads=2, head_dim=64, dtype=B.CASCADE_BF16, n_sink=2,
                        cascade_sizes=[70] + [9] * 15, ema_beta=0.9, rope_base=10000.0, max_chunk=96,
                        accept_period=[1] * 16, keep_update_scores=1)
    tol_out, tol_score = _tolerances(cfg)
    rng = np.random.default_rng(16)
    run = ParityRun(cfg, one_step_ahead=True)
    plan = [("p", 96)] * 5 + [("p", 37)] + [("d", 1)] * 5 + [("p", 96)] * 2
    worst_out = worst_score = 0.0
    for i, (kind, n) in enumerate(plan):
        q, k, v = _inputs(rng, cfg, n)
        rep = run.step(q, k, v, decode=(kind == "d"))
        assert rep.replay_exact, i
        worst_out, worst_score = max(worst_out, rep.out_err), max(worst_score, rep.score_err)
    st = run.gpu.read_state()
    assert st.counts.tolist() == [2, 70] + [9] * 15      # every ring is full
    print(f"sixteen cascades: out {worst_out:.3e} score {worst_score:.3e}")
    assert worst_out <= tol_out and worst_score <= tol_score
    run.close()


def test_decode_steps_between_tile_aligned_chunks(oracle_mod, monkeypatch):
    """Decode steps write cache rows without touching the packed K/V tiles of the prefill path, so
    the chunk after them must not reuse any tile (rings of whole tiles, as above)."""
    from gpu_harness import ParityRun
    monkeypatch.setenv("CASCADE_KV_PACK_REUSE", "1")
    cfg = B.make_config(batch=1, n_q_heads=4, n_kv_heads=2, head_dim=128, dtype=B.CASCADE_BF16, n_sink=64,
                        cascade_sizes=[128, 128], ema_beta=0.9, rope_base=10000.0, max_chunk=256, keep_update_scores=1)
    tol_out, tol_score = _tolerances(cfg)
    rng = np.random.default_rng(21)
    run = ParityRun(cfg, one_step_ahead=True)
    plan = [("p", 256)] * 4 + [("d", 1)] * 64 + [("p", 256)] * 3 + [("d", 1)] * 7 + [("p", 256)] * 2
    worst_out = worst_score = 0.0
    for i, (kind, n) in enumerate(plan):
        q, k, v = _inputs(rng, cfg, n)
        rep = run.step(q, k, v, decode=(kind == "d"))
        assert rep.replay_exact, i
        worst_out, worst_score = max(worst_out, rep.out_err), max(worst_score, rep.score_err)
    print(f"decode between aligned chunks: out {worst_out:.3e} score {worst_score:.3e}")
    assert worst_out <= tol_out and worst_score <= tol_score
    run.close()


@pytest.mark.parametrize("dtype,d,hq,hkv", [(B.CASCADE_F32, 64, 8, 2), (B.CASCADE_BF16, 128, 8, 2),
                                            (B.CASCADE_BF16, 64, 8, 1), (B.CASCADE_BF16, 64, 2, 2),
                                            (B.CASCADE_BF16, 128, 4, 2), (B.CASCADE_BF16, 128, 3, 1)])
def test_prefill_then_decode(oracle_mod, dtype, d, hq, hkv):
    """A decode step has the semantics of a chunk of one token (Eq. 2); group sizes 1, 2, 3, 4, 8."""
    from gpu_harness import ParityRun
    cfg = B.make_config(batch=2, n_q_heads=hq, n_kv_heads=hkv, head_dim=d, dtype=dtype, n_sink=4,
                        cascade_sizes=[20, 12, 12], ema_beta=0.9, rope_base=10000.0, max_chunk=64,
                        keep_update_scores=1)
    tol_out, tol_score = _tolerances(cfg)
    rng = np.random.default_rng(8)
    run = ParityRun(cfg, one_step_ahead=True)
    # decode from an empty cache, prefill, decode again
    plan = [("d", 1)] * 6 + [("p", 64), ("p", 37)] + [("d", 1)] * 40
    worst_out = worst_score = 0.0
    for i, (kind, n) in enumerate(plan):
        q, k, v = _inputs(rng, cfg, n)
        rep = run.step(q, k, v, decode=(kind == "d"))
        assert rep.replay_exact, i
        worst_out, worst_score = max(worst_out, rep.out_err), max(worst_score, rep.score_err)
    print(f"prefill_then_decode {dtype} d={d} {hq}/{hkv}: out {worst_out:.3e} score {worst_score:.3e}")
    assert worst_out <= tol_out and worst_score <= tol_score
    run.close()


@pytest.mark.parametrize("dtype,d,G,policy", [(B.CASCADE_BF16, 128, 4, 0), (B.CASCADE_BF16, 64, 2, 1)])
def test_long_decode(oracle_mod, dtype, d, G, policy):
    """Three hundred decode steps after one chunk, every step compared one step ahead: the rings of 37, 64
    and 50 slots turn over several times, every acceptance phase of the three cascades comes up."""
    from gpu_harness import ParityRun
    cfg = B.make_config(batch=2, n_q_heads=2 * G, n_kv_heads=2, head_dim=d, dtype=dtype, n_sink=3,
                        cascade_sizes=[37, 64, 50], ema_beta=0.97, rope_base=10000.0, max_chunk=64,
                        keep_update_scores=1, head_policy=policy)
    rng = np.random.default_rng(77)
    run = ParityRun(cfg, one_step_ahead=True)
    worst_out = worst_score = 0.0

    def inputs(n):
        sh_q = (cfg.batch, n, cfg.n_q_heads, d)
        sh_k = (cfg.batch, n, cfg.n_kv_heads, d)
        f = lambda sh: rng.standard_normal(sh).astype(np.float32)
        q, k, v = f(sh_q), f(sh_k), f(sh_k)
        if dtype == B.CASCADE_BF16:
            from paper_2406_17808_amd.workloads import round_to_bf16
            q, k, v = round_to_bf16(q), round_to_bf16(k), round_to_bf16(v)
        return q, k, v

    rep = run.step(*inputs(50))
    for step in range(300):
        rep = run.step(*inputs(1), decode=True)
        assert rep.replay_exact, step
        assert rep.flips_mismatch == 0, (step, rep)
        worst_out, worst_score = max(worst_out, rep.out_err), max(worst_score, rep.score_err)
    print(f"long decode dtype {dtype} d={d} G={G} head policy {policy}: out {worst_out:.3e} score {worst_score:.3e}")
    tol_out, tol_score = _tolerances(cfg)
    assert worst_out <= tol_out and worst_score <= tol_score
    assert int(run.gpu.read_state().discards.sum()) > 100
    run.close()


@pytest.mark.parametrize("seed", list(range(12)))
def test_random_geometries(oracle_mod, seed, monkeypatch):
    """Seeded random geometries (heads, head_dim, sinks, cascade count and sizes, periods, chunk
    mix, decay) through prefill and decode, one step ahead of the oracle: sizes that are not
    multiples of any tile, partly filled cascades, chunks from 1 token to several tiles.  Even
    seeds pack every K/V tile for every chunk, odd seeds keep the tiles no update has written."""
    from gpu_harness import ParityRun
    monkeypatch.setenv("CASCADE_KV_PACK_REUSE", str(seed % 2))
    # small launches take the score kernel with 32 keys per wave; half of the seeds force the 64-key form
    monkeypatch.setenv("CASCADE_KV_SCORE_NARROW", str(seed // 2 % 2))
    rng = np.random.default_rng(1000 + seed)
    d = int(rng.choice([64, 128]))
    hkv = int(rng.choice([1, 2, 3]))
    G = int(rng.choice([1, 2, 4, 5, 8]))
    N = int(rng.integers(1, 6))
    sizes = [int(rng.integers(3, 150)) for _ in range(N)]
    periods = None
    if rng.random() < 0.4:
        periods = [1] + [int(rng.integers(1, 5)) for _ in range(N - 1)]
    max_chunk = int(rng.choice([17, 64, 130, 300]))
    cfg = B.make_config(batch=int(rng.choice([1, 2])), n_q_heads=hkv * G, n_kv_heads=hkv, head_dim=d,
                        dtype=B.CASCADE_BF16, n_sink=int(rng.integers(0, 9)), cascade_sizes=sizes,
                        ema_beta=float(rng.choice([0.5, 0.9, 0.99, 0.999])), rope_base=10000.0, max_chunk=max_chunk,
                        accept_period=periods, head_reduce=int(rng.integers(0, 2)),
                        token_selection=int(rng.random() < 0.85), keep_update_scores=1)
    tol_out, tol_score = _tolerances(cfg)
    run = ParityRun(cfg, one_step_ahead=True)
    worst_out = worst_score = 0.0
    drift = compared = 0
    for step in range(14):
        decode = rng.random() < 0.3
        n = 1 if decode else int(rng.integers(1, max_chunk + 1))
        q, k, v = _inputs(rng, cfg, n)
        rep = run.step(q, k, v, decode=decode)
        assert rep.replay_exact, (seed, step)
        assert rep.flips_mismatch == 0, (seed, step, rep)
        worst_out, worst_score = max(worst_out, rep.out_err), max(worst_score, rep.score_err)
        drift += rep.drift
        compared += rep.compared
    print(f"random geometry {seed}: d={d} heads {hkv * G}/{hkv} sinks {cfg.n_sink} sizes {sizes} periods {periods} "
          f"max_chunk {max_chunk}: out {worst_out:.3e} score {worst_score:.3e} drift {drift}/{compared}")
    assert worst_out <= tol_out and worst_score <= tol_score
    run.close()


@pytest.mark.parametrize("dtype,reduce,hkv,G,d", [(B.CASCADE_BF16, B.CASCADE_REDUCE_MAX, 4, 2, 128), (B.CASCADE_BF16, B.CASCADE_REDUCE_MEAN, 2, 4, 64),
                                                  (B.CASCADE_F32, B.CASCADE_REDUCE_MAX, 3, 1, 64)])
def test_homogeneous_heads(oracle_mod, dtype, reduce, hkv, G, d):
    """Homogeneous heads (Appendix "Head Policy and Head Reduction"): the scores are reduced over all
    heads, every KV head takes the same decisions.  Prefill chunks and decode steps against the
    oracle's homogeneous policy; all KV heads of the library must hold the same tokens throughout."""
    from gpu_harness import ParityRun
    cfg = B.make_config(batch=2, n_q_heads=hkv * G, n_kv_heads=hkv, head_dim=d, dtype=dtype, n_sink=3,
                        cascade_sizes=[40, 24, 24], ema_beta=0.9, rope_base=10000.0, max_chunk=64, head_reduce=reduce,
                        keep_update_scores=1, head_policy=B.CASCADE_HEADS_HOMOGENEOUS)
    assert cfg.head_policy == 1
    tol_out, tol_score = _tolerances(cfg)
    rng = np.random.default_rng(31)
    run = ParityRun(cfg, one_step_ahead=True)
    plan = [("p", 64), ("p", 50)] + [("d", 1)] * 3 + [("p", 64)] * 3 + [("d", 1)] * 4 + [("p", 17), ("p", 64)]
    worst_out = worst_score = 0.0
    for i, (kind, n) in enumerate(plan):
        q, k, v = _inputs(rng, cfg, n)
        rep = run.step(q, k, v, decode=(kind == "d"))
        assert rep.replay_exact, i
        assert rep.flips_mismatch == 0, (i, rep)
        worst_out, worst_score = max(worst_out, rep.out_err), max(worst_score, rep.score_err)
        st = run.prev
        for b in range(cfg.batch):
            for g in range(1, hkv):
                assert np.array_equal(st.ids[b, g], st.ids[b, 0]) and np.array_equal(st.mu[b, g], st.mu[b, 0]), (i, b, g)
    print(f"homogeneous heads reduce {reduce}: out {worst_out:.3e} score {worst_score:.3e}")
    assert worst_out <= tol_out and worst_score <= tol_score
    assert int(run.gpu.read_state().discards.sum()) > 100      # the policy was at work
    run.close()


@pytest.mark.parametrize("case", [
    # every row of a chunk carries weight; rings of whole and of ragged tiles, two row blocks per head
    dict(name="sp_all_rows_d128", d=128, Hq=8, Hkv=2, n_sink=64, sizes=[256, 256, 192], beta=0.999, chunks=[512] * 7),
    # head_dim 64, three row blocks per head, rings that are no multiples of a tile
    dict(name="sp_all_rows_d64", d=64, Hq=4, Hkv=2, n_sink=5, sizes=[300, 200], beta=0.9999, chunks=[768] * 5),
    # beta = 0.5: only the last 40 rows of a chunk carry weight: the exact pass is short, and taken
    dict(name="sp_short_tail_takes_exact", d=64, Hq=4, Hkv=2, n_sink=5, sizes=[300, 200], beta=0.5, chunks=[768] * 3, never=True),
    # chunks that do not qualify (not a multiple of 256) take the exact pass in between; mean reduction
    dict(name="sp_mixed_chunks_mean", d=128, Hq=4, Hkv=1, n_sink=4, sizes=[128, 128, 128], beta=0.99,
         chunks=[256, 256, 100, 256, 37, 512, 256], head_reduce=B.CASCADE_REDUCE_MEAN),
], ids=lambda c: c["name"])
def test_single_pass_scores(oracle_mod, case, monkeypatch):
    """score_mode = CASCADE_SCORES_SINGLE_PASS: the scores of Alg. 3, added up while the attention
    kernel sweeps the keys, against the oracle's single-pass scores on the kernel's visiting
    schedule (gpu_harness.visiting_schedule); outputs, decisions and cached rows as in every other
    case.  How far the approximation moves the cache is counted against an exact-score twin."""
    from gpu_harness import ParityRun
    monkeypatch.setenv("CASCADE_KV_ATTN_SPLITS", "1")     # small launches are otherwise split over the keys (exact pass)
    cfg = B.make_config(batch=1, n_q_heads=case["Hq"], n_kv_heads=case["Hkv"], head_dim=case["d"], dtype=B.CASCADE_BF16,
                        n_sink=case["n_sink"], cascade_sizes=case["sizes"], ema_beta=case["beta"], rope_base=10000.0,
                        max_chunk=max(case["chunks"]), head_reduce=case.get("head_reduce", 0), keep_update_scores=1,
                        score_mode=B.CASCADE_SCORES_SINGLE_PASS)
    tol_out, tol_score = _tolerances(cfg)
    rng = np.random.default_rng(41)
    run = ParityRun(cfg, one_step_ahead=True)
    worst_out = worst_score = 0.0
    diverged = compared = taken = 0
    for i, n in enumerate(case["chunks"]):
        q, k, v = _inputs(rng, cfg, n)
        rep = run.step(q, k, v, exact_twin=True)
        assert rep.single_pass == (n % 256 == 0 and not case.get("never", False)), (i, n)
        assert rep.replay_exact, (case["name"], i)
        assert rep.flips_mismatch == 0, (case["name"], i, rep)
        worst_out, worst_score = max(worst_out, rep.out_err), max(worst_score, rep.score_err)
        if rep.single_pass:
            taken += 1
            diverged += rep.diverged_from_exact
            compared += rep.compared
    print(f"{case['name']}: out {worst_out:.3e} score {worst_score:.3e}; {taken} single-pass chunks, cache positions that "
          f"differ from the exact-score oracle's: {diverged}/{compared}")
    assert worst_out <= tol_out and worst_score <= tol_score
    assert taken >= (0 if case.get("never", False) else 4)
    run.close()


@pytest.mark.parametrize("seed", list(range(8)))
def test_random_single_pass(oracle_mod, seed, monkeypatch):
    """Seeded random geometries with score_mode single_pass: chunks of 256, 512 and 768 tokens take the
    column sums inside the attention kernel (rings that are no multiples of a tile, several row blocks per
    head, both head policies), ragged chunks and decode steps in between take the exact pass."""
    from gpu_harness import ParityRun
    monkeypatch.setenv("CASCADE_KV_ATTN_SPLITS", "1")
    monkeypatch.setenv("CASCADE_KV_PACK_REUSE", str(seed % 2))
    rng = np.random.default_rng(5000 + seed)
    d = int(rng.choice([64, 128]))
    hkv = int(rng.choice([1, 2]))
    G = int(rng.choice([1, 2, 4]))
    N = int(rng.integers(1, 5))
    sizes = [int(rng.integers(40, 400)) for _ in range(N)]
    max_chunk = int(rng.choice([256, 512, 768]))
    cfg = B.make_config(batch=1, n_q_heads=hkv * G, n_kv_heads=hkv, head_dim=d,
                        dtype=B.CASCADE_BF16, n_sink=int(rng.integers(0, 70)), cascade_sizes=sizes,
                        ema_beta=float(rng.choice([0.999, 0.9999])), rope_base=10000.0, max_chunk=max_chunk,
                        head_reduce=int(rng.integers(0, 2)), keep_update_scores=1,
                        head_policy=int(rng.random() < 0.3), score_mode=B.CASCADE_SCORES_SINGLE_PASS)
    tol_out, tol_score = _tolerances(cfg)
    run = ParityRun(cfg, one_step_ahead=True)
    worst_out = worst_score = 0.0
    taken = 0
    for step in range(6):
        n = int(rng.choice([256, 512, 768, 100, 1]))
        n = min(n, max_chunk)
        q, k, v = _inputs(rng, cfg, n)
        rep = run.step(q, k, v, decode=(n == 1 and rng.random() < 0.5))
        assert rep.replay_exact, (seed, step)
        assert rep.flips_mismatch == 0, (seed, step, rep)
        taken += int(rep.single_pass)
        worst_out, worst_score = max(worst_out, rep.out_err), max(worst_score, rep.score_err)
    print(f"random single pass {seed}: d={d} heads {hkv * G}/{hkv} sizes {sizes} max_chunk {max_chunk}: out {worst_out:.3e} score {worst_score:.3e} taken {taken}")
    assert worst_out <= tol_out and worst_score <= tol_score
    run.close()


def test_single_pass_needs_bf16():
    cfg = B.make_config(batch=1, n_q_heads=2, n_kv_heads=1, head_dim=64, dtype=B.CASCADE_F32, n_sink=1, cascade_sizes=[4],
                        ema_beta=0.9, rope_base=10000.0, max_chunk=8, score_mode=B.CASCADE_SCORES_SINGLE_PASS)
    assert B.cascade_workspace_bytes(cfg) == 0
    with pytest.raises(B.CascadeError) as e:
        B.cascade_init(cfg, 256, 1 << 20)
    assert e.value.code == B.CASCADE_E_UNSUPPORTED


def test_layers_share_scratch_without_interfering(oracle_mod):
    """Three layers over one workspace (the layer loop of Alg. 1), fed different inputs in turn,
    prefill and decode: the middle layer is compared with the oracle at every step, the outer
    ones must end exactly where independent single-layer contexts fed the same inputs end."""
    import torch
    from gpu_harness import ParityRun, to_device
    from paper_2406_17808_amd.cache import CascadeKVCache, CascadeKVLayers
    cfg = B.make_config(batch=2, n_q_heads=8, n_kv_heads=2, head_dim=128, dtype=B.CASCADE_BF16, n_sink=4,
                        cascade_sizes=[20, 12, 12], ema_beta=0.9, rope_base=10000.0, max_chunk=48,
                        keep_update_scores=1)
    tol_out, tol_score = _tolerances(cfg)
    layers = CascadeKVLayers(cfg, 3)
    assert layers.workspace_bytes < 3 * B.cascade_workspace_bytes(cfg)
    solo = [CascadeKVCache(cfg), None, CascadeKVCache(cfg)]
    run = ParityRun(cfg, one_step_ahead=True, gpu=layers[1])
    rngs = [np.random.default_rng(100 + i) for i in range(3)]
    plan = [("p", 48), ("p", 31), ("d", 1), ("d", 1), ("p", 48), ("d", 1), ("p", 7)] + [("d", 1)] * 6
    worst_out = worst_score = 0.0
    for step, (kind, n) in enumerate(plan):
        for i in range(3):
            q, k, v = _inputs(rngs[i], cfg, n)
            if i == 1:
                rep = run.step(q, k, v, decode=(kind == "d"))
                assert rep.replay_exact, step
                worst_out, worst_score = max(worst_out, rep.out_err), max(worst_score, rep.score_err)
                continue
            dq, dk, dv = (to_device(x, cfg) for x in (q, k, v))
            if kind == "d":
                a = layers[i].decode_step(dq[:, 0].contiguous(), dk[:, 0].contiguous(), dv[:, 0].contiguous())
                b = solo[i].decode_step(dq[:, 0].contiguous(), dk[:, 0].contiguous(), dv[:, 0].contiguous())
            else:
                a = layers[i].prefill_chunk(dq, dk, dv)
                b = solo[i].prefill_chunk(dq, dk, dv)
            assert torch.equal(a, b), (step, i)
    print(f"layers: out {worst_out:.3e} score {worst_score:.3e}")
    assert worst_out <= tol_out and worst_score <= tol_score
    for i in (0, 2):
        sa, sb = layers[i].read_state(with_kv=True), solo[i].read_state(with_kv=True)
        assert sa.count == sb.count and sa.t == sb.t and sa.n_seen == sb.n_seen
        for name in ("ids", "mu", "k", "v"):
            assert np.array_equal(getattr(sa, name), getattr(sb, name)), (i, name)
        solo[i].close()
    run.close()
    layers.close()


def test_error_paths_on_device(oracle_mod):
    import torch
    from paper_2406_17808_amd.cache import CascadeKVCache
    cfg = B.make_config(batch=1, n_q_heads=2, n_kv_heads=1, head_dim=64, dtype=B.CASCADE_F32, n_sink=1,
                        cascade_sizes=[4], ema_beta=0.9, rope_base=10000.0, max_chunk=8)
    c = CascadeKVCache(cfg)
    q = torch.zeros(1, 9, 2, 64, device="cuda:0")
    kv = torch.zeros(1, 9, 1, 64, device="cuda:0")
    with pytest.raises(B.CascadeError) as e:
        c.prefill_chunk(q, kv, kv)
    assert e.value.code == B.CASCADE_E_BAD_ARG
    with pytest.raises(B.CascadeError) as e:
        B.cascade_prefill_chunk(c.ctx, 0, kv.data_ptr(), kv.data_ptr(), 4, q.data_ptr())
    assert e.value.code == B.CASCADE_E_NULL_ARG
    st = c.read_state()
    assert st.count == 0 and st.n_seen == 0
    c.close()
