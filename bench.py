#!/usr/bin/env python3
"""Benchmark of the cascading KV cache hot path on one MI355X.

A step is one pass of the whole prefill hot path over one chunk of the workload: query/key
rotation, chunk attention, exact EMA score sums and the cascade update (one call of
cascade_prefill_chunk).  The default workload is the 1M-token / 65K-slot prefill.  Whatever
--warmup and --steps say, the first chunks of the stream are run untimed as SETUP until every
slot of the cache is occupied (33 chunks for that workload); the warm-up chunks and then the
timed chunks follow, so every timed chunk attends to a full cache.
The single JSON line also carries the decode-step latency of the batch-32 decode workload, the
roofline figures of the dominant kernel of each, and the CPU oracle timed on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK = 2.5e15     # dense bf16 MFMA FLOP/s of one MI355X
HBM_PEAK = 8.0e12           # bytes/s
HEADLINE = "prefill_1m"     # the workload the metric is quoted on: its timed chunks must see a full cache


def stored_traffic(name):
    """HBM bytes per launch of a kernel as measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE,
    scaled by a copy of known size); the figures live with the profile summaries, or None."""
    path = os.path.join(ROOT, "profiles", name)
    try:
        with open(path) as f:
            return json.load(f).get("hbm_bytes_per_launch")
    except (OSError, ValueError):
        return None


def calibration_copy(torch, mib):
    """A plain device-to-device copy of known size, for scaling the HBM counters of a profiler run."""
    n = mib << 20
    a = torch.full((n,), 1, dtype=torch.uint8, device="cuda:0")
    b = torch.empty_like(a)
    for _ in range(3):
        b.copy_(a)
    torch.cuda.synchronize()
    del a, b


def measured_ceilings(torch, B):
    """What this very device sustains, measured in this run (untimed leg): streaming read, copy, pure MFMA loop."""
    nbytes = 9 << 30      # a half is the size of the decode workload's K (or V) cache; single-launch figures use the first half
    buf = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    buf.fill_(1)
    torch.cuda.synchronize()
    c = B.cascade_measure_ceilings(buf.data_ptr(), nbytes, torch.cuda.current_stream().cuda_stream)
    del buf
    torch.cuda.empty_cache()
    return {"compute_units": c["compute_units"], "core_clock_mhz": c["core_clock_mhz"], "memory_clock_mhz": c["memory_clock_mhz"],
            "memory_bus_bits": c["memory_bus_bits"], "hbm_read_gb_s": c["read_gb_s"], "hbm_copy_gb_s_read_plus_write": c["copy_gb_s"],
            "hbm_read_regions_gb_s": c["read_regions_gb_s"], "hbm_read_with_1_16_stores_gb_s": c["read_with_stores_gb_s"],
            "hbm_two_pass_read_gb_s": c["two_pass_read_gb_s"],
            "mfma_bf16_tflops": c["mfma_bf16_tflops"], "buffer_bytes": nbytes}


def prefill_bench(args, torch, B, wl):
    from paper_2406_17808_amd.cache import CascadeKVCache, config_of
    from paper_2406_17808_amd.workloads import chunk_inputs_torch
    dev = "cuda:0"
    W, K = args.warmup, args.steps
    cfg = config_of(wl, score_mode=B.CASCADE_SCORES_SINGLE_PASS if args.score_mode == "single_pass" else B.CASCADE_SCORES_EXACT)
    # cached rows before every chunk (host arithmetic; the fill does not depend on the scores)
    n_before = [B.cascade_simulate_structure(cfg, [wl.chunk] * c).count if c else 0 for c in range(wl.n_chunks + 1)]
    # setup chunks: the stream from its start until every slot is occupied
    F = next((c for c in range(wl.n_chunks + 1) if n_before[c] == wl.n_slots), None)
    if F is None and wl.name != HEADLINE:
        # a stream too short to fill its cache (Eq. 4: the span of the cascades exceeds it): time its last
        # chunks but sixteen, which the per-family breakdown takes
        F = max(wl.n_chunks - W - K - 16, 0)
    if F is None or F + W + K > wl.n_chunks:
        print(f"bench.py: {wl.name} has {wl.n_chunks} chunks; {F} fill the cache, so --warmup + --steps "
              f"must not exceed {wl.n_chunks - (F or 0)}", file=sys.stderr)
        sys.exit(2)
    cache = CascadeKVCache(cfg, dev)
    out = None
    for c in range(F):      # untimed, generated and dropped one at a time
        qkv = chunk_inputs_torch(wl, args.seed, c, dev)
        out = torch.empty_like(qkv[0]) if out is None else out
        cache.prefill_chunk(*qkv, out=out)
    chunks = {c: chunk_inputs_torch(wl, args.seed, c, dev) for c in range(F, F + W + K)}
    out = torch.empty_like(chunks[F][0]) if out is None else out
    for c in range(F, F + W):
        cache.prefill_chunk(*chunks[c], out=out)
    W += F                  # index of the first timed chunk
    torch.cuda.synchronize()
    accepted_before = cache.read_state().accepted.copy()
    # In the timed region only the dominant kernel is bracketed by events (its duration is the
    # denominator of `roofline`): two events between two kernels leave the GPU idle for about ten
    # microseconds, which the throughput should not pay four times per step.
    B.cascade_profile_begin(cache.ctx, ["attention"])
    t0 = time.perf_counter()
    for c in range(W, W + K):
        cache.prefill_chunk(*chunks[c], out=out)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    prof = B.cascade_profile_end(cache.ctx)
    seconds = t1 - t0
    tokens = K * wl.chunk * wl.batch
    Q, d = wl.chunk, wl.head_dim
    # algorithmic work of the attention kernel: one QK^T and one PV over the visible pairs
    flops = [4.0 * d * wl.n_q_heads * wl.batch * (Q * n_before[c] + Q * (Q + 1) / 2) for c in range(W, W + K)]
    moved_timed = int((cache.read_state().accepted - accepted_before).sum()) * wl.n_kv_heads * wl.batch
    # The other kernel families: an untimed pass over the chunks that follow, every family bracketed.
    K2 = min(16, wl.n_chunks - (W + K))
    breakdown = {}
    moved = upd_ms = 0.0
    upd_n = 0
    if K2 > 0:
        acc0 = cache.read_state().accepted.copy()
        B.cascade_profile_begin(cache.ctx)
        for c in range(W + K, W + K + K2):
            qkv = chunk_inputs_torch(wl, args.seed, c, dev)
            # (the last chunk of a stream may be ragged)
            cache.prefill_chunk(*qkv, out=out if qkv[0].shape == out.shape else torch.empty_like(qkv[0]))
        torch.cuda.synchronize()
        prof2 = B.cascade_profile_end(cache.ctx)
        breakdown = {k: v[0] / max(v[1], 1) for k, v in prof2.items() if v[1]}
        upd_ms, upd_n = prof2["update"]
        moved = int((cache.read_state().accepted - acc0).sum()) * wl.n_kv_heads * wl.batch
    # cache update (Alg. 2 as row moves): rows that arrived at an accepting step of a cascade (the
    # host-visible count; a token that wins a selection moves one more row, so this is a lower
    # bound).  Two bases: `roofline_update` counts the algorithmic bytes of a move,
    # 520 B per row (K, V, score, id) read once and written once; `bytes_incl_rotated_copy`
    # also counts the rotated key copy the library writes for its own use.
    esz = 2 if wl.dtype == "bf16" else 4
    row_bytes = 2 * d * esz + 8
    upd_rate = moved * 2 * row_bytes / (upd_ms / 1e3) if upd_ms > 0 else 0.0
    upd_rate_incl = moved * (2 * row_bytes + d * esz) / (upd_ms / 1e3) if upd_ms > 0 else 0.0
    attn_ms, attn_n = prof["attention"]
    avg_s = attn_ms / 1e3 / max(attn_n, 1)
    achieved = (sum(flops) / K) / avg_s
    rows_first, rows_last = n_before[W], n_before[W + K - 1]
    if min(rows_first, rows_last) < wl.n_slots and wl.name == HEADLINE:     # cannot happen after the setup above
        print(f"bench.py: timed chunks saw {rows_first}..{rows_last} cached rows, below the {wl.n_slots} slots", file=sys.stderr)
        sys.exit(3)
    res = {
        "setup_chunks": F, "timed_chunks": [W, W + K], "cache_rows_first_timed": rows_first, "cache_rows_last_timed": rows_last,
        "tokens_per_s": tokens / seconds, "ms_per_step": seconds * 1e3 / K,
        "kernel_ms_per_step": dict(breakdown, attention=avg_s * 1e3),
        "kernel_ms_per_step_source": f"attention: events in the timed chunks; the others: an untimed pass over the {K2} chunks that follow, every family bracketed by events",
        "roofline": {"bound": "mfma", "kernel": "attn_stream_kernel", "achieved": achieved / 1e12,
                     "peak": MFMA_BF16_PEAK / 1e12, "unit": "TFLOP/s", "frac": achieved / MFMA_BF16_PEAK,
                     "traffic": stored_traffic("attn_stream_kernel_prefill_1m_hbm_traffic.json") if wl.name == "prefill_1m" else None,
                     "traffic_source": "profiles/attn_stream_kernel_prefill_1m_hbm_traffic.json (rocprofv3 --pmc runs, not this run)",
                     "flop_per_launch": sum(flops) / K, "avg_launch_ms": avg_s * 1e3},
        "end_to_end_mfma_frac": (sum(flops) / seconds) / MFMA_BF16_PEAK,
        "roofline_update": {"bound": "hbm", "kernel": "gather_direct_kernel + scatter_kernel (plan_kernel + gather_kernel + scatter_kernel when a ring turns over within one chunk)",
                            "achieved": upd_rate / 1e9, "peak": HBM_PEAK / 1e9, "unit": "GB/s", "frac": upd_rate / HBM_PEAK,
                            "basis": f"rows moved x {row_bytes} B (K, V, score, id) read once and written once",
                            "achieved_incl_rotated_copy": upd_rate_incl / 1e9,
                            "rows_moved_per_step": moved / max(K2, 1), "rows_moved_per_timed_step": moved_timed / max(K, 1),
                            "avg_ms_per_step": upd_ms / max(upd_n, 1)},
    }
    return res, cache, [chunks[c] for c in sorted(chunks)], cfg


def cpu_baseline(args, torch, B, wl, cache, cfg, chunks):
    """The oracle as it stands, timed on the host cores on a bounded sample of the same workload:
    `sample_tokens` tokens against the cache the GPU run ended with, all KV heads."""
    import numpy as np
    from oracle import OracleConfig, OracleSeq
    st = cache.read_state(with_kv=True)
    o = OracleSeq(OracleConfig(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.n_sink, list(wl.cascade_sizes),
                               float(np.float32(wl.ema_beta)), wl.rope_base))
    n = st.count
    for g in range(wl.n_kv_heads):
        o.set_state(g, st.ids[0, g, :n].astype(np.int64), st.mu[0, g, :n].astype(np.float64), st.counts,
                    st.k[0, g, :n], st.v[0, g, :n], st.t, st.n_seen)
    m = args.cpu_sample_tokens
    q, k, v = (x[0, :m].float().cpu().numpy() for x in chunks[-1])
    t0 = time.perf_counter()
    o.chunk(q, k, v)
    dt = time.perf_counter() - t0
    threads = min(int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)), wl.n_kv_heads)
    o.close()
    return {"value": m / dt, "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": f"{m} tokens of {wl.name} against the {n}-row cache the GPU run ended with, "
                      f"all {wl.n_kv_heads} KV heads ({dt:.1f} s)"}


def decode_bench(args, torch, B):
    from paper_2406_17808_amd.cache import CascadeKVCache, config_of
    from paper_2406_17808_amd.workloads import WORKLOADS
    wl = WORKLOADS["decode_b32"]
    dev = "cuda:0"
    cfg = config_of(wl, max_chunk=1)
    slots, d = wl.n_slots, wl.head_dim
    gen = torch.Generator(device=dev)
    gen.manual_seed(args.seed + 12345)
    shape = (wl.batch, wl.n_kv_heads, slots, d)
    k0 = torch.randn(shape, generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    v0 = torch.randn(shape, generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    mu0 = torch.rand(shape[:3], generator=gen, device=dev, dtype=torch.float32)
    total = 4 * slots
    ids0 = torch.cat([torch.arange(wl.n_sink), torch.arange(total - (slots - wl.n_sink), total)]).to(torch.int32)
    ids0 = ids0.to(dev).expand(wl.batch, wl.n_kv_heads, slots).contiguous()
    st = B.cascade_init_state()
    st.dev_k, st.dev_v, st.dev_mu, st.dev_ids = k0.data_ptr(), v0.data_ptr(), mu0.data_ptr(), ids0.data_ptr()
    st.counts[0] = wl.n_sink
    for i, c in enumerate(wl.cascade_sizes):
        st.counts[1 + i] = c
    st.t, st.n_seen = total - wl.n_sink, total
    cache = CascadeKVCache(cfg, dev, st)
    torch.cuda.synchronize()
    del k0, v0
    steps, warm = args.decode_steps, args.decode_warmup
    n_in = 64   # distinct step inputs, cycled
    qs = torch.randn((n_in, wl.batch, wl.n_q_heads, d), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    ks = torch.randn((n_in, wl.batch, wl.n_kv_heads, d), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    vs = torch.randn((n_in, wl.batch, wl.n_kv_heads, d), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    out = torch.empty_like(qs[0])
    for i in range(warm):
        cache.decode_step(qs[i % n_in], ks[i % n_in], vs[i % n_in], out=out)
    torch.cuda.synchronize()
    B.cascade_profile_begin(cache.ctx, ["decode_qk"])     # the timed steps bracket the roofline kernel only
    t0 = time.perf_counter()
    for i in range(warm, warm + steps):
        cache.decode_step(qs[i % n_in], ks[i % n_in], vs[i % n_in], out=out)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = B.cascade_profile_end(cache.ctx)
    B.cascade_profile_begin(cache.ctx)                     # untimed: every family
    for i in range(warm + steps, warm + steps + 32):
        cache.decode_step(qs[i % n_in], ks[i % n_in], vs[i % n_in], out=out)
    torch.cuda.synchronize()
    prof2 = B.cascade_profile_end(cache.ctx)
    BH = wl.batch * wl.n_kv_heads
    # algorithmic bytes of a step: every cached K and V row once, scores read and written once
    bytes_step = BH * slots * (2 * d * 2 + 8)
    qk_ms, qk_n = prof["decode_qk"]
    k_bytes = BH * slots * d * 2
    res = {
        "decode_step_us": dt / steps * 1e6, "decode_steps": steps, "decode_tokens_per_s": wl.batch * steps / dt,
        "decode_hbm_frac": bytes_step / (dt / steps) / HBM_PEAK,
        "decode_kernel_us": {k: v[0] / max(v[1], 1) * 1e3 for k, v in prof2.items() if v[1]},
        "roofline_decode": {"bound": "hbm", "kernel": "decode_qk_stream_kernel", "achieved": k_bytes / (qk_ms / 1e3 / max(qk_n, 1)) / 1e9,
                            "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                            "frac": k_bytes / (qk_ms / 1e3 / max(qk_n, 1)) / HBM_PEAK,
                            "traffic": stored_traffic("decode_qk_stream_kernel_decode_b32_hbm_traffic.json"),
                            "traffic_source": "profiles/decode_qk_stream_kernel_decode_b32_hbm_traffic.json (rocprofv3 --pmc runs, not this run)"},
    }
    cache.close()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="prefill_1m")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--cpu-sample-tokens", type=int, default=640)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--score-mode", choices=["exact", "single_pass"], default="exact",
                    help="exact: the EMA scores use the final softmax probabilities (default, the mode parity is stated for); "
                         "single_pass: the scores of Alg. 3, accumulated inside the attention kernel")
    ap.add_argument("--no-decode", action="store_true")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the untimed leg that measures read / copy / MFMA ceilings")
    ap.add_argument("--only-decode", action="store_true")
    ap.add_argument("--decode-steps", type=int, default=256)
    ap.add_argument("--decode-warmup", type=int, default=16)
    ap.add_argument("--copy-calibration-mib", type=int, default=0,
                    help="profiler runs: also do a plain device copy of this size (scales the HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this path runs on ONE GPU (no collectives, no sharding); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2406_17808_amd import binding as B
    from paper_2406_17808_amd.workloads import WORKLOADS
    B.load_library()   # fails loudly if the HIP library has not been built
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    wl = WORKLOADS[args.workload]
    if args.copy_calibration_mib:
        calibration_copy(torch, args.copy_calibration_mib)
    if args.only_decode:   # development aid: the decode section alone, not the contract line
        print(json.dumps(decode_bench(args, torch, B)))
        return
    ceilings = None if args.no_ceilings else measured_ceilings(torch, B)
    res, cache, chunks, cfg = prefill_bench(args, torch, B, wl)
    line = {
        "metric": "prefill_tokens_per_s_per_layer", "value": res["tokens_per_s"], "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "seq_len": wl.seq_len, "chunk": wl.chunk, "n_sink": wl.n_sink,
                   "cascades": list(wl.cascade_sizes), "n_q_heads": wl.n_q_heads, "n_kv_heads": wl.n_kv_heads,
                   "head_dim": wl.head_dim, "ema_beta": wl.ema_beta, "score_mode": args.score_mode, "n_slots": wl.n_slots, "setup_chunks": res["setup_chunks"],
                   "timed_chunks": res["timed_chunks"], "cache_rows_first_timed": res["cache_rows_first_timed"],
                   "cache_rows_last_timed": res["cache_rows_last_timed"]},
        "roofline": res["roofline"], "kernel_ms_per_step": res["kernel_ms_per_step"],
        "end_to_end_mfma_frac": res["end_to_end_mfma_frac"], "roofline_update": res["roofline_update"],
    }
    if ceilings is not None:
        line["measured_ceilings"] = ceilings
        line["roofline"]["frac_of_measured_mfma"] = line["roofline"]["achieved"] / ceilings["mfma_bf16_tflops"]
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(args, torch, B, wl, cache, cfg, chunks)
    cache.close()
    del cache, chunks
    torch.cuda.empty_cache()
    if not args.no_decode:
        line.update(decode_bench(args, torch, B))
        if ceilings is not None:
            # the dominant decode kernel writes one byte of logits for every sixteen of keys it reads: next to
            # the plain streaming reads, the ceiling of that very mix (rate of the bytes read, as `achieved` is
            # the rate of the key bytes)
            rd = max(ceilings["hbm_read_gb_s"], ceilings["hbm_read_regions_gb_s"])
            line["roofline_decode"]["frac_of_measured_read"] = line["roofline_decode"]["achieved"] / rd
            line["roofline_decode"]["frac_of_measured_read_with_stores"] = (line["roofline_decode"]["achieved"]
                                                                            / ceilings["hbm_read_with_1_16_stores_gb_s"])
            line["decode_frac_of_measured_read"] = line["decode_hbm_frac"] * HBM_PEAK / 1e9 / rd
            # the whole step against its two passes as traffic alone (a read with stores, then a plain read,
            # alternating): bytes of K and V read per second over the measured rate of that pair
            kv_rate = 2 * line["roofline_decode"]["achieved"] * (line["decode_kernel_us"]["decode_qk"] / line["decode_step_us"])
            line["decode_frac_of_measured_two_pass_read"] = kv_rate / ceilings["hbm_two_pass_read_gb_s"]
    print(json.dumps(line))


if __name__ == "__main__":
    main()
