#!/usr/bin/env python3
"""Benchmark of the mixed-batch layer step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

A step is one pass of the whole layer (RMSNorm, q/k/v projection + rotary + KV append,
attention over the paged cache, W_o, SwiGLU MLP) over one synthetic relQuery batch
that is already resident in HBM.  Consecutive steps rotate over several independent
(weights, cache) sets, as consecutive layers of a model would, so that a layer's
weights are not served from the last-level cache left warm by the previous step.
Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_FP8_TFLOPS = 5000.0    # MI355X dense fp8 MFMA (the quantised-projection variant)
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E


def build_workload(name: str):
    from paper_2601_11546_amd import workloads as W
    table = {
        "relquery_13b": W.workload_relquery_13b,                       # configs[1]: the headline workload
        "relquery_decode_13b": lambda: W.workload_relquery_13b(n_rows=256, n_prefill=0),   # a pure decode batch of one relQuery
        "relquery_32b": W.workload_relquery_32b,                       # the same batch on the 32B (5 q heads per kv head) shape
        "relquery_70b_tp4_share": lambda: W.workload_tp_share("70b_tp4"),   # one GPU's share of the 70B layer at TP = 4
        "relquery_32b_tp2_share": lambda: W.workload_tp_share("32b_tp2"),   # one GPU's share of the 32B layer at TP = 2
        "tiny": W.workload_tiny,                                       # configs[0]
        "decode_heavy_70b": W.workload_decode_heavy_70b,               # configs[2]
        "decode_only_70b": lambda: W.workload_decode_heavy_70b(with_chunk=False),
        "prefill_only_13b": W.workload_prefill_only_13b,               # configs[3]
        "decode128_13b": lambda: W.workload_decode_plus_chunk_13b(0),  # configs[4], one layer, chunk 0
    }
    for c in (512, 1024, 2048, 4096):                                  # configs[4] with a prefill chunk of c tokens
        table[f"decode128_chunk{c}_13b"] = (lambda c=c: W.workload_decode_plus_chunk_13b(c))
    import re
    m = re.fullmatch(r"prefill_chunk(\d+)_13b", name)                   # one prefill chunk of any size, no decode rows
    if m:
        table[name] = lambda: W.workload_decode_plus_chunk_13b(int(m.group(1)), n_dec=0)
    if name not in table:
        raise SystemExit(f"unknown workload {name!r}; choose from {sorted(table)}")
    wl = table[name]()
    wl.extra["bench_key"] = name          # the key profiles/traffic.json files this workload under
    return wl


def algorithmic_counts(shape, batch, kv_elem_bytes: int = 2, w_elem_bytes: int = 2) -> dict:
    """FLOPs and HBM bytes one step must do/move, counted from the definition (kv_elem_bytes: 2 for the 16-bit
    cache, 1 for the quantised one; w_elem_bytes: 2 for 16-bit projections, 1 for the quantised ones, whose inputs
    are one byte per element too)."""
    T, H, I = batch.T, shape.hidden, shape.mlp_dim
    d, nq, nkv = shape.head_dim, shape.n_q_heads, shape.n_kv_heads
    gemm = {"gemm_qkv_rope_append": 2 * T * shape.qkv_dim * H, "gemm_o": 2 * T * H * shape.q_dim,
            "gemm_gate_up": 2 * T * 2 * I * H, "gemm_down": 2 * T * H * I}
    q_len, past = batch.q_len.astype(np.int64), batch.past.astype(np.int64)
    visible = int(sum(int(q) * int(p) + int(q) * (int(q) + 1) // 2 for q, p in zip(q_len, past)))
    attn_flops = 4 * d * nq * visible
    # unique KV bytes: a shared prefix once per group, every other cached key/value once
    kv_tok = 2 * nkv * d * kv_elem_bytes
    pl = batch.prefix_len
    grouped = [p for p in range(len(pl)) if int((batch.prefix_id == p).sum()) >= 2]
    uniq_tokens = int(sum(int(pl[p]) for p in grouped))
    own_tokens = {"decode": 0, "prefill": 0}
    for r in range(batch.num_reqs):
        own = int(batch.ctx_len[r]) - (int(pl[batch.prefix_id[r]]) if batch.prefix_id[r] in grouped else 0)
        own_tokens["decode" if q_len[r] == 1 else "prefill"] += own
    uniq_tokens += own_tokens["decode"] + own_tokens["prefill"]
    wb = w_elem_bytes
    weights = shape.params * wb
    bytes_total = weights + uniq_tokens * kv_tok + 2 * T * H * 2 + T * kv_tok
    qd = nq * d
    # bytes one launch of each GEMM must move: its weights, its input, its output, its residual input
    gemm_bytes = {"gemm_qkv_rope_append": wb * (shape.qkv_dim * H + T * H) + 2 * T * shape.qkv_dim,
                  "gemm_o": wb * (H * qd + T * qd) + 2 * T * H + 4 * T * H,
                  "gemm_gate_up": wb * (2 * I * H + T * H + T * I),
                  "gemm_down": wb * (H * I + T * I) + 2 * T * H + 4 * T * H}
    return {"gemm_flops": gemm, "gemm_bytes": gemm_bytes, "attn_flops": attn_flops, "flops_total": sum(gemm.values()) + attn_flops,
            "weight_bytes": weights, "kv_unique_bytes": uniq_tokens * kv_tok, "bytes_total": bytes_total,
            "kv_decode_own_bytes": own_tokens["decode"] * kv_tok, "kv_prefill_own_bytes": own_tokens["prefill"] * kv_tok,
            "kv_naive_bytes": int(batch.ctx_len.astype(np.int64).sum()) * kv_tok}


def cpu_baseline(wl, weights, x, budget_tokens: int) -> dict:
    """The oracle, as it stands, timed on this host on a bounded sample of the same batch."""
    from oracle import relserve_oracle
    from paper_2601_11546_amd import workloads as W
    orc = relserve_oracle.load("f32")
    b = wl.batch
    # sample with the batch's own mix of prefill and decode TOKENS: the shortest prefill requests up to the prefill
    # share of the token budget, then decode requests in batch order for the rest
    pre = sorted((r for r in range(b.num_reqs) if b.q_len[r] > 1), key=lambda r: int(b.q_len[r]))
    dec = [r for r in range(b.num_reqs) if b.q_len[r] == 1]
    pre_tokens = int(b.q_len[pre].sum()) if pre else 0
    picked, tokens = [], 0
    for r in pre:
        if picked and tokens + int(b.q_len[r]) > budget_tokens * pre_tokens / max(b.T, 1):
            break
        picked.append(r)
        tokens += int(b.q_len[r])
    n_pre = len(picked)
    want_dec = max(1 if dec else 0, int(round(tokens * (b.T - pre_tokens) / pre_tokens))) if pre_tokens else budget_tokens
    picked += dec[:want_dec]
    picked.sort()
    sub = b.select(picked)
    rows = b.token_rows(picked)
    kp, vp = W.make_cache(wl.shape, b.num_pages, wl.seed)
    t0 = time.perf_counter()
    orc.layer_step(wl.shape, sub, weights, x[rows], kp, vp)
    dt = time.perf_counter() - t0
    del n_pre
    return {"value": sub.T / dt, "unit": "tokens/s", "cores": orc.num_threads, "kind": "oracle",
            "seconds": round(dt, 3),
            "sample": f"{len(picked)} of {b.num_reqs} requests of the same batch ({sub.T} of {b.T} query tokens: "
                      f"{int((sub.q_len > 1).sum())} prefill rows, {int((sub.q_len == 1).sum())} decode rows), one layer step"}


def cpu_baseline_tiny_single_thread() -> dict:
    """The whole tiny configuration (configs[0]) through the oracle on ONE host thread."""
    import ctypes
    from oracle import relserve_oracle
    from paper_2601_11546_amd import workloads as W
    orc = relserve_oracle.load("f32")
    omp = ctypes.CDLL("libgomp.so.1")
    omp.omp_get_max_threads.restype = ctypes.c_int
    before = omp.omp_get_max_threads()
    wl = W.workload_tiny()
    x = W.make_activations(wl.batch.T, wl.shape.hidden, wl.seed)
    weights = wl.weights()
    omp.omp_set_num_threads(1)
    try:
        best = float("inf")
        for _ in range(3):
            kp, vp = W.make_cache(wl.shape, wl.batch.num_pages, wl.seed)
            t0 = time.perf_counter()
            orc.layer_step(wl.shape, wl.batch, weights, x, kp, vp)
            best = min(best, time.perf_counter() - t0)
    finally:
        omp.omp_set_num_threads(before)
    return {"workload": "tiny", "query_tokens": wl.batch.T, "seconds": round(best, 5), "tokens_per_s": round(wl.batch.T / best, 1),
            "cores": 1}


def peak_probes(rs, torch) -> dict:
    """What this GPU sustains (not the figures fractions are reported against): a loop of independent
    32x32x16 bf16 MFMAs on random operands, and a streaming read of 4 GiB."""
    sink = torch.zeros(64, dtype=torch.float32, device="cuda")
    buf = torch.empty(1 << 32, dtype=torch.uint8, device="cuda")
    buf.view(torch.int32).random_()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    rs.relserve_peak_probe_mfma(sink, 2000)
    rs.relserve_peak_probe_stream(buf, buf.numel(), sink)
    torch.cuda.synchronize()
    best_tf, best_gb = 0.0, 0.0
    for _ in range(3):
        e0.record()
        flops = rs.relserve_peak_probe_mfma(sink, 100000)
        e1.record()
        torch.cuda.synchronize()
        best_tf = max(best_tf, flops / (e0.elapsed_time(e1) * 1e-3) / 1e12)
        e0.record()
        rs.relserve_peak_probe_stream(buf, buf.numel(), sink)
        e1.record()
        torch.cuda.synchronize()
        best_gb = max(best_gb, buf.numel() / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    del buf
    return {"mfma_issue_loop_tflops": round(best_tf, 1), "stream_read_gbs": round(best_gb, 1),
            "note": "random bf16 operands, 16 independent accumulators per wave; 4 GiB read with 16-byte non-temporal loads"}


def stream_patterns(rs, torch) -> dict:
    """A 4 GiB read of HBM in five access patterns (relserve_peak_probe_stream_pattern): what the choice of the
    non-temporal hint for bytes that are read once rests on."""
    names = ["grid-stride, plain 16-byte loads", "32 KB pieces per workgroup, plain loads", "32 KB pieces, non-temporal loads",
             "32 KB pieces direct to LDS, plain", "32 KB pieces direct to LDS, non-temporal"]
    sink = torch.zeros(64, dtype=torch.float32, device="cuda")
    buf = torch.empty(1 << 32, dtype=torch.uint8, device="cuda")
    buf.view(torch.int32).random_()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    out = {}
    for pat, name in enumerate(names):
        best = 0.0
        for _ in range(5):
            e0.record()
            rs.relserve_peak_probe_stream_pattern(buf, buf.numel(), pat, sink)
            e1.record()
            torch.cuda.synchronize()
            best = max(best, buf.numel() / (e0.elapsed_time(e1) * 1e-3) / 1e9)
        out[name] = round(best, 1)
    return {"metric": "stream_read_gbs", "bytes": buf.numel(), "best_of": 5, "patterns": out}


def model_step_bench(args, rs, W, torch) -> dict:
    """The model step (Sec. 2.3 "LLM Inference": embedding, layer stack, output layer on the last hidden states)
    at full depth.  Weights and caches are drawn on the device (a 40-layer 13B stack with 128 contexts of 1024
    tokens is 25 GB of weights and 107 GB of KV cache); values follow the same distributions as the
    host-seeded workloads, seeded with torch's generator."""
    wl = build_workload(args.workload)
    shape, b, n_layers, vocab = wl.shape, wl.batch, args.model_layers, 32000
    g = torch.Generator(device="cuda")
    g.manual_seed(wl.seed)

    def randn(*size, std=1.0, mean=0.0):
        return (torch.randn(*size, generator=g, device="cuda", dtype=torch.float32) * std + mean).to(torch.bfloat16)

    H, I, qd, qkv = shape.hidden, shape.mlp_dim, shape.n_q_heads * shape.head_dim, shape.qkv_dim
    res_std = 0.02 / (2 * n_layers) ** 0.5
    layers, caches = [], []
    pool = (b.num_pages, shape.page_size, shape.n_kv_heads, shape.head_dim)
    for _ in range(n_layers):
        w = {"w_in_norm": randn(H, std=0.02, mean=1.0), "w_qkv": randn(qkv, H, std=0.02), "w_o": randn(H, qd, std=res_std),
             "w_post_norm": randn(H, std=0.02, mean=1.0), "w_gate_up": randn(2 * I, H, std=0.02), "w_down": randn(H, I, std=res_std)}
        if args.w8a8:
            from paper_2601_11546_amd import duration_model
            w = duration_model.quantise_layer_on_device(torch, w)
            layers.append(w if args.row_major_weights else rs.pack_layer_weights_w8a8(w))
        else:
            layers.append(w if args.row_major_weights else rs.pack_layer_weights(w))
        caches.append((randn(*pool), randn(*pool)))
    model = {"embedding": randn(vocab, H), "layers": layers, "caches": caches, "w_final_norm": randn(H, std=0.02, mean=1.0),
             "w_lm_head": randn(vocab, H, std=0.02)}
    ids = torch.randint(0, vocab, (b.T,), generator=g, device="cuda", dtype=torch.int32)
    layer = rs.relserve_layer_create(shape)
    pb = rs.relserve_batch_prepare(layer, b)
    ws = torch.empty(rs.relserve_model_workspace_bytes(layer, b.T, b.num_reqs), dtype=torch.uint8, device="cuda")
    logits = torch.empty(b.num_reqs, vocab, dtype=torch.float32, device="cuda")
    steps, warm = max(1, min(args.steps, 10)), max(1, min(args.warmup, 2))
    for _ in range(warm):
        rs.relserve_model_step(layer, pb, model, ids, logits, ws)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        rs.relserve_model_step(layer, pb, model, ids, logits, ws)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / steps * 1e3
    assert bool(torch.isfinite(logits).all())
    c = algorithmic_counts(shape, b, 2, 1 if args.w8a8 else 2)
    peak = PEAK_FP8_TFLOPS if args.w8a8 else PEAK_BF16_TFLOPS
    flops = n_layers * c["flops_total"] + 2 * b.num_reqs * vocab * H
    nbytes = n_layers * c["bytes_total"] + (vocab * H + b.T * H) * 2
    hbm = torch.cuda.max_memory_allocated() / 1e9
    return {"metric": "model_step_tokens_per_s", "value": round(b.T / (ms * 1e-3), 1), "unit": "tokens/s", "n_gpus": 1,
            "steps": steps, "warmup": warm, "ms_per_step": round(ms, 3), "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "fp8 (1-4-3) projections, bf16 elsewhere" if args.w8a8 else "bf16",
            "data": "synthetic (drawn on the device)",
            "config": {"workload": f"model_step_{wl.name}" + ("_w8a8" if args.w8a8 else ""), "layers": n_layers, "vocab": vocab, "query_tokens": b.T,
                       "requests": b.num_reqs, "weight_layout": "row-major" if args.row_major_weights else "packed",
                       "hbm_allocated_gb": round(hbm, 1)},
            "step": {"ms_per_layer": round(ms / n_layers, 4), "tflops": round(flops / (ms * 1e-3) / 1e12, 1),
                     "frac_mfma_peak": round(flops / (ms * 1e-3) / 1e12 / peak, 4),
                     "algorithmic_gbs": round(nbytes / (ms * 1e-3) / 1e9, 1),
                     "frac_hbm_peak": round(nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)}}


def serve_gpu(rs, W, w8a8: bool = False) -> dict:
    """The scheduler loop with its batches executed on the GPU (Sec. 4.1): FCFS against the RelServe policy."""
    from paper_2601_11546_amd import duration_model, scheduler, serving
    layers, vocab = 4, 32000
    fit = duration_model.run(n_prefill=32, decode_sizes=(1, 16, 32, 64, 96, 128, 160, 192, 224, 256), steps=3, warmup=1, w8a8=w8a8)
    mp = {k: fit["prefill"]["uncached_tokens"][k] * layers for k in ("alpha", "beta")}     # what the policy predicts with
    md = {k: fit["decode"]["requests"][k] * layers for k in ("alpha", "beta")}
    lim = scheduler.Limits(cap=65536, max_num_seqs=256, max_num_batched_tokens=8192)
    worker = serving.GpuWorker(W.LLAMA_13B, layers, vocab, num_pages=6144, max_tokens=8192 + 1200, max_reqs=256, seed=5, w8a8=w8a8)
    rows = []
    for rate in (20.0, 40.0, 60.0, 80.0):
        trace = scheduler.poisson_trace(80, rate, seed=int(rate))
        row = {"relqueries_per_s": rate}
        for policy in ("fcfs", "relserve"):
            t0 = time.perf_counter()
            kw = {"starvation_threshold": 0.2} if policy == "relserve" else {}
            res = scheduler.serve(trace, mp, md, policy, lim, execute=worker, **kw)
            row[policy + "_mean_latency_s"] = round(res["mean_latency"], 4)
            row[policy + "_batches"] = len(res["log"])
            row[policy + "_wall_s"] = round(time.perf_counter() - t0, 1)
            worker.cache.check()
            assert not worker.pages
        row["ratio"] = round(row["fcfs_mean_latency_s"] / row["relserve_mean_latency_s"], 3)
        rows.append(row)
    return {"metric": "mean_relquery_latency_s", "clock": "sum of the measured GPU durations of the executed batches",
            "model": f"13B layer shape x {layers} layers, vocab {vocab}, random-init" + (", quantised projections" if w8a8 else ""),
            "prefill_model": mp, "decode_model": md,
            "trace": "80 relQueries per run, 1-100 requests each, templates 256-1024 tokens, suffixes 30-120, output 5 or 50 tokens",
            "prefix_cache": {"tokens_served_from_cache": worker.cache.hits, "tokens_computed": worker.cache.misses},
            "results": rows}


def _stats(ms: list) -> dict:
    a = np.sort(np.asarray(ms, np.float64))
    return {"median": round(float(np.median(a)), 4), "p10": round(float(np.percentile(a, 10)), 4),
            "p90": round(float(np.percentile(a, 90)), 4), "min": round(float(a[0]), 4), "max": round(float(a[-1]), 4),
            "repeats": len(a)}


def measure_layer_step(rs, W, torch, args, wl, host_draws: bool, kv_fp8: bool = False, w8a8: bool = False) -> dict:
    """Times the layer step of one workload.  host_draws: weights, cache and activations are the seeded host draws the
    parity tests use (needed for the oracle leg); otherwise they are drawn on the device from the same distributions.
    w8a8: the quantised-projection variant (8-bit codes of the same weight distribution, one scale per output row)."""
    shape, b = wl.shape, wl.batch
    counts = algorithmic_counts(shape, b, 1 if kv_fp8 else 2, 1 if w8a8 else 2)
    H, I, qd = shape.hidden, shape.mlp_dim, shape.n_q_heads * shape.head_dim
    assert not ((kv_fp8 or w8a8) and host_draws), "the quantised variants are timed on device draws"
    peak_tflops = PEAK_FP8_TFLOPS if w8a8 else PEAK_BF16_TFLOPS

    def dev(bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)

    # enough sets that the rotating working set exceeds the 256 MB last-level cache several times
    n_sets = args.layer_sets or max(2, min(4, int(np.ceil(2.5e9 / counts["weight_bytes"]))))
    packed = not args.row_major_weights and all(v % (128 if w8a8 else 64) == 0 for v in (H, qd, I))
    weights0 = x_bits = None
    pool = (b.num_pages, shape.page_size, shape.n_kv_heads, shape.head_dim)
    if host_draws:
        weights0 = wl.weights()
        x_bits = W.make_activations(b.T, H, wl.seed)
        kp, vp = W.make_cache(shape, b.num_pages, wl.seed)
        base = ({k: dev(v) for k, v in weights0.items()}, dev(kp), dev(vp))
        del kp, vp
        x = dev(x_bits)
    else:
        g = torch.Generator(device="cuda")
        g.manual_seed(wl.seed)

        def randn(*size, std=1.0, mean=0.0):
            return (torch.randn(*size, generator=g, device="cuda", dtype=torch.float32) * std + mean).to(torch.bfloat16)

        res_std = 0.02 / (2 * wl.n_layers) ** 0.5 if wl.n_layers else 0.02
        base = ({"w_in_norm": randn(H, std=0.02, mean=1.0), "w_qkv": randn(shape.qkv_dim, H, std=0.02),
                 "w_o": randn(H, qd, std=res_std), "w_post_norm": randn(H, std=0.02, mean=1.0),
                 "w_gate_up": randn(2 * I, H, std=0.02), "w_down": randn(H, I, std=res_std)}, randn(*pool), randn(*pool))
        x = randn(b.T, H)
        if kv_fp8:   # pools of 8-bit codes: exponent fields 0..11 (magnitudes under 32 code units), random signs
            def codes():
                c = torch.randint(0, 96, pool, generator=g, device="cuda", dtype=torch.uint8)
                return c | (torch.randint(0, 2, pool, generator=g, device="cuda", dtype=torch.uint8) << 7)
            base = (base[0], codes(), codes())
        if w8a8:
            from paper_2601_11546_amd import duration_model
            base = (duration_model.quantise_layer_on_device(torch, base[0]), base[1], base[2])
    # set 0 holds the draws; the other sets are row-rotated device copies of it (same values and
    # distribution at other addresses), which keeps set-up time short
    sets = []
    for i in range(n_sets):
        wts = base[0] if i == 0 else {k: (torch.roll(v, 7 * i, 0) if torch.is_tensor(v) else v) for k, v in base[0].items()}
        if packed:   # one-time conversion at model load (relserve_pack_weight); the row-major copy is dropped
            wts = rs.pack_layer_weights_w8a8(wts) if w8a8 else rs.pack_layer_weights(wts)
        sets.append((wts,
                     base[1] if i == 0 else torch.roll(base[1].view(-1, base[1].shape[-1]), 5 * i, 0).view(base[1].shape).contiguous(),
                     base[2] if i == 0 else torch.roll(base[2].view(-1, base[2].shape[-1]), 5 * i, 0).view(base[2].shape).contiguous()))
    if packed:
        base = (None, base[1], base[2])
    layer = rs.relserve_layer_create(shape)
    rs.relserve_batch_prepare(layer, b).close()          # the first call of a process also pays the runtime's set-up
    t0 = time.perf_counter()
    pb = rs.relserve_batch_prepare(layer, b)
    prepare_ms = (time.perf_counter() - t0) * 1e3
    y = torch.empty_like(x)
    ws = torch.empty(rs.relserve_workspace_bytes(layer, b.T), dtype=torch.uint8, device="cuda")

    if kv_fp8:
        sets = [(w, rs.QuantPool(k, 2.0 ** -4), rs.QuantPool(v, 2.0 ** -5)) for w, k, v in sets]

    layer_step = rs.relserve_layer_step_w8a8 if w8a8 else rs.relserve_layer_step

    def step(i):
        wts, kd, vd = sets[i % n_sets]
        layer_step(layer, pb, wts, x, y, kd, vd, ws)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    if args.calibration_copy:     # a kernel of known traffic: reads 1 GiB, writes 1 GiB
        src = torch.ones(1 << 29, dtype=torch.bfloat16, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    # untimed pass with HIP events around every kernel: the per-kernel table, and which kernel dominates
    rs.relserve_profile_enable(layer, True)
    for i in range(min(args.steps, 10)):
        step(i)
    prof = rs.relserve_profile_read(layer, reset=True)
    dom = max(prof, key=lambda n: prof[n]["ms_sum"] / prof[n]["launches"])
    # timed region: `repeats` times exactly K steps, each bracketed by a device synchronisation; HIP events (recorded
    # by the library on the launch stream) around the dominant kernel only, since every event pair costs stream time
    rs.relserve_profile_enable(layer, [dom])
    per_loop = []
    for _ in range(args.repeats):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(i)
        torch.cuda.synchronize()
        per_loop.append((time.perf_counter() - t0) / args.steps * 1e3)
    prof_timed = rs.relserve_profile_read(layer, reset=True)
    rs.relserve_profile_enable(layer, False)
    prof[dom] = prof_timed[dom]
    # the same K steps without any events, to show what the pair costs
    plain = []
    for _ in range(max(1, args.repeats // 2)):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(i)
        torch.cuda.synchronize()
        plain.append((time.perf_counter() - t0) / args.steps * 1e3)
    stats = _stats(per_loop)
    ms_step = stats["median"]

    kv_bytes = {"attn_own_keys": counts["kv_decode_own_bytes"] + counts["kv_prefill_own_bytes"],
                "attn_split": counts["kv_decode_own_bytes"], "attn_tile": counts["kv_prefill_own_bytes"]}
    kernels = {}
    for name, v in prof.items():
        avg_ms = v["ms_sum"] / v["launches"]
        k = {"avg_ms": round(avg_ms, 4), "launches": v["launches"]}
        if name in counts["gemm_flops"]:
            k["tflops"] = round(counts["gemm_flops"][name] / (avg_ms * 1e-3) / 1e12, 1)
            k["frac_mfma_peak"] = round(k["tflops"] / peak_tflops, 4)
            k["gbs"] = round(counts["gemm_bytes"][name] / (avg_ms * 1e-3) / 1e9, 1)
            k["frac_hbm_peak"] = round(k["gbs"] / PEAK_HBM_GBS, 4)
        elif kv_bytes.get(name):
            k["kv_gbs"] = round(kv_bytes[name] / (avg_ms * 1e-3) / 1e9, 1)
            k["frac_hbm_peak"] = round(k["kv_gbs"] / PEAK_HBM_GBS, 4)
        kernels[name] = k
    attn_ms = sum(kernels[n]["avg_ms"] for n in ("attn_prefix", "attn_own_keys", "attn_tile", "attn_split") if n in kernels)
    if attn_ms > 0:
        kernels["attention_all"] = {"avg_ms": round(attn_ms, 4),
                                    "tflops": round(counts["attn_flops"] / (attn_ms * 1e-3) / 1e12, 1),
                                    "kv_unique_gbs": round(counts["kv_unique_bytes"] / (attn_ms * 1e-3) / 1e9, 1)}

    step_tflops = counts["flops_total"] / (ms_step * 1e-3) / 1e12
    step_gbs = counts["bytes_total"] / (ms_step * 1e-3) / 1e9
    hbm_bound = (counts["bytes_total"] / (PEAK_HBM_GBS * 1e9)) > (counts["flops_total"] / (peak_tflops * 1e12))
    traffic, traffic_source = None, None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    key = wl.extra.get("bench_key")
    traffic_step = None
    if os.path.exists(tpath) and key:
        recorded = json.load(open(tpath)).get(key + ("_w8a8" if w8a8 else "") + ("_fp8kv" if kv_fp8 else ""), {})
        traffic, traffic_step = recorded.get(dom), recorded.get("whole_step")
        if traffic is not None:
            traffic_source = "recorded: profiles/traffic.json (rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE of an earlier run of this command)"
    dk = kernels[dom]
    if hbm_bound or dom not in counts["gemm_flops"]:
        # the dominant kernel against the bytes it must move, and the whole step beside it (also when an attention kernel
        # dominates a step whose GEMMs make it matrix-bound as a whole: that kernel's own bound is its K/V stream)
        dom_bytes = counts["gemm_bytes"].get(dom) or kv_bytes.get(dom) or 0
        roofline = {"bound": "hbm", "achieved": round(dom_bytes / (dk["avg_ms"] * 1e-3) / 1e9, 1), "peak": PEAK_HBM_GBS,
                    "unit": "GB/s", "frac": round(dom_bytes / (dk["avg_ms"] * 1e-3) / 1e9 / PEAK_HBM_GBS, 4), "traffic": traffic,
                    "traffic_source": traffic_source, "kernel": dom, "bytes_per_launch": dom_bytes, "avg_launch_ms": dk["avg_ms"],
                    "whole_step": {"achieved": round(step_gbs, 1), "frac": round(step_gbs / PEAK_HBM_GBS, 4),
                                   "bytes": counts["bytes_total"], "traffic": traffic_step}}
    else:
        roofline = {"bound": "mfma", "achieved": dk["tflops"], "peak": peak_tflops, "unit": "TFLOP/s",
                    "frac": dk["frac_mfma_peak"], "traffic": traffic, "traffic_source": traffic_source, "kernel": dom,
                    "flops_per_launch": counts["gemm_flops"][dom], "avg_launch_ms": dk["avg_ms"],
                    "whole_step": {"achieved": round(step_tflops, 1), "frac": round(step_tflops / peak_tflops, 4),
                                   "flops": counts["flops_total"], "traffic": traffic_step}}
    line = {
        "metric": "mixed_batch_layer_step_tokens_per_s", "value": round(b.T / (ms_step * 1e-3), 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "fp8 (1-4-3) projections, bf16 elsewhere" if w8a8 else "bf16", "data": "synthetic",
        "config": {"workload": wl.name + ("_w8a8" if w8a8 else "") + ("_fp8kv" if kv_fp8 else ""),
                   "projections": "8-bit codes, one scale per output row and per input tensor" if w8a8 else "bf16", "layer": f"H{shape.hidden} q{shape.n_q_heads}/kv{shape.n_kv_heads}x{shape.head_dim} "
                   f"I{shape.mlp_dim} P{shape.page_size}", "query_tokens": b.T, "requests": b.num_reqs,
                   "prefill_rows": int((b.q_len > 1).sum()), "decode_rows": int((b.q_len == 1).sum()),
                   "layer_sets_rotated": n_sets, "weight_layout": "packed" if packed else "row-major",
                   "kv_cache": "8-bit codes, one scale per pool" if kv_fp8 else "bf16", "batch_info": pb.info},
        "ms_per_step_stats": stats,
        "roofline": roofline,
        "step": {"tflops": round(step_tflops, 1), "frac_mfma_peak": round(step_tflops / peak_tflops, 4),
                 "algorithmic_gbs": round(step_gbs, 1), "frac_hbm_peak": round(step_gbs / PEAK_HBM_GBS, 4),
                 "ms_per_step_without_events": round(float(np.median(plain)), 4),
                 "batch_prepare_ms": round(prepare_ms, 3)},
        "kernels": kernels,
    }
    pb.close()
    del sets, base, ws, x, y
    torch.cuda.empty_cache()
    return {"line": line, "weights0": weights0, "x_bits": x_bits}


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="relquery_13b")
    ap.add_argument("--layer-sets", type=int, default=0, help="independent (weights, cache) sets to rotate over (0 = auto)")
    ap.add_argument("--row-major-weights", action="store_true",
                    help="feed the projections row-major [out, in] weights instead of the packed streaming layout")
    ap.add_argument("--model-layers", type=int, default=0,
                    help="time the model step (embedding, this many layers, final norm, output layer) instead of one layer step; "
                         "device-generated weights and caches, e.g. --workload decode128_13b --model-layers 40 (133 GB of HBM)")
    ap.add_argument("--duration-model", action="store_true",
                    help="instead of the benchmark line: time the 13B layer step over seeded prefill and decode batches and "
                         "print the fitted batch-duration model (slope, intercept, R^2 against uncached and total tokens)")
    ap.add_argument("--serve-sim", action="store_true",
                    help="fit the batch-duration model on this GPU (short sweep), then serve seeded Poisson traces of relQueries "
                         "on the virtual clock under the FCFS and the RelServe policies and print their mean latencies")
    ap.add_argument("--serve-gpu", action="store_true",
                    help="serve seeded Poisson traces of relQueries for real: every scheduled batch runs through "
                         "relserve_model_step on a 4-layer model of the 13B layer shape; the clock is the measured GPU time")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-peak-probes", action="store_true", help="skip the MFMA issue loop and the streaming read")
    ap.add_argument("--stream-patterns", action="store_true",
                    help="instead of the benchmark line: a 4 GiB read of HBM in five access patterns (GB/s each)")
    ap.add_argument("--kv-fp8", action="store_true", help="time the quantised-cache variant (8-bit K/V pools) of the workload")
    ap.add_argument("--w8a8", action="store_true", help="time the quantised-projection variant (8-bit codes for the four matrices and their inputs)")
    ap.add_argument("--repeats", type=int, default=9, help="how many times the K timed steps are repeated (median, p10, p90)")
    ap.add_argument("--no-regimes", action="store_true",
                    help="headline workload only (by default the line also carries the prefill-only and the decode-only regimes)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (reference for rocprofv3's FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--cpu-tokens", type=int, default=0, help="token budget of the oracle sample (0 = auto)")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py measures the layer step on ONE MI355X; this build has no multi-GPU path "
                         "(run with --gpus 1)")

    import torch
    from paper_2601_11546_amd import binding as rs
    from paper_2601_11546_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs an MI355X"
    torch.cuda.set_device(0)
    if args.stream_patterns:
        print(json.dumps(stream_patterns(rs, torch)))
        return
    if args.model_layers > 0:
        print(json.dumps(model_step_bench(args, rs, W, torch)))
        return
    if args.serve_gpu:
        print(json.dumps(serve_gpu(rs, W, args.w8a8)))
        return
    if args.serve_sim:
        from paper_2601_11546_amd import duration_model, scheduler
        fit = duration_model.run(n_prefill=32, decode_sizes=(1, 16, 32, 64, 96, 128, 160, 192, 224, 256), steps=3, warmup=1)
        layers = 40
        mp = {k: fit["prefill"]["uncached_tokens"][k] * layers for k in ("alpha", "beta")}
        md = {k: fit["decode"]["requests"][k] * layers for k in ("alpha", "beta")}
        print(json.dumps({"metric": "mean_relquery_latency_s", "model": "13B layer shape x 40 layers (durations from the fitted lines)",
                          "prefill_model": mp, "decode_model": md, "trace": "80 relQueries per run, 3 seeds, 1-100 requests each, "
                          "templates 256-1024 tokens, suffixes 30-120, output 5 or 50 tokens",
                          "results": scheduler.compare_policies(mp, md)}))
        return
    if args.duration_model:
        from paper_2601_11546_amd import duration_model
        print(json.dumps(duration_model.run(steps=max(1, min(args.steps, 10)), warmup=max(1, min(args.warmup, 3)), w8a8=args.w8a8)))
        return
    wl = build_workload(args.workload)
    variant = args.kv_fp8 or args.w8a8
    res = measure_layer_step(rs, W, torch, args, wl, host_draws=not variant, kv_fp8=args.kv_fp8, w8a8=args.w8a8)
    out = res["line"]
    if not args.no_regimes and args.workload == "relquery_13b" and not variant:
        # the two regimes the roofline targets are stated on, each with its own roofline object, and the decode-dominated
        # one on the quantised-cache variant
        out["regimes"] = {}
        for name, fp8, q8 in (("prefill_only_13b", False, False), ("decode128_13b", False, False), ("decode_only_70b", False, False),
                              ("decode128_13b", True, False), ("prefill_only_13b", False, True), ("decode128_13b", True, True)):
            r = measure_layer_step(rs, W, torch, args, build_workload(name), host_draws=False, kv_fp8=fp8, w8a8=q8)["line"]
            out["regimes"][name + ("_w8a8" if q8 else "") + ("_fp8kv" if fp8 else "")] = {"ms_per_step": r["ms_per_step"], "ms_per_step_stats": r["ms_per_step_stats"],
                                    "tokens_per_s": r["value"], "query_tokens": r["config"]["query_tokens"],
                                    "requests": r["config"]["requests"], "layer": r["config"]["layer"],
                                    "data": "synthetic (drawn on the device)", "roofline": r["roofline"], "step": r["step"],
                                    "kernels": r["kernels"]}
    if not args.no_peak_probes:
        out["measured_peaks"] = peak_probes(rs, torch)
    if not args.no_cpu_baseline and not variant:
        budget = args.cpu_tokens or max(8, int(1.6e11 / (2 * wl.shape.params)))   # about 160 GFLOP of dense work, ~10 s
        out["cpu_baseline"] = cpu_baseline(wl, res["weights0"], res["x_bits"], budget)
        out["cpu_baseline"]["tiny_single_thread"] = cpu_baseline_tiny_single_thread()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
