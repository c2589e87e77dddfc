"""Fits the batch-duration model (Sec. 4.2, Eq. 9) to layer-step durations measured on this GPU.

    from paper_2601_11546_amd import duration_model
    result = duration_model.run()          # needs an MI355X; bench.py --duration-model prints it

The paper's scheduler predicts how long a prefill or a decode batch takes from a line in the batch's
uncached tokens, or in its request count, fitted to offline runs.  This module is those offline runs:
it times `relserve_layer_step` over seeded synthetic batches and hands the points to the library's
`relserve_duration_fit`.  Durations are per layer step; a model of n layers scales both coefficients by n.
"""
from __future__ import annotations

import numpy as np

from . import binding as rs
from . import workloads as W

DECODE_SIZES = (1, 2, 4, 8, 12, 16, 24, 32, 48, 64, 80, 96, 112, 128, 144, 160, 176, 192, 208, 224, 240, 256)


def quantise_layer_on_device(torch, w: dict) -> dict:
    """A layer's four bf16 matrices as 8-bit codes of W[n, :] / s[n], s[n] = the row's largest magnitude / 448 (device
    tensors; the norm weights stay bf16; static input scales from workloads.W8A8_INPUT_SCALES)."""
    q = {"w_in_norm": w["w_in_norm"], "w_post_norm": w["w_post_norm"], **W.W8A8_INPUT_SCALES}
    for name in ("qkv", "o", "gate_up", "down"):
        wf = w["w_" + name].float()
        sc = wf.abs().amax(dim=1) / 448.0
        q["w_" + name] = (wf / sc[:, None]).clamp(-448.0, 448.0).to(torch.float8_e4m3fn).view(torch.uint8)
        q["s_" + name] = sc.contiguous()
        del wf
    return q


def device_layer_sets(torch, shape, n_sets: int, n_layers: int, seed: int, packed: bool = True, w8a8: bool = False) -> list:
    """n_sets independent random-init weight sets of one layer, drawn on the device (w8a8: with quantised projections)."""
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)

    def randn(*size, std=1.0, mean=0.0):
        return (torch.randn(*size, generator=g, device="cuda", dtype=torch.float32) * std + mean).to(torch.bfloat16)

    H, I, qd = shape.hidden, shape.mlp_dim, shape.n_q_heads * shape.head_dim
    res_std = 0.02 / (2 * n_layers) ** 0.5 if n_layers > 0 else 0.02
    sets = []
    for _ in range(n_sets):
        w = {"w_in_norm": randn(H, std=0.02, mean=1.0), "w_qkv": randn(shape.qkv_dim, H, std=0.02),
             "w_o": randn(H, qd, std=res_std), "w_post_norm": randn(H, std=0.02, mean=1.0),
             "w_gate_up": randn(2 * I, H, std=0.02), "w_down": randn(H, I, std=res_std)}
        if w8a8:
            w = quantise_layer_on_device(torch, w)
            sets.append(rs.pack_layer_weights_w8a8(w) if packed else w)
        else:
            sets.append(rs.pack_layer_weights(w) if packed else w)
    return sets


def measure(torch, shape, batches, weight_sets, steps: int = 5, warmup: int = 2, seed: int = 0) -> np.ndarray:
    """Seconds per layer step of every batch (tensors resident; consecutive steps rotate over the weight sets)."""
    g = torch.Generator(device="cuda")
    g.manual_seed(seed + 17)
    t_max = max(b.T for b in batches)
    pages = max(b.num_pages for b in batches)
    pool = (pages, shape.page_size, shape.n_kv_heads, shape.head_dim)
    k_pages = torch.randn(*pool, generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    v_pages = torch.randn(*pool, generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    x_all = torch.randn(t_max, shape.hidden, generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    y_all = torch.empty_like(x_all)
    layer = rs.relserve_layer_create(shape)
    step = rs.relserve_layer_step_w8a8 if "s_qkv" in weight_sets[0] else rs.relserve_layer_step
    ws = torch.empty(rs.relserve_workspace_bytes(layer, t_max), dtype=torch.uint8, device="cuda")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    out = np.zeros(len(batches))
    n = 0
    if batches:     # the process's first steps also pay one-time costs of the runtime (first launches, clocks): not timed
        pb = rs.relserve_batch_prepare(layer, batches[0])
        for _ in range(len(weight_sets) + warmup):
            step(layer, pb, weight_sets[n % len(weight_sets)], x_all[:batches[0].T], y_all[:batches[0].T], k_pages, v_pages, ws)
            n += 1
        torch.cuda.synchronize()
        pb.close()
    for i, b in enumerate(batches):
        pb = rs.relserve_batch_prepare(layer, b)
        x, y = x_all[:b.T], y_all[:b.T]
        for _ in range(warmup):
            step(layer, pb, weight_sets[n % len(weight_sets)], x, y, k_pages, v_pages, ws)
            n += 1
        e0.record()
        for _ in range(steps):
            step(layer, pb, weight_sets[n % len(weight_sets)], x, y, k_pages, v_pages, ws)
            n += 1
        e1.record()
        torch.cuda.synchronize()
        out[i] = e0.elapsed_time(e1) * 1e-3 / steps
        pb.close()
    layer.close()
    return out


def _fit(units, seconds) -> dict:
    m = rs.relserve_duration_fit(units, seconds)
    pred = np.array([rs.relserve_duration_predict(m, u) for u in units])
    m["mean_abs_rel_error"] = float(np.mean(np.abs(pred - seconds) / seconds))
    return m


def run(n_prefill: int = 64, decode_sizes=DECODE_SIZES, shape=W.LLAMA_13B, n_layers: int = 40, steps: int = 5,
        warmup: int = 2, seed: int = 1100, max_tokens: int = 8192, w8a8: bool = False) -> dict:
    import torch
    assert torch.cuda.is_available(), "the duration model is fitted to measurements on the GPU"
    n_sets = max(2, min(4, int(np.ceil(2.5e9 / (2 * shape.params)))))
    packed = all(d % (128 if w8a8 else 64) == 0 for d in (shape.hidden, shape.n_q_heads * shape.head_dim, shape.mlp_dim))
    sets = device_layer_sets(torch, shape, n_sets, n_layers, seed, packed, w8a8)
    pre = W.duration_sweep_prefill(n_prefill, seed, max_tokens, shape=shape)
    dec = W.duration_sweep_decode(decode_sizes, seed + 100, shape=shape)
    t_pre = measure(torch, shape, pre, sets, steps, warmup, seed)
    t_dec = measure(torch, shape, dec, sets, steps, warmup, seed + 1)
    utok = np.array([W.prefill_tokens(b)[0] for b in pre], np.float64)
    total = np.array([W.prefill_tokens(b)[1] for b in pre], np.float64)
    req = np.array([b.num_reqs for b in dec], np.float64)
    return {
        "layer": f"H{shape.hidden} q{shape.n_q_heads}/kv{shape.n_kv_heads}x{shape.head_dim} I{shape.mlp_dim}"
                 + (", quantised projections" if w8a8 else ""),
        "seconds_are": "per layer step (multiply alpha and beta by the number of layers for a model step)",
        "prefill": {"uncached_tokens": _fit(utok, t_pre), "total_tokens": _fit(total, t_pre),
                    "points": [[int(u), int(t), float(s)] for u, t, s in zip(utok, total, t_pre)],
                    "point_columns": ["utok", "total_tokens", "seconds"]},
        "decode": {"requests": _fit(req, t_dec),
                   "points": [[int(r), float(s)] for r, s in zip(req, t_dec)], "point_columns": ["req", "seconds"]},
    }
