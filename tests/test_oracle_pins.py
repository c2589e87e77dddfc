"""Pins for the CPU oracle: each piece is checked against something that is not
the oracle itself -- a PyTorch/numpy library routine in fp64, a brute-force
evaluation of Eq. 4-5 (Sec. 2.3) on contiguous tensors, a closed form, or an
invariant that the paper's caching statements imply (Sec. 2.3 "KV Cache",
"Prefix Cache"; chunked prefill, Sec. 5.1 baselines).  No GPU needed.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from paper_2601_11546_amd import workloads as W
from tests.dense_reference import dense_layer, dense_model_logits, rope_complex
from tests.flows import gather_kv, make_flow, run_flow, run_model_flow

SHAPES = {"mha": W.TINY, "gqa": W.TINY_GQA, "d128": W.TINY_D128}


def oracle_stepper(oracle, shape, weights, k_pages, v_pages, what="y_f32"):
    def step(batch, x):
        res = oracle.layer_step(shape, batch, weights, x, k_pages, v_pages)
        return getattr(res, what)
    return step


# ---------------------------------------------------------------------------
# number format
# ---------------------------------------------------------------------------
def test_bf16_round_matches_torch(oracle):
    rng = np.random.default_rng(0)
    vals = np.concatenate([
        rng.standard_normal(4000).astype(np.float32) * np.float32(10.0) ** rng.integers(-30, 30, 4000).astype(np.float32),
        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, -1.00390625, 3.3895314e38, 3.4e38,
                  np.inf, -np.inf, 1e-40, 65504.0, 1.0 + 2.0 ** -8 + 2.0 ** -20], np.float32)])
    want = torch.from_numpy(vals).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([oracle.f32_to_bf16(v) for v in vals], np.uint16)
    np.testing.assert_array_equal(got, want)
    np.testing.assert_array_equal(W.f32_to_bf16_bits(vals), want)          # the input generator's rounding too
    back = np.array([oracle.bf16_to_f32(b) for b in want], np.float32)
    np.testing.assert_array_equal(back, torch.from_numpy(want.view(np.int16)).view(torch.bfloat16).float().numpy())
    assert np.isnan(oracle.bf16_to_f32(oracle.f32_to_bf16(float("nan"))))


# ---------------------------------------------------------------------------
# elementwise pieces against library routines and closed forms
# ---------------------------------------------------------------------------
def test_rmsnorm_matches_torch_and_invariants(oracle):
    rng = np.random.default_rng(1)
    x = rng.standard_normal((5, 96)).astype(np.float32) * 3
    w = W.f32_to_bf16_bits(1 + 0.1 * rng.standard_normal(96).astype(np.float32))
    got = oracle.rmsnorm(x, w, 1e-5)
    want = F.rms_norm(torch.from_numpy(x).double(), (96,), torch.from_numpy(W.bf16_bits_to_f32(w)).double(), eps=1e-5)
    np.testing.assert_allclose(got, want.numpy(), rtol=2e-6, atol=1e-6)
    # unit weights, eps -> 0: rows have unit RMS, and positive rescaling of x changes nothing
    ones = W.f32_to_bf16_bits(np.ones(96, np.float32))
    y = oracle.rmsnorm(x, ones, 0.0)
    np.testing.assert_allclose(np.sqrt((y.astype(np.float64) ** 2).mean(1)), 1.0, rtol=1e-6)
    np.testing.assert_allclose(oracle.rmsnorm(x * 7.5, ones, 0.0), y, rtol=2e-6)
    # eps sits inside the root: a zero row stays zero and a tiny row is damped by sqrt(eps)
    tiny = np.full((1, 96), 1e-4, np.float32)
    np.testing.assert_allclose(oracle.rmsnorm(tiny, ones, 1e-2), 1e-4 / np.sqrt(1e-8 + 1e-2), rtol=1e-5)


def test_linear_orientation_matches_matmul(oracle):
    rng = np.random.default_rng(2)
    Wt = W.f32_to_bf16_bits(rng.standard_normal((7, 13)).astype(np.float32))
    x = rng.standard_normal((3, 13)).astype(np.float32)
    want = x.astype(np.float64) @ W.bf16_bits_to_f32(Wt).astype(np.float64).T
    np.testing.assert_allclose(oracle.linear(Wt, x), want, rtol=1e-5, atol=1e-5)
    # a one-hot input row reads out one column of W
    e = np.zeros((1, 13), np.float32)
    e[0, 4] = 1
    np.testing.assert_array_equal(oracle.linear(Wt, e)[0], W.bf16_bits_to_f32(Wt)[:, 4])


@pytest.mark.parametrize("d", [8, 64, 128])
def test_rope_closed_forms(oracle, d):
    rng = np.random.default_rng(3)
    q = rng.standard_normal(d).astype(np.float32)
    k = rng.standard_normal(d).astype(np.float32)
    base = 10000.0
    np.testing.assert_array_equal(oracle.rope(q, 0, base), q)                       # position 0 = identity
    for pos in (1, 17, 513, 4095):
        r = oracle.rope(q, pos, base)
        want = rope_complex(torch.from_numpy(q).double()[None, None], torch.tensor([pos]), base)[0, 0]
        np.testing.assert_allclose(r, want.numpy(), rtol=0, atol=2e-6)
        np.testing.assert_allclose(np.linalg.norm(r.astype(np.float64)), np.linalg.norm(q.astype(np.float64)), rtol=1e-6)
    # <rope(q, m), rope(k, n)> depends only on m - n
    a = float(oracle.rope(q, 40, base).astype(np.float64) @ oracle.rope(k, 25, base).astype(np.float64))
    b = float(oracle.rope(q, 1015, base).astype(np.float64) @ oracle.rope(k, 1000, base).astype(np.float64))
    assert abs(a - b) < 2e-4
    # first pair turns by exactly pos radians (theta_0 = 1), the last pair hardly moves
    e = np.zeros(d, np.float32)
    e[0] = 1
    r = oracle.rope(e, 3, base)
    np.testing.assert_allclose([r[0], r[d // 2]], [np.cos(3.0), np.sin(3.0)], atol=1e-7)
    e = np.zeros(d, np.float32)
    e[d // 2 - 1] = 1
    r = oracle.rope(e, 1, base)
    th = base ** (-(d - 2) / d)
    np.testing.assert_allclose([r[d // 2 - 1], r[d - 1]], [np.cos(th), np.sin(th)], atol=1e-7)


# ---------------------------------------------------------------------------
# cache placement
# ---------------------------------------------------------------------------
def test_kv_append_slots_brute_force(oracle):
    shape = W.TINY_GQA
    wl = W.workload_tiny_prefix(shape=shape)
    b = wl.batch
    rng = np.random.default_rng(4)
    k = rng.integers(0, 2 ** 16, (b.T, shape.n_kv_heads, shape.head_dim)).astype(np.uint16)
    v = rng.integers(0, 2 ** 16, (b.T, shape.n_kv_heads, shape.head_dim)).astype(np.uint16)
    kp, vp = W.make_cache(shape, b.num_pages, 5)
    kp0, vp0 = kp.copy(), vp.copy()
    slots = oracle.kv_append(shape, b, k, v, kp, vp)
    P = shape.page_size
    want_k, want_v = kp0.reshape(-1, shape.n_kv_heads, shape.head_dim).copy(), vp0.reshape(-1, shape.n_kv_heads, shape.head_dim).copy()
    seen = set()
    for r in range(b.num_reqs):
        for j in range(b.q_len[r]):
            pos = int(b.past[r]) + j
            slot = int(b.block_table[r, pos // P]) * P + pos % P
            t = int(b.q_start[r]) + j
            assert slots[t] == slot
            assert slot not in seen
            seen.add(slot)
            want_k[slot] = k[t]
            want_v[slot] = v[t]
    np.testing.assert_array_equal(kp.reshape(want_k.shape), want_k)     # written slots hold the rows, all others untouched
    np.testing.assert_array_equal(vp.reshape(want_v.shape), want_v)
    assert len(seen) == b.T


# ---------------------------------------------------------------------------
# attention: brute force of Eq. 4-5 and closed forms
# ---------------------------------------------------------------------------
def _one_request_batch(shape, L, seed):
    return W.build_batch(shape, [1], [L], seed=seed)


@pytest.mark.parametrize("name", list(SHAPES))
def test_attention_token_brute_force(oracle, name):
    shape = SHAPES[name]
    L = 37
    b = _one_request_batch(shape, L, 6)
    kp, vp = W.make_cache(shape, b.num_pages, 7)
    rng = np.random.default_rng(8)
    q = rng.standard_normal((shape.n_q_heads, shape.head_dim)).astype(np.float32)
    kc, vc = gather_kv(shape, b.block_table[0], L, kp, vp)
    K = W.bf16_bits_to_f32(kc).astype(np.float64)
    V = W.bf16_bits_to_f32(vc).astype(np.float64)
    g = shape.n_q_heads // shape.n_kv_heads
    for pos in (0, 1, 15, 16, 36):
        got = oracle.attention_token(shape, b, 0, pos, q, kp, vp)
        for a in range(shape.n_q_heads):
            s = K[:pos + 1, a // g] @ q[a].astype(np.float64) / np.sqrt(shape.head_dim)
            alpha = np.exp(s) / np.exp(s).sum()                      # Eq. 4 exactly as printed (no max shift)
            want = alpha @ V[:pos + 1, a // g]                        # Eq. 5 before W_o
            np.testing.assert_allclose(got[a], want, rtol=2e-5, atol=2e-6)


def test_attention_closed_forms(oracle):
    shape = W.TINY
    L = 20
    b = _one_request_batch(shape, L, 9)
    kp, vp = W.make_cache(shape, b.num_pages, 10)
    rng = np.random.default_rng(11)
    q = rng.standard_normal((shape.n_q_heads, shape.head_dim)).astype(np.float32)
    kc, vc = gather_kv(shape, b.block_table[0], L, kp, vp)
    # one visible key: output is that value exactly
    got = oracle.attention_token(shape, b, 0, 0, q, kp, vp)
    np.testing.assert_array_equal(got, W.bf16_bits_to_f32(vc[0]))
    # q = 0: uniform weights, output is the mean of the visible values
    got = oracle.attention_token(shape, b, 0, L - 1, np.zeros_like(q), kp, vp)
    np.testing.assert_allclose(got, W.bf16_bits_to_f32(vc).astype(np.float64).mean(0), rtol=1e-5, atol=1e-6)
    # all values equal: output is that row whatever the scores are
    vp2 = vp.copy()
    flat = vp2.reshape(-1, shape.n_kv_heads, shape.head_dim)
    flat[:] = vc[3]
    got = oracle.attention_token(shape, b, 0, L - 1, q, kp, vp2)
    np.testing.assert_allclose(got, W.bf16_bits_to_f32(vc[3]), rtol=1e-6, atol=1e-7)
    # two keys whose scores differ by ln 2: weights 1/3 and 2/3 (scale 1/sqrt(d) included)
    shape2 = W.LayerShape(8, 1, 1, 4, 8, page_size=2)
    b2 = _one_request_batch(shape2, 2, 12)
    kp2 = np.zeros((b2.num_pages, 2, 1, 4), np.uint16)
    vp2 = np.zeros_like(kp2)
    P = 2
    s0, s1 = (int(b2.block_table[0, p // P]) * P + p % P for p in (0, 1))
    kf, vf = kp2.reshape(-1, 4), vp2.reshape(-1, 4)
    kf[s1] = W.f32_to_bf16_bits(np.array([1, 0, 0, 0], np.float32))
    vf[s0] = W.f32_to_bf16_bits(np.array([3, 0, 0, 0], np.float32))
    vf[s1] = W.f32_to_bf16_bits(np.array([0, 3, 0, 0], np.float32))
    qq = np.array([[np.log(2.0) * np.sqrt(4.0), 5, 5, 5]], np.float32)
    got = oracle.attention_token(shape2, b2, 0, 1, qq, kp2, vp2)
    np.testing.assert_allclose(got[0], [1.0, 2.0, 0, 0], atol=1e-6)


# ---------------------------------------------------------------------------
# whole step against the dense library implementation
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("name", list(SHAPES))
def test_layer_step_matches_dense_recompute(oracle, oracle64, name):
    """Chunked prefill then decode through the paged oracle == each request's
    whole sequence recomputed at once with torch fp64 library routines."""
    shape = SHAPES[name]
    weights = W.make_weights(shape, 20)
    seq = [41, 23, 50]
    sched = [[(0, 30), (1, 23)], [(0, 9), (2, 17), (1, 0)][:2], [(2, 32), (0, 1)], [(0, 1), (2, 1)]]
    flow = make_flow(shape, seq, sched, seed=21)
    for orc, tol in ((oracle, 3e-4), (oracle64, 3e-4)):
        kp, vp = W.make_cache(shape, flow.num_pages, 22)
        ys = run_flow(flow, oracle_stepper(orc, shape, weights, kp, vp))
        for r, L in enumerate(seq):
            ref = dense_layer(shape, weights, flow.x_full[r])
            # keys/values in the cache are the recomputed ones up to rare 1-ulp rounding flips
            kc, vc = gather_kv(shape, flow.block_table[r], L, kp, vp)
            for got, want in ((kc, ref["k"]), (vc, ref["v"])):
                g = W.bf16_bits_to_f32(got).astype(np.float64)
                wv = want.numpy()
                assert np.mean(g == wv) > 0.995
                np.testing.assert_allclose(g, wv, rtol=2 ** -7, atol=1e-6)   # atol: cancellation in the rotation
            # with the oracle's own cached bits fed back, the rest must agree tightly
            kv = (torch.from_numpy(W.bf16_bits_to_f32(kc).astype(np.float64)),
                  torch.from_numpy(W.bf16_bits_to_f32(vc).astype(np.float64)))
            ref2 = dense_layer(shape, weights, flow.x_full[r], kv_override=kv)
            np.testing.assert_allclose(ys[r], ref2["y"].numpy(), rtol=tol, atol=tol)
            # and against the fully independent recompute within the slack of those flips
            np.testing.assert_allclose(ys[r], ref["y"].numpy(), rtol=3e-3, atol=3e-3)


def test_taps_match_dense(oracle):
    shape = W.TINY_GQA
    weights = W.make_weights(shape, 30)
    flow = make_flow(shape, [19], [[(0, 19)]], seed=31)
    kp, vp = W.make_cache(shape, flow.num_pages, 32)
    b = W.Batch(np.array([0, 19], np.int32), np.array([19], np.int32), flow.block_table, flow.prefix_id,
                flow.prefix_len, flow.num_pages)
    res = oracle.layer_step(shape, b, weights, flow.x_full[0], kp, vp)
    kc, vc = gather_kv(shape, flow.block_table[0], 19, kp, vp)
    kv = (torch.from_numpy(W.bf16_bits_to_f32(kc).astype(np.float64)),
          torch.from_numpy(W.bf16_bits_to_f32(vc).astype(np.float64)))
    ref = dense_layer(shape, weights, flow.x_full[0], kv_override=kv)
    np.testing.assert_allclose(res.attn_out, ref["attn_out"].numpy(), rtol=1e-4, atol=1e-5)
    np.testing.assert_allclose(res.x1, ref["x1"].numpy(), rtol=1e-4, atol=1e-5)
    np.testing.assert_array_equal(res.y_bf16, W.f32_to_bf16_bits(res.y_f32))
    # row selection returns the same rows
    sel = np.array([18, 0, 7], np.int32)
    kp2, vp2 = W.make_cache(shape, flow.num_pages, 32)
    res2 = oracle.layer_step(shape, b, weights, flow.x_full[0], kp2, vp2, rows=sel)
    np.testing.assert_array_equal(res2.y_f32, res.y_f32[sel])
    np.testing.assert_array_equal(kp2, kp)


# ---------------------------------------------------------------------------
# invariants the paper's caching statements imply (exact in the oracle, reading R5)
# ---------------------------------------------------------------------------
def _run(oracle, shape, weights, flow, cache_seed=40):
    kp, vp = W.make_cache(shape, flow.num_pages, cache_seed)
    ys = run_flow(flow, oracle_stepper(oracle, shape, weights, kp, vp))
    return ys, kp, vp


@pytest.mark.parametrize("name", ["mha", "gqa"])
def test_incremental_decode_equals_full_causal(oracle, name):
    shape = SHAPES[name]
    weights = W.make_weights(shape, 41)
    L = 35
    full, _, _ = _run(oracle, shape, weights, make_flow(shape, [L], [[(0, L)]], seed=42))
    inc, _, _ = _run(oracle, shape, weights, make_flow(shape, [L], [[(0, 1)] for _ in range(L)], seed=42))
    np.testing.assert_array_equal(inc[0], full[0])


def test_chunked_prefill_equals_one_shot(oracle):
    shape = W.TINY
    weights = W.make_weights(shape, 43)
    L = 128
    one, kp1, vp1 = _run(oracle, shape, weights, make_flow(shape, [L], [[(0, L)]], seed=44))
    for chunks in ([64, 64], [1, 127], [50, 30, 48]):
        ys, kp, vp = _run(oracle, shape, weights, make_flow(shape, [L], [[(0, c)] for c in chunks], seed=44))
        np.testing.assert_array_equal(ys[0], one[0])
        np.testing.assert_array_equal(kp, kp1)
        np.testing.assert_array_equal(vp, vp1)


def test_page_permutation_leaves_outputs_unchanged(oracle):
    shape = W.TINY_GQA
    weights = W.make_weights(shape, 45)
    seq = [40, 21, 33]
    sched = [[(0, 40), (1, 20)], [(1, 1), (2, 33)]]
    f1 = make_flow(shape, seq, sched, seed=46)
    f2 = make_flow(shape, seq, sched, seed=46, page_perm_seed=999)
    assert not np.array_equal(f1.block_table, f2.block_table)
    y1, kp1, vp1 = _run(oracle, shape, weights, f1)
    y2, kp2, vp2 = _run(oracle, shape, weights, f2)
    for r, L in enumerate(seq):
        np.testing.assert_array_equal(y1[r], y2[r])
        a = gather_kv(shape, f1.block_table[r], L, kp1, vp1)
        b = gather_kv(shape, f2.block_table[r], L, kp2, vp2)
        np.testing.assert_array_equal(a[0], b[0])
        np.testing.assert_array_equal(a[1], b[1])


def test_page_size_independence(oracle):
    weights = W.make_weights(W.TINY, 47)
    outs = []
    for P in (8, 16, 32):
        shape = W.LayerShape(256, 4, 4, 64, 688, page_size=P)
        ys, _, _ = _run(oracle, shape, weights, make_flow(shape, [45, 30], [[(0, 44), (1, 30)], [(0, 1)]], seed=48))
        outs.append(ys)
    for ys in outs[1:]:
        for a, b in zip(ys, outs[0]):
            np.testing.assert_array_equal(a, b)


def test_shared_prefix_equals_private_recompute(oracle):
    """One copy of the template's keys/values referenced by several block tables
    gives the same outputs as every request prefilling its own copy."""
    shape = W.TINY_GQA
    weights = W.make_weights(shape, 49)
    P = shape.page_size
    pl = 2 * P
    seq = [pl + 20, pl + 7, pl + 13]
    # shared: request 0 writes the prefix once, the others start after it
    shared = make_flow(shape, seq, [[(0, pl + 20)], [(1, 7), (2, 13)]], seed=50, shared_prefix=(pl, [0, 1, 2]),
                       start=[0, pl, pl])
    assert np.array_equal(shared.block_table[0, :2], shared.block_table[1, :2])
    ys_s, _, _ = _run(oracle, shape, weights, shared)
    private = make_flow(shape, seq, [[(0, pl + 20), (1, pl + 7), (2, pl + 13)]], seed=50)
    private.x_full = shared.x_full
    ys_p, _, _ = _run(oracle, shape, weights, private)
    np.testing.assert_array_equal(ys_s[0], ys_p[0])
    np.testing.assert_array_equal(ys_s[1][pl:], ys_p[1][pl:])
    np.testing.assert_array_equal(ys_s[2][pl:], ys_p[2][pl:])


def test_batch_order_independence(oracle):
    shape = W.TINY
    weights = W.make_weights(shape, 51)
    seq = [30, 12, 25, 1]
    y1, _, _ = _run(oracle, shape, weights, make_flow(shape, seq, [[(0, 30), (1, 12), (2, 25), (3, 1)]], seed=52))
    y2, _, _ = _run(oracle, shape, weights, make_flow(shape, seq, [[(3, 1), (2, 25), (0, 30), (1, 12)]], seed=52))
    for a, b in zip(y1, y2):
        np.testing.assert_array_equal(a, b)


def test_gqa_equals_mha_with_replicated_kv_heads(oracle):
    gqa = W.TINY_GQA
    mha = W.LayerShape(gqa.hidden, gqa.n_q_heads, gqa.n_q_heads, gqa.head_dim, gqa.mlp_dim)
    wg = W.make_weights(gqa, 53)
    d, rep = gqa.head_dim, gqa.n_q_heads // gqa.n_kv_heads
    qkv = wg["w_qkv"]
    wq = qkv[:gqa.q_dim]
    wk = qkv[gqa.q_dim:gqa.q_dim + gqa.kv_dim].reshape(gqa.n_kv_heads, d, -1)
    wv = qkv[gqa.q_dim + gqa.kv_dim:].reshape(gqa.n_kv_heads, d, -1)
    wm = dict(wg)
    wm["w_qkv"] = np.concatenate([wq, np.repeat(wk, rep, 0).reshape(-1, gqa.hidden),
                                  np.repeat(wv, rep, 0).reshape(-1, gqa.hidden)], 0)
    seq, sched = [26, 9], [[(0, 25), (1, 9)], [(0, 1)]]
    yg, _, _ = _run(oracle, gqa, wg, make_flow(gqa, seq, sched, seed=54))
    ym, _, _ = _run(oracle, mha, wm, make_flow(mha, seq, sched, seed=54))
    for a, b in zip(yg, ym):
        np.testing.assert_array_equal(a, b)


def test_zero_weights_special_cases(oracle):
    shape = W.TINY
    weights = W.make_weights(shape, 55)
    flow = make_flow(shape, [18], [[(0, 18)]], seed=56)
    x = W.bf16_bits_to_f32(flow.x_full[0])
    # W_o = 0 and W_down = 0: the layer is the identity on the residual stream
    w0 = dict(weights, w_o=np.zeros_like(weights["w_o"]), w_down=np.zeros_like(weights["w_down"]))
    ys, _, _ = _run(oracle, shape, w0, flow)
    np.testing.assert_array_equal(ys[0], x)
    # zero gate rows: silu(0) = 0, so y = x1
    wgu = weights["w_gate_up"].copy()
    wgu[:shape.mlp_dim] = 0
    kp, vp = W.make_cache(shape, flow.num_pages, 40)
    b = W.Batch(np.array([0, 18], np.int32), np.array([18], np.int32), flow.block_table, flow.prefix_id,
                flow.prefix_len, flow.num_pages)
    res = oracle.layer_step(shape, b, dict(weights, w_gate_up=wgu), flow.x_full[0], kp, vp)
    np.testing.assert_array_equal(res.y_f32, res.x1)
    # the full layer does move the stream (guards against the cases above passing vacuously)
    ys, _, _ = _run(oracle, shape, weights, flow)
    assert np.abs(ys[0] - x).max() > 1e-2


def test_oracle_own_rounding_error_is_small(oracle, oracle64):
    """fp32 accumulators against fp64 accumulators: the oracle's own error is far
    below the parity tolerance (max-abs 2e-2, rel-L2 1e-2)."""
    wl = W.workload_tiny()
    weights = W.make_weights(wl.shape, wl.seed)
    x = W.make_activations(wl.batch.T, wl.shape.hidden, wl.seed)
    outs = []
    for orc in (oracle, oracle64):
        kp, vp = W.make_cache(wl.shape, wl.batch.num_pages, wl.seed)
        outs.append(orc.layer_step(wl.shape, wl.batch, weights, x, kp, vp).y_f32.astype(np.float64))
    err = np.abs(outs[0] - outs[1]).max()
    rel = np.linalg.norm(outs[0] - outs[1]) / np.linalg.norm(outs[1])
    assert err < 2e-4 and rel < 1e-5, (err, rel)


# ---------------------------------------------------------------------------
# the stack: embedding -> layers -> final norm -> output layer on the last token
# ---------------------------------------------------------------------------
def _model_caches(shape, flow, n_layers, seed):
    ks, vs = [], []
    for l in range(n_layers):
        k, v = W.make_cache(shape, flow.num_pages, seed + l)
        ks.append(k)
        vs.append(v)
    return ks, vs


@pytest.mark.parametrize("name", ["mha", "gqa"])
def test_model_step_matches_dense_stack(oracle, name):
    """Chunked prefill + decode through the paged 3-layer oracle == torch fp64 recompute of
    each request's whole token sequence (next-token logits of the last token)."""
    shape = SHAPES[name]
    n_layers, vocab = 3, 211
    model = W.make_model(shape, n_layers, vocab, seed=70)
    seq = [29, 18, 33]
    sched = [[(0, 20), (1, 18)], [(0, 8), (2, 33)], [(0, 1)]]
    flow = make_flow(shape, seq, sched, seed=71)
    ids = [W.make_token_ids(L, vocab, 72 + r) for r, L in enumerate(seq)]
    ks, vs = _model_caches(shape, flow, n_layers, 73)
    final = run_model_flow(flow, ids, lambda b, t: oracle.model_step(shape, b, model, t, ks, vs)[0])
    for r in range(len(seq)):
        want = dense_model_logits(shape, model, ids[r]).numpy()
        # slack: rare one-ulp bf16 flips of cached k/v and of the stream between layers
        np.testing.assert_allclose(final[r], want, rtol=0, atol=2e-2 * np.abs(want).max())
        assert np.corrcoef(final[r], want)[0, 1] > 0.9999


def test_model_step_is_the_composition_of_pinned_pieces(oracle):
    """Exact identity: model step == embedding rows -> layer step (bf16 out) per layer ->
    rmsnorm -> linear on each request's last row, all of them pinned above."""
    shape = W.TINY_GQA
    n_layers, vocab = 2, 97
    model = W.make_model(shape, n_layers, vocab, seed=80)
    wl = W.workload_tiny_prefix(shape=shape)
    b = wl.batch
    ids = W.make_token_ids(b.T, vocab, 81)
    flowless_k = [W.make_cache(shape, b.num_pages, 82 + l) for l in range(n_layers)]
    ks, vs = [k.copy() for k, _ in flowless_k], [v.copy() for _, v in flowless_k]
    logits, hidden = oracle.model_step(shape, b, model, ids, ks, vs)
    x = model["embedding"][ids]
    ks2, vs2 = [k.copy() for k, _ in flowless_k], [v.copy() for _, v in flowless_k]
    for l in range(n_layers):
        x = oracle.layer_step(shape, b, model["layers"][l], x, ks2[l], vs2[l]).y_bf16
    np.testing.assert_array_equal(hidden, x)
    last = W.bf16_bits_to_f32(x[b.q_start[1:] - 1])
    want = oracle.linear(model["w_lm_head"], oracle.rmsnorm(last, model["w_final_norm"], shape.rms_eps))
    np.testing.assert_array_equal(logits, want)
    for l in range(n_layers):
        np.testing.assert_array_equal(ks[l], ks2[l])
        np.testing.assert_array_equal(vs[l], vs2[l])
    # a token id outside the vocabulary is refused
    bad = ids.copy()
    bad[3] = vocab
    with pytest.raises(ValueError):
        oracle.model_step(shape, b, model, bad, ks, vs)


def test_greedy_sample_is_the_first_largest_logit(oracle):
    """Sec. 2.3 "LLM Inference": the next token from the output layer's logits.  Pins: numpy's argmax on random
    rows, hand-written rows, planted ties (lowest id wins), extreme values, NaN never chosen."""
    rng = np.random.default_rng(5)
    logits = rng.standard_normal((37, 1000)).astype(np.float32)
    np.testing.assert_array_equal(oracle.greedy_sample(logits), np.argmax(logits, axis=1))
    hand = np.array([[0.0, 1.0, -1.0, 0.5], [3.0, 3.0, 2.0, 3.0], [-5.0, -4.0, -4.0, -6.0], [-np.inf, -np.inf, -1e30, -np.inf],
                     [np.nan, 2.0, np.inf, np.inf], [np.nan, np.nan, np.nan, np.nan]], np.float32)
    np.testing.assert_array_equal(oracle.greedy_sample(hand), [1, 0, 1, 2, 2, 0])
    tied = logits.copy()
    for r in range(tied.shape[0]):           # copy the row maximum to a later and to an earlier position
        m = int(np.argmax(tied[r]))
        tied[r, (m + 17) % 1000] = tied[r, m]
        want = min(m, (m + 17) % 1000)
        assert oracle.greedy_sample(tied[r:r + 1])[0] == want
    last = np.full((1, 64), -1.0, np.float32)
    last[0, 63] = 0.0                        # the maximum in the last position
    assert oracle.greedy_sample(last)[0] == 63


# ---------------------------------------------------------------------------
# quantised cache (reading R15)
# ---------------------------------------------------------------------------
def test_e4m3_format_matches_the_library_type(oracle):
    """The 8-bit format against torch's float8_e4m3fn: every code decodes to the same value; random and boundary values
    encode to the same code (round to nearest even); exact midpoints go to the even neighbour; round trips are exact;
    above 448 the code saturates (the library type has no saturation: checked by definition)."""
    codes = np.arange(256, dtype=np.uint8)
    lib = torch.from_numpy(codes).view(torch.float8_e4m3fn).float().numpy()
    mine = np.array([oracle.e4m3_to_f32(int(c)) for c in codes], np.float32)
    np.testing.assert_array_equal(np.isnan(mine), np.isnan(lib))
    np.testing.assert_array_equal(mine[~np.isnan(lib)], lib[~np.isnan(lib)])
    assert mine[0x7e] == 448.0 and mine[0x01] == 2.0 ** -9 and mine[0x08] == 2.0 ** -6 and mine[0x38] == 1.0
    finite = [int(c) for c in codes if not np.isnan(lib[c])]
    for c in finite:                                                       # round trip, both signs of zero included
        assert oracle.f32_to_e4m3(float(lib[c])) == c
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.standard_normal(4000) * 3, rng.standard_normal(2000) * 0.01, rng.uniform(-448, 448, 2000),
                        [448.0, -448.0, 447.9, 2.0 ** -10, 2.0 ** -10 * 1.0001, 2.0 ** -10 * 0.9999, 0.0]]).astype(np.float32)
    want = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = np.array([oracle.f32_to_e4m3(float(v)) for v in x], np.uint8)
    np.testing.assert_array_equal(got, want)
    pos = sorted(set(float(lib[c]) for c in finite if lib[c] >= 0))
    for lo, hi in zip(pos[:-1], pos[1:]):                                  # the midpoint of two neighbours goes to the even code
        mid = np.float32((np.float64(lo) + np.float64(hi)) / 2)
        c = oracle.f32_to_e4m3(float(mid))
        assert c % 2 == 0 and oracle.e4m3_to_f32(c) in (lo, hi)
        assert oracle.f32_to_e4m3(float(np.nextafter(mid, np.float32(1e9)))) == oracle.f32_to_e4m3(hi)
        assert oracle.f32_to_e4m3(float(np.nextafter(mid, np.float32(-1e9)))) == oracle.f32_to_e4m3(lo)
    for big in (448.1, 464.0, 480.0, 1e9, float("inf")):                    # saturation
        assert oracle.f32_to_e4m3(big) == 0x7e and oracle.f32_to_e4m3(-big) == 0xfe
    assert oracle.f32_to_e4m3(float("nan")) & 0x7f == 0x7f


def test_quantised_cache_reads_like_the_16_bit_cache_holding_the_same_values(oracle):
    """With power-of-two scales every code x scale is a bf16 number, so a 16-bit cache can hold exactly what the
    quantised one represents: attention over the two must agree bit for bit (same sums in the same order)."""
    shape = W.TINY_GQA
    b = W.workload_tiny_prefix(shape=shape).batch
    k8, v8 = W.make_cache_fp8(shape, b.num_pages, 7)
    ks, vs = 0.25, 2.0
    deq = np.array([oracle.e4m3_to_f32(c) for c in range(256)], np.float32)
    kp, vp = W.f32_to_bf16_bits(deq[k8] * np.float32(ks)), W.f32_to_bf16_bits(deq[v8] * np.float32(vs))
    np.testing.assert_array_equal(W.bf16_bits_to_f32(kp), deq[k8] * np.float32(ks))         # representable: nothing was rounded
    rng = np.random.default_rng(8)
    for r in range(b.num_reqs):
        pos = int(b.ctx_len[r]) - 1
        q = rng.standard_normal((shape.n_q_heads, shape.head_dim)).astype(np.float32)
        got = oracle.attention_token_fp8kv(shape, b, r, pos, q, k8, v8, ks, vs)
        want = oracle.attention_token(shape, b, r, pos, q, kp, vp)
        np.testing.assert_array_equal(got, want)
    # a scale that is not a power of two: the dequantised values in fp64, Eq. 4-5 written out
    ks, vs = 0.3, 0.7
    r, pos = 0, int(b.ctx_len[0]) - 1
    q = rng.standard_normal((shape.n_q_heads, shape.head_dim)).astype(np.float32)
    got = oracle.attention_token_fp8kv(shape, b, r, pos, q, k8, v8, ks, vs)
    P, group = shape.page_size, shape.n_q_heads // shape.n_kv_heads
    slots = [int(b.block_table[r][j // P]) * P + j % P for j in range(pos + 1)]
    K = deq[k8.reshape(-1, shape.n_kv_heads, shape.head_dim)[slots]].astype(np.float64) * np.float64(np.float32(ks))
    V = deq[v8.reshape(-1, shape.n_kv_heads, shape.head_dim)[slots]].astype(np.float64) * np.float64(np.float32(vs))
    for a in range(shape.n_q_heads):
        s = K[:, a // group] @ q[a].astype(np.float64) / np.sqrt(shape.head_dim)
        w = np.exp(s - s.max())
        np.testing.assert_allclose(got[a], (w / w.sum()) @ V[:, a // group], rtol=2e-5, atol=2e-6)


def test_quantised_cache_layer_step(oracle):
    """The step with the quantised cache: the appended codes are the library type's rounding of (rotated key x 1 / scale)
    and (value x 1 / scale); the attention output is the pinned 16-bit attention over a cache holding the same values;
    caching stays a memo (decoding one token at a time = one pass over the prompt, exactly); a pool of other codes at
    unused slots changes nothing."""
    shape = W.TINY_GQA
    wl = W.workload_tiny_prefix(shape=shape)
    b, weights = wl.batch, wl.weights()
    x = W.make_activations(b.T, shape.hidden, 3)
    ks, vs = 0.25, 0.125                                                     # powers of two
    k8, v8 = W.make_cache_fp8(shape, b.num_pages, 9)
    k0, v0 = k8.copy(), v8.copy()
    res = oracle.layer_step(shape, b, weights, x, k8, v8, kv_scales=(ks, vs))
    # what must have been written: pieces that are pinned on their own
    h = oracle.rmsnorm(W.bf16_bits_to_f32(x), weights["w_in_norm"], shape.rms_eps)
    h = W.bf16_bits_to_f32(W.f32_to_bf16_bits(h))                            # R15: bf16 inputs to the projection in this variant
    qkv = oracle.linear(weights["w_qkv"], h)
    d, nq, nkv, P = shape.head_dim, shape.n_q_heads, shape.n_kv_heads, shape.page_size
    pos = np.concatenate([np.arange(p, p + q) for p, q in zip(b.past, b.q_len)])
    for t in range(b.T):
        for hd in range(nq + nkv):
            qkv[t, hd * d:(hd + 1) * d] = oracle.rope(qkv[t, hd * d:(hd + 1) * d], int(pos[t]), shape.rope_base)
    slots = oracle.kv_append(shape, b, np.zeros((b.T, nkv, d), np.uint16), np.zeros((b.T, nkv, d), np.uint16),
                             np.zeros(k8.shape, np.uint16), np.zeros(k8.shape, np.uint16))
    want_k = torch.from_numpy(qkv[:, nq * d:(nq + nkv) * d] * np.float32(1 / ks)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    want_v = torch.from_numpy(qkv[:, (nq + nkv) * d:] * np.float32(1 / vs)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    np.testing.assert_array_equal(k8.reshape(-1, nkv * d)[slots], want_k)
    np.testing.assert_array_equal(v8.reshape(-1, nkv * d)[slots], want_v)
    mask = np.ones(k8.shape[0] * P, bool)
    mask[slots] = False
    np.testing.assert_array_equal(k8.reshape(-1, nkv * d)[mask], k0.reshape(-1, nkv * d)[mask])     # nothing else was written
    np.testing.assert_array_equal(v8.reshape(-1, nkv * d)[mask], v0.reshape(-1, nkv * d)[mask])
    # attention over the quantised cache = the 16-bit attention over the same values
    deq = np.array([oracle.e4m3_to_f32(c) for c in range(256)], np.float32)
    kp, vp = W.f32_to_bf16_bits(deq[k8] * np.float32(ks)), W.f32_to_bf16_bits(deq[v8] * np.float32(vs))
    t = 0
    for r in range(b.num_reqs):
        for j in range(int(b.q_len[r])):
            want = oracle.attention_token(shape, b, r, int(b.past[r]) + j, qkv[t, :nq * d].reshape(nq, d), kp, vp)
            np.testing.assert_array_equal(res.attn_out[t], want.reshape(-1))
            t += 1
    # a saturating scale: codes stop at the largest magnitude
    k9, v9 = W.make_cache_fp8(shape, b.num_pages, 9)
    oracle.layer_step(shape, b, weights, x, k9, v9, kv_scales=(1e-4, 1e-4))
    assert set(np.unique(k9.reshape(-1, nkv * d)[slots] & 0x7f)) <= set(range(0x7f)) and (k9.reshape(-1, nkv * d)[slots] & 0x7f).max() == 0x7e
    # memoisation: one token at a time == one pass, exactly
    L = 30
    outs = []
    for sched in ([[(0, L)]], [[(0, 1)] for _ in range(L)], [[(0, 11)], [(0, 19)]]):
        flow = make_flow(shape, [L], sched, seed=50)
        kq, vq = W.make_cache_fp8(shape, flow.num_pages, 51)
        ys = run_flow(flow, lambda bb, xx: oracle.layer_step(shape, bb, weights, xx, kq, vq, kv_scales=(ks, vs)).y_f32)
        outs.append((ys[0], kq, vq))
    for y, kq, vq in outs[1:]:
        np.testing.assert_array_equal(y, outs[0][0])
        np.testing.assert_array_equal(kq, outs[0][1])
        np.testing.assert_array_equal(vq, outs[0][2])
    # and close to the 16-bit step: the quantisation is fine enough not to change the output by more than a few percent
    kp16 = W.f32_to_bf16_bits(deq[k0] * np.float32(ks))
    vp16 = W.f32_to_bf16_bits(deq[v0] * np.float32(vs))
    y16 = oracle.layer_step(shape, b, weights, x, kp16, vp16).y_f32
    assert np.linalg.norm(res.y_f32 - y16) / np.linalg.norm(y16) < 3e-2


# ---------------------------------------------------------------------------
# quantised projections (reading R16 of the oracle header)
# ---------------------------------------------------------------------------
def _codes_to_f64(codes: np.ndarray) -> torch.Tensor:
    """Values of 8-bit codes through the library's own type."""
    return torch.from_numpy(codes.copy()).view(torch.float8_e4m3fn).to(torch.float64)


def _torch_quantise(values: torch.Tensor, scale: float) -> np.ndarray:
    """fp32 values -> codes of values / scale through the library's conversion (which does not saturate: clamp first)."""
    inv = np.float32(1.0 / np.float64(scale))
    scaled = (values.to(torch.float32) * torch.tensor(inv)).clamp(-448.0, 448.0)
    return scaled.to(torch.float8_e4m3fn).view(torch.uint8).numpy()


def test_quantise_matches_the_library_type(oracle):
    rng = np.random.default_rng(70)
    vals = (rng.standard_normal(20000) * 10.0 ** rng.integers(-4, 3, 20000)).astype(np.float32)
    for scale in (1.0, 0.0133, 3.7, 8.0 / 448.0):
        got = oracle.quantise(vals, scale)
        np.testing.assert_array_equal(got, _torch_quantise(torch.from_numpy(vals), scale))
    # beyond the range: the largest magnitude, with the sign
    np.testing.assert_array_equal(oracle.quantise(np.array([1e6, -1e6, 449.0 * 0.5], np.float32), 0.5), [0x7e, 0xfe, 0x7e])
    assert oracle.quantise(np.array([1.0], np.float32), 2.0)[0] == oracle.f32_to_e4m3(0.5)      # divides by the scale


def test_linear_w8a8_matches_matmul_of_the_code_values(oracle):
    rng = np.random.default_rng(71)
    N, K, T = 37, 192, 11
    wc = W.nearest_e4m3_codes(rng.standard_normal((N, K)).astype(np.float32) * 100)
    xc = W.nearest_e4m3_codes(rng.standard_normal((T, K)).astype(np.float32) * 30)
    s_w = (0.5 + rng.random(N)).astype(np.float32) * np.float32(1e-3)
    a = 0.037
    got = oracle.linear_w8a8(wc, s_w, xc, a)
    want = F.linear(_codes_to_f64(xc), _codes_to_f64(wc)) * torch.from_numpy(s_w.astype(np.float64))[None, :] * float(np.float32(a))
    np.testing.assert_allclose(got, want.numpy(), rtol=2e-6, atol=1e-9)
    # small whole numbers: every product and sum is exact, the result is the integer dot product times the scales
    vals = W.e4m3_code_values()
    small = np.array([c for c in range(256) if np.isfinite(vals[c]) and vals[c] == np.round(vals[c]) and abs(vals[c]) <= 16], np.uint8)
    wc = small[rng.integers(0, len(small), (N, 64))]
    xc = small[rng.integers(0, len(small), (T, 64))]
    ints = vals[xc].astype(np.int64) @ vals[wc].astype(np.int64).T
    got = oracle.linear_w8a8(wc, np.full(N, 0.25, np.float32), xc, 2.0)
    np.testing.assert_array_equal(got, (ints * 0.5).astype(np.float32))
    # which index the row scale follows: a matrix that picks input k(n) for output n
    pick = rng.integers(0, 64, N)
    wc = np.zeros((N, 64), np.uint8)
    wc[np.arange(N), pick] = 0x38                                    # the code of 1.0
    got = oracle.linear_w8a8(wc, s_w, xc, 1.0)
    np.testing.assert_array_equal(got, vals[xc][:, pick] * s_w[None, :])


_W8A8_SHAPE = W.LayerShape(256, 4, 2, 64, 384)
_W8A8_SCALES = {"a_qkv": 0.019, "a_o": 0.0071, "a_gate_up": 0.023, "a_down": 0.041}     # all different: a swap shows


def _w8a8_weights(seed):
    w = W.make_weights_w8a8(_W8A8_SHAPE, seed)
    w.update({k: np.float32(v) for k, v in _W8A8_SCALES.items()})
    return w


def test_layer_step_w8a8_is_the_composition_of_pinned_pieces(oracle):
    """The step with quantised projections, re-assembled here from the oracle's separately pinned pieces (norm,
    quantiser, code matmul, rotary embedding, append, attention): pins WHAT is quantised with WHICH scale."""
    shape = _W8A8_SHAPE
    wl = W.workload_tiny_prefix(shape=shape)
    b = wl.batch
    w = _w8a8_weights(72)
    x = W.make_activations(b.T, shape.hidden, 73)
    kp, vp = W.make_cache(shape, b.num_pages, 74)
    k1, v1 = kp.copy(), vp.copy()
    res = oracle.layer_step(shape, b, w, x, kp, vp)
    d, nh, nkv, I = shape.head_dim, shape.n_q_heads, shape.n_kv_heads, shape.mlp_dim
    xf = W.bf16_bits_to_f32(x)
    h = oracle.rmsnorm(xf, w["w_in_norm"], shape.rms_eps)
    qkv = oracle.linear_w8a8(w["w_qkv"], w["s_qkv"], oracle.quantise(h, w["a_qkv"]), w["a_qkv"])
    tok_req = np.repeat(np.arange(b.num_reqs), np.diff(b.q_start))
    tok_pos = np.concatenate([np.arange(b.ctx_len[r] - (b.q_start[r + 1] - b.q_start[r]), b.ctx_len[r]) for r in range(b.num_reqs)])
    for t in range(b.T):
        for a in range(nh + nkv):
            qkv[t, a * d:(a + 1) * d] = oracle.rope(qkv[t, a * d:(a + 1) * d], int(tok_pos[t]), shape.rope_base)
    kb = W.f32_to_bf16_bits(qkv[:, nh * d:(nh + nkv) * d]).reshape(b.T, nkv, d)
    vb = W.f32_to_bf16_bits(qkv[:, (nh + nkv) * d:]).reshape(b.T, nkv, d)
    oracle.kv_append(shape, b, kb, vb, k1, v1)
    np.testing.assert_array_equal(k1, kp)
    np.testing.assert_array_equal(v1, vp)
    attn = np.stack([oracle.attention_token(shape, b, int(tok_req[t]), int(tok_pos[t]), qkv[t, :nh * d].reshape(nh, d), k1, v1).reshape(-1)
                     for t in range(b.T)])
    np.testing.assert_array_equal(res.attn_out, attn)
    attn16 = W.bf16_bits_to_f32(W.f32_to_bf16_bits(attn))            # it exists as bf16 before it is quantised
    x1 = xf + oracle.linear_w8a8(w["w_o"], w["s_o"], oracle.quantise(attn16, w["a_o"]), w["a_o"])
    np.testing.assert_array_equal(res.x1, x1)
    h2 = oracle.rmsnorm(x1, w["w_post_norm"], shape.rms_eps)
    gu = oracle.linear_w8a8(w["w_gate_up"], w["s_gate_up"], oracle.quantise(h2, w["a_gate_up"]), w["a_gate_up"])
    g, u = gu[:, :I].astype(np.float64), gu[:, I:].astype(np.float64)
    act = (g / (1.0 + np.exp(-g)) * u).astype(np.float32)
    codes = oracle.quantise(act, w["a_down"])
    mine = oracle.linear_w8a8(w["w_down"], w["s_down"], codes, w["a_down"])
    # silu in fp64 here, fp32 there: an activation next to a rounding boundary may take the neighbouring code
    np.testing.assert_allclose(res.y_f32, x1 + mine, rtol=0, atol=2e-3)
    assert np.mean(np.abs(res.y_f32 - (x1 + mine)) > 1e-6) < 0.3


def test_layer_step_w8a8_matches_dense_recompute_through_library_types(oracle):
    """The same step on contiguous sequences with torch's own 8-bit type and fp64 matmuls.  Codes are decided in fp32
    there and in fp64 here, so a few inputs fall on the other side of a rounding boundary: a tolerance, far below
    the effect of any wiring mistake (which the composition pin above catches exactly)."""
    shape = _W8A8_SHAPE
    w = _w8a8_weights(75)
    L = 40
    flow = make_flow(shape, [L, 23], [[(0, L), (1, 23)]], seed=76)
    kp, vp = W.make_cache(shape, flow.num_pages, 77)
    ys = run_flow(flow, lambda bb, xx: oracle.layer_step(shape, bb, w, xx, kp, vp).y_f32)
    for r, n in enumerate([L, 23]):
        want = dense_layer(shape, w, flow.x_full[r], quantise=_torch_quantise, code_values=_codes_to_f64)["y"].numpy()
        got = ys[r]
        rel = np.linalg.norm(got - want) / np.linalg.norm(want)
        xin = W.bf16_bits_to_f32(flow.x_full[r])
        crel = np.linalg.norm(got - want) / np.linalg.norm(want - xin)
        print(f"request {r}: rel {rel:.2e}, on the layer's contribution {crel:.2e}")
        assert rel < 1e-4 and crel < 2e-3, (r, rel, crel)


def test_layer_step_w8a8_saturates_and_rejects_bad_scales(oracle):
    shape = _W8A8_SHAPE
    wl = W.workload_tiny(shape=shape)
    b = wl.batch
    w = _w8a8_weights(78)
    x = W.make_activations(b.T, shape.hidden, 79)
    kp, vp = W.make_cache(shape, b.num_pages, 80)
    base = oracle.layer_step(shape, b, w, x, kp.copy(), vp.copy()).y_f32
    tiny = dict(w, a_qkv=np.float32(1e-3))      # every normed activation beyond 0.448 becomes 0.448: a different, finite output
    sat = oracle.layer_step(shape, b, tiny, x, kp.copy(), vp.copy()).y_f32
    assert np.isfinite(sat).all() and np.abs(sat - base).max() > 1e-2
    with pytest.raises(ValueError):
        oracle.layer_step(shape, b, dict(w, a_o=np.float32(0.0)), x, kp.copy(), vp.copy())


def test_model_step_w8a8_is_the_composition_of_pinned_pieces(oracle):
    """The stack with quantised projections == embedding rows -> the (pinned) quantised layer step per layer, its output
    rounded to bf16 -> 16-bit final norm and output layer on each request's last row.  Exact."""
    shape = _W8A8_SHAPE
    n_layers, vocab = 3, 89
    model = W.make_model_w8a8(shape, n_layers, vocab, seed=84, scaled=False)
    for l, layer in enumerate(model["layers"]):                 # different input scales per layer: a mixed-up layer shows
        layer.update({k: np.float32(v * (1.0 + 0.1 * l)) for k, v in _W8A8_SCALES.items()})
    wl = W.workload_tiny_prefix(shape=shape)
    b = wl.batch
    ids = W.make_token_ids(b.T, vocab, 85)
    pools = [W.make_cache(shape, b.num_pages, 86 + l) for l in range(n_layers)]
    ks, vs = [k.copy() for k, _ in pools], [v.copy() for _, v in pools]
    logits, hidden = oracle.model_step(shape, b, model, ids, ks, vs)
    x = model["embedding"][ids]
    ks2, vs2 = [k.copy() for k, _ in pools], [v.copy() for _, v in pools]
    for l in range(n_layers):
        x = oracle.layer_step(shape, b, model["layers"][l], x, ks2[l], vs2[l]).y_bf16
    np.testing.assert_array_equal(hidden, x)
    last = W.bf16_bits_to_f32(x[b.q_start[1:] - 1])
    np.testing.assert_array_equal(logits, oracle.linear(model["w_lm_head"], oracle.rmsnorm(last, model["w_final_norm"], shape.rms_eps)))
    for l in range(n_layers):
        np.testing.assert_array_equal(ks[l], ks2[l])
        np.testing.assert_array_equal(vs[l], vs2[l])


def test_layer_step_w8a8_keeps_the_memoisation_invariant(oracle):
    """Static scales quantise every token by itself, so the cache stays a pure memo (Sec. 2.3 "KV Cache") under the
    quantised projections too: a prompt processed token by token, in two chunks or in one pass gives the same outputs
    and the same cache, exactly."""
    shape = _W8A8_SHAPE
    w = _w8a8_weights(88)
    L = 29
    outs = []
    for sched in ([[(0, L)]], [[(0, 1)] for _ in range(L)], [[(0, 13)], [(0, 16)]]):
        flow = make_flow(shape, [L], sched, seed=89)
        kp, vp = W.make_cache(shape, flow.num_pages, 90)
        ys = run_flow(flow, lambda bb, xx: oracle.layer_step(shape, bb, w, xx, kp, vp).y_f32)
        outs.append((ys[0], kp, vp))
    for y, kp, vp in outs[1:]:
        np.testing.assert_array_equal(y, outs[0][0])
        np.testing.assert_array_equal(kp, outs[0][1])
        np.testing.assert_array_equal(vp, outs[0][2])


def test_golden_tiny_layer_step_is_stable():
    """The frozen oracle outputs (written by tests/golden/make_golden.py) still hold."""
    import os
    from tests.golden.make_golden import compute
    res, kp, vp = compute()
    path = os.path.join(os.path.dirname(__file__), "golden", "tiny_layer_step.txt")
    for line in open(path):
        if line.startswith("#"):
            continue
        f = line.split()
        if f[0] == "y":
            # libm's expf/cos may differ in the last place between machines
            np.testing.assert_allclose(res.y_f32[int(f[1]), int(f[2])], float.fromhex(f[3]), rtol=1e-5, atol=1e-6)
        elif f[0] == "sum_k_pages":
            assert abs(int(kp.astype(np.uint64).sum()) - int(f[1])) < 4096
        elif f[0] == "sum_v_pages":
            assert abs(int(vp.astype(np.uint64).sum()) - int(f[1])) < 4096
