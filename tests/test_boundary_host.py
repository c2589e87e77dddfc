"""Host-side behaviour of the C-ABI library: it loads, exports what the header
declares, validates descriptors with a distinct status per rule, and places KV
slots exactly where the oracle does.  No GPU needed.
"""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2601_11546_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def rs():
    from paper_2601_11546_amd import binding
    return binding


def test_library_exports_every_declared_symbol(rs):
    header = open(os.path.join(ROOT, "include", "relserve.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(relserve_[a-z0-9_]+)\s*\(", header))
    assert len(declared) >= 18
    lib = C.CDLL(rs.LIB_PATH)
    for name in sorted(declared):
        assert hasattr(lib, name), f"{name} declared in relserve.h but not exported"
    assert declared == set(rs.EXPORTS)
    assert rs.relserve_version() >= 100
    assert rs.relserve_strerror(0) == "ok"
    assert "slot" in rs.relserve_strerror(-8)


def test_config_validation(rs):
    ok = W.TINY
    assert rs.relserve_config_validate(ok) == 0
    from dataclasses import replace
    bad = [replace(ok, head_dim=96), replace(ok, n_q_heads=6, n_kv_heads=4), replace(ok, page_size=12),
           replace(ok, page_size=4), replace(ok, hidden=250), replace(ok, mlp_dim=100), replace(ok, n_kv_heads=0),
           replace(ok, rope_base=0.0), replace(ok, n_q_heads=32, n_kv_heads=1)]
    for b in bad:
        assert rs.relserve_config_validate(b) == -2, b
    for good in (W.TINY_GQA, W.TINY_D128, W.TINY_G5, W.TINY_G3_D128, W.LLAMA_13B, W.LLAMA_70B, W.QWEN_32B, W.LLAMA_70B_TP4, W.QWEN_32B_TP2,
                 replace(ok, page_size=256)):
        assert rs.relserve_config_validate(good) == 0


def test_layer_handle_needs_no_device(rs):
    layer = rs.relserve_layer_create(W.LLAMA_70B)
    assert rs.relserve_workspace_bytes(layer, 0) >= 0
    n1, n2 = rs.relserve_workspace_bytes(layer, 100), rs.relserve_workspace_bytes(layer, 200)
    assert n2 > n1 > 100 * 8192 * 2
    layer.close()
    with pytest.raises(rs.RelserveError):
        rs.relserve_layer_create(W.LayerShape(256, 4, 4, 80, 688))


def _tiny_prefix():
    return W.workload_tiny_prefix().batch


def test_batch_validation_status_per_rule(rs):
    shape = W.TINY
    b = _tiny_prefix()
    assert rs.relserve_batch_validate(shape, b) == 0
    from dataclasses import replace

    def mut(**kw):
        c = replace(b, **{k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in kw.items()})
        return rs.relserve_batch_validate(shape, c)

    qs = b.q_start.copy(); qs[0] = 1
    assert mut(q_start=qs) == -3
    qs = b.q_start.copy(); qs[2] = qs[1]
    assert mut(q_start=qs) == -3                      # an empty request
    ctx = b.ctx_len.copy(); ctx[0] = 3
    assert mut(ctx_len=ctx) == -4                     # shorter than its own query tokens
    ctx = b.ctx_len.copy(); ctx[4] = b.block_table.shape[1] * shape.page_size + 1
    assert mut(ctx_len=ctx) == -5
    bt = b.block_table.copy(); bt[4, 0] = b.num_pages
    assert mut(block_table=bt) == -6
    bt = b.block_table.copy(); bt[4, 1] = -1
    assert mut(block_table=bt) == -6
    pid = b.prefix_id.copy(); pid[0] = 3
    assert mut(prefix_id=pid) == -7                   # unknown prefix id
    assert mut(prefix_len=np.array([24], np.int32)) == -7   # not a multiple of the page size
    assert mut(prefix_len=np.array([48], np.int32)) == -7   # longer than a member's past
    bt = b.block_table.copy(); bt[1, 0] = bt[4, 0]
    assert mut(block_table=bt) == -7                  # members disagree on the prefix pages
    bt = b.block_table.copy(); bt[4, 4] = bt[5, 5]
    # request 4 (ctx 70, q 1) writes position 69 -> block 4; request 5 (ctx 97, q 33) writes 64..96 -> blocks 4..6
    ctx = b.ctx_len.copy()
    bt = b.block_table.copy(); bt[4, 4] = bt[5, 4]; ctx[4] = 70
    assert mut(block_table=bt, ctx_len=ctx) == -8     # two tokens into one slot (pos 69 of both)
    bt = b.block_table.copy(); bt[4, 4] = bt[0, 0]
    assert mut(block_table=bt) == -7                  # a write into a shared prefix page
    assert mut(num_pages=1 << 28) == -12
    # empty batch is fine
    e = W.Batch(np.zeros(1, np.int32), np.zeros(0, np.int32), np.zeros((0, 1), np.int32), np.zeros(0, np.int32),
                np.zeros(0, np.int32), 4)
    assert rs.relserve_batch_validate(shape, e) == 0


@pytest.mark.parametrize("make", [W.workload_tiny, W.workload_tiny_prefix, W.workload_tiny_long_prefixes,
                                  W.workload_relquery_13b, lambda: W.workload_relquery_13b(n_rows=256, n_prefill=0),
                                  W.workload_decode_heavy_70b, W.workload_prefill_only_13b])
def test_slot_placement_matches_oracle_bit_exactly(rs, oracle, make):
    wl = make()
    # small stand-in shape with the same page size: slot placement does not depend on widths
    shape = W.LayerShape(64, 1, 1, 64, 64, page_size=wl.shape.page_size)
    b = wl.batch
    got = rs.relserve_batch_slots(shape, b)
    k = np.zeros((b.T, 1, 64), np.uint16)
    kp = np.zeros((b.num_pages, shape.page_size, 1, 64), np.uint16)
    want = oracle.kv_append(shape, b, k, k, kp, kp.copy())
    np.testing.assert_array_equal(got, want)
    assert len(set(got.tolist())) == b.T


def test_prepare_without_device_reports_it(rs):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    layer = rs.relserve_layer_create(W.TINY)
    d, keep = rs._desc(W.workload_tiny().batch)
    h = C.c_void_p()
    rc = rs._lib.relserve_batch_prepare(layer.handle, C.byref(d), None, C.byref(h))
    assert rc == -11 and not h
