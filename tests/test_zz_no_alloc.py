"""The allocation-free variant of the layer step (fixed device array as workspace) against the entry point
that takes the caller's workspace: same kernels, so the outputs and the appended cache rows agree bit for bit.
Two calls in a row, the second on a smaller batch (the array keeps the first call's contents)."""
import numpy as np
import pytest
import torch

from paper_2601_11546_amd import workloads as W
from tests.gpu_harness import assert_close, dev_bf16, host_bits, host_f32

pytestmark = pytest.mark.gpu


def _both(rs, shape, batch, weights_dev, x_bits, cache_seed):
    layer = rs.relserve_layer_create(shape)
    pb = rs.relserve_batch_prepare(layer, batch)
    x = dev_bf16(x_bits)
    outs = []
    for static in (False, True):
        kp, vp = W.make_cache(shape, batch.num_pages, cache_seed)
        kd, vd = dev_bf16(kp), dev_bf16(vp)
        y = torch.empty_like(x)
        if static:
            rs.relserve_layer_step_static(layer, pb, weights_dev, x, y, kd, vd)
        else:
            ws = torch.empty(rs.relserve_workspace_bytes(layer, batch.T), dtype=torch.uint8, device="cuda")
            rs.relserve_layer_step(layer, pb, weights_dev, x, y, kd, vd, ws)
        torch.cuda.synchronize()
        outs.append((host_bits(y), host_bits(kd), host_bits(vd), kp, vp))
    pb.close()
    return outs


def test_static_scratch_layer_step_matches_workspace_entry_point(oracle):
    from paper_2601_11546_amd import binding as rs
    assert torch.cuda.is_available()
    assert rs.relserve_static_scratch_bytes() == 80 << 20
    shape = W.LLAMA_13B
    weights = W.make_weights(shape, 1013, n_layers=40)
    wd = rs.pack_layer_weights({k: dev_bf16(v) for k, v in weights.items()})
    # first call: 200 decode rows of one relQuery behind a 512-token template (T = 200, two token tiles);
    # second call: a smaller mixed batch (T = 77: 13 decode rows and one 64-token prefill chunk)
    first = W.workload_relquery_13b(seed=1013, n_rows=200, n_prefill=0).batch
    second = W.workload_decode_plus_chunk_13b(64, n_dec=13, ctx=300, seed=1014).batch
    for i, b in enumerate((first, second)):
        print(f"[case] static scratch call {i}: T={b.T} reqs={b.num_reqs}", flush=True)
        x = W.make_activations(b.T, shape.hidden, 1015 + i)
        (y0, k0, v0, _, _), (y1, k1, v1, kp, vp) = _both(rs, shape, b, wd, x, 1016 + i)
        assert np.array_equal(y0, y1) and np.array_equal(k0, k1) and np.array_equal(v0, v1)
        # and against the oracle on sampled requests, to the parity bar of the layer step
        reqs = [0, b.num_reqs // 2, b.num_reqs - 1]
        sub, rows = b.select(reqs), b.token_rows(reqs)
        res = oracle.layer_step(shape, sub, weights, x[rows], kp, vp)
        assert_close(W.bf16_bits_to_f32(y1)[rows], res.y_f32, f"static scratch call {i}")
    # a batch beyond the fixed array is refused, nothing is launched
    big = W.build_batch(shape, [400], [400], seed=3)
    layer = rs.relserve_layer_create(shape)
    pb = rs.relserve_batch_prepare(layer, big)
    xb = dev_bf16(W.make_activations(400, shape.hidden, 4))
    kd, vd = (dev_bf16(a) for a in W.make_cache(shape, big.num_pages, 5))
    y = torch.zeros_like(xb)
    with pytest.raises(rs.RelserveError) as e:
        rs.relserve_layer_step_static(layer, pb, wd, xb, y, kd, vd)
    assert e.value.status == -12
    torch.cuda.synchronize()
    assert float(y.float().abs().max()) == 0.0


def test_static_scratch_layer_step_replays_from_a_graph():
    """What the allocation-free entry point is for: the step captured into a HIP graph (kernels only: no allocation, no
    memset, no host synchronisation) and replayed, with the program's own eager work between the replays; every replay
    gives the bits of the eager call on the same inputs."""
    from paper_2601_11546_amd import binding as rs
    shape = W.LLAMA_13B
    weights = W.make_weights(shape, 1021, n_layers=40)
    wd = rs.pack_layer_weights({k: dev_bf16(v) for k, v in weights.items()})
    b = W.workload_relquery_13b(seed=1022, n_rows=96, n_prefill=2).batch
    layer = rs.relserve_layer_create(shape)
    pb = rs.relserve_batch_prepare(layer, b)
    kp, vp = W.make_cache(shape, b.num_pages, 1023)
    k0, v0 = dev_bf16(kp), dev_bf16(vp)
    xs = [dev_bf16(W.make_activations(b.T, shape.hidden, 1024 + i)) for i in range(3)]

    def eager(x):
        kd, vd, y = k0.clone(), v0.clone(), torch.empty_like(x)
        rs.relserve_layer_step_static(layer, pb, wd, x, y, kd, vd)
        torch.cuda.synchronize()
        return host_bits(y), host_bits(kd)
    want = [eager(x) for x in xs]            # also the warm-up: kernel attributes and the scratch address are set here
    # static buffers of the graph
    x_in, y_out, kd, vd = torch.empty_like(xs[0]), torch.empty_like(xs[0]), k0.clone(), v0.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        x_in.copy_(xs[0])
        rs.relserve_layer_step_static(layer, pb, wd, x_in, y_out, kd, vd)     # once more on the capture stream, uncaptured
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            rs.relserve_layer_step_static(layer, pb, wd, x_in, y_out, kd, vd)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for rep in range(2):
        for i, x in enumerate(xs):
            kd.copy_(k0)
            vd.copy_(v0)
            x_in.copy_(x)
            y_out.zero_()
            graph.replay()
            torch.cuda.synchronize()
            assert np.array_equal(host_bits(y_out), want[i][0]), (rep, i)
            assert np.array_equal(host_bits(kd), want[i][1]), (rep, i)
            eager(xs[(i + 1) % 3])      # eager work on the same scratch array between replays
    pb.close()
