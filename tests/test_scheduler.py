"""Iteration-level relQuery scheduler on the virtual clock (Sec. 4.1-4.3): conservation and limits, agreement of the
engine loop with Algorithm 1's decomposition (Eq. 10), the head-of-line case the paper is about, starvation."""
import numpy as np
import pytest

from oracle import pem as opem

MP, MD = {"alpha": 2.2e-5, "beta": 8.6e-3}, {"alpha": 4.0e-5, "beta": 6.6e-3}     # 40-layer 13B on this GPU, seconds


@pytest.fixture(scope="module")
def sch():
    from paper_2601_11546_amd import scheduler
    return scheduler


def _check_log(sch, trace, res, lim):
    pre = sum(r[3] for r in res["log"] if r[1] == "prefill")
    dec = sum(r[3] for r in res["log"] if r[1] == "decode")
    assert pre == sum(q.n for q in trace)                                  # every request prefilled once
    assert dec == sum(q.n * q.out_len for q in trace)                      # and decoded OL times
    for t, kind, rid, reqs, toks in res["log"]:
        if kind == "prefill":
            assert toks <= lim.max_num_batched_tokens or reqs == 1
        else:
            assert reqs <= lim.max_num_seqs
    assert all(v > 0 for v in res["latency"].values()) and len(res["latency"]) == len(trace)
    times = [r[0] for r in res["log"]]
    assert times == sorted(times)


def test_tiny_trace_by_hand(sch):
    # one relQuery, cold template of 100 tokens, suffixes 10 and 20, two decode iterations
    q = sch.RelQuery(0, 0.0, 100, [10, 20], 2)
    res = sch.serve([q], MP, MD, "fcfs")
    kinds = [(r[1], r[3], r[4]) for r in res["log"]]
    assert kinds == [("prefill", 2, 130), ("decode", 2, 2), ("decode", 2, 2)]          # the first request computes the template
    want = MP["alpha"] * 130 + MP["beta"] + 2 * (MD["alpha"] * 2 + MD["beta"])
    assert abs(res["latency"][0] - want) < 1e-12
    assert sch.serve([q], MP, MD, "relserve")["latency"][0] == pytest.approx(want, abs=1e-12)


@pytest.mark.parametrize("policy", ["fcfs", "relserve"])
def test_lone_relquery_runs_as_algorithm_1_decomposes_it(sch, policy):
    """The engine loop on a single relQuery executes exactly the batches Algorithm 1 predicts, so its duration is the
    Priority Estimation Model's value (Eq. 10) computed by the independent oracle."""
    rng = np.random.default_rng(5)
    for _ in range(40):
        n = int(rng.integers(1, 120))
        q = sch.RelQuery(0, 0.0, int(rng.choice([256, 512, 1024])), [int(x) for x in rng.integers(30, 121, n)], int(rng.integers(1, 8)))
        lim = sch.Limits(cap=int(rng.integers(1200, 9000)), max_num_seqs=int(rng.integers(2, 64)),
                         max_num_batched_tokens=int(rng.integers(1200, 4096)))
        res = sch.serve([q], MP, MD, policy, lim)
        utok = [q.prefix + q.suffix[0]] + q.suffix[1:]
        want = opem.pem(utok, q.out_len, lim.cap, lim.max_num_seqs, lim.max_num_batched_tokens,
                        (MP["alpha"], MP["beta"]), (MD["alpha"], MD["beta"]))
        assert res["latency"][0] == pytest.approx(want, rel=1e-9)
        _check_log(sch, [q], res, lim)


@pytest.mark.parametrize("policy", ["fcfs", "static", "relserve"])
def test_conservation_and_limits_on_poisson_traces(sch, policy):
    for seed in range(4):
        trace = sch.poisson_trace(25, rate=0.5, seed=seed)
        lim = sch.Limits(cap=20000, max_num_seqs=64, max_num_batched_tokens=4096)
        res = sch.serve(trace, MP, MD, policy, lim)
        _check_log(sch, trace, res, lim)


def test_short_relqueries_are_not_blocked_behind_a_long_one(sch):
    long_q = sch.RelQuery(0, 0.0, 1024, [100] * 100, 50)
    short = [sch.RelQuery(1 + i, 0.05 + 0.01 * i, 512, [60] * 3, 5) for i in range(5)]
    lim = sch.Limits(cap=65536, max_num_seqs=64, max_num_batched_tokens=4096)
    fcfs = sch.serve([long_q] + short, MP, MD, "fcfs", lim)
    rel = sch.serve([long_q] + short, MP, MD, "relserve", lim)
    assert rel["mean_latency"] < 0.7 * fcfs["mean_latency"]
    for i in range(1, 6):                                                  # each short relQuery finishes earlier
        assert rel["latency"][i] < fcfs["latency"][i]


def test_starvation_threshold_bounds_the_wait_of_a_long_relquery(sch):
    # short relQueries arrive a little faster than they can be served; a long one, entirely waiting, is passed over
    # by each of them until its waiting time per request exceeds the threshold
    stream = [sch.RelQuery(i, 0.045 * i, 256, [40] * 4, 5) for i in range(100)]
    long_q = sch.RelQuery(1000, 0.01, 1024, [100] * 60, 20)
    lim = sch.Limits(cap=65536, max_num_seqs=64, max_num_batched_tokens=4096)
    free = sch.serve(stream + [long_q], MP, MD, "relserve", lim)
    fair = sch.serve(stream + [long_q], MP, MD, "relserve", lim, starvation_threshold=0.02)
    assert free["latency"][1000] > 3.0                                     # starved until the stream dries up
    assert fair["latency"][1000] < 0.75 * free["latency"][1000]
    first_long = min(r[0] for r in fair["log"] if r[1] == "prefill" and r[2] == 1000)
    assert first_long >= 0.01 + 0.02 * 60                                  # not before the threshold is crossed


# ---------------------------------------------------------------- the loop executing its batches on the GPU
@pytest.mark.gpu
@pytest.mark.parametrize("policy,w8a8", [("fcfs", False), ("relserve", False), ("relserve", True)],
                         ids=["fcfs", "relserve", "relserve-quantised-projections"])
def test_serving_loop_executes_its_batches_on_the_gpu(sch, policy, w8a8):
    """A short trace served for real: every batch goes through relserve_batch_prepare (which validates block tables,
    prefix groups and write slots) and relserve_model_step; the page pool is whole again at the end; and a request
    that read its relQuery's template from pages shared with (and written by) another request gets the logits of a
    private recomputation and the CPU oracle's for the same prompt.  w8a8: the worker quantises its layers and every
    batch runs the quantised model step; the bounds are those of the quantised tiny model steps (two implementations
    of a quantised layer differ by codes that fall on the other side of a rounding boundary)."""
    from paper_2601_11546_amd import serving
    from paper_2601_11546_amd import workloads as W
    # the quantised projections need inner dimensions that are multiples of 128
    shape, vocab = (W.LayerShape(256, 4, 2, 64, 384) if w8a8 else W.TINY_GQA), 512
    rng = np.random.default_rng(9)
    trace = [sch.RelQuery(i, 0.002 * i, int(rng.choice([32, 48, 64])), [int(x) for x in rng.integers(5, 21, int(rng.integers(2, 9)))],
                          int(rng.integers(2, 5))) for i in range(6)]
    trace.append(sch.RelQuery(6, 0.02, trace[0].prefix, [7, 19, 12], 3, template=0))      # a second relQuery behind relQuery 0's template
    trace[0].template = 0
    lim = sch.Limits(cap=600, max_num_seqs=12, max_num_batched_tokens=160)
    print(f"serving loop, policy {policy}, w8a8 {w8a8}: {sum(q.n for q in trace)} requests", flush=True)
    worker = serving.GpuWorker(shape, n_layers=2, vocab=vocab, num_pages=256, max_tokens=256, max_reqs=16, seed=3, keep_logits=True,
                               w8a8=w8a8)
    res = sch.serve(trace, MP, MD, policy, lim, execute=worker)
    _check_log(sch, trace, res, lim)
    assert worker.batches == len(res["log"]) and res["makespan"] > 0
    worker.cache.check()
    assert not worker.pages and all(r == 0 for r in worker.cache.refs)
    # every relQuery's template was computed once: by its first request, or not at all behind a cached template
    computed = sum(r[4] for r in res["log"] if r[1] == "prefill")
    assert computed == sum(sum(q.suffix) for q in trace) + sum(q.prefix for q in trace[:6])
    assert worker.cache.misses == computed and worker.cache.hits == sum(q.prefix * q.n for q in trace) - sum(q.prefix for q in trace[:6])
    checked, worst = 0, 0.0
    for q in trace:
        for req in (0, q.n - 1):                      # the template's writer (or first reader), and a reader of the shared pages
            want = worker.standalone_logits(q, req)
            got = worker.logits[(q.rid, req)]
            dev = float(np.abs(got - want).max() / max(1.0, np.abs(want).max()))
            assert dev <= 2e-2, (q.rid, req, dev)
            worst = max(worst, dev)
            checked += 1
    assert checked == 14
    worker.cache.check()
    assert all(r == 0 for r in worker.cache.refs)
    # and the oracle, run privately on the same prompts with the same weights, gives those logits: the writer of a
    # template, a reader within its relQuery, and a reader from another relQuery
    from oracle import relserve_oracle
    orc = relserve_oracle.load("f32")
    import torch
    bits = lambda t: t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)

    def host(v):   # bf16 tensors as their bit patterns; the codes, their fp32 scales and the static input scales as they are
        if not torch.is_tensor(v):
            return v
        return bits(v) if v.dtype == torch.bfloat16 else v.detach().cpu().contiguous().numpy()

    model = {"embedding": bits(worker.model["embedding"]), "w_final_norm": bits(worker.model["w_final_norm"]),
             "w_lm_head": bits(worker.model["w_lm_head"]),
             "layers": [{k: host(v) for k, v in w.items()} for w in worker.model["layers"]]}
    for q, req in ((trace[0], 0), (trace[0], trace[0].n - 1), (trace[6], 1)):
        ids = worker.prompt(q, req)
        b = W.build_batch(shape, [len(ids)], [len(ids)], seed=1)
        pools = [W.make_cache(shape, b.num_pages, 0, fill=False) for _ in range(2)]
        want, _ = orc.model_step(shape, b, model, ids, [k for k, _ in pools], [v for _, v in pools])
        got = worker.logits[(q.rid, req)]
        scale = float(np.sqrt(np.mean(want[0].astype(np.float64) ** 2)))
        rel = float(np.linalg.norm(got - want[0]) / np.linalg.norm(want[0]))
        print(f"  relQuery {q.rid} request {req}: logits rel-L2 {rel:.2e} against the oracle (worst served vs private {worst:.2e})", flush=True)
        assert rel <= 1e-2 and np.abs(got - want[0]).max() <= 6e-2 * scale, (q.rid, req, rel)


def test_sampled_miss_ratio_estimates_uncached_tokens(sch):
    """Eq. 11: the estimate for the unsampled requests is their prompt length times the miss ratio of a random sample
    (the oracle's formula on the same draws), and the priorities built on it stay close to the exactly counted ones."""
    from oracle import pem as opem
    from paper_2601_11546_amd import workloads as W
    rng = np.random.default_rng(2)
    q = sch.RelQuery(0, 0.0, 512, [int(x) for x in rng.integers(30, 121, 60)], 5)
    draw = W.sample_positions(11)
    exact = sch.Engine(MP, MD).waiting_utok(q)
    eng = sch.Engine(MP, MD, sample_size=8, draw=draw)
    est = eng.waiting_utok(q)
    assert est[0] == exact[0] == 512 + q.suffix[0]                        # the first request brings the template
    rest = list(range(1, 60))
    sample = [rest[p] for p in draw(0, 0, len(rest), 8)]
    assert len(set(sample)) == 8
    want = opem.utok_estimate([512 + q.suffix[i] for i in rest], [q.suffix[i] for i in sample], [512 + q.suffix[i] for i in sample])
    assert est[1:] == [int(round(w)) for w in want]
    assert abs(sum(est) - sum(exact)) <= 0.25 * sum(exact)                 # eight samples of suffixes spread over 30-120
    trace = sch.poisson_trace(30, rate=4.0, seed=7)
    a = sch.serve(trace, MP, MD, "relserve")["mean_latency"]
    b = sch.serve(trace, MP, MD, "relserve", sample_size=8, draw=draw)["mean_latency"]
    assert abs(a - b) <= 0.15 * a


# ---------------------------------------------------------------- the loop against its oracle, batch by batch
def _oracle_log(trace, policy, lim, **kw):
    from oracle import scheduler as osch
    return osch.serve(trace, (MP["alpha"], MP["beta"]), (MD["alpha"], MD["beta"]), policy, lim.cap, lim.max_num_seqs,
                      lim.max_num_batched_tokens, **kw)


def _same_logs(got, want):
    assert len(got) == len(want)
    for i, (g, w) in enumerate(zip(got, want)):
        assert g[1:] == w[1:], (i, g, w)                                   # kind, relQuery, requests, tokens: exact
        assert g[0] == pytest.approx(w[0], rel=1e-12, abs=1e-12), (i, g, w)


@pytest.mark.parametrize("policy", ["fcfs", "static", "relserve"])
def test_every_batch_is_the_one_the_oracle_loop_runs(sch, policy):
    """Seeded Poisson traces (own templates and templates shared between relQueries, loose and tight limits, with and
    without the sampled miss ratio and the starvation rule): the engine executes, batch by batch, what the plain-Python
    oracle of Sec. 4.1's iteration executes."""
    from paper_2601_11546_amd import workloads as W
    cases = 0
    for seed in range(6):
        for n_templates in (0, 3):
            trace = W.poisson_trace(18, rate=(3.0, 8.0, 20.0)[seed % 3], seed=seed, max_requests=40, n_templates=n_templates)
            for lim in (sch.Limits(cap=65536, max_num_seqs=256, max_num_batched_tokens=8192),
                        sch.Limits(cap=3000, max_num_seqs=24, max_num_batched_tokens=1500)):
                variants = [{}]
                if policy == "relserve":
                    variants = [{}, {"threshold": 0.03}, {"sample_size": 4, "draw": W.sample_positions(seed)},
                                {"cache_tokens": 1200, "threshold": 0.05}]
                for v in variants:
                    kw = {("starvation_threshold" if k == "threshold" else k): x for k, x in v.items()}
                    res = sch.serve(trace, MP, MD, policy, lim, **kw)
                    log, lat = _oracle_log(trace, policy, lim, **v)
                    _same_logs(res["log"], log)
                    assert res["latency"].keys() == lat.keys()
                    for rid in lat:
                        assert res["latency"][rid] == pytest.approx(lat[rid], rel=1e-12)
                    cases += 1
    assert cases >= 24


def test_scheduler_primitives_match_their_oracles(sch):
    """Eq. 6-7, Eq. 11, Eq. 12 and the candidate prefill batch of Sec. 4.3: the library's functions against the plain ones."""
    from oracle import pem as opem
    from oracle import scheduler as osch
    from paper_2601_11546_amd import binding as rs
    rng = np.random.default_rng(3)
    # hand-worked: two requests of 110 and 120 prompt tokens, OL 3, L1(x) = 2x + 1, L2(x) = x / 2: (221 + 1.5) + (241 + 1.5)
    assert rs.relserve_static_priority([110, 120], 3, {"alpha": 2.0, "beta": 1.0}, {"alpha": 0.5, "beta": 0.0}) == 465.0
    assert osch.static_priority([110, 120], 3, (2.0, 1.0), (0.5, 0.0)) == 465.0
    # hand-worked candidate: limits 1000 free tokens, 3 free slots, 300 tokens per batch
    assert rs.relserve_prefill_candidate([100, 200, 50, 40], 1000, 3, 0, 300) == (2, 300)      # the third would exceed the batch
    assert rs.relserve_prefill_candidate([100, 100, 50, 40], 1000, 3, 0, 300) == (3, 250)      # the fourth has no slot
    assert rs.relserve_prefill_candidate([100, 100, 50, 40], 220, 9, 0, 300) == (2, 200)       # the third exceeds the cache room
    assert rs.relserve_prefill_candidate([500, 10], 1000, 9, 0, 300) == (1, 500)               # alone above the batch limit
    assert rs.relserve_prefill_candidate([500, 10], 1000, 9, 40, 300) == (0, 0)                # ... but not into a started batch
    for _ in range(300):
        n = int(rng.integers(0, 30))
        tok = [int(x) for x in rng.integers(0, 900, n)]
        ol = int(rng.integers(0, 60))
        l1, l2 = (float(rng.random()), float(rng.random())), (float(rng.random()), float(rng.random()))
        got = rs.relserve_static_priority(tok, ol, {"alpha": l1[0], "beta": l1[1]}, {"alpha": l2[0], "beta": l2[1]})
        assert got == pytest.approx(osch.static_priority(tok, ol, l1, l2), rel=1e-12, abs=1e-12)
        args = (int(rng.integers(0, 3000)), int(rng.integers(0, 12)), int(rng.integers(0, 500)), int(rng.integers(1, 1500)))
        assert rs.relserve_prefill_candidate(tok, *args) == osch.prefill_candidate(tok, *args)
        ns = int(rng.integers(1, 6))
        st = [int(x) for x in rng.integers(1, 900, ns)]
        su = [int(rng.integers(0, t + 1)) for t in st]
        want = [int(round(x)) for x in opem.utok_estimate(tok, su, st)]
        assert list(rs.relserve_utok_estimate(tok, st, su)) == want
        sub = int(rng.integers(1, 50))
        before = int(rng.integers(0, sub + 1))
        nowv = int(rng.integers(0, before + 1))
        assert rs.relserve_priority_reuse(sub, before, nowv) == osch.priority_reuse(sub, before, nowv)
    with pytest.raises(rs.RelserveError):
        rs.relserve_utok_estimate([5], [10], [11])                       # more uncached than prompt tokens
    with pytest.raises(rs.RelserveError):
        rs.relserve_priority_reuse(4, 3, 4)                              # waiting requests cannot come back


def test_three_relqueries_by_hand(sch):
    """A hand-worked trace under the RelServe policy, batch by batch.  Lines: prefill 1 ms per token + 10 ms, decode
    1 ms per request + 5 ms.  A (2 requests, template 100, suffixes 10 / 10, OL 2) arrives at 0; B (1 request, template
    20, suffix 5, OL 1) at 0.05; C (3 requests, A's template, suffixes 10 / 10 / 10, OL 1) at 0.06.
      t = 0      only A: prefill A (110 + 10 tokens: 120 ms + 10 ms) -> 0.130 s; B and C have arrived meanwhile.
      t = 0.130  priorities: A = 2 decode iterations of 2 requests = 2 x 7 ms = 0.014; B = (25 + 10) ms + 6 ms = 0.041;
                 C: A's template is cached, so 30 tokens: (30 + 10) ms + (3 + 5) ms = 0.048.  m+ = 0.014 < m- = 0.041:
                 transitional case, delta+ = L_prefill(B) x 1 + 1 ms x 1 x min(2, 1) = 0.036, delta- = 2 waiting x 5 ms x
                 min(1, 2) = 0.010: delta > 0, decode A -> 0.137; the same again -> 0.144, A done (latency 0.144).
      t = 0.144  nothing runs: prefill B (25 tokens, 35 ms) -> 0.179; now m+ = B = 0.006 < m- = C = 0.048, delta+ = 0.040 +
                 0.003 > delta- = 0.005: decode B (6 ms) -> 0.185, B done (latency 0.135).
      t = 0.185  prefill C (30 tokens, 40 ms) -> 0.225; decode C (3 requests, 8 ms) -> 0.233 (latency 0.173)."""
    mp, md = {"alpha": 1e-3, "beta": 1e-2}, {"alpha": 1e-3, "beta": 5e-3}
    trace = [sch.RelQuery(0, 0.0, 100, [10, 10], 2, template=7), sch.RelQuery(1, 0.05, 20, [5], 1),
             sch.RelQuery(2, 0.06, 100, [10, 10, 10], 1, template=7)]
    res = sch.serve(trace, mp, md, "relserve")
    want = [(0.130, "prefill", 0, 2, 120), (0.137, "decode", -1, 2, 2), (0.144, "decode", -1, 2, 2),
            (0.179, "prefill", 1, 1, 25), (0.185, "decode", -1, 1, 1), (0.225, "prefill", 2, 3, 30), (0.233, "decode", -1, 3, 3)]
    _same_logs(res["log"], want)
    assert res["latency"] == pytest.approx({0: 0.144, 1: 0.135, 2: 0.173}, abs=1e-9)
    from oracle import scheduler as osch
    log, lat = osch.serve(trace, (1e-3, 1e-2), (1e-3, 5e-3), "relserve", 65536, 256, 8192)
    _same_logs(log, want)
    # static priorities (Eq. 6-7 with the default lines: 1 ms per prompt token + 1 ms per output token):
    # A = 2 x (110 + 2) ms = 0.224, B = 26 ms, C = 3 x 111 ms = 0.333.  After A's prefill the queue is B, C; prefill comes
    # first and a batch may span relQueries: B's request (25 tokens) and C's three (30) run as one prefill batch, then
    # all six requests decode together; A needs a second iteration.
    st = sch.serve(trace, mp, md, "static")
    want = [(0.130, "prefill", 0, 2, 120), (0.195, "prefill", -1, 4, 55), (0.206, "decode", -1, 6, 6), (0.213, "decode", -1, 2, 2)]
    _same_logs(st["log"], want)
    log, _ = osch.serve(trace, (1e-3, 1e-2), (1e-3, 5e-3), "static", 65536, 256, 8192)
    _same_logs(log, want)
