"""Iteration-level scheduler for relQueries (Sec. 4.1 overview, Sec. 4.2 Dynamic Priority Updater, Sec. 4.3
Adaptive Batch Arranger) over the library's primitives, with a virtual clock.

Every iteration runs one prefill batch or one decode batch (Sec. 4.1 step 1).  The policy decides which:

  "fcfs"      the engine default the paper starts from (Sec. 2.3): waiting requests in arrival order, prefill
              first whenever a request can be admitted, otherwise decode all running requests;
  "static"    the static-priority baseline (Sec. 3, Eq. 6-7): a relQuery's priority value is computed once, at
              arrival (`relserve_static_priority`), and orders the waiting queue; otherwise as "fcfs";
  "relserve"  priorities = predicted remaining duration of each relQuery (`relserve_pem_estimate` over the current
              prefix-cache state — uncached tokens counted exactly or estimated from a random sample's miss ratio
              (Eq. 11, `relserve_utok_estimate`) — reused while a relQuery is entirely waiting (Eq. 12,
              `relserve_priority_reuse`) and its template's cached state is unchanged, zeroed by the starvation rule
              (Eq. 13)); the candidate prefill batch holds requests of the first waiting relQuery only
              (`relserve_prefill_candidate`); the arranger (`relserve_aba_decide`) picks between it and the candidate
              decode batch.

This module only keeps the queues and calls the library: every formula of the method sits behind the C ABI.

What a batch costs comes from the fitted batch-duration model (Eq. 9), so a run needs no GPU: the same loop can
drive `relserve_model_step` by passing `execute=` (`serving.GpuWorker`), which is called with every batch and returns
the measured duration that then moves the clock instead of the prediction.
The prefix cache is modelled per template: once a request of a relQuery has been prefilled, its template's tokens
are cached (least-recently-used templates are dropped beyond `cache_tokens`) and later requests compute their
suffix only.  Block-level prefix matching is not modelled.
"""
from __future__ import annotations

from collections import OrderedDict
from dataclasses import dataclass, field

from . import binding as rs


@dataclass
class RelQuery:
    rid: int
    arrival: float                 # seconds
    prefix: int                    # template tokens shared by all requests
    suffix: list                   # private tokens per request
    out_len: int                   # OL(R): decode iterations per request
    template: int = -1             # relQueries with the same template id share its tokens (-1: its own)
    # run state
    next_req: int = 0              # requests [0, next_req) have been prefilled
    running: list = field(default_factory=list)    # [remaining decode iterations, tokens admitted] of the prefilled, unfinished requests
    finished: int = 0
    finish_time: float = -1.0
    priority: float = 0.0
    priority_valid: bool = False
    priority_cached: bool = False  # whether the template was cached when `priority` was computed
    priority_waiting: int = 0      # requests waiting when `priority` was computed / last checked
    effective: float = 0.0         # priority after the starvation rule
    static_priority: float = -1.0  # Eq. 6-7, fixed at arrival

    @property
    def n(self) -> int:
        return len(self.suffix)

    @property
    def waiting(self) -> int:
        return self.n - self.next_req

    @property
    def done(self) -> bool:
        return self.finished == self.n


@dataclass
class Limits:
    cap: int = 65536                       # tokens the KV cache manager holds for admitted requests (their uncached tokens, as in Algorithm 1)
    max_num_seqs: int = 256
    max_num_batched_tokens: int = 8192


class Engine:
    def __init__(self, prefill_model: dict, decode_model: dict, limits: Limits = Limits(), policy: str = "relserve",
                 cache_tokens: int = 1 << 20, starvation_threshold: float = float("inf"), execute=None, sample_size: int = 0,
                 draw=None, l1: dict | None = None, l2: dict | None = None):
        assert policy in ("fcfs", "static", "relserve")
        self.mp, self.md, self.lim, self.policy = prefill_model, decode_model, limits, policy
        self.cache_tokens, self.threshold, self.execute = cache_tokens, starvation_threshold, execute
        self.sample_size = sample_size               # Eq. 11: requests sampled per relQuery for the miss ratio (0 = count exactly)
        self.draw = draw                             # draw(rid, key, n, k) -> k distinct positions in range(n): the random sample
        assert not sample_size or draw is not None
        # Eq. 6: L1 and L2 as lines; by default the slopes of the fitted duration lines (tokens and output lengths in seconds)
        self.l1 = l1 or {"alpha": prefill_model["alpha"], "beta": 0.0}
        self.l2 = l2 or {"alpha": decode_model["alpha"], "beta": 0.0}
        self.cache: OrderedDict = OrderedDict()      # template id -> template tokens, in LRU order
        self.now = 0.0
        self.log = []                                # (time, kind, rid or -1, requests, tokens)

    # ---- prefix cache (template granularity)
    @staticmethod
    def tid(q: RelQuery) -> int:
        return q.template if q.template >= 0 else -1 - q.rid

    def cached(self, q: RelQuery) -> bool:
        return self.tid(q) in self.cache

    def touch(self, q: RelQuery) -> None:
        self.cache[self.tid(q)] = q.prefix
        self.cache.move_to_end(self.tid(q))
        while sum(self.cache.values()) > self.cache_tokens and len(self.cache) > 1:
            self.cache.popitem(last=False)

    def utok(self, q: RelQuery, i: int, cached: bool) -> int:
        if self.execute is not None and hasattr(self.execute, "uncached_tokens"):
            exact = self.execute.uncached_tokens(q, i)       # the worker's block-level cache as it stands
            return min(exact, q.suffix[i]) if cached else exact
        return q.suffix[i] + (0 if cached else q.prefix)

    # ---- admission limits shared by both policies
    def admitted_tokens(self, active) -> int:
        return sum(r[1] for q in active for r in q.running)

    def take_prefill(self, q: RelQuery, budget_left: int, seqs_left: int, tokens_in_batch: int):
        """Requests of q, in order, that fit the limits; returns their uncached token counts."""
        cached = self.cached(q)
        # the first request of a cold template computes it for the rest
        u = [self.utok(q, i, cached or i > q.next_req) for i in range(q.next_req, q.n)]
        k, _ = rs.relserve_prefill_candidate(u, budget_left, seqs_left, tokens_in_batch, self.lim.max_num_batched_tokens)
        return u[:k]

    # ---- priorities (Sec. 4.2)
    def waiting_utok(self, q: RelQuery) -> list:
        """Uncached tokens of the waiting requests of q: counted exactly, or (Eq. 11) for the first waiting request
        exactly and for the others as their prompt length times the cache miss ratio of a small sample of them."""
        cached = self.cached(q)
        first, rest = q.next_req, list(range(q.next_req + 1, q.n))
        out = [self.utok(q, first, cached)] if first < q.n else []
        if not self.sample_size or len(rest) <= self.sample_size:
            return out + [self.utok(q, i, True) for i in rest]
        sample = [rest[p] for p in self.draw(q.rid, q.next_req, len(rest), self.sample_size)]
        est = rs.relserve_utok_estimate([q.prefix + q.suffix[i] for i in rest], [q.prefix + q.suffix[i] for i in sample],
                                        [self.utok(q, i, True) for i in sample])
        return out + [int(e) for e in est]

    def update_priorities(self, active) -> None:
        for q in active:
            cached = self.cached(q)
            reuse = (q.priority_valid and rs.relserve_priority_reuse(q.n, q.priority_waiting, q.waiting)     # Eq. 12
                     and q.priority_cached == cached)         # and nobody else has cached (or evicted) its template meanwhile
            q.priority_waiting = q.waiting
            if not reuse:
                utok = [0] * q.next_req + self.waiting_utok(q)
                decodes = [0] * q.n
                for i in range(q.next_req, q.n):
                    decodes[i] = 1
                first_running = q.next_req - len(q.running)
                for i in range(first_running, q.next_req):
                    decodes[i] = 1
                q.priority = rs.relserve_pem_estimate(utok, q.out_len, self.lim.cap, self.lim.max_num_seqs,
                                                      self.lim.max_num_batched_tokens, self.mp, self.md, decodes)
                q.priority_valid, q.priority_cached = True, cached
            if q.waiting:
                q.effective = rs.relserve_starved_priority(q.priority, self.now - q.arrival, q.n, self.threshold)
            else:
                q.effective = q.priority

    # ---- one iteration
    def step(self, active) -> bool:
        """Runs one batch; False if nothing can run (idle)."""
        running = [q for q in active if q.running]
        n_running = sum(len(q.running) for q in running)
        budget = self.lim.cap - self.admitted_tokens(active)
        seqs = self.lim.max_num_seqs - n_running
        if self.policy in ("fcfs", "static"):
            cand = []                                                  # [(q, uncached tokens of the requests taken)] in queue order
            toks = 0
            if self.policy == "static":
                for q in active:
                    if q.static_priority < 0:                          # once, when the relQuery is first seen
                        q.static_priority = rs.relserve_static_priority([q.prefix + x for x in q.suffix], q.out_len, self.l1, self.l2)
            order = (lambda q: (q.arrival, q.rid)) if self.policy == "fcfs" else (lambda q: (q.static_priority, q.arrival, q.rid))
            for q in sorted((q for q in active if q.waiting), key=order):
                taken = self.take_prefill(q, budget, seqs, toks)
                if not taken:
                    break
                cand.append((q, taken))
                toks += sum(taken)
                budget -= sum(taken)
                seqs -= len(taken)
                if len(taken) < q.waiting:
                    break
            if cand:
                self.run_prefill(cand)
                return True
            if n_running:
                self.run_decode(running)
                return True
            return False
        # relserve
        self.update_priorities(active)
        waiting = sorted((q for q in active if q.waiting), key=lambda q: (q.effective, q.arrival, q.rid))
        cand, taken = None, []
        if waiting:
            cand = waiting[0]
            taken = self.take_prefill(cand, budget, seqs, 0)
        m_run = min((q.effective for q in running), default=0.0)
        m_wait = cand.effective if cand is not None else 0.0
        decision, _ = rs.relserve_aba_decide(m_run, m_wait, n_running, len(taken), sum(taken), cand.out_len if cand else 0,
                                             [q.out_len for q in running], len(waiting), self.mp, self.md)
        if decision == 1:
            self.run_prefill([(cand, taken)])
        elif decision == 2:
            self.run_decode(running)
        return decision != 0

    def run_prefill(self, cand) -> None:
        reqs, toks = sum(len(t) for _, t in cand), sum(sum(t) for _, t in cand)
        measured = self.execute("prefill", cand) if self.execute else None
        self.now += rs.relserve_duration_predict(self.mp, toks) if measured is None else measured
        for q, taken in cand:
            q.running += [[q.out_len, u] for u in taken]
            q.next_req += len(taken)
            self.touch(q)
            self.retire(q)
        self.log.append((self.now, "prefill", cand[0][0].rid if len(cand) == 1 else -1, reqs, toks))

    def run_decode(self, running) -> None:
        reqs = sum(len(q.running) for q in running)
        measured = self.execute("decode", running) if self.execute else None
        self.now += rs.relserve_duration_predict(self.md, reqs) if measured is None else measured
        for q in running:
            for r in q.running:
                r[0] -= 1
            self.retire(q)
        self.log.append((self.now, "decode", -1, reqs, reqs))

    def retire(self, q: RelQuery) -> None:
        left = [r for r in q.running if r[0] > 0]
        q.finished += len(q.running) - len(left)
        q.running = left
        if q.done and q.finish_time < 0:
            q.finish_time = self.now


def serve(relqueries, prefill_model: dict, decode_model: dict, policy: str, limits: Limits = Limits(), **kw) -> dict:
    """Runs the trace to completion; returns per-relQuery latencies and the iteration log."""
    qs = sorted((RelQuery(q.rid, q.arrival, q.prefix, list(q.suffix), q.out_len, q.template) for q in relqueries),
                key=lambda q: (q.arrival, q.rid))
    eng = Engine(prefill_model, decode_model, limits, policy, **kw)
    arrived, i = [], 0
    while i < len(qs) or any(not q.done for q in arrived):
        while i < len(qs) and qs[i].arrival <= eng.now:
            arrived.append(qs[i])
            i += 1
        active = [q for q in arrived if not q.done]
        if not active or not eng.step(active):
            if i < len(qs):
                eng.now = max(eng.now, qs[i].arrival)         # idle until the next arrival
            else:
                raise RuntimeError("scheduler stalled: a request fits no batch under the limits")
    lat = {q.rid: q.finish_time - q.arrival for q in arrived}
    return {"latency": lat, "mean_latency": sum(lat.values()) / max(1, len(lat)), "makespan": eng.now, "log": eng.log}


def poisson_trace(n_relqueries: int, rate: float, seed: int = 0, max_requests: int = 100, out_lens=(5, 50)):
    """The seeded synthetic trace of workloads.poisson_trace as run-state records."""
    from . import workloads as W
    return [RelQuery(s.rid, s.arrival, s.prefix, list(s.suffix), s.out_len, s.template)
            for s in W.poisson_trace(n_relqueries, rate, seed, max_requests, out_lens)]


def compare_policies(prefill_model: dict, decode_model: dict, rates=(2.0, 4.0, 6.0, 8.0), n_relqueries: int = 80, seeds=(0, 1, 2),
                     limits: Limits = Limits(cap=65536, max_num_seqs=256, max_num_batched_tokens=8192),
                     starvation_threshold: float = 2.0) -> list:
    """Mean relQuery latency under both policies on seeded Poisson traces, one row per arrival rate."""
    rows = []
    for rate in rates:
        acc = {"fcfs": [], "static": [], "relserve": []}
        for seed in seeds:
            trace = poisson_trace(n_relqueries, rate, seed)
            for policy in acc:
                kw = {"starvation_threshold": starvation_threshold} if policy == "relserve" else {}
                acc[policy].append(serve(trace, prefill_model, decode_model, policy, limits, **kw)["mean_latency"])
        f, st, r = (sum(acc[k]) / len(seeds) for k in ("fcfs", "static", "relserve"))
        rows.append({"relqueries_per_s": rate, "fcfs_mean_latency_s": round(f, 4), "static_priority_mean_latency_s": round(st, 4),
                     "relserve_mean_latency_s": round(r, 4), "speedup": round(f / r, 3), "speedup_over_static": round(st / r, 3)})
    return rows
