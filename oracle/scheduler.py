"""Oracle of the serving loop (test infrastructure, not product code): one iteration of the scheduler as Sec. 4.1
lists it, step by step, in plain Python, for the three policies the evaluation compares.

  "fcfs"      the engine default (Sec. 5.1 "Baselines", first item): waiting requests in arrival order,
              prefill first whenever a waiting request can be admitted, otherwise decode all running requests;
  "static"    the static-priority baseline (Sec. 3, Eq. 6-7; Sec. 5.1 "Baselines", third item: the same engine
              with the dynamic priority update and the adaptive arrangement switched off): a relQuery's
              priority value is computed once, when it arrives, as the sum over its requests of
              L1(tok) + L2(OL); the waiting queue is ordered by it; prefill first as in "fcfs";
  "relserve"  Sec. 4.1 steps 2-5: priorities from the Priority Estimation Model at every iteration (Sec. 4.2,
              Eq. 8-10), with the two shortcuts (Eq. 11 sampled miss ratio, Eq. 12 reuse) and the
              starvation rule (Eq. 13); waiting queue in ascending priority; candidate prefill batch from the
              first waiting relQuery only; the arranger (Sec. 4.3, Eq. 14-17) picks the batch.

Readings (the product takes the same ones):
  * L1 and L2 of Eq. 6 are linear, given as (slope, intercept) pairs ("simple linear functions"; identity and
    constant mappings are special cases);
  * priority ties are broken by arrival time, then by relQuery id;
  * Eq. 12's reuse also needs the cached state of the relQuery's template to be what it was when the value was
    computed: this engine lets two relQueries name the same template, so a waiting relQuery's workload can drop
    when another one caches its template (the paper's argument for the reuse assumes distinct templates);
  * Eq. 11: the first waiting request is counted exactly (it is the one that may have to compute the template),
    the others through the miss ratio of the sample; the sample positions are random draws passed in by the
    caller (`draw(rid, iteration, n, k)` -> k distinct positions in range(n));
  * the prefix cache is per template, least recently used first out beyond `cache_tokens` tokens;
  * a batch costs what Eq. 9 predicts (virtual clock).

Only tests import this module; it imports nothing of the product.
"""
from __future__ import annotations

from . import aba as oaba
from . import pem as opem


class _Q:
    def __init__(self, spec):
        self.rid, self.arrival, self.prefix = spec.rid, spec.arrival, spec.prefix
        self.suffix, self.out_len = list(spec.suffix), spec.out_len
        self.tid = spec.template if getattr(spec, "template", -1) >= 0 else -1 - spec.rid
        self.n = len(self.suffix)
        self.prefilled = 0            # requests [0, prefilled) have left the waiting queue
        self.running = []             # [remaining decode iterations, tokens admitted] per running request
        self.finished = 0
        self.finish_time = None
        self.prio = None              # last Priority Estimation Model value
        self.prio_cached = None       # whether the template was cached when it was computed
        self.prio_waiting = None      # requests waiting when it was computed
        self.static = None


def static_priority(tok, out_len, l1, l2):
    """Eq. 6-7."""
    return sum((l1[0] * t + l1[1]) + (l2[0] * out_len + l2[1]) for t in tok)


def priority_reuse(n_submitted, n_waiting_before, n_waiting_now):
    """Eq. 12: every request of the relQuery was waiting, and still is."""
    return n_waiting_before == n_submitted and n_waiting_now == n_submitted


def prefill_candidate(utok, tokens_free, seqs_free, tokens_in_batch, mnbt):
    """Sec. 4.3: requests from the front of one relQuery's waiting requests under the three limits."""
    taken, toks = 0, 0
    for u in utok:
        if seqs_free - taken < 1:                # max_num_seqs
            break
        if u > tokens_free - toks:               # the KV cache manager's capacity
            break
        if tokens_in_batch + toks + u > mnbt and (taken > 0 or tokens_in_batch > 0):     # max_num_batched_tokens
            break
        taken += 1
        toks += u
    return taken, toks


def serve(trace, prefill_model, decode_model, policy, cap, mns, mnbt, threshold=float("inf"), sample_size=0, draw=None,
          cache_tokens=1 << 20, l1=None, l2=None):
    """Runs the trace to completion.  Models are (alpha, beta).  Returns (log, latency): log = one
    (time, kind, relQuery id or -1, requests, tokens) per executed batch."""
    ap, bp = prefill_model
    ad, bd = decode_model
    l1 = (ap, 0.0) if l1 is None else l1
    l2 = (ad, 0.0) if l2 is None else l2
    pending = sorted((_Q(s) for s in trace), key=lambda q: (q.arrival, q.rid))
    arrived, cache, log = [], [], []          # cache: [template id, tokens], least recently used first
    now, it = 0.0, 0

    def cached(q):
        return any(t == q.tid for t, _ in cache)

    def touch(q):
        cache[:] = [e for e in cache if e[0] != q.tid] + [[q.tid, q.prefix]]
        while sum(e[1] for e in cache) > cache_tokens and len(cache) > 1:
            cache.pop(0)

    def utok(q, i, template_cached):
        return q.suffix[i] + (0 if template_cached else q.prefix)

    def waiting_utok(q):
        c = cached(q)
        first, rest = q.prefilled, list(range(q.prefilled + 1, q.n))
        out = [utok(q, first, c)] if first < q.n else []
        if not sample_size or len(rest) <= sample_size:
            return out + [utok(q, i, True) for i in rest]
        pos = draw(q.rid, q.prefilled, len(rest), sample_size)
        sample = [rest[p] for p in pos]
        est = opem.utok_estimate([q.prefix + q.suffix[i] for i in rest], [utok(q, i, True) for i in sample],
                                 [q.prefix + q.suffix[i] for i in sample])
        return out + [int(round(e)) for e in est]

    def retire(q):
        left = [r for r in q.running if r[0] > 0]
        q.finished += len(q.running) - len(left)
        q.running = left
        if q.finished == q.n and q.finish_time is None:
            q.finish_time = now

    while pending or any(q.finished < q.n for q in arrived):
        while pending and pending[0].arrival <= now:
            q = pending.pop(0)
            q.static = static_priority([q.prefix + s for s in q.suffix], q.out_len, l1, l2)
            arrived.append(q)
        active = [q for q in arrived if q.finished < q.n]
        it += 1
        running = [q for q in active if q.running]
        n_running = sum(len(q.running) for q in running)
        tokens_free = cap - sum(r[1] for q in active for r in q.running)
        seqs_free = mns - n_running
        batch = None                                            # ("prefill", [(q, [utok...])]) or ("decode", running)
        if policy in ("fcfs", "static"):
            key = (lambda q: (q.arrival, q.rid)) if policy == "fcfs" else (lambda q: (q.static, q.arrival, q.rid))
            cand, toks = [], 0
            for q in sorted((q for q in active if q.prefilled < q.n), key=key):
                c = cached(q)
                u = [utok(q, i, c or i > q.prefilled) for i in range(q.prefilled, q.n)]
                k, t = prefill_candidate(u, tokens_free, seqs_free, toks, mnbt)
                if k == 0:
                    break
                cand.append((q, u[:k]))
                toks += t
                tokens_free -= t
                seqs_free -= k
                if k < q.n - q.prefilled:
                    break
            if cand:
                batch = ("prefill", cand)
            elif n_running:
                batch = ("decode", running)
        else:
            # step 2: priority values, waiting queue in ascending order
            eff = {}
            for q in active:
                n_wait = q.n - q.prefilled
                c = cached(q)
                keep = (q.prio is not None and priority_reuse(q.n, q.prio_waiting, n_wait) and q.prio_cached == c)
                if not keep:
                    u = [0] * q.prefilled + waiting_utok(q)
                    dec = [0] * q.n
                    for i in range(q.prefilled - len(q.running), q.n):
                        dec[i] = 1
                    q.prio = opem.pem(u, q.out_len, cap, mns, mnbt, prefill_model, decode_model, dec)
                    q.prio_cached, q.prio_waiting = c, n_wait
                else:
                    q.prio_waiting = n_wait
                eff[q.rid] = oaba.starved_priority(q.prio, now - q.arrival, q.n, threshold) if n_wait else q.prio
            waiting = sorted((q for q in active if q.prefilled < q.n), key=lambda q: (eff[q.rid], q.arrival, q.rid))
            # step 3: the two candidates and the arranger's choice
            cand_q, u_taken = None, []
            if waiting:
                cand_q = waiting[0]
                c = cached(cand_q)
                u = [utok(cand_q, i, c or i > cand_q.prefilled) for i in range(cand_q.prefilled, cand_q.n)]
                k, _ = prefill_candidate(u, tokens_free, seqs_free, 0, mnbt)
                u_taken = u[:k]
            m_run = min((eff[q.rid] for q in running), default=0.0)
            m_wait = eff[cand_q.rid] if cand_q is not None else 0.0
            choice = oaba.decide(m_run, m_wait, n_running, len(u_taken), sum(u_taken), cand_q.out_len if cand_q else 0,
                                 [q.out_len for q in running], len(waiting), prefill_model, decode_model)
            if choice == oaba.PREFILL:
                batch = ("prefill", [(cand_q, u_taken)])
            elif choice == oaba.DECODE:
                batch = ("decode", running)
        if batch is None:                                         # idle: wait for the next arrival
            if not pending:
                raise RuntimeError("stalled")
            now = max(now, pending[0].arrival)
            continue
        # steps 4 and 5: run the batch on the virtual clock (Eq. 9), update the queues
        if batch[0] == "prefill":
            reqs = sum(len(u) for _, u in batch[1])
            toks = sum(sum(u) for _, u in batch[1])
            now += ap * toks + bp
            for q, u in batch[1]:
                q.running += [[q.out_len, x] for x in u]
                q.prefilled += len(u)
                touch(q)
                retire(q)
            log.append((now, "prefill", batch[1][0][0].rid if len(batch[1]) == 1 else -1, reqs, toks))
        else:
            reqs = sum(len(q.running) for q in batch[1])
            now += ad * reqs + bd
            for q in batch[1]:
                for r in q.running:
                    r[0] -= 1
                retire(q)
            log.append((now, "decode", -1, reqs, reqs))
    return log, {q.rid: q.finish_time - q.arrival for q in arrived}
