"""Executes the scheduler's batches on the GPU: the `execute=` side of `scheduler.Engine`.

The scheduler (Sec. 4.1 step 4) hands over a configured batch; this module owns what a GPU worker owns: the model
weights, the paged KV cache of every layer, the page allocator, the block tables.  A relQuery's template occupies
one run of pages, written by its first request and named by the block tables of all its requests (stored once,
Sec. 2.3 "Prefix Cache"); every request has private pages for its suffix and generated tokens.  Each batch becomes
one `relserve_batch_prepare` + `relserve_model_step`; the measured GPU time is returned to the scheduler's clock.
Token ids are a fixed function of (relQuery, request, position): there is no tokenizer and no sampling loop here,
a request decodes for its output length.
"""
from __future__ import annotations

import numpy as np

from . import binding as rs
from . import workloads as W


def token_ids(rid: int, req: int, first: int, n: int, prefix: int, vocab: int) -> np.ndarray:
    """Deterministic synthetic tokens of positions [first, first + n) of a request: template positions (below
    `prefix`) depend on the relQuery only, so all its requests share them."""
    pos = np.arange(first, first + n, dtype=np.int64)
    who = np.where(pos < prefix, 0, req + 1)
    h = (rid * 1000003 + who * 7919 + pos * 104729 + 12345) & 0x7FFFFFFF
    return ((h * 2654435761 >> 7) % vocab).astype(np.int32)


class GpuWorker:
    def __init__(self, shape: W.LayerShape, n_layers: int, vocab: int, num_pages: int, max_tokens: int, max_reqs: int,
                 seed: int = 0, keep_logits: bool = False):
        import torch
        self.torch, self.shape, self.vocab, self.n_layers = torch, shape, vocab, n_layers
        g = torch.Generator(device="cuda")
        g.manual_seed(seed)

        def randn(*size, std=1.0, mean=0.0):
            return (torch.randn(*size, generator=g, device="cuda", dtype=torch.float32) * std + mean).to(torch.bfloat16)

        H, I, qd = shape.hidden, shape.mlp_dim, shape.n_q_heads * shape.head_dim
        res_std = 0.02 / (2 * max(1, n_layers)) ** 0.5
        pool = (num_pages, shape.page_size, shape.n_kv_heads, shape.head_dim)
        layers = [{"w_in_norm": randn(H, std=0.02, mean=1.0), "w_qkv": randn(shape.qkv_dim, H, std=0.02),
                   "w_o": randn(H, qd, std=res_std), "w_post_norm": randn(H, std=0.02, mean=1.0),
                   "w_gate_up": randn(2 * I, H, std=0.02), "w_down": randn(H, I, std=res_std)} for _ in range(n_layers)]
        self.model = {"embedding": randn(vocab, H), "layers": layers,
                      "caches": [(torch.zeros(pool, dtype=torch.bfloat16, device="cuda"),
                                  torch.zeros(pool, dtype=torch.bfloat16, device="cuda")) for _ in range(n_layers)],
                      "w_final_norm": randn(H, std=0.02, mean=1.0), "w_lm_head": randn(vocab, H, std=0.02)}
        self.layer = rs.relserve_layer_create(shape)
        self.ws = torch.empty(rs.relserve_model_workspace_bytes(self.layer, max_tokens, max_reqs), dtype=torch.uint8, device="cuda")
        self.max_tokens, self.max_reqs, self.num_pages = max_tokens, max_reqs, num_pages
        self.free = list(range(num_pages - 1, -1, -1))          # page allocator: a stack of free page ids
        self.template_pages = {}                                # rid -> pages of the relQuery's template
        self.req_pages = {}                                     # (rid, req) -> private pages
        self.generated = {}                                     # (rid, req) -> tokens generated so far
        self.keep_logits, self.logits = keep_logits, {}         # (rid, req) -> logits row after its prefill
        self.e0, self.e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        self.batches = 0

    # ---- pages
    def take(self, n: int) -> list:
        if n > len(self.free):
            raise RuntimeError("KV page pool exhausted: lower the scheduler's cap or enlarge the pool")
        return [self.free.pop() for _ in range(n)]

    def give(self, pages) -> None:
        self.free.extend(pages)

    # ---- the scheduler's hook
    def __call__(self, kind: str, what) -> float:
        P = self.shape.page_size
        rows = []            # (q, req index, first position computed, positions computed, context length after the step)
        if kind == "prefill":
            for q, taken in what:
                assert q.prefix % P == 0, "templates are whole pages"
                for j, u in enumerate(taken):
                    req = q.next_req + j
                    cold = u > q.suffix[req]                     # this request computes the template too
                    if q.rid not in self.template_pages:
                        assert cold or q.prefix == 0, "a request reads a template nobody has written"
                        self.template_pages[q.rid] = self.take(q.prefix // P)
                    self.req_pages[(q.rid, req)] = self.take((q.suffix[req] + q.out_len + P - 1) // P)
                    self.generated[(q.rid, req)] = 0
                    rows.append((q, req, 0 if cold else q.prefix, u, q.prefix + q.suffix[req]))
        else:
            for q in what:
                first = q.next_req - len(q.running)
                for req in range(first, q.next_req):
                    ctx = q.prefix + q.suffix[req] + self.generated[(q.rid, req)] + 1
                    rows.append((q, req, ctx - 1, 1, ctx))
        # descriptor: a template written in an EARLIER batch is declared as a prefix group (its pages are read once
        # for all its readers); one that a request of this batch is writing is only shared through the block
        # tables, since a declared prefix must already be in the cache
        written_now = {q.rid for q, _, first, _, _ in rows if first == 0 and q.prefix > 0}
        rids = sorted({q.rid for q, _, first, _, _ in rows if first > 0 and q.rid not in written_now})
        pid_of = {rid: i for i, rid in enumerate(rids)}
        prefix_len = np.array([next(q.prefix for q, *_ in rows if q.rid == rid) for rid in rids], np.int32)
        q_len = np.array([n for *_, n, _ in rows], np.int32)
        ctx = np.array([c for *_, c in rows], np.int32)
        max_blocks = int(((ctx + P - 1) // P).max())
        bt = np.zeros((len(rows), max_blocks), np.int32)
        ids = np.empty(int(q_len.sum()), np.int32)
        o = 0
        for r, (q, req, first, n, c) in enumerate(rows):
            pages = self.template_pages[q.rid] + self.req_pages[(q.rid, req)]
            nb = (c + P - 1) // P
            bt[r, :nb] = pages[:nb]
            ids[o:o + n] = token_ids(q.rid, req, first, n, q.prefix, self.vocab)
            o += n
        qs = np.zeros(len(rows) + 1, np.int32)
        qs[1:] = np.cumsum(q_len)
        pid = np.array([pid_of[q.rid] if first > 0 and q.rid in pid_of else -1 for q, _, first, _, _ in rows], np.int32)
        batch = W.Batch(qs, ctx, bt, pid, prefix_len, self.num_pages, f"{kind}_{self.batches}")
        assert batch.T <= self.max_tokens and batch.num_reqs <= self.max_reqs
        torch = self.torch
        pb = rs.relserve_batch_prepare(self.layer, batch)
        tok = torch.from_numpy(ids).cuda()
        logits = torch.empty(batch.num_reqs, self.vocab, dtype=torch.float32, device="cuda")
        self.e0.record()
        rs.relserve_model_step(self.layer, pb, self.model, tok, logits, self.ws)
        self.e1.record()
        torch.cuda.synchronize()
        pb.close()
        self.batches += 1
        if not bool(torch.isfinite(logits).all()):
            raise RuntimeError(f"non-finite logits in {batch.name}")
        # bookkeeping: generated tokens, logits of prefills, pages of finished requests
        for r, (q, req, first, n, c) in enumerate(rows):
            key = (q.rid, req)
            if kind == "prefill":
                if self.keep_logits:
                    self.logits[key] = logits[r].cpu().numpy()
                done = q.out_len == 0
            else:
                self.generated[key] += 1
                done = self.generated[key] == q.out_len
            if done:
                self.give(self.req_pages.pop(key))
                del self.generated[key]
        return self.e0.elapsed_time(self.e1) * 1e-3

    def relquery_done(self, q) -> None:
        """Called by the scheduler when the last request of a relQuery has finished: its template pages are free."""
        self.give(self.template_pages.pop(q.rid, []))

    def standalone_logits(self, q, req: int) -> np.ndarray:
        """Next-token logits of one request computed privately (template and suffix in fresh pages, no sharing): what
        the serving run must reproduce for that request's prefill."""
        P, torch = self.shape.page_size, self.torch
        n = q.prefix + q.suffix[req]
        pages = self.take((n + P - 1) // P)
        bt = np.array([pages], np.int32)
        batch = W.Batch(np.array([0, n], np.int32), np.array([n], np.int32), bt, np.array([-1], np.int32), np.zeros(0, np.int32),
                        self.num_pages, "standalone")
        ids = token_ids(q.rid, req, 0, n, q.prefix, self.vocab)
        pb = rs.relserve_batch_prepare(self.layer, batch)
        logits = torch.empty(1, self.vocab, dtype=torch.float32, device="cuda")
        rs.relserve_model_step(self.layer, pb, self.model, torch.from_numpy(ids).cuda(), logits, self.ws)
        torch.cuda.synchronize()
        pb.close()
        self.give(pages)
        return logits[0].cpu().numpy()
