"""Executes the scheduler's batches on the GPU: the `execute=` side of `scheduler.Engine`.

The scheduler (Sec. 4.1 step 4) hands over a configured batch; this module owns what a GPU worker owns: the model
weights, the paged KV cache of every layer, the block tables, and a block-level prefix cache over the page pool
(`prefix_cache.BlockPrefixCache`): the full blocks of a prompt are keyed by their tokens, so the template of a relQuery
is written by the first request that brings it and named by the block tables of all later ones (stored once,
Sec. 2.3 "Prefix Cache"); what a request does not find cached it computes into pages of its own.  Each batch becomes
one `relserve_batch_prepare` + `relserve_model_step`; the measured GPU time is returned to the scheduler's clock.
Token ids are a fixed function of (relQuery, request, position): there is no tokenizer and no sampling loop here,
a request decodes for its output length.
"""
from __future__ import annotations

import numpy as np

from . import binding as rs
from . import workloads as W
from .prefix_cache import BlockPrefixCache


def token_ids(template: int, rid: int, req: int, first: int, n: int, prefix: int, vocab: int) -> np.ndarray:
    """Deterministic synthetic tokens of positions [first, first + n) of a request: template positions (below
    `prefix`) depend on the template only, so every request behind that template shares them."""
    pos = np.arange(first, first + n, dtype=np.int64)
    who = np.where(pos < prefix, template * 1000003, (rid * 1000003 + (req + 1) * 7919) ^ 0x5bd1e995)
    h = (who + pos * 104729 + 12345) & 0x7FFFFFFF
    return ((h * 2654435761 >> 7) % vocab).astype(np.int32)


class GpuWorker:
    def __init__(self, shape: W.LayerShape, n_layers: int, vocab: int, num_pages: int, max_tokens: int, max_reqs: int,
                 seed: int = 0, keep_logits: bool = False, w8a8: bool = False):
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
        if w8a8:     # the quantised-projection variant of every layer (the model step then runs relserve_model_step_w8a8)
            from .duration_model import quantise_layer_on_device
            layers = [quantise_layer_on_device(torch, w) for w in layers]
        self.model = {"embedding": randn(vocab, H), "layers": layers,
                      "caches": [(torch.zeros(pool, dtype=torch.bfloat16, device="cuda"),
                                  torch.zeros(pool, dtype=torch.bfloat16, device="cuda")) for _ in range(n_layers)],
                      "w_final_norm": randn(H, std=0.02, mean=1.0), "w_lm_head": randn(vocab, H, std=0.02)}
        self.layer = rs.relserve_layer_create(shape)
        self.ws = torch.empty(rs.relserve_model_workspace_bytes(self.layer, max_tokens, max_reqs), dtype=torch.uint8, device="cuda")
        self.max_tokens, self.max_reqs, self.num_pages = max_tokens, max_reqs, num_pages
        self.cache = BlockPrefixCache(num_pages, shape.page_size)     # page allocator and block-level prefix cache
        self.pages = {}                                         # (rid, req) -> pages of a live request
        self.generated = {}                                     # (rid, req) -> tokens generated so far
        self.keep_logits, self.logits = keep_logits, {}         # (rid, req) -> logits row after its prefill
        self.e0, self.e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        self.batches = 0

    def prompt(self, q, req: int) -> np.ndarray:
        tid = q.template if q.template >= 0 else q.rid
        return token_ids(tid, q.rid, req, 0, q.prefix + q.suffix[req], q.prefix, self.vocab)

    def uncached_tokens(self, q, req: int) -> int:
        """utok(r) against the cache as it stands (what the scheduler asks before it forms a batch)."""
        toks = self.prompt(q, req)
        return len(toks) - self.cache.match(toks)

    # ---- the scheduler's hook
    def __call__(self, kind: str, what) -> float:
        P, cache = self.shape.page_size, self.cache
        rows = []            # (q, req index, first position computed, positions computed, context length after the step)
        ready_blocks = []    # leading blocks of the row's block table that an earlier batch wrote and that carry a key
        tokens = []
        if kind == "prefill":
            for q, taken in what:
                for j, _ in enumerate(taken):
                    req = q.next_req + j
                    toks = self.prompt(q, req)
                    pages, cached, n_ready = cache.acquire(toks, q.out_len)
                    self.pages[(q.rid, req)] = pages
                    self.generated[(q.rid, req)] = 0
                    rows.append((q, req, cached, len(toks) - cached, len(toks)))
                    ready_blocks.append(n_ready // P)
                    tokens.append(toks[cached:])
        else:
            for q in what:
                first = q.next_req - len(q.running)
                for req in range(first, q.next_req):
                    g = self.generated[(q.rid, req)]
                    ctx = q.prefix + q.suffix[req] + g + 1
                    rows.append((q, req, ctx - 1, 1, ctx))
                    pages = self.pages[(q.rid, req)]
                    nb = 0
                    while nb < len(pages) and cache.key_of[pages[nb]] is not None and cache.ready[pages[nb]]:
                        nb += 1
                    ready_blocks.append(nb)
                    tid = q.template if q.template >= 0 else q.rid
                    tokens.append(token_ids(tid, q.rid, req, ctx - 1, 1, q.prefix, self.vocab))
        # descriptor: rows whose block tables begin with the same cached blocks, written by EARLIER batches, are
        # declared as a shared-prefix group of their common length (those pages are then read once for the group);
        # blocks that a request of this batch is writing are shared through the block tables only, since a
        # declared prefix must already be in the cache
        groups = {}
        for r, (q, req, *_rest) in enumerate(rows):
            if ready_blocks[r] > 0:
                groups.setdefault(self.pages[(q.rid, req)][0], []).append(r)
        pid = np.full(len(rows), -1, np.int32)
        prefix_len = []
        for members in groups.values():
            if len(members) < 2:
                continue
            first_pages = self.pages[(rows[members[0]][0].rid, rows[members[0]][1])]
            common = min(ready_blocks[r] for r in members)
            for r in members[1:]:
                pr = self.pages[(rows[r][0].rid, rows[r][1])]
                k = 0
                while k < common and pr[k] == first_pages[k]:
                    k += 1
                common = k
            pid[members] = len(prefix_len)
            prefix_len.append(common * P)
        prefix_len = np.array(prefix_len, np.int32)
        q_len = np.array([n for *_, n, _ in rows], np.int32)
        ctx = np.array([c for *_, c in rows], np.int32)
        max_blocks = int(((ctx + P - 1) // P).max())
        bt = np.zeros((len(rows), max_blocks), np.int32)
        ids = np.empty(int(q_len.sum()), np.int32)
        o = 0
        for r, (q, req, first, n, c) in enumerate(rows):
            pages = self.pages[(q.rid, req)]
            nb = (c + P - 1) // P
            bt[r, :nb] = pages[:nb]
            ids[o:o + n] = tokens[r]
            o += n
        qs = np.zeros(len(rows) + 1, np.int32)
        qs[1:] = np.cumsum(q_len)
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
        # bookkeeping: written blocks become shareable, generated tokens, logits of prefills, pages of finished requests
        for r, (q, req, first, n, c) in enumerate(rows):
            key = (q.rid, req)
            if kind == "prefill":
                cache.mark_ready(self.pages[key])
                if self.keep_logits:
                    self.logits[key] = logits[r].cpu().numpy()
                done = q.out_len == 0
            else:
                self.generated[key] += 1
                done = self.generated[key] == q.out_len
            if done:
                cache.release(self.pages.pop(key))
                del self.generated[key]
        return self.e0.elapsed_time(self.e1) * 1e-3

    def standalone_logits(self, q, req: int) -> np.ndarray:
        """Next-token logits of one request computed privately (template and suffix in fresh pages, no sharing): what
        the serving run must reproduce for that request's prefill."""
        P, torch = self.shape.page_size, self.torch
        ids = self.prompt(q, req)
        n = len(ids)
        pages = self.cache.acquire_private((n + P - 1) // P)
        bt = np.array([pages], np.int32)
        batch = W.Batch(np.array([0, n], np.int32), np.array([n], np.int32), bt, np.array([-1], np.int32), np.zeros(0, np.int32),
                        self.num_pages, "standalone")
        pb = rs.relserve_batch_prepare(self.layer, batch)
        logits = torch.empty(1, self.vocab, dtype=torch.float32, device="cuda")
        rs.relserve_model_step(self.layer, pb, self.model, torch.from_numpy(ids).cuda(), logits, self.ws)
        torch.cuda.synchronize()
        pb.close()
        self.cache.release(pages)
        return logits[0].cpu().numpy()
