"""Multi-step request flows (prefill chunks, then decode steps) over one paged
cache.  A flow is run through any `step(batch, x_bits) -> y rows` callable, so the
same schedule can drive the oracle and the GPU library.  Test helper only.
"""
from dataclasses import dataclass

import numpy as np

from paper_2601_11546_amd import workloads as W


@dataclass
class Flow:
    shape: W.LayerShape
    seq_len: list            # full length of each request
    x_full: list             # per request [L_r, H] bf16 bits
    block_table: np.ndarray  # [R, max_blocks]
    prefix_id: np.ndarray
    prefix_len: np.ndarray
    num_pages: int
    schedule: list           # list of steps; a step = list of (request, n_tokens)
    start: list = None       # tokens of each request already in the cache before the first step


def make_flow(shape, seq_len, schedule, seed, shared_prefix=None, page_perm_seed=None, start=None):
    """shared_prefix = (length, [member requests]) makes the members' first `length`
    tokens identical and backed by the same pages."""
    R = len(seq_len)
    rng = np.random.default_rng(seed)
    x_full = [W.f32_to_bf16_bits(rng.standard_normal((L, shape.hidden), dtype=np.float32)) for L in seq_len]
    pid = np.full(R, -1, np.int32)
    plen = np.zeros(0, np.int32)
    if shared_prefix is not None:
        n, members = shared_prefix
        for m in members[1:]:
            x_full[m][:n] = x_full[members[0]][:n]
        pid[list(members)] = 0
        plen = np.array([n], np.int32)
    b = W.build_batch(shape, np.ones(R, np.int32), np.asarray(seq_len, np.int32), pid, plen,
                      seed=seed if page_perm_seed is None else page_perm_seed)
    return Flow(shape, list(seq_len), x_full, b.block_table, pid, plen, b.num_pages, schedule, start)


def run_flow(flow: Flow, step_fn):
    """step_fn(batch, x_bits[T,H]) -> array-like [T, H] (any dtype).  Returns
    per-request list of [L_r, H] outputs assembled from all steps."""
    R = len(flow.seq_len)
    done = list(flow.start) if flow.start else [0] * R
    outs = [None] * R
    for step in flow.schedule:
        reqs = [r for r, _ in step]
        q_len = np.array([n for _, n in step], np.int32)
        ctx = np.array([done[r] + n for r, n in step], np.int32)
        qs = np.zeros(len(step) + 1, np.int32)
        qs[1:] = np.cumsum(q_len)
        # a request that is still writing its template prefix does not claim it as shared
        pid = np.array([flow.prefix_id[r] if flow.prefix_id[r] >= 0 and done[r] >= flow.prefix_len[flow.prefix_id[r]]
                        else -1 for r in reqs], np.int32)
        batch = W.Batch(qs, ctx, np.ascontiguousarray(flow.block_table[reqs]), pid,
                        flow.prefix_len, flow.num_pages)
        x = np.concatenate([flow.x_full[r][done[r]:done[r] + n] for r, n in step], axis=0)
        y = np.asarray(step_fn(batch, x))
        for i, (r, n) in enumerate(step):
            if outs[r] is None:
                outs[r] = np.zeros((flow.seq_len[r], y.shape[1]), y.dtype)
            outs[r][done[r]:done[r] + n] = y[qs[i]:qs[i + 1]]
            done[r] += n
    assert done == flow.seq_len, (done, flow.seq_len)
    return outs


def gather_kv(shape, block_table_row, L, k_pages, v_pages):
    """Contiguous [L, n_kv, d] bits of one request, read through its block-table row."""
    P = shape.page_size
    pos = np.arange(L)
    slots = block_table_row[pos // P].astype(np.int64) * P + pos % P
    kf = k_pages.reshape(-1, shape.n_kv_heads, shape.head_dim)
    vf = v_pages.reshape(-1, shape.n_kv_heads, shape.head_dim)
    return kf[slots], vf[slots]


def run_model_flow(flow: Flow, token_ids: list, model_step_fn):
    """Like run_flow for a whole stack: model_step_fn(batch, ids[T]) -> logits [B, V].
    Returns, per request, the logits produced by the step that consumed its LAST token."""
    R = len(flow.seq_len)
    done = list(flow.start) if flow.start else [0] * R
    final = [None] * R
    for step in flow.schedule:
        reqs = [r for r, _ in step]
        q_len = np.array([n for _, n in step], np.int32)
        ctx = np.array([done[r] + n for r, n in step], np.int32)
        qs = np.zeros(len(step) + 1, np.int32)
        qs[1:] = np.cumsum(q_len)
        pid = np.array([flow.prefix_id[r] if flow.prefix_id[r] >= 0 and done[r] >= flow.prefix_len[flow.prefix_id[r]]
                        else -1 for r in reqs], np.int32)
        batch = W.Batch(qs, ctx, np.ascontiguousarray(flow.block_table[reqs]), pid, flow.prefix_len, flow.num_pages)
        ids = np.concatenate([token_ids[r][done[r]:done[r] + n] for r, n in step]).astype(np.int32)
        logits = np.asarray(model_step_fn(batch, ids))
        for i, (r, n) in enumerate(step):
            done[r] += n
            if done[r] == flow.seq_len[r]:
                final[r] = logits[i]
    return final
