"""Oracle of the Priority Estimation Model (test infrastructure, not product code).

Sec. 4.2: Algorithm 1 (Batch Decomposition) walks the requests of a relQuery in order and simulates the
engine: requests join the current prefill batch p and the current decode batch d; p is closed when the next
request would push it over max_num_batched_tokens; when the next request would push the tokens held on the
GPU over `cap` or the decode batch over max_num_seqs, p is closed and d is decoded to completion (OL copies
of d), after which both start empty again; what is left at the end is closed the same way.  Eq. 10: the
priority of the relQuery is the sum of the predicted durations (Eq. 9) of all these batches.

Readings where the algorithm's text leaves a choice (the product takes the same ones):
  * the running token count `accum` starts again at zero together with p and d after a decode-to-completion
    (the listing does not say; if it kept growing, every later request would force a flush);
  * an empty batch is never emitted (a flush can find p empty right after a max_num_batched_tokens close);
  * a request larger than max_num_batched_tokens forms a prefill batch of its own;
  * a request with utok = 0 (already prefilled) joins no prefill batch; a request flagged as not decoding any
    more joins no decode batch (Sec. 4.2, last sentence of the Algorithm 1 walk-through).

Pure Python loops.  Only tests import this.
"""
from __future__ import annotations


def _segments(utok, decodes, cap, mns):
    """First pass: where the engine has to decode to completion.  A segment is a longest run of consecutive requests
    whose uncached tokens together fit `cap` and of which at most `mns` still decode; the next request opens a new
    segment as soon as it would break either limit (a request that breaks a limit alone is a segment of its own)."""
    segs, start, tokens, decoding = [], 0, 0, 0
    for i in range(len(utok)):
        if i > start and (tokens + utok[i] > cap or decoding + decodes[i] > mns):
            segs.append((start, i))
            start, tokens, decoding = i, 0, 0
        tokens += utok[i]
        decoding += decodes[i]
    if len(utok) > start:
        segs.append((start, len(utok)))
    return segs


def _prefill_batches(utok, lo, hi, mnbt):
    """Second pass, inside one segment: its requests that still have tokens to compute, in order, cut into prefill
    batches of at most `mnbt` tokens (a longer request is a batch of its own)."""
    batches, cur, cur_tokens = [], [], 0
    for i in range(lo, hi):
        if utok[i] + cur_tokens > mnbt and cur:
            batches.append(cur)
            cur, cur_tokens = [], 0
        if utok[i] > 0:
            cur.append(i)
            cur_tokens += utok[i]
    if cur:
        batches.append(cur)
    return batches


def batch_decompose(utok, out_len, cap, mns, mnbt, decodes=None):
    """Returns (P, D): P = list of prefill batches (lists of request indices), D = list of decode batches
    (each decode group repeated out_len times).  Derived in two passes (segments between decodes-to-completion,
    then the prefill batches of each segment) rather than as one walk: same batches as Algorithm 1."""
    n = len(utok)
    decodes = [1] * n if decodes is None else [1 if x else 0 for x in decodes]
    P, D = [], []
    for lo, hi in _segments(utok, decodes, cap, mns):
        P.extend(_prefill_batches(utok, lo, hi, mnbt))
        group = [i for i in range(lo, hi) if decodes[i]]
        if group:
            D.extend([list(group) for _ in range(out_len)])
    return P, D


def pem(utok, out_len, cap, mns, mnbt, prefill_model, decode_model, decodes=None):
    """Eq. 10 with Eq. 9's lines: models are (alpha, beta) pairs."""
    P, D = batch_decompose(utok, out_len, cap, mns, mnbt, decodes)
    ap, bp = prefill_model
    ad, bd = decode_model
    total = 0.0
    for p in P:
        total += ap * sum(utok[r] for r in p) + bp
    for d in D:
        total += ad * len(d) + bd
    return total


def utok_estimate(tok, sample_utok, sample_tok):
    """Eq. 11: uncached tokens of a request estimated from the cache miss ratio of a sample of its relQuery."""
    ratio = sum(sample_utok) / sum(sample_tok)
    return [t * ratio for t in tok]
