"""Oracle of the Adaptive Batch Arranger's decision and of the starvation rule (test infrastructure only).

Sec. 4.3: at every iteration the arranger chooses between the candidate decode batch (all running requests)
and the candidate prefill batch (requests of the first waiting relQuery).  Empty candidates: run the other
one, or idle.  Otherwise compare the smallest priority values m+ (running) and m- (waiting), Eq. 14:
m+ > m- (a shorter relQuery waits: preempt) and m+ = m- (same relQuery: keep prefilling) run the prefill
candidate; m+ < m- (the running relQuery only has decode left) weighs the latency added to the running
relQueries (Eq. 15) against the latency saved for the waiting ones (Eq. 16) and prefills iff the total change
is negative.

Reading: Eq. 16 defines a latency REDUCTION as a positive quantity and Eq. 17 prints the total as a sum; the
total change used here is delta = delta_plus - delta_minus (with the printed sum the prefill candidate could
never win, which contradicts the text around the equation).

Sec. 4.2 "Starvation Prevention", Eq. 13: unit waiting time = waiting time / requests of the relQuery as
submitted; above a threshold the priority value becomes zero.
"""
from __future__ import annotations

IDLE, PREFILL, DECODE = 0, 1, 2


def delta(prefill_model, decode_model, cand_utok, cand_reqs, cand_out_len, running_out_lens, n_waiting):
    ap, bp = prefill_model
    ad, bd = decode_model
    l_prefill = ap * cand_utok + bp                                           # Eq. 9
    d_plus = l_prefill * len(running_out_lens)                                # Eq. 15, first term
    for ol in running_out_lens:                                               # Eq. 15, second term
        d_plus += ad * cand_reqs * min(ol, cand_out_len)
    d_minus = n_waiting * bd * min(cand_out_len, max(running_out_lens))       # Eq. 16
    return d_plus - d_minus


def decide(m_running, m_waiting, n_running_reqs, cand_reqs, cand_utok, cand_out_len, running_out_lens, n_waiting,
           prefill_model, decode_model):
    if n_running_reqs == 0 and cand_reqs == 0:
        return IDLE
    if n_running_reqs == 0:
        return PREFILL
    if cand_reqs == 0:
        return DECODE
    if m_running >= m_waiting:                                                # preemption, or the same relQuery
        return PREFILL
    d = delta(prefill_model, decode_model, cand_utok, cand_reqs, cand_out_len, running_out_lens, n_waiting)
    return PREFILL if d < 0 else DECODE


def starved_priority(priority, waiting_time, n_requests_submitted, threshold):
    """Eq. 13 and the rule below it."""
    return 0.0 if waiting_time / n_requests_submitted > threshold else priority
