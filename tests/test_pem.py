"""Priority Estimation Model (Sec. 4.2: Algorithm 1, Eq. 10, Eq. 11): the oracle against hand-worked cases and
invariants, and the library's host-side implementation against the oracle."""
import numpy as np
import pytest

from oracle import pem as opem

BIG = 10 ** 9
MP, MD = (5.5e-7, 2.1e-4), (1.2e-6, 1.7e-4)


# ---------------------------------------------------------------- oracle pins
def test_no_limit_binds_one_prefill_batch_and_out_len_decode_batches():
    P, D = opem.batch_decompose([100, 100, 100], 2, BIG, BIG, BIG)
    assert P == [[0, 1, 2]] and D == [[0, 1, 2], [0, 1, 2]]
    want = MP[0] * 300 + MP[1] + 2 * (MD[0] * 3 + MD[1])          # closed form of Eq. 10 for this case
    assert abs(opem.pem([100, 100, 100], 2, BIG, BIG, BIG, MP, MD) - want) < 1e-15


def test_prefill_batch_size_limit_closes_prefill_batches_only():
    # 100 + 100 > 150: every request gets its own prefill batch; all three decode together
    P, D = opem.batch_decompose([100, 100, 100], 3, BIG, BIG, 150)
    assert P == [[0], [1], [2]] and D == [[0, 1, 2]] * 3
    P, D = opem.batch_decompose([100, 40, 30, 90], 1, BIG, BIG, 150)     # 100+40 fits, +30 does not; 30+90 fits
    assert P == [[0, 1], [2, 3]] and D == [[0, 1, 2, 3]]


def test_decode_batch_size_limit_decodes_to_completion():
    # the third request would be the third sequence: the first two are prefilled and decoded out first
    P, D = opem.batch_decompose([100, 100, 100], 2, BIG, 2, BIG)
    assert P == [[0, 1], [2]] and D == [[0, 1], [0, 1], [2], [2]]


def test_capacity_limit_decodes_to_completion_and_restarts_the_count():
    # cap 250: 100, 200, then 300 > 250 -> flush; the count restarts, so requests 2 and 3 share the next round
    P, D = opem.batch_decompose([100, 100, 100, 100, 100], 1, 250, BIG, BIG)
    assert P == [[0, 1], [2, 3], [4]] and D == [[0, 1], [2, 3], [4]]


def test_both_limits_in_one_step_emit_no_empty_batch():
    # request 2 trips cap (flush: p = [0, 1] closed) and then fits the fresh prefill batch
    P, D = opem.batch_decompose([80, 80, 80], 1, 200, BIG, 100)
    assert P == [[0], [1], [2]] and D == [[0, 1], [2]]
    assert all(len(p) > 0 for p in P) and all(len(d) > 0 for d in D)


def test_oversized_and_prefilled_and_finished_requests():
    P, D = opem.batch_decompose([500, 10], 1, BIG, BIG, 100)                # larger than the batch limit: alone
    assert P == [[0], [1]] and D == [[0, 1]]
    P, D = opem.batch_decompose([0, 50, 0], 2, BIG, BIG, BIG)               # already prefilled: decode only
    assert P == [[1]] and D == [[0, 1, 2]] * 2
    P, D = opem.batch_decompose([0, 50, 0], 2, BIG, BIG, BIG, decodes=[False, True, True])
    assert P == [[1]] and D == [[1, 2]] * 2
    assert opem.batch_decompose([], 3, 10, 10, 10) == ([], [])


def test_invariants_on_random_relqueries():
    rng = np.random.default_rng(0)
    for _ in range(200):
        n = int(rng.integers(1, 60))
        utok = [int(x) for x in rng.integers(0, 400, n)]
        ol = int(rng.integers(1, 6))
        cap, mns, mnbt = int(rng.integers(300, 4000)), int(rng.integers(1, 20)), int(rng.integers(100, 2000))
        P, D = opem.batch_decompose(utok, ol, cap, mns, mnbt)
        flat = [r for p in P for r in p]
        assert flat == [i for i in range(n) if utok[i] > 0]                  # each request prefilled once, in order
        for p in P:
            assert sum(utok[r] for r in p) <= mnbt or len(p) == 1
        assert len(D) % ol == 0
        groups = D[::ol]
        assert [r for g in groups for r in g] == list(range(n))            # each request decoded in one group
        for k, g in enumerate(groups):
            assert D[k * ol:(k + 1) * ol] == [g] * ol and 1 <= len(g) <= mns
            assert sum(utok[r] for r in g) <= cap or len(g) == 1
        # Eq. 10 is additive over the batches
        want = sum(MP[0] * sum(utok[r] for r in p) + MP[1] for p in P) + sum(MD[0] * len(d) + MD[1] for d in D)
        assert abs(opem.pem(utok, ol, cap, mns, mnbt, MP, MD) - want) < 1e-12


def test_utok_estimate_is_the_sample_miss_ratio():
    est = opem.utok_estimate([100, 200, 50], sample_utok=[30, 10], sample_tok=[100, 100])    # miss ratio 0.2
    assert est == pytest.approx([20.0, 40.0, 10.0])
