"""Adaptive Batch Arranger decision (Sec. 4.3, Eq. 14-17) and starvation rule (Eq. 13): oracle pins, and the
library's host-side functions against the oracle."""
import numpy as np
import pytest

from oracle import aba as oaba

MP, MD = (2.0e-5, 8.0e-3), (5.0e-5, 7.0e-3)          # seconds; of the order fitted for a 40-layer 13B step


def test_empty_candidates():
    args = dict(cand_utok=0, cand_out_len=5, running_out_lens=[5], n_waiting=1, prefill_model=MP, decode_model=MD)
    assert oaba.decide(1.0, 2.0, 0, 0, **args) == oaba.IDLE
    assert oaba.decide(1.0, 2.0, 0, 3, **args) == oaba.PREFILL
    assert oaba.decide(1.0, 2.0, 4, 0, **args) == oaba.DECODE


def test_preemption_and_internal_execution_prefill_first():
    args = dict(cand_utok=3000, cand_out_len=5, running_out_lens=[5], n_waiting=1, prefill_model=MP, decode_model=MD)
    assert oaba.decide(9.0, 2.0, 4, 3, **args) == oaba.PREFILL       # a shorter relQuery waits
    assert oaba.decide(2.0, 2.0, 4, 3, **args) == oaba.PREFILL       # requests of the running relQuery itself


def test_delta_hand_worked():
    # one running relQuery (OL 5); candidate: 10 requests, 1000 uncached tokens, OL 3; two waiting relQueries
    # L_prefill = 2e-5 * 1000 + 8e-3 = 0.028;  delta+ = 0.028 * 1 + 5e-5 * 10 * min(5, 3) = 0.028 + 0.0015 = 0.0295
    # delta- = 2 * 7e-3 * min(3, 5) = 0.042;   delta = -0.0125 < 0 -> prefill first
    d = oaba.delta(MP, MD, 1000, 10, 3, [5], 2)
    assert abs(d - (0.0295 - 0.042)) < 1e-15
    assert oaba.decide(1.0, 2.0, 4, 10, 1000, 3, [5], 2, MP, MD) == oaba.PREFILL
    # the same candidate with 4000 tokens and one waiting relQuery: 0.088 + 0.0015 - 0.021 > 0 -> decode first
    assert abs(oaba.delta(MP, MD, 4000, 10, 3, [5], 1) - (0.0895 - 0.021)) < 1e-15
    assert oaba.decide(1.0, 2.0, 4, 10, 4000, 3, [5], 1, MP, MD) == oaba.DECODE


def test_delta_monotonicities():
    base = oaba.delta(MP, MD, 1000, 10, 4, [5, 8], 2)
    assert oaba.delta(MP, MD, 2000, 10, 4, [5, 8], 2) > base       # a longer prefill delays the running ones more
    assert oaba.delta(MP, MD, 1000, 20, 4, [5, 8], 2) > base       # more joining requests slow their decode steps
    assert oaba.delta(MP, MD, 1000, 10, 4, [5, 8], 5) < base       # more waiting relQueries gain
    assert oaba.delta(MP, MD, 1000, 10, 4, [5, 8, 8], 2) > base    # more running relQueries pay


def test_starvation_rule():
    assert oaba.starved_priority(3.5, 10.0, 100, 2.0) == 3.5       # 0.1 s per request
    assert oaba.starved_priority(3.5, 300.0, 100, 2.0) == 0.0      # 3 s per request > 2
    assert oaba.starved_priority(3.5, 200.0, 100, 2.0) == 3.5      # exactly at the threshold: not above it


# ---------------------------------------------------------------- the library against the oracle
@pytest.fixture(scope="module")
def rs():
    from paper_2601_11546_amd import binding
    return binding


def test_library_aba_matches_oracle(rs):
    rng = np.random.default_rng(3)
    mp, md = {"alpha": MP[0], "beta": MP[1]}, {"alpha": MD[0], "beta": MD[1]}
    seen = set()
    for _ in range(2000):
        n_run = int(rng.integers(0, 3)) * int(rng.integers(1, 50))
        cand = int(rng.integers(0, 3)) * int(rng.integers(1, 40))
        utok = int(rng.integers(0, 8192))
        ol = int(rng.integers(1, 100))
        run_ol = [int(x) for x in rng.integers(1, 100, int(rng.integers(1, 5)))]
        n_wait = int(rng.integers(1, 8))
        m_run, m_wait = float(rng.integers(0, 4)), float(rng.integers(0, 4))
        want = oaba.decide(m_run, m_wait, n_run, cand, utok, ol, run_ol, n_wait, MP, MD)
        got, d = rs.relserve_aba_decide(m_run, m_wait, n_run, cand, utok, ol, run_ol, n_wait, mp, md)
        assert got == want
        if n_run and cand and m_run < m_wait:
            wd = oaba.delta(MP, MD, utok, cand, ol, run_ol, n_wait)
            assert abs(d - wd) <= 1e-12 * max(1.0, abs(wd))
        seen.add(got)
    assert seen == {oaba.IDLE, oaba.PREFILL, oaba.DECODE}
    got, d = rs.relserve_aba_decide(1.0, 2.0, 4, 10, 1000, 3, [5], 2, mp, md)
    assert got == oaba.PREFILL and abs(d + 0.0125) < 1e-15


def test_library_starvation_matches_oracle(rs):
    for prio, wait, n, thr in ((3.5, 10.0, 100, 2.0), (3.5, 300.0, 100, 2.0), (3.5, 200.0, 100, 2.0), (0.2, 5.0, 1, 4.9)):
        assert rs.relserve_starved_priority(prio, wait, n, thr) == oaba.starved_priority(prio, wait, n, thr)
    with pytest.raises(rs.RelserveError):
        rs.relserve_starved_priority(1.0, 1.0, 0, 1.0)
