"""Batch-duration model (Sec. 4.2, Eq. 9): the fit's oracle against what the mathematics fixes, the
library's host-side fit against the oracle, and (GPU) the fit of measured layer-step durations."""
import numpy as np
import pytest

from oracle import duration_model as odm


def _noisy(seed, n=40, alpha=3.5e-7, beta=2.1e-4, noise=2e-5):
    rng = np.random.default_rng(seed)
    u = rng.integers(1, 8192, n).astype(np.float64)
    return u, alpha * u + beta + rng.standard_normal(n) * noise


# ---------------------------------------------------------------- the oracle against its pins
def test_oracle_recovers_an_exact_line():
    u = np.array([1.0, 5.0, 9.0, 100.0])
    a, b = odm.fit_line(u, 3.0 * u + 2.0)
    assert abs(a - 3.0) < 1e-12 and abs(b - 2.0) < 1e-12
    assert abs(odm.r_squared(u, 3.0 * u + 2.0, a, b) - 1.0) < 1e-12


def test_oracle_hand_worked_three_points():
    # points (0,0), (1,1), (2,1): means 1 and 2/3, Sxy = 1, Sxx = 2 -> slope 1/2, intercept 1/6;
    # residuals -1/6, 1/3, -1/6 -> SSres 1/6, SStot 2/3 -> R^2 = 3/4
    a, b = odm.fit_line([0, 1, 2], [0, 1, 1])
    assert abs(a - 0.5) < 1e-15 and abs(b - 1.0 / 6.0) < 1e-15
    assert abs(odm.r_squared([0, 1, 2], [0, 1, 1], a, b) - 0.75) < 1e-15


def test_oracle_is_the_least_squares_minimiser():
    u, s = _noisy(1)
    a, b = odm.fit_line(u, s)
    sse = lambda aa, bb: float(np.sum((s - aa * u - bb) ** 2))
    best = sse(a, b)
    for da in (-1e-9, 0.0, 1e-9):
        for db in (-1e-6, 0.0, 1e-6):
            if da or db:
                assert sse(a + da, b + db) > best
    res = s - odm.predict(a, b, u)              # normal equations: residuals orthogonal to 1 and to u
    assert abs(res.sum()) < 1e-12 and abs((res * u).sum()) < 1e-9


def test_oracle_matches_library_routines():
    from scipy import stats
    for seed in range(5):
        u, s = _noisy(seed)
        a, b = odm.fit_line(u, s)
        pa, pb = np.polyfit(u, s, 1)
        lr = stats.linregress(u, s)
        assert abs(a - pa) <= 1e-9 * abs(pa) and abs(b - pb) <= 1e-9 * abs(pb)
        assert abs(a - lr.slope) <= 1e-9 * abs(lr.slope) and abs(b - lr.intercept) <= 1e-9 * abs(lr.intercept)
        assert abs(odm.r_squared(u, s, a, b) - lr.rvalue ** 2) < 1e-9      # R^2 of a line fit = Pearson r squared


def test_oracle_invariances():
    u, s = _noisy(7)
    a, b = odm.fit_line(u, s)
    r2 = odm.r_squared(u, s, a, b)
    a2, b2 = odm.fit_line(u + 100.0, s)                   # shifted abscissa: same slope, intercept moves by -100 a
    assert abs(a2 - a) <= 1e-9 * abs(a) and abs(b2 - (b - 100.0 * a)) <= 1e-9 * abs(b)
    a3, b3 = odm.fit_line(u, 1e3 * s)                     # durations in other units scale both coefficients
    assert abs(a3 - 1e3 * a) <= 1e-9 * abs(a3) and abs(b3 - 1e3 * b) <= 1e-9 * abs(b3)
    assert abs(odm.r_squared(u, 1e3 * s, a3, b3) - r2) < 1e-9
    # durations that do not depend on the abscissa: slope 0 and nothing explained
    a4, b4 = odm.fit_line([1, 2, 3, 4], [5, 7, 7, 5])
    assert abs(a4) < 1e-15 and abs(b4 - 6.0) < 1e-15 and abs(odm.r_squared([1, 2, 3, 4], [5, 7, 7, 5], a4, b4)) < 1e-15


def test_oracle_rejects_degenerate_input():
    with pytest.raises(ValueError):
        odm.fit_line([1.0], [2.0])
    with pytest.raises(ValueError):
        odm.fit_line([3.0, 3.0, 3.0], [1.0, 2.0, 3.0])


# ---------------------------------------------------------------- the library's host-side fit against the oracle
@pytest.fixture(scope="module")
def rs():
    from paper_2601_11546_amd import binding
    return binding


def _same_fit(rs, u, s):
    m = rs.relserve_duration_fit(u, s)
    a, b = odm.fit_line(u, s)
    r2 = odm.r_squared(u, s, a, b)
    assert abs(m["alpha"] - a) <= 1e-9 * abs(a) + 1e-300
    assert abs(m["beta"] - b) <= 1e-9 * abs(b) + 1e-12 * float(np.abs(s).max())
    assert abs(m["r2"] - r2) < 1e-9
    assert m["n"] == len(u)
    return m


def test_library_fit_matches_oracle(rs):
    for seed in range(8):
        u, s = _noisy(seed, n=3 + 11 * seed)
        _same_fit(rs, u, s)
    # abscissae far from zero with a small spread: uncentred sums would lose the slope
    u = 1e6 + np.arange(20.0)
    _same_fit(rs, u, 2e-7 * u + 1e-3 + 1e-8 * np.sin(np.arange(20.0)))
    _same_fit(rs, np.array([0.0, 1.0, 2.0]), np.array([0.0, 1.0, 1.0]))
    m = _same_fit(rs, np.array([1.0, 2.0, 3.0, 4.0]), np.array([5.0, 5.0, 5.0, 5.0]))   # constant durations
    assert m["alpha"] == 0.0 and m["r2"] == 1.0


def test_library_predict_is_eq9(rs):
    u, s = _noisy(3)
    m = rs.relserve_duration_fit(u, s)
    for x in (0.0, 1.0, 777.0, 8192.0):
        assert abs(rs.relserve_duration_predict(m, x) - float(odm.predict(m["alpha"], m["beta"], x))) < 1e-15


def test_library_fit_rejects_degenerate_input(rs):
    for u, s in (([1.0], [2.0]), ([3.0, 3.0, 3.0], [1.0, 2.0, 3.0]), ([1.0, 2.0], [1.0, float("nan")]),
                 ([1.0, float("inf")], [1.0, 2.0])):
        with pytest.raises(rs.RelserveError) as e:
            rs.relserve_duration_fit(np.array(u), np.array(s))
        assert e.value.status == -14


# ---------------------------------------------------------------- measured durations (GPU)
@pytest.mark.gpu
def test_measured_durations_follow_eq9(rs):
    """Layer-step durations of seeded 13B-shaped batches: the line in uncached tokens explains the prefill
    durations and does so better than the line in total tokens (the paper's observation, Sec. 4.2); the
    decode durations grow with the request count; the library's fit of the measured points is the oracle's."""
    import torch
    from paper_2601_11546_amd import duration_model as dm
    from paper_2601_11546_amd import workloads as W
    print("duration model: 20 prefill and 10 decode batches, 13B layer shape", flush=True)
    res = dm.run(n_prefill=20, decode_sizes=(1, 8, 32, 64, 96, 128, 160, 192, 224, 256), steps=3, warmup=1)
    pts = np.array(res["prefill"]["points"])
    fu, ft = res["prefill"]["uncached_tokens"], res["prefill"]["total_tokens"]
    for fit, col in ((fu, 0), (ft, 1)):
        a, b = odm.fit_line(pts[:, col], pts[:, 2])
        assert abs(fit["alpha"] - a) <= 1e-9 * abs(a) and abs(fit["beta"] - b) <= 1e-9 * abs(b) + 1e-15
        assert abs(fit["r2"] - odm.r_squared(pts[:, col], pts[:, 2], a, b)) < 1e-9
    assert fu["alpha"] > 0 and fu["r2"] > 0.97, fu
    assert fu["r2"] > ft["r2"], (fu, ft)
    dpts = np.array(res["decode"]["points"])
    fd = res["decode"]["requests"]
    a, b = odm.fit_line(dpts[:, 0], dpts[:, 1])
    assert abs(fd["alpha"] - a) <= 1e-9 * abs(a) and abs(fd["beta"] - b) <= 1e-9 * abs(b)
    assert fd["alpha"] > 0 and fd["beta"] > 0 and fd["r2"] > 0.8, fd
    assert dpts[-1, 1] > dpts[0, 1]
