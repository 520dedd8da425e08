"""Pins for the oracle's latency model (Section 3.3 of arXiv 2109.00170, Eqs. (2), (4)-(6)).

Compared with things other than the oracle: numpy's library interpolation (the estimate is
the piecewise-linear interpolant of the measured points, clamped at both ends), values
worked out by hand, and properties the equations fix (exact at every knot, t_1 at s = 0,
linear inside an interval, additive over layers)."""
import numpy as np
import pytest

import oracle


def test_hand_worked_example():
    # three knots: 0 -> 2.0, 10 -> 4.0, 30 -> 5.0; slopes 0.2 and 0.05
    k, t = [0, 10, 30], [2.0, 4.0, 5.0]
    assert oracle.latency_estimate(k, t, 0) == 2.0
    assert oracle.latency_estimate(k, t, 5) == pytest.approx(3.0, abs=1e-15)          # 2 + 0.2*5
    assert oracle.latency_estimate(k, t, 10) == pytest.approx(4.0, abs=1e-15)
    assert oracle.latency_estimate(k, t, 14) == pytest.approx(4.2, abs=1e-15)         # 2 + 0.2*10 + 0.05*4
    assert oracle.latency_estimate(k, t, 30) == pytest.approx(5.0, abs=1e-15)
    assert oracle.latency_estimate(k, t, 100) == pytest.approx(5.0, abs=1e-15)        # min() caps the last interval


@pytest.mark.parametrize("seed", range(6))
def test_equals_library_interpolation(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(2, 14))
    k = np.cumsum(rng.integers(1, 1000, size=n)).astype(np.float64)
    k[0] = 0.0
    t = rng.random(n) * 50 + 1                      # run times need not be monotone
    for s in np.concatenate([k, rng.random(200) * k[-1], [k[-1] * 1.5]]):
        want = float(np.interp(s, k, t))
        assert oracle.latency_estimate(k, t, s) == pytest.approx(want, rel=1e-12, abs=1e-12)


def test_paper_knots_eleven_points():
    """The paper's choice: knots at 0, 0.1 N, ..., N (eleven measurements per layer)."""
    N = 512 * 512
    k = np.arange(11) * 0.1 * N
    t = 3.0 + 40.0 * (np.arange(11) / 10.0) ** 1.3
    for i in range(11):
        assert oracle.latency_estimate(k, t, k[i]) == pytest.approx(t[i], rel=1e-13)
    mid = 0.5 * (k[3] + k[4])
    assert oracle.latency_estimate(k, t, mid) == pytest.approx(0.5 * (t[3] + t[4]), rel=1e-13)
    # a dropped term, a wrong slope or an off-by-one interval would break one of these
    assert oracle.latency_estimate(k, t, k[4] - 1e-6 * N) < t[4] < oracle.latency_estimate(k, t, k[4] + 1e-6 * N)


def test_network_is_tau_plus_sum_over_layers():
    rng = np.random.default_rng(3)
    tables, nnz, want = [], [], 7.5
    for l in range(5):
        n = int(rng.integers(2, 12))
        k = np.concatenate([[0.0], np.cumsum(rng.integers(1, 500, size=n - 1))]).astype(np.float64)
        t = np.sort(rng.random(n) * 30)
        s = float(rng.random() * k[-1])
        tables.append((k, t))
        nnz.append(s)
        want += float(np.interp(s, k, t))
    assert oracle.network_latency(7.5, tables, nnz) == pytest.approx(want, rel=1e-12)
    assert oracle.network_latency(1.25, [], []) == 1.25


def test_rejects_bad_tables():
    with pytest.raises(ValueError):
        oracle.latency_estimate([0.0], [1.0], 0.0)
    with pytest.raises(ValueError):
        oracle.latency_estimate([0.0, 5.0, 5.0], [1.0, 2.0, 3.0], 1.0)
    with pytest.raises(ValueError):
        oracle.network_latency(0.0, [([0, 1], [1, 2])], [])
