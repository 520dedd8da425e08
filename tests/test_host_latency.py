"""The library's latency model (host code, no GPU) against the oracle's term-by-term sum of
Section 3.3, Eqs. (2), (4)-(6)."""
import numpy as np
import pytest

import oracle
import paper_2109_00170_amd as alcs


def random_table(rng, n=None):
    n = int(rng.integers(2, 14)) if n is None else n
    k = np.concatenate([[0.0], np.cumsum(rng.integers(1, 100000, size=n - 1))]).astype(np.float64)
    t = rng.random(n) * 100 + 0.5
    return k, t


@pytest.mark.parametrize("seed", range(8))
def test_estimate_matches_oracle(seed):
    rng = np.random.default_rng(100 + seed)
    k, t = random_table(rng)
    probes = np.concatenate([k, 0.5 * (k[1:] + k[:-1]), rng.random(300) * k[-1], [k[-1] * 2, k[-1] + 1]])
    for s in probes:
        got = alcs.alcs_latency_estimate(k, t, s)
        want = oracle.latency_estimate(k, t, s)
        assert abs(got - want) <= 1e-12 * max(1.0, abs(want)), (s, got, want)


def test_eleven_point_tables_of_a_network():
    rng = np.random.default_rng(7)
    tables, nnz = [], []
    for l in range(13):
        N = int(rng.integers(1000, 10 ** 6))
        k = np.arange(11) * 0.1 * N
        t = 4.0 + np.sort(rng.random(11)) * 30
        tables.append((k, t))
        nnz.append(float(rng.integers(0, N + 1)))
    got = alcs.alcs_network_latency(12.5, tables, nnz)
    want = oracle.network_latency(12.5, tables, nnz)
    assert abs(got - want) <= 1e-12 * want
    assert alcs.alcs_network_latency(3.0, [], []) == 3.0


def test_rejected_tables():
    E = alcs.AlcsError
    with pytest.raises(E):
        alcs.alcs_latency_estimate([0.0], [1.0], 0.0)                       # fewer than two knots
    with pytest.raises(E):
        alcs.alcs_latency_estimate([0.0, 2.0, 2.0], [1.0, 2.0, 3.0], 1.0)   # knots not increasing
    with pytest.raises(E):
        alcs.alcs_latency_estimate([0.0, 2.0], [1.0, float("nan")], 1.0)
    with pytest.raises(E):
        alcs.alcs_latency_estimate([0.0, 2.0], [1.0, 2.0], float("nan"))
    with pytest.raises(E):
        alcs.alcs_network_latency(float("inf"), [([0.0, 1.0], [1.0, 2.0])], [0.5])
    with pytest.raises(E):
        alcs.alcs_network_latency(0.0, [([0.0, 1.0], [1.0, 2.0]), ([1.0, 0.0], [1.0, 2.0])], [0.5, 0.5])
