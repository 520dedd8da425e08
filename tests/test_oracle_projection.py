"""Pins for the oracle's projection with bisection (Section 3.4, Algorithm 1 of arXiv
2109.00170): block scores, top-N selection and the bisection itself, against things other than
the routines: float64 norms from numpy's library routine, exact integer cases, a selection
written with a plain Python sort, and brute force over every N on small networks."""
import numpy as np
import pytest

import oracle


def test_block_scores_against_library_norm_and_exact_integers():
    rng = np.random.default_rng(41)
    for (Cout, Cin, k, V) in [(8, 5, 1, 4), (10, 3, 3, 4), (7, 4, 1, 2), (16, 2, 3, 16), (5, 5, 1, 1)]:
        W = rng.standard_normal((Cout, Cin, k, k)).astype(np.float32)
        s = oracle.block_scores(W, V)
        G = oracle.n_groups(Cout, V)
        assert s.shape == (G, Cin, k, k) and s.dtype == np.float32
        Wp = np.zeros((G * V, Cin, k, k), dtype=np.float64)
        Wp[:Cout] = W
        ref = np.linalg.norm(Wp.reshape(G, V, Cin, k, k), axis=1) ** 2
        assert np.max(np.abs(s - ref)) <= 1e-6 * np.max(ref)
        # integer weights: every product and sum is exact in float32
        Wi = rng.integers(-9, 10, size=(Cout, Cin, k, k)).astype(np.float32)
        si = oracle.block_scores(Wi, V)
        Wp[:] = 0
        Wp[:Cout] = Wi
        assert np.array_equal(si, (Wp.reshape(G, V, Cin, k, k) ** 2).sum(axis=1).astype(np.float32))


def test_block_scores_is_the_sequential_float32_sum():
    # values chosen so that the order of the additions shows: 1 + 2^-24 rounds back to 1
    W = np.zeros((4, 1, 1, 1), dtype=np.float32)
    W[:, 0, 0, 0] = [1.0, 2.0 ** -12, 2.0 ** -12, 2.0 ** -12]
    assert oracle.block_scores(W, 4)[0, 0, 0, 0] == np.float32(1.0)
    # the same four values, small ones first: 2^-24 + 2^-24 = 2^-23 survives the final + 1
    W[:, 0, 0, 0] = [2.0 ** -12, 2.0 ** -12, 0.0, 1.0]
    assert oracle.block_scores(W, 4)[0, 0, 0, 0] == np.float32(1.0 + 2.0 ** -23)
    W[:, 0, 0, 0] = [1.0, 2.0 ** -12, 2.0 ** -12, 0.0]
    assert oracle.block_scores(W, 4)[0, 0, 0, 0] == np.float32(1.0)


def test_topn_mask_against_a_plain_sort():
    rng = np.random.default_rng(42)
    s = rng.random(500).astype(np.float32)
    s[rng.integers(0, 500, 60)] = np.float32(0.25)          # ties
    s[rng.integers(0, 500, 20)] = np.float32(0.0)
    order = sorted(range(500), key=lambda i: (-float(s[i]), i))
    for N in (0, 1, 7, 250, 499, 500):
        want = np.zeros(500, dtype=np.uint8)
        want[order[:N]] = 1
        got = oracle.topn_mask(s, N)
        assert np.array_equal(got, want)
        assert int(got.sum()) == N
        if 0 < N < 500:
            assert s[got == 1].min() >= s[got == 0].max()
    # hand-made: two equal maxima, the lower index wins
    assert list(oracle.topn_mask(np.array([1, 3, 3, 2], np.float32), 1)) == [0, 1, 0, 0]
    assert list(oracle.topn_mask(np.array([1, 3, 3, 2], np.float32), 3)) == [0, 1, 1, 1]
    with pytest.raises(ValueError):
        oracle.topn_mask(s, 501)


def linear_tables(sizes, Vs, slopes, t_empty):
    tables = []
    for n, V, a, t in zip(sizes, Vs, slopes, t_empty):
        k = np.arange(11) * 0.1 * n * V
        tables.append((k, t + a * k))
    return tables


@pytest.mark.parametrize("seed", range(5))
def test_bisection_against_brute_force_over_every_n(seed):
    """With latency tables that grow with the number of kept weights, the latency of top-N grows
    with N; the bisection must end next to the largest N whose latency is below the budget."""
    rng = np.random.default_rng(50 + seed)
    sizes = [int(x) for x in rng.integers(20, 80, size=3)]
    Vs = [4, 4, 2]
    scores = [rng.random(n).astype(np.float32) for n in sizes]
    tables = linear_tables(sizes, Vs, rng.random(3) * 0.05 + 0.01, rng.random(3) * 2 + 1)
    tau = 1.5
    total = sum(sizes)
    allscores = np.concatenate(scores)
    starts = np.concatenate([[0], np.cumsum(sizes)])

    def T(N):
        m = oracle.topn_mask(allscores, N)
        nnz = [float(m[starts[l]:starts[l + 1]].sum()) * Vs[l] for l in range(3)]
        return tau + sum(float(np.interp(nnz[l], *tables[l])) for l in range(3))

    lat = [T(N) for N in range(total + 1)]
    assert all(b >= a for a, b in zip(lat, lat[1:]))
    budget = 0.5 * (lat[0] + lat[-1])
    best = max(N for N in range(total + 1) if lat[N] < budget)
    N, masks, t0, t1 = oracle.project_latency(scores, Vs, tables, tau, budget, eps=1e-9)
    assert best <= N <= best + 1
    assert t0 < budget <= t1
    assert sum(int(m.sum()) for m in masks) == N
    assert [m.shape for m in masks] == [s.shape for s in scores]
    got = np.concatenate([m.reshape(-1) for m in masks])
    assert np.array_equal(got, oracle.topn_mask(allscores, N))
    # a loose tolerance stops early but still brackets the budget
    N2, _, t0, t1 = oracle.project_latency(scores, Vs, tables, tau, budget, eps=0.5 * (lat[-1] - lat[0]))
    assert t0 <= budget <= t1 or t1 - t0 <= 0.5 * (lat[-1] - lat[0])
    assert 0 <= N2 <= total


def test_bisection_closed_form_single_layer():
    # one layer, 100 blocks of 4 weights, latency 2 + 0.01 * nnz: budget 4.02 admits nnz < 202, i.e. 50 blocks
    scores = [np.arange(100, dtype=np.float32)]
    k = np.arange(11) * 40.0
    tables = [(k, 2.0 + 0.01 * k)]
    N, masks, t0, t1 = oracle.project_latency(scores, [4], tables, 0.0, 4.02, eps=1e-12)
    assert N == 50 and t0 == pytest.approx(4.0) and t1 == pytest.approx(4.04)
    assert np.array_equal(np.nonzero(masks[0])[0], np.arange(50, 100))     # the 50 largest scores
    # budgets outside the reachable range keep nothing / everything (up to the final halving)
    N, _, _, _ = oracle.project_latency(scores, [4], tables, 0.0, 1.0, eps=1e-12)
    assert N == 0
    N, _, _, _ = oracle.project_latency(scores, [4], tables, 0.0, 100.0, eps=1e-12)
    assert N >= 99
