"""GPU parity of the projection with bisection (Section 3.4, Algorithm 1 of arXiv 2109.00170):
block scores, top-N selection and the bisection against the oracle - integer and index work, so
everything is compared bit for bit (scores included: their arithmetic order is part of the
definition)."""
import ctypes

import numpy as np
import pytest

import oracle
import paper_2109_00170_amd as alcs

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("Cout,Cin,k,V", [(8, 5, 1, 4), (10, 3, 3, 4), (7, 4, 1, 2), (33, 2, 3, 16), (5, 5, 1, 1),
                                          (64, 129, 1, 8), (256, 257, 1, 4), (30, 64, 3, 4)])
def test_block_scores_bit_exact(Cout, Cin, k, V):
    import torch
    rng = np.random.default_rng(3000 + Cout + Cin)
    W = (rng.standard_normal((Cout, Cin, k, k)) * rng.random((Cout, 1, 1, 1)) * 3).astype(np.float32)
    W[rng.random(W.shape) < 0.1] = 0
    got = alcs.alcs_block_scores(torch.from_numpy(W).cuda(), V)
    torch.cuda.synchronize()
    want = oracle.block_scores(W, V)
    assert got.cpu().numpy().tobytes() == want.tobytes()


def scores_with_ties(n, seed):
    rng = np.random.default_rng(seed)
    s = (rng.random(n) ** 3).astype(np.float32)
    if n >= 8:
        s[rng.integers(0, n, n // 8)] = np.float32(0.125)      # many equal scores
        s[rng.integers(0, n, n // 16)] = np.float32(0.0)
        s[rng.integers(0, n, 2)] = np.float32(np.inf)
    return s


@pytest.mark.parametrize("n", [1, 2, 255, 256, 257, 5000, 70001, 600000])
def test_topn_mask_bit_exact(n):
    import torch
    s = scores_with_ties(n, 3100 + n)
    sd = torch.from_numpy(s).cuda()
    cuts = sorted(set([0, n] + [int(x) for x in np.random.default_rng(n).integers(0, n + 1, 5)]))
    for N in sorted(set([0, 1, n // 3, n // 2, max(n - 1, 0), n])):
        if N > n:
            continue
        mask, counts = alcs.alcs_topn_mask(sd, N, seg_starts=cuts)
        want = oracle.topn_mask(s, N)
        got = mask.cpu().numpy()
        assert got.tobytes() == want.tobytes(), "n=%d N=%d" % (n, N)
        assert list(counts) == [int(want[a:b].sum()) for a, b in zip(cuts, cuts[1:])]
        _, c2 = alcs.alcs_topn_mask(sd, N, want_mask=False)
        assert list(c2) == [N]


def test_topn_with_nan_scores_ranks_them_above_infinity():
    import torch
    s = np.array([1.0, np.nan, np.inf, 0.5, np.nan, 3.0], dtype=np.float32)
    for N in range(7):
        mask, _ = alcs.alcs_topn_mask(torch.from_numpy(s).cuda(), N)
        assert mask.cpu().numpy().tobytes() == oracle.topn_mask(s, N).tobytes()
    mask, _ = alcs.alcs_topn_mask(torch.from_numpy(s).cuda(), 2)
    assert list(mask.cpu().numpy()) == [0, 1, 0, 0, 1, 0]


def test_topn_all_scores_equal_keeps_the_lowest_indices():
    import torch
    s = np.full(1000, 2.5, dtype=np.float32)
    mask, _ = alcs.alcs_topn_mask(torch.from_numpy(s).cuda(), 300)
    got = mask.cpu().numpy()
    assert got[:300].all() and not got[300:].any()


def synthetic_network(seed, scale=1):
    """Layer shapes of the MobileNetV1 pointwise convs (scaled down), Gaussian weights with a
    per-layer magnitude, and latency tables shaped like measured ones (a floor plus a slope)."""
    rng = np.random.default_rng(seed)
    shapes = [(32, 64), (64, 128), (128, 128), (128, 256), (256, 256), (256, 512)] + [(512, 512)] * 5 + \
             [(512, 1024), (1024, 1024)]
    Ws, tables = [], []
    for (ci, co) in shapes:
        ci, co = max(4, ci // scale), max(4, co // scale)
        Ws.append((rng.standard_normal((co, ci, 1, 1)) * (0.05 + rng.random() * 0.2)).astype(np.float32))
        nw = float(co * ci)
        k = np.arange(11) * 0.1 * nw
        floor, slope = 8.0 + 10 * rng.random(), (20 + 40 * rng.random()) / nw
        t = floor + slope * k * (1.0 + 0.1 * np.sin(np.arange(11)))      # locally linear, not globally
        tables.append((k, np.maximum.accumulate(t)))
    return Ws, tables


@pytest.mark.parametrize("seed,scale,frac", [(1, 8, 0.5), (2, 8, 0.2), (3, 4, 0.8), (4, 1, 0.45)])
def test_projection_matches_the_oracle(seed, scale, frac):
    import torch
    Ws, tables = synthetic_network(3200 + seed, scale)
    V = 4
    sc_dev = [alcs.alcs_block_scores(torch.from_numpy(W).cuda(), V) for W in Ws]
    sc_ref = [oracle.block_scores(W, V) for W in Ws]
    for a, b in zip(sc_dev, sc_ref):
        assert a.cpu().numpy().tobytes() == b.tobytes()
    starts = np.concatenate([[0], np.cumsum([s.size for s in sc_ref])]).astype(np.int64)
    allsc = torch.cat([s.reshape(-1) for s in sc_dev])
    tau = 25.0
    t_none = tau + sum(t[0] for _, t in tables)
    t_all = tau + sum(t[-1] for _, t in tables)
    budget = t_none + frac * (t_all - t_none)
    eps = 1e-3
    N, mask, t0, t1 = alcs.alcs_project_latency(allsc, starts, [V] * len(Ws), tables, tau, budget, eps)
    Nr, masks_r, t0r, t1r = oracle.project_latency(sc_ref, [V] * len(Ws), tables, tau, budget, eps)
    assert N == Nr
    assert abs(t0 - t0r) <= 1e-9 * t0r and abs(t1 - t1r) <= 1e-9 * t1r
    assert t0 < budget <= t1 or t1 - t0 <= eps
    want = np.concatenate([m.reshape(-1) for m in masks_r])
    assert mask.cpu().numpy().tobytes() == want.tobytes()
    # the projected network can be packed and its latency estimate honours the bracket
    nnz = [float(int(m.sum()) * V) for m in masks_r]
    assert t0 - 1e-9 <= alcs.alcs_network_latency(tau, tables, nnz) <= t1 + 1e-9


def test_projection_feeds_the_packer():
    """The mask that comes out of the projection is the mask alcs_pack_weights takes."""
    import torch
    rng = np.random.default_rng(3300)
    W = rng.standard_normal((64, 48, 1, 1)).astype(np.float32)
    sc = alcs.alcs_block_scores(torch.from_numpy(W).cuda(), 4)
    k = np.arange(11) * 0.1 * W.size
    N, mask, _, _ = alcs.alcs_project_latency(sc.reshape(-1), [0, sc.numel()], [4], [(k, 5.0 + 0.01 * k)], 0.0,
                                              5.0 + 0.01 * 0.3 * W.size, 1e-6)
    m = mask.cpu().numpy().reshape(16, 48, 1, 1)
    assert abs(int(m.sum()) - round(0.3 * 16 * 48)) <= 1
    packed = alcs.alcs_pack_weights(W, m, 4)
    assert packed.nnzb == int(m.sum())
    for got, want in zip(packed.export(), oracle.pack(W, m, 4)):
        assert got.tobytes() == want.tobytes()
    packed.free()


def test_rejected_arguments():
    import torch
    lib = alcs.load_library()
    s = torch.zeros(100, device="cuda")
    ws = torch.zeros(1024, dtype=torch.int64, device="cuda")
    P = lambda t: ctypes.c_void_p(t.data_ptr())
    LL = ctypes.c_longlong
    assert lib.alcs_topn_mask(P(s), LL(100), LL(101), None, 0, None, None, P(ws), None) < 0
    assert lib.alcs_topn_mask(P(s), LL(100), LL(-1), None, 0, None, None, P(ws), None) < 0
    assert lib.alcs_topn_mask(None, LL(100), LL(5), None, 0, None, None, P(ws), None) < 0
    assert lib.alcs_topn_mask(P(s), LL(100), LL(5), None, 0, None, None, None, None) < 0
    bad = (ctypes.c_longlong * 3)(0, 120, 100)
    assert lib.alcs_topn_mask(P(s), LL(100), LL(5), bad, 2, None, None, P(ws), None) < 0
    assert lib.alcs_block_scores(P(s), 4, 4, 1, 3, P(s), None) < 0          # V = 3
    assert lib.alcs_block_scores(P(s), 4, 4, 5, 4, P(s), None) < 0          # kernel = 5
    torch.cuda.synchronize()
