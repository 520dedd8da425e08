"""GPU parity on seeded random layer shapes: kernel size, stride, group size, channel
counts (including counts that are no multiple of anything), image sizes down to one
pixel, batch, sparsity from 0 to 1, with and without bias, plain and fused epilogue.
Every case is a valid call; the point is to reach combinations the hand-picked cases miss."""
import numpy as np
import pytest

import oracle
import paper_2109_00170_amd as alcs
import workloads
from gpu_util import TOL, assert_close_after_activation

pytestmark = pytest.mark.gpu


def draw(seed):
    rng = np.random.default_rng(seed)
    k = int(rng.choice([1, 1, 3]))
    stride = int(rng.choice([1, 1, 2]))
    V = int(rng.choice([1, 2, 4, 4, 8, 16]))
    wide = rng.random() < 0.15
    Cin = int(rng.integers(640, 1400)) if (wide and k == 1) else int(rng.integers(1, 130))
    Cout = int(rng.integers(1, 100))
    H = int(rng.integers(1, 34))
    W = int(rng.integers(1, 34))
    N = int(rng.integers(1, 5))
    sparsity = float(rng.choice([0.0, 0.3, 0.6, 0.8, 0.9, 0.97, 1.0]))
    kind = str(rng.choice(["exact", "exact", "zipf"]))
    if kind == "zipf":
        sparsity = min(max(sparsity, 0.3), 0.95)
    L = workloads.Layer("rnd%d" % seed, Cin, Cout, H, W, k=k, stride=stride, N=N, V=V, sparsity=sparsity,
                        w_std=0.2, mask_kind=kind, tap_shared=bool(rng.random() < 0.5))
    return L, bool(rng.random() < 0.5), str(rng.choice(["plain", "relu", "relu6+res", "res"]))


@pytest.mark.parametrize("seed", range(72))
def test_random_layer(seed):
    import torch
    L, with_bias, epi = draw(7000 + seed)
    d = workloads.make_layer(L, 7000 + seed, with_bias=with_bias)
    packed = alcs.alcs_pack_weights(d.W, d.mask, L.V)
    for got, want in zip(packed.export(), oracle.pack(d.W, d.mask, L.V)):
        assert got.tobytes() == want.tobytes()
    assert packed.selfcheck() == 0
    X = torch.from_numpy(d.X).cuda()
    b = None if d.bias is None else torch.from_numpy(d.bias).cuda()
    Y = torch.full((L.N, L.Cout, L.Ho, L.Wo), float("nan"), dtype=torch.float32, device="cuda")
    R = None
    act = None
    if epi == "plain":
        alcs.alcs_sparse_conv(packed, X, b, Y, stride=L.stride)
    else:
        act = {"relu": "relu", "relu6+res": "relu6", "res": None}[epi]
        if "res" in epi:
            R = np.random.default_rng(seed).standard_normal((L.N, L.Cout, L.Ho, L.Wo)).astype(np.float32)
        Rd = None if R is None else torch.from_numpy(R).cuda()
        alcs.alcs_sparse_conv_fused(packed, X, b, Rd, Y, stride=L.stride, activation=act)
    torch.cuda.synchronize()
    info = alcs.alcs_last_launch()
    got = Y.cpu().numpy()
    packed.free()
    assert not np.isnan(got).any(), "%s %s: some outputs were never written" % (L, info)
    ref = oracle.sparse_conv(d.W, d.mask, d.X, L.V, bias=d.bias, stride=L.stride, residual=R, act=act)
    pre = oracle.sparse_conv(d.W, d.mask, d.X, L.V, bias=d.bias, stride=L.stride, residual=R, act=None)
    assert_close_after_activation(got, ref, pre, "%s %s %s" % (L, info, epi))
