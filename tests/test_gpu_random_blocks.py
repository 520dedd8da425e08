"""Seeded random shapes through the MobileNet-block kernel and the bfloat16 entry point: group
size, channel counts, image sizes down to one pixel, both depthwise strides, every epilogue,
sparsity from 0 to 1.  Every case is a valid call."""
import numpy as np
import pytest

import oracle
import paper_2109_00170_amd as alcs
import workloads
from gpu_util import TOL, assert_close_after_activation

pytestmark = pytest.mark.gpu


def draw(seed):
    rng = np.random.default_rng(seed)
    V = int(rng.choice([1, 2, 4, 4, 8, 16]))
    wide = rng.random() < 0.2
    Cin = int(rng.integers(512, 1300)) if (wide and V >= 4) else int(rng.integers(1, 140))
    Cout = int(rng.integers(1, 90))
    s = int(rng.choice([1, 1, 2]))
    Hin, Win = int(rng.integers(1, 30)), int(rng.integers(1, 30))
    N = int(rng.integers(1, 5))
    sparsity = float(rng.choice([0.0, 0.5, 0.8, 0.9, 0.97, 1.0]))
    acts = [None, "relu", "relu6"]
    return dict(V=V, Cin=Cin, Cout=Cout, s=s, Hin=Hin, Win=Win, N=N, sparsity=sparsity,
                dw_act=acts[int(rng.integers(0, 3))], act=acts[int(rng.integers(0, 3))],
                res=bool(rng.random() < 0.4), bias=bool(rng.random() < 0.6), dw_bias=bool(rng.random() < 0.6),
                ws=bool(rng.random() < 0.3))


@pytest.mark.parametrize("seed", range(48))
def test_random_block(seed):
    import torch
    c = draw(9000 + seed)
    H, W = oracle.out_size(c["Hin"], 3, c["s"]), oracle.out_size(c["Win"], 3, c["s"])
    L = workloads.Layer("rb%d" % seed, c["Cin"], c["Cout"], H, W, N=c["N"], V=c["V"], sparsity=c["sparsity"], w_std=0.2)
    d = workloads.make_layer(L, 9000 + seed, with_bias=c["bias"])
    packed = alcs.alcs_pack_weights(d.W, d.mask, L.V)
    rng = np.random.default_rng(9500 + seed)
    D = (rng.standard_normal((L.Cin, 3, 3)) * 0.4).astype(np.float32)
    X = (rng.standard_normal((L.N, L.Cin, c["Hin"], c["Win"])) * 1.5).astype(np.float32)
    b1 = rng.standard_normal(L.Cin).astype(np.float32) if c["dw_bias"] else None
    R = (rng.standard_normal((L.N, L.Cout, H, W)) * 2).astype(np.float32) if c["res"] else None
    Y = torch.full((L.N, L.Cout, H, W), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty((L.N, L.Cin, H, W), dtype=torch.float32, device="cuda") if c["ws"] else None
    t = lambda a: None if a is None else torch.from_numpy(a).cuda()
    try:
        alcs.alcs_dw_sparse_conv_fused(packed, t(D), t(b1), t(X), t(d.bias), t(R), Y, dw_stride=c["s"],
                                       dw_activation=c["dw_act"], activation=c["act"], workspace=ws)
    except alcs.AlcsError as e:
        # only layouts the one-kernel path does not cover may be refused, and only without a workspace
        assert e.status == -2 and ws is None and (L.V < 4 and L.Cin > 639), (c, str(e))
        packed.free()
        return
    torch.cuda.synchronize()
    got = Y.cpu().numpy()
    packed.free()
    assert not np.isnan(got).any(), c
    Z = oracle.depthwise(D, X, bias=b1, stride=c["s"], act=c["dw_act"])
    ref = oracle.sparse_conv(d.W, d.mask, Z, L.V, bias=d.bias, residual=R, act=c["act"])
    pre = oracle.sparse_conv(d.W, d.mask, Z, L.V, bias=d.bias, residual=R)
    assert_close_after_activation(got, ref, pre, str(c))


@pytest.mark.parametrize("seed", range(32))
def test_random_bf16(seed):
    import torch
    c = draw(9700 + seed)
    stride = c["s"]
    L = workloads.Layer("rf%d" % seed, c["Cin"], c["Cout"], c["Hin"], c["Win"], stride=stride, N=c["N"], V=c["V"],
                        sparsity=c["sparsity"], w_std=0.2)
    d = workloads.make_layer(L, 9700 + seed, with_bias=c["bias"])
    packed = alcs.alcs_pack_weights(d.W, d.mask, L.V)
    Xb = oracle.round_bf16(d.X)
    rng = np.random.default_rng(9800 + seed)
    Rb = oracle.round_bf16((rng.standard_normal((L.N, L.Cout, L.Ho, L.Wo)) * 2).astype(np.float32)) if c["res"] else None
    Y = torch.full((L.N, L.Cout, L.Ho, L.Wo), float("nan"), dtype=torch.bfloat16, device="cuda")
    tb = lambda a: None if a is None else torch.from_numpy(a).cuda().to(torch.bfloat16)
    try:
        alcs.alcs_sparse_conv_bf16(packed, tb(Xb), None if d.bias is None else torch.from_numpy(d.bias).cuda(), tb(Rb), Y,
                                   stride=stride, activation=c["act"])
    except alcs.AlcsError as e:
        assert e.status == -2 and (L.V < 4 and L.Cin > 639), (c, str(e))
        packed.free()
        return
    torch.cuda.synchronize()
    got = Y.float().cpu().numpy()
    packed.free()
    assert not np.isnan(got).any(), c
    Wd = oracle.densify(d.W, d.mask, L.V)
    ref = oracle.conv_fused(Wd, Xb, bias=d.bias, residual=Rb, act=c["act"], stride=stride).astype(np.float64)
    pre = oracle.conv_fused(Wd, Xb, bias=d.bias, residual=Rb, act=None, stride=stride)
    # half a bfloat16 unit of the element plus the float32 bound, relative to max |ref| and max |pre|
    bound = 2.0 ** -8 * np.abs(ref) + TOL * min(float(np.max(np.abs(pre))), float(np.max(np.abs(ref))))
    assert float(np.max(np.abs(got - ref) - bound)) <= 0.0, c
