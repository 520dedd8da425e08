"""Pins for the oracle's fused epilogue, act(conv + bias + residual): the element-wise layers
behind the constant tau of Section 3.3, Eq. (2) of arXiv 2109.00170 folded into the
convolution.

Compared with things other than the oracle: a library convolution followed by library
element-wise ops (torch CPU, float64), a brute-force evaluation written here with exact
integer inputs, and closed forms (cancelling residual, saturating inputs)."""
import numpy as np
import pytest
import torch

import oracle

ACTS = [None, "relu", "relu6"]


def torch_ref(Wd, X, bias, residual, act, stride):
    k = Wd.shape[2]
    y = torch.nn.functional.conv2d(torch.from_numpy(X).double(), torch.from_numpy(Wd).double(),
                                   None if bias is None else torch.from_numpy(bias).double(),
                                   stride=stride, padding=(k - 1) // 2)
    if residual is not None:
        y = y + torch.from_numpy(residual).double()
    if act == "relu":
        y = torch.relu(y)
    elif act == "relu6":
        y = torch.clamp(y, 0.0, 6.0)
    return y.numpy()


@pytest.mark.parametrize("act", ACTS)
@pytest.mark.parametrize("k,stride", [(1, 1), (1, 2), (3, 1), (3, 2)])
@pytest.mark.parametrize("with_res", [False, True])
def test_against_library_conv_and_elementwise_ops(act, k, stride, with_res):
    rng = np.random.default_rng(31 + 7 * k + stride + (3 if with_res else 0))
    Cout, Cin, H, Wi, N = 10, 6, 9, 8, 2
    Wd = (rng.standard_normal((Cout, Cin, k, k)) * 0.8).astype(np.float32)
    Wd[rng.random(Wd.shape) < 0.4] = 0
    X = (rng.standard_normal((N, Cin, H, Wi)) * 2).astype(np.float32)
    bias = rng.standard_normal(Cout).astype(np.float32)
    Ho, Wo = oracle.out_size(H, k, stride), oracle.out_size(Wi, k, stride)
    R = (rng.standard_normal((N, Cout, Ho, Wo)) * 3).astype(np.float32) if with_res else None
    got = oracle.conv_fused(Wd, X, bias=bias, residual=R, act=act, stride=stride)
    ref = torch_ref(Wd, X, bias, R, act, stride)
    assert got.shape == ref.shape and got.dtype == np.float32
    # the oracle rounds a double result once: it is the float nearest to the reference
    assert np.array_equal(got, ref.astype(np.float32)) or \
        np.max(np.abs(got.astype(np.float64) - ref)) <= 1e-6 * max(1.0, float(np.max(np.abs(ref))))
    if act is not None:
        assert got.min() >= 0.0
    if act == "relu6":
        assert got.max() <= 6.0


@pytest.mark.parametrize("act", ACTS)
def test_tiny_integer_inputs_bit_exact_against_loops(act):
    """Integer-valued tensors: every sum is exact, so plain Python loops written here must
    agree bit for bit (pins the order of bias, residual and activation and the indexing of R)."""
    rng = np.random.default_rng(5)
    Cout, Cin, H, Wi, N, k, stride = 3, 2, 4, 5, 2, 3, 2
    Wd = rng.integers(-3, 4, size=(Cout, Cin, k, k)).astype(np.float32)
    X = rng.integers(-4, 5, size=(N, Cin, H, Wi)).astype(np.float32)
    bias = rng.integers(-2, 3, size=(Cout,)).astype(np.float32)
    Ho, Wo = oracle.out_size(H, k, stride), oracle.out_size(Wi, k, stride)
    R = rng.integers(-9, 10, size=(N, Cout, Ho, Wo)).astype(np.float32)
    want = np.zeros((N, Cout, Ho, Wo), dtype=np.float32)
    for n in range(N):
        for o in range(Cout):
            for ho in range(Ho):
                for wo in range(Wo):
                    t = float(bias[o]) + float(R[n, o, ho, wo])
                    for c in range(Cin):
                        for r in range(k):
                            for s in range(k):
                                hi, wi = ho * stride + r - 1, wo * stride + s - 1
                                if 0 <= hi < H and 0 <= wi < Wi:
                                    t += float(Wd[o, c, r, s]) * float(X[n, c, hi, wi])
                    if act is not None:
                        t = max(t, 0.0)
                    if act == "relu6":
                        t = min(t, 6.0)
                    want[n, o, ho, wo] = t
    got = oracle.conv_fused(Wd, X, bias=bias, residual=R, act=act, stride=stride)
    assert got.tobytes() == want.tobytes()


def test_identity_epilogue_is_the_plain_convolution():
    rng = np.random.default_rng(8)
    Wd = rng.standard_normal((8, 5, 3, 3)).astype(np.float32)
    X = rng.standard_normal((2, 5, 7, 7)).astype(np.float32)
    b = rng.standard_normal(8).astype(np.float32)
    assert oracle.conv_fused(Wd, X, bias=b).tobytes() == oracle.conv(Wd, X, bias=b).tobytes()


def test_cancelling_residual_and_saturation():
    rng = np.random.default_rng(9)
    Wd = rng.standard_normal((8, 16, 1, 1)).astype(np.float32)
    X = rng.standard_normal((2, 16, 5, 5)).astype(np.float32)
    y = oracle.conv(Wd, X)
    # residual = -conv: what is left is the rounding of y itself, far below one ulp of the terms
    z = oracle.conv_fused(Wd, X, residual=-y, act=None)
    assert np.max(np.abs(z)) <= 1e-6 * np.max(np.abs(y))
    # relu of (conv - conv - 1) is exactly zero, relu6 of (conv - conv + 100) exactly six
    assert not oracle.conv_fused(Wd, X, residual=-y - 1.0, act="relu").any()
    assert np.all(oracle.conv_fused(Wd, X, residual=-y + 100.0, act="relu6") == np.float32(6.0))
    # the residual may be the output's own previous contents (in place, element-wise)
    buf = (-y + 2.0).astype(np.float32)
    out = oracle.conv_fused(Wd, X, residual=buf, act="relu6")
    assert np.max(np.abs(out - 2.0)) <= 1e-5


def test_sparse_conv_routes_the_epilogue():
    rng = np.random.default_rng(10)
    W = rng.standard_normal((8, 8, 1, 1)).astype(np.float32)
    mask = (rng.random((2, 8, 1, 1)) < 0.5).astype(np.uint8)
    X = rng.standard_normal((1, 8, 4, 4)).astype(np.float32)
    R = rng.standard_normal((1, 8, 4, 4)).astype(np.float32)
    a = oracle.sparse_conv(W, mask, X, 4, residual=R, act="relu")
    b = np.maximum(oracle.sparse_conv(W, mask, X, 4).astype(np.float64) + R, 0)
    assert np.max(np.abs(a - b)) <= 1e-6
    with pytest.raises(KeyError):
        oracle.sparse_conv(W, mask, X, 4, act="gelu")


def test_round_bf16_against_the_library_conversion():
    rng = np.random.default_rng(12)
    x = np.concatenate([rng.standard_normal(5000).astype(np.float32) * np.float32(10.0) ** rng.integers(-20, 20, 5000),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, np.inf, -np.inf, 3.3895314e38], np.float32)])
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    got = oracle.round_bf16(x)
    assert got.tobytes() == want.tobytes()
    # ties go to the even neighbour: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert oracle.round_bf16(np.float32(1.00390625)) == np.float32(1.0)
    assert oracle.round_bf16(np.float32(1.01171875)) == np.float32(1.015625)
    assert np.isnan(oracle.round_bf16(np.float32(np.nan)))
