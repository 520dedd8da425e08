"""Pins for the oracle's depthwise convolution (the layer in front of every pointwise
convolution of the MobileNet that arXiv 2109.00170 prunes; the convolution equation of its
Section 3.2.2 with one filter per channel).

Compared with things other than the routine itself: a library grouped convolution (torch CPU,
float64, groups = C), exact integer loops written here, impulse responses, and the already
pinned full convolution run on block-diagonal weights."""
import numpy as np
import pytest
import torch

import oracle


def torch_ref(D, X, bias, stride, act):
    C, k = D.shape[0], D.shape[1]
    y = torch.nn.functional.conv2d(torch.from_numpy(X).double(), torch.from_numpy(D).double().reshape(C, 1, k, k),
                                   None if bias is None else torch.from_numpy(bias).double(),
                                   stride=stride, padding=(k - 1) // 2, groups=C)
    if act == "relu":
        y = torch.relu(y)
    elif act == "relu6":
        y = torch.clamp(y, 0.0, 6.0)
    return y.numpy()


@pytest.mark.parametrize("act", [None, "relu", "relu6"])
@pytest.mark.parametrize("stride", [1, 2])
@pytest.mark.parametrize("H,W", [(9, 8), (7, 7), (1, 5), (2, 2)])
def test_against_library_grouped_convolution(act, stride, H, W):
    rng = np.random.default_rng(17 + stride + H * 31 + W)
    C, N = 5, 3
    D = rng.standard_normal((C, 3, 3)).astype(np.float32)
    X = (rng.standard_normal((N, C, H, W)) * 3).astype(np.float32)
    b = rng.standard_normal(C).astype(np.float32)
    for bias in (None, b):
        got = oracle.depthwise(D, X, bias=bias, stride=stride, act=act)
        ref = torch_ref(D, X, bias, stride, act)
        assert got.shape == ref.shape and got.dtype == np.float32
        assert np.max(np.abs(got.astype(np.float64) - ref)) <= 1e-6 * max(1.0, float(np.max(np.abs(ref))))


@pytest.mark.parametrize("stride", [1, 2])
def test_integer_inputs_bit_exact_against_loops(stride):
    rng = np.random.default_rng(23)
    C, N, H, W = 3, 2, 6, 5
    D = rng.integers(-3, 4, size=(C, 3, 3)).astype(np.float32)
    X = rng.integers(-5, 6, size=(N, C, H, W)).astype(np.float32)
    b = rng.integers(-2, 3, size=(C,)).astype(np.float32)
    Ho, Wo = oracle.out_size(H, 3, stride), oracle.out_size(W, 3, stride)
    want = np.zeros((N, C, Ho, Wo), dtype=np.float32)
    for n in range(N):
        for c in range(C):
            for ho in range(Ho):
                for wo in range(Wo):
                    t = float(b[c])
                    for r in range(3):
                        for q in range(3):
                            hi, wi = ho * stride + r - 1, wo * stride + q - 1
                            if 0 <= hi < H and 0 <= wi < W:
                                t += float(D[c, r, q]) * float(X[n, c, hi, wi])
                    want[n, c, ho, wo] = max(t, 0.0)
    got = oracle.depthwise(D, X, bias=b, stride=stride, act="relu")
    assert got.tobytes() == want.tobytes()


def test_impulse_reproduces_the_filter_reversed_and_stays_in_its_channel():
    C, H, W = 4, 7, 7
    D = np.arange(1, C * 9 + 1, dtype=np.float32).reshape(C, 3, 3)
    X = np.zeros((1, C, H, W), dtype=np.float32)
    X[0, 2, 3, 3] = 1.0
    Z = oracle.depthwise(D, X)
    # output (h, w) sees the impulse through tap (3 - h + 1, 3 - w + 1): the filter, reversed
    assert np.array_equal(Z[0, 2, 2:5, 2:5], D[2, ::-1, ::-1])
    Z[0, 2, 2:5, 2:5] = 0
    assert not Z.any()                       # nothing leaks into other channels or pixels


def test_equals_full_convolution_on_block_diagonal_weights():
    rng = np.random.default_rng(29)
    C = 6
    D = rng.standard_normal((C, 3, 3)).astype(np.float32)
    X = rng.standard_normal((2, C, 8, 9)).astype(np.float32)
    b = rng.standard_normal(C).astype(np.float32)
    Wd = np.zeros((C, C, 3, 3), dtype=np.float32)
    for c in range(C):
        Wd[c, c] = D[c]
    for stride in (1, 2):
        assert oracle.depthwise(D, X, bias=b, stride=stride).tobytes() == \
            oracle.conv(Wd, X, bias=b, stride=stride).tobytes()


def test_rejects_bad_shapes():
    with pytest.raises(ValueError):
        oracle.depthwise(np.zeros((3, 3, 2), np.float32), np.zeros((1, 3, 4, 4), np.float32))
    with pytest.raises(ValueError):
        oracle.depthwise(np.zeros((3, 3, 3), np.float32), np.zeros((1, 4, 4, 4), np.float32))
