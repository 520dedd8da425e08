"""Pins for the oracle's convolution (equation of Section 3.2.2 of arXiv 2109.00170,
extended with batch, zero padding, stride and bias).

The oracle is compared with things other than itself: a brute-force shifted-slice
evaluation written here, a library convolution (torch CPU, float64), closed forms
(identity and impulse inputs, all-dropped masks), and algebraic invariants.
"""
import itertools

import numpy as np
import pytest
import torch

import oracle
import workloads


def brute_force(Wd, X, bias, stride):
    """sum over taps of (weight slice) x (shifted, strided view of the padded input),
    in float64.  Written independently of the oracle's loop nest."""
    Cout, Cin, k, _ = Wd.shape
    N, _, H, Wi = X.shape
    pad = (k - 1) // 2
    Ho = (H + 2 * pad - k) // stride + 1
    Wo = (Wi + 2 * pad - k) // stride + 1
    Xp = np.zeros((N, Cin, H + 2 * pad, Wi + 2 * pad), dtype=np.float64)
    Xp[:, :, pad:pad + H, pad:pad + Wi] = X
    Y = np.zeros((N, Cout, Ho, Wo), dtype=np.float64)
    for r in range(k):
        for s in range(k):
            view = Xp[:, :, r:r + stride * (Ho - 1) + 1:stride, s:s + stride * (Wo - 1) + 1:stride]
            Y += np.einsum("oc,nchw->nohw", Wd[:, :, r, s].astype(np.float64), view)
    if bias is not None:
        Y += bias.astype(np.float64)[None, :, None, None]
    return Y


def masked(W, mask, V):
    """W with dropped blocks zeroed, built with numpy broadcasting (not the oracle)."""
    if mask is None:
        return W.copy()
    keep = np.repeat(mask, V, axis=0)[: W.shape[0]].astype(bool)
    return np.where(keep, W, np.float32(0))


TINY = [c for c in itertools.product((1, 3), (1, 2), (1, 2, 4), (3, 8), (2, 5), (1, 4, 5))]


@pytest.mark.parametrize("k,stride,V,Cout,Cin,HW", TINY)
def test_tiny_integer_inputs_bit_exact(k, stride, V, Cout, Cin, HW):
    """Integer-valued inputs make every partial sum exact in double and in float, so
    the oracle, the brute force and the grouped-CSR walker must agree bit for bit."""
    rng = np.random.default_rng(1000 * k + 100 * stride + 10 * V + Cout + Cin + HW)
    H, Wi = HW, HW + 1
    G = oracle.n_groups(Cout, V)
    W = rng.integers(-4, 5, size=(Cout, Cin, k, k)).astype(np.float32)
    mask = (rng.random((G, Cin, k, k)) < 0.5).astype(np.uint8)
    X = rng.integers(-8, 9, size=(2, Cin, H, Wi)).astype(np.float32)
    bias = rng.integers(-3, 4, size=(Cout,)).astype(np.float32)
    Wd = masked(W, mask, V)
    ref = brute_force(Wd, X, bias, stride).astype(np.float32)
    got = oracle.sparse_conv(W, mask, X, V, bias=bias, stride=stride)
    assert got.shape == ref.shape
    assert got.tobytes() == ref.tobytes()
    rp, ci, vals = oracle.pack(W, mask, V)
    walk = oracle.conv_csr(rp, ci, vals, X, Cout, k, V, bias=bias, stride=stride)
    assert walk.tobytes() == ref.tobytes()


def test_hand_computed_two_group_example():
    """V=2, two groups, 1x1, 2 input channels, 2 pixels; worked out by hand."""
    W = np.array([[1, 2], [3, 4], [5, 6], [7, 8]], dtype=np.float32).reshape(4, 2, 1, 1)
    mask = np.array([[1, 0], [0, 1]], dtype=np.uint8).reshape(2, 2, 1, 1)
    X = np.array([[10, 20], [1, 2]], dtype=np.float32).reshape(1, 2, 1, 2)
    # group 0 keeps channel 0 only: rows (1*x0, 3*x0); group 1 keeps channel 1: (6*x1, 8*x1)
    expect = np.array([[10, 20], [30, 60], [6, 12], [8, 16]], dtype=np.float32).reshape(1, 4, 1, 2)
    got = oracle.sparse_conv(W, mask, X, 2)
    assert np.array_equal(got, expect)


@pytest.mark.parametrize("k,stride", [(1, 1), (1, 2), (3, 1), (3, 2)])
def test_sparsity_zero_is_library_dense_conv(k, stride):
    rng = np.random.default_rng(11 + k + stride)
    W = rng.standard_normal((12, 10, k, k)).astype(np.float32)
    X = rng.standard_normal((3, 10, 9, 11)).astype(np.float32)
    b = rng.standard_normal(12).astype(np.float32)
    ref = torch.nn.functional.conv2d(torch.from_numpy(X).double(), torch.from_numpy(W).double(),
                                     torch.from_numpy(b).double(), stride=stride,
                                     padding=(k - 1) // 2).numpy()
    got = oracle.sparse_conv(W, None, X, 4, bias=b, stride=stride)
    assert np.max(np.abs(got - ref)) <= 2e-7 * np.max(np.abs(ref))
    if k == 1 and stride == 1:       # for 1x1 it is the matrix product W . X_n
        mm = np.einsum("oc,ncp->nop", W.reshape(12, 10).astype(np.float64),
                       X.reshape(3, 10, -1).astype(np.float64)) + b[None, :, None]
        assert np.max(np.abs(got.reshape(3, 12, -1) - mm)) <= 2e-7 * np.max(np.abs(mm))


@pytest.mark.parametrize("k,stride,V", [(1, 1, 4), (3, 1, 4), (3, 2, 2), (1, 1, 16), (1, 2, 1)])
def test_pruned_weights_against_library_conv(k, stride, V):
    rng = np.random.default_rng(5 + k + stride + V)
    Cout, Cin = 24, 13
    G = oracle.n_groups(Cout, V)
    W = rng.standard_normal((Cout, Cin, k, k)).astype(np.float32)
    mask = (rng.random((G, Cin, k, k)) < 0.3).astype(np.uint8)
    X = rng.standard_normal((2, Cin, 8, 7)).astype(np.float32)
    Wd = masked(W, mask, V)
    ref = torch.nn.functional.conv2d(torch.from_numpy(X).double(), torch.from_numpy(Wd).double(),
                                     stride=stride, padding=(k - 1) // 2).numpy()
    got = oracle.sparse_conv(W, mask, X, V, stride=stride)
    assert np.max(np.abs(got - ref)) <= 2e-7 * max(np.max(np.abs(ref)), 1e-30)


def test_everything_dropped_gives_bias_exactly():
    rng = np.random.default_rng(2)
    W = rng.standard_normal((8, 6, 3, 3)).astype(np.float32)
    X = rng.standard_normal((2, 6, 5, 5)).astype(np.float32)
    b = rng.standard_normal(8).astype(np.float32)
    mask = np.zeros((2, 6, 3, 3), np.uint8)
    got = oracle.sparse_conv(W, mask, X, 4, bias=b)
    assert np.array_equal(got, np.broadcast_to(b[None, :, None, None], got.shape))
    got0 = oracle.sparse_conv(W, mask, X, 4)
    assert not got0.any()


def test_linearity_in_x_and_in_disjoint_masks():
    rng = np.random.default_rng(4)
    W = rng.standard_normal((8, 9, 3, 3)).astype(np.float32)
    m1 = (rng.random((2, 9, 3, 3)) < 0.4).astype(np.uint8)
    m2 = ((rng.random((2, 9, 3, 3)) < 0.4) & (m1 == 0)).astype(np.uint8)
    X1 = rng.standard_normal((1, 9, 6, 6)).astype(np.float32)
    X2 = rng.standard_normal((1, 9, 6, 6)).astype(np.float32)
    a, b = np.float32(0.75), np.float32(-2.5)
    y = oracle.sparse_conv(W, m1, a * X1 + b * X2, 4)
    y12 = a * oracle.sparse_conv(W, m1, X1, 4) + b * oracle.sparse_conv(W, m1, X2, 4)
    assert np.max(np.abs(y - y12)) <= 2e-6 * np.max(np.abs(y))
    ym = oracle.sparse_conv(W, m1, X1, 4) + oracle.sparse_conv(W, m2, X1, 4)
    yu = oracle.sparse_conv(W, m1 | m2, X1, 4)
    assert np.max(np.abs(ym - yu)) <= 2e-6 * np.max(np.abs(yu))


def test_identity_input_reads_back_the_pruned_weights():
    """1x1 with H*W = Cin and X one-hot per channel: every sum has a single term, so
    Y[n,:,p] is column p of the pruned weight matrix, exactly."""
    rng = np.random.default_rng(6)
    Cout, Cin, V = 12, 16, 4
    W = rng.standard_normal((Cout, Cin, 1, 1)).astype(np.float32)
    mask = (rng.random((3, Cin, 1, 1)) < 0.5).astype(np.uint8)
    X = np.eye(Cin, dtype=np.float32).reshape(1, Cin, 4, 4)
    got = oracle.sparse_conv(W, mask, X, V)
    assert got.reshape(Cout, Cin).tobytes() == masked(W, mask, V).reshape(Cout, Cin).tobytes()


@pytest.mark.parametrize("stride", [1, 2])
def test_impulse_pins_no_flip_padding_and_stride_phase(stride):
    """A unit impulse at (hi,wi): output (ho,wo) sees tap (r,s) with ho*stride+r-1=hi,
    wo*stride+s-1=wi; i.e. the taps appear mirrored around the impulse (correlation,
    not convolution), and at the border only the taps that still overlap."""
    k, H, Wi = 3, 6, 7
    W = (np.arange(9, dtype=np.float32) + 1).reshape(1, 1, 3, 3)
    for hi, wi in [(2, 3), (0, 0), (5, 6), (4, 1)]:
        X = np.zeros((1, 1, H, Wi), np.float32)
        X[0, 0, hi, wi] = 1
        got = oracle.sparse_conv(W, None, X, 1, stride=stride)[0, 0]
        Ho, Wo = got.shape
        expect = np.zeros((Ho, Wo), np.float32)
        for ho in range(Ho):
            for wo in range(Wo):
                r, s = hi - ho * stride + 1, wi - wo * stride + 1
                if 0 <= r < k and 0 <= s < k:
                    expect[ho, wo] = W[0, 0, r, s]
        assert np.array_equal(got, expect)
    assert got.shape == ((H + 2 - 3) // stride + 1, (Wi + 2 - 3) // stride + 1)


def test_channel_and_group_permutation_symmetry():
    rng = np.random.default_rng(8)
    Cout, Cin, V = 16, 10, 4
    W = rng.standard_normal((Cout, Cin, 3, 3)).astype(np.float32)
    mask = (rng.random((4, Cin, 3, 3)) < 0.5).astype(np.uint8)
    X = rng.standard_normal((2, Cin, 5, 5)).astype(np.float32)
    y = oracle.sparse_conv(W, mask, X, V)
    pc = rng.permutation(Cin)
    y2 = oracle.sparse_conv(W[:, pc], mask[:, pc], X[:, pc], V)
    assert np.max(np.abs(y - y2)) <= 2e-6 * np.max(np.abs(y))
    pg = rng.permutation(4)
    rows = (pg[:, None] * V + np.arange(V)[None, :]).reshape(-1)
    y3 = oracle.sparse_conv(W[rows], mask[pg], X, V)
    assert np.array_equal(y3, y[:, rows])


def test_conv_at_matches_full_conv():
    rng = np.random.default_rng(9)
    W = rng.standard_normal((8, 6, 3, 3)).astype(np.float32)
    X = rng.standard_normal((3, 6, 7, 5)).astype(np.float32)
    b = rng.standard_normal(8).astype(np.float32)
    Wd = masked(W, (rng.random((2, 6, 3, 3)) < 0.5).astype(np.uint8), 4)
    ref = brute_force(Wd, X, b, 2).astype(np.float32)
    idx = rng.choice(ref.size, size=50, replace=False)
    got = oracle.conv_at(Wd, X, idx, bias=b, stride=2)
    assert np.max(np.abs(got - ref.reshape(-1)[idx])) <= 1e-6 * np.max(np.abs(ref))


def test_im2col_rows_are_shifted_inputs():
    X1 = np.arange(2 * 4 * 5, dtype=np.float32).reshape(2, 4, 5)
    I = oracle.im2col(X1, 3, 1)
    assert I.shape == (18, 20)
    # the centre tap of channel 1 is the channel itself
    assert np.array_equal(I[1 * 9 + 1 * 3 + 1].reshape(4, 5), X1[1])
    # tap (0,0) looks one up and one left: first row and column come from the padding
    t = I[0].reshape(4, 5)
    assert not t[0].any() and not t[:, 0].any() and np.array_equal(t[1:, 1:], X1[0, :-1, :-1])


def test_threads_do_not_change_the_result():
    rng = np.random.default_rng(10)
    W = rng.standard_normal((16, 12, 1, 1)).astype(np.float32)
    X = rng.standard_normal((4, 12, 6, 6)).astype(np.float32)
    a = oracle.conv(W, X, nthreads=1)
    b = oracle.conv(W, X, nthreads=4)
    assert a.tobytes() == b.tobytes()


def test_shape_tables_match_the_papers_operation_counts():
    """The paper counts 569 M multiply-accumulates for MobileNet and 4.1 G for
    ResNet-50 (Table 3); the pointwise / bottleneck convs listed here are the bulk."""
    mb = workloads.macs_per_image(workloads.mobilenet_v1_pointwise(1, 0.9))
    assert abs(mb - 539.5e6) < 0.2e6 and 0.94 < mb / 569e6 < 0.96
    rn = workloads.macs_per_image(workloads.resnet50_bottlenecks(1))
    assert abs(rn - 3.61e9) < 0.02e9 and rn < 4.1e9
    assert sum(L.repeats for L in workloads.resnet50_bottlenecks(1)) == 48
    v2 = workloads.macs_per_image(workloads.mobilenet_v2_pointwise(1, 4))
    assert abs(v2 - 247.9e6) < 0.5e6
