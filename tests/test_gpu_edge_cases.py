"""GPU parity on the corners of the argument space: empty batch, images smaller than the
filter or than one tile, very few channels, very many columns, side streams, and the
argument checks that must reject a call before anything is launched."""
import numpy as np
import pytest

import oracle
import paper_2109_00170_amd as alcs
import workloads
from gpu_util import TOL, oracle_ref, rel_err, run_sparse

pytestmark = pytest.mark.gpu


def check(L, seed, with_bias=True):
    d = workloads.make_layer(L, seed, with_bias=with_bias)
    got, info = run_sparse(d)
    ref = oracle_ref(d)
    assert got.shape == ref.shape
    assert not np.isnan(got).any(), "some outputs were never written"
    err = rel_err(got, ref)
    assert err <= TOL, "%s %s: rel err %.3g" % (L.name, info, err)
    return info


def test_empty_batch_is_a_no_op():
    import torch
    L = workloads.Layer("n0", 8, 8, 5, 5, k=1, stride=1, N=1, V=4, sparsity=0.5)
    d = workloads.make_layer(L, 900)
    packed = alcs.alcs_pack_weights(d.W, d.mask, L.V)
    X = torch.empty((0, 8, 5, 5), dtype=torch.float32, device="cuda")
    Y = torch.empty((0, 8, 5, 5), dtype=torch.float32, device="cuda")
    alcs.alcs_sparse_conv(packed, X, None, Y)
    torch.cuda.synchronize()
    packed.free()


@pytest.mark.parametrize("k,stride,hw", [(1, 1, 1), (1, 2, 1), (3, 1, 1), (3, 2, 1), (3, 1, 2), (3, 2, 2),
                                         (3, 2, 3), (1, 2, 2)])
@pytest.mark.parametrize("V", [1, 4, 16])
def test_images_smaller_than_the_filter_or_one_tile(k, stride, hw, V):
    # Cout = 7: ragged last group for every V > 1; three images, so a tile spans images
    L = workloads.Layer("tiny_k%d_s%d_%d_v%d" % (k, stride, hw, V), 5, 7, hw, hw, k=k, stride=stride, N=3,
                        V=V, sparsity=0.4)
    check(L, 910 + 10 * k + stride + hw + V)


def test_non_square_single_row_and_single_column_images():
    for j, (H, W) in enumerate(((1, 37), (37, 1), (2, 65))):
        for k in (1, 3):
            for stride in (1, 2):
                L = workloads.Layer("thin_%dx%d_k%d_s%d" % (H, W, k, stride), 6, 12, H, W, k=k, stride=stride,
                                    N=2, V=4, sparsity=0.5)
                check(L, 930 + j + k + stride)


def test_three_input_channels_on_a_large_image():
    """Stem-like layer: 3 channels (fewer than one chunk), 224x224, stride 2."""
    L = workloads.Layer("stem", 3, 32, 224, 224, k=3, stride=2, N=2, V=4, sparsity=0.3, w_std=0.1)
    info = check(L, 940)
    assert info["mode"] == 3


def test_many_columns_3x3():
    """600 input channels = 5400 columns per group, 19 chunks, the last one short."""
    L = workloads.Layer("wide3", 600, 16, 9, 9, k=3, stride=1, N=1, V=4, sparsity=0.9, w_std=0.05)
    check(L, 941)


def test_one_group_one_kept_column():
    import torch
    L = workloads.Layer("single", 16, 4, 6, 6, k=1, stride=1, N=2, V=4, sparsity=0.0)
    d = workloads.make_layer(L, 942)
    mask = np.zeros((1, 16, 1, 1), dtype=np.uint8)
    mask[0, 11] = 1
    packed = alcs.alcs_pack_weights(d.W, mask, 4)
    X = torch.from_numpy(d.X).cuda()
    Y = torch.full((2, 4, 6, 6), float("nan"), dtype=torch.float32, device="cuda")
    alcs.alcs_sparse_conv(packed, X, None, Y)
    torch.cuda.synchronize()
    want = d.W[:, 11, 0, 0][None, :, None, None] * d.X[:, 11:12]
    assert Y.cpu().numpy().tobytes() == want.astype(np.float32).tobytes()   # one product per output: exact
    packed.free()


def test_side_stream_and_two_streams_share_a_handle():
    import torch
    L = workloads.Layer("streams", 64, 64, 28, 28, k=1, stride=1, N=4, V=4, sparsity=0.8)
    d = workloads.make_layer(L, 943)
    ref = oracle_ref(d)
    packed = alcs.alcs_pack_weights(d.W, d.mask, L.V)
    X = torch.from_numpy(d.X).cuda()
    torch.cuda.synchronize()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    Y1 = torch.full((4, 64, 28, 28), float("nan"), dtype=torch.float32, device="cuda")
    Y2 = torch.full_like(Y1, float("nan"))
    torch.cuda.synchronize()
    for _ in range(3):
        alcs.alcs_sparse_conv(packed, X, None, Y1, stream=s1)
        alcs.alcs_sparse_conv(packed, X, None, Y2, stream=s2)
    s1.synchronize()
    s2.synchronize()
    assert rel_err(Y1.cpu().numpy(), ref) <= TOL
    assert Y1.cpu().numpy().tobytes() == Y2.cpu().numpy().tobytes()
    packed.free()


def test_calls_that_must_be_rejected_before_any_launch():
    import torch
    L = workloads.Layer("rej", 16, 16, 8, 8, k=1, stride=1, N=2, V=4, sparsity=0.5)
    d = workloads.make_layer(L, 944)
    packed = alcs.alcs_pack_weights(d.W, d.mask, L.V)
    X = torch.from_numpy(d.X).cuda()
    Y = torch.zeros((2, 16, 8, 8), dtype=torch.float32, device="cuda")
    lib = alcs.load_library()
    import ctypes
    vp = ctypes.c_void_p

    def call(x_ptr, y_ptr, N=2, Cin=16, Cout=16, H=8, W=8, k=1, stride=1):
        return lib.alcs_sparse_conv(packed.handle, vp(x_ptr), vp(None), vp(y_ptr), N, Cin, Cout, H, W, k, stride,
                                    vp(None))

    xp, yp = X.data_ptr(), Y.data_ptr()
    assert call(xp, yp) == 0
    assert call(xp, yp, Cin=17) == -1            # shape differs from the packed one
    assert call(xp, yp, Cout=12) == -1
    assert call(xp, yp, k=3) == -1
    assert call(xp, yp, stride=3) == -2
    assert call(xp, yp, H=0) == -1
    assert call(xp, yp, N=-1) == -1
    assert call(None, yp) == -1
    assert call(xp, None) == -1
    assert call(xp + 4, yp) == -1                # not 16-byte aligned
    assert call(xp, yp + 8) == -1
    torch.cuda.synchronize()
    assert rel_err(Y.cpu().numpy(), oracle_ref(d)) <= TOL   # the one valid call produced the result
    packed.free()
