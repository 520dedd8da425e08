"""3x3 handles whose pattern is shared by the nine taps (every kept input channel keeps all its
taps): the kernel that walks channel records (one selector and nine reads at fixed offsets per
kept channel) against the oracle, full tensors; handles with independent taps and groups of 16
channels keep the column-by-column kernel."""
import numpy as np
import pytest

import oracle
import paper_2109_00170_amd as alcs
import workloads
from gpu_util import TOL, rel_err

pytestmark = pytest.mark.gpu


def run(L, seed, options=None, on_device=False, expect_mode=7):
    import torch
    d = workloads.make_layer(L, seed, with_bias=True)
    if expect_mode == 7:
        options = dict(options or {}, path=7)       # the record walk also where it is not the default
    if on_device:
        packed = alcs.alcs_pack_weights_device(torch.from_numpy(d.W).cuda(), torch.from_numpy(d.mask).cuda(), L.V, options=options)
    else:
        packed = alcs.alcs_pack_weights(d.W, d.mask, L.V, options=options)
    X = torch.from_numpy(d.X).cuda()
    b = torch.from_numpy(d.bias).cuda()
    Y = torch.full((L.N, L.Cout, L.Ho, L.Wo), float("nan"), device="cuda")
    alcs.alcs_sparse_conv(packed, X, b, Y, stride=L.stride)
    torch.cuda.synchronize()
    info = alcs.alcs_last_launch()
    assert info["mode"] == expect_mode, info
    got = Y.cpu().numpy()
    assert not np.isnan(got).any()
    ref = oracle.sparse_conv(d.W, d.mask, d.X, L.V, bias=d.bias, stride=L.stride)
    assert rel_err(got, ref) <= TOL, (L.name, info, rel_err(got, ref))
    # the fused entry point shares the kernel
    Y2 = torch.full_like(Y, float("nan"))
    alcs.alcs_sparse_conv_fused(packed, X, b, None, Y2, stride=L.stride, activation="relu")
    torch.cuda.synchronize()
    assert rel_err(Y2.cpu().numpy(), np.maximum(ref, 0)) <= TOL
    packed.free()
    return info, got


@pytest.mark.parametrize("V", [4, 8, 16])
@pytest.mark.parametrize("H,W", [(16, 16), (14, 14), (12, 29), (33, 17), (56, 56)])
def test_tap_shared_images(V, H, W):
    L = workloads.Layer("ts_%d_%dx%d" % (V, H, W), 24, 2 * V + 4, H, W, k=3, N=2, V=V, sparsity=0.6, w_std=0.2, tap_shared=True)
    run(L, 6100 + V + H + W, expect_mode=7 if V <= 8 else 3)


@pytest.mark.parametrize("stride", [1, 2])
@pytest.mark.parametrize("tile_width", [8, 16, 32])
def test_tap_shared_tile_shapes_and_strides(tile_width, stride):
    L = workloads.Layer("ts_tw%d_s%d" % (tile_width, stride), 40, 24, 30, 27, k=3, stride=stride, N=2, V=4, sparsity=0.6,
                        w_std=0.2, tap_shared=True)
    info, _ = run(L, 6140 + tile_width + stride, options={"tile_width": tile_width})
    assert info["tile_width"] == tile_width


@pytest.mark.parametrize("pv", [1, 2])
@pytest.mark.parametrize("ug", [2, 4])
def test_tap_shared_launch_shapes(pv, ug):
    L = workloads.Layer("ts_shapes", 70, 72, 20, 20, k=3, N=3, V=4, sparsity=0.7, w_std=0.2, tap_shared=True)   # three chunks
    info, _ = run(L, 6150, options={"pixels_per_lane": pv, "groups_per_wave": ug})
    assert info["pv"] == pv


def test_more_than_64_channels_in_a_chunk():
    """A chunk of 100 input channels, all kept: the records' channel indices are fetched 64 at a time."""
    L = workloads.Layer("ts_long", 100, 12, 14, 14, k=3, N=2, V=4, sparsity=0.0, w_std=0.1, tap_shared=True)
    run(L, 6160, options={"chunk_channels": 100})


def test_small_images_and_the_column_kernel_on_request():
    L = workloads.Layer("ts_small", 32, 16, 7, 7, k=3, N=4, V=4, sparsity=0.7, w_std=0.2, tap_shared=True)
    run(L, 6170)
    run(L, 6170, options={"path": 6}, expect_mode=3)
    run(L, 6170, options={}, expect_mode=3)               # one pixel per lane: the column walk by default


def test_tall_tiles_walk_records_by_default():
    import torch
    L = workloads.Layer("ts_default", 32, 16, 28, 28, k=3, N=2, V=4, sparsity=0.7, w_std=0.2, tap_shared=True)
    d = workloads.make_layer(L, 6175)
    packed = alcs.alcs_pack_weights(d.W, d.mask, 4)
    Y = torch.empty((2, 16, 28, 28), device="cuda")
    alcs.alcs_sparse_conv(packed, torch.from_numpy(d.X).cuda(), None, Y)
    torch.cuda.synchronize()
    info = alcs.alcs_last_launch()
    assert info["mode"] == 7 and info["pv"] == 2, info
    assert rel_err(Y.cpu().numpy(), oracle.sparse_conv(d.W, d.mask, d.X, 4)) <= TOL
    packed.free()


def test_independent_taps_keep_the_column_kernel():
    L = workloads.Layer("ts_indep", 32, 16, 28, 28, k=3, N=2, V=4, sparsity=0.7, w_std=0.2, tap_shared=False)
    run(L, 6181, expect_mode=3)


def test_device_built_handle_gets_channel_records():
    L = workloads.Layer("ts_dev", 48, 40, 28, 28, k=3, N=2, V=8, sparsity=0.75, w_std=0.2, tap_shared=True)
    _, a = run(L, 6190)
    _, b = run(L, 6190, on_device=True)
    assert np.array_equal(a, b)
    L = workloads.Layer("ts_dev_indep", 48, 40, 28, 28, k=3, N=2, V=8, sparsity=0.75, w_std=0.2, tap_shared=False)
    run(L, 6191, on_device=True, expect_mode=3)


def test_resnet_shaped_layers_at_two_images():
    for (c, hw) in ((64, 56), (128, 28), (256, 14)):
        L = workloads.Layer("ts_rn_%d" % c, c, c, hw, hw, k=3, N=2, V=4, sparsity=0.8, w_std=0.1, tap_shared=True)
        run(L, 6200 + c)


def test_more_than_1024_segments():
    """520 groups x 3 chunks: the scan that numbers the channel records takes two rounds."""
    L = workloads.Layer("ts_many", 96, 2080, 12, 12, k=3, N=1, V=4, sparsity=0.9, w_std=0.2, tap_shared=True)
    run(L, 6210)
    run(L, 6210, on_device=True)
