"""GPU parity of alcs_sparse_conv_bf16_mfma (bfloat16 tensors AND bfloat16 weights on the 16-bit
matrix instruction, float32 sums) against the oracle: inputs and weights are rounded to bfloat16
(values held in float32 arrays), the oracle evaluates the definition on them in double, and the
kernel's output must be that value rounded to bfloat16, give or take the float32 summation error
(which can move a result that sits on a rounding boundary to the neighbouring bfloat16 value)."""
import numpy as np
import pytest

import oracle
import paper_2109_00170_amd as alcs
import workloads
from gpu_util import TOL

pytestmark = pytest.mark.gpu


def run_m16(L, seed, act=None, with_res=False, with_bias=True, in_place=False, options=None, on_device=False):
    import torch
    d = workloads.make_layer(L, seed, with_bias=with_bias)
    if on_device:
        packed = alcs.alcs_pack_weights_device(torch.from_numpy(d.W).cuda(), torch.from_numpy(d.mask).cuda(), L.V,
                                               options=options)
    else:
        packed = alcs.alcs_pack_weights(d.W, d.mask, L.V, options=options)
    packed.add_bf16_weights()
    packed.add_bf16_weights()                                   # a second call does nothing
    Xb = oracle.round_bf16(d.X)
    Wb = oracle.round_bf16(d.W)
    rng = np.random.default_rng(seed + 1)
    Rb = oracle.round_bf16((rng.standard_normal((L.N, L.Cout, L.Ho, L.Wo)) * 2).astype(np.float32)) if with_res else None
    X = torch.from_numpy(Xb).cuda().to(torch.bfloat16)
    assert np.array_equal(X.float().cpu().numpy(), Xb)
    b = None if d.bias is None else torch.from_numpy(d.bias).cuda()
    if in_place:
        Y = torch.from_numpy(Rb).cuda().to(torch.bfloat16)
        R = Y
    else:
        Y = torch.full((L.N, L.Cout, L.Ho, L.Wo), float("nan"), dtype=torch.bfloat16, device="cuda")
        R = None if Rb is None else torch.from_numpy(Rb).cuda().to(torch.bfloat16)
    alcs.alcs_sparse_conv_bf16_mfma(packed, X, b, R, Y, stride=L.stride, activation=act)
    torch.cuda.synchronize()
    info = alcs.alcs_last_launch()
    assert info["mode"] == 6
    got = Y.float().cpu().numpy()
    packed.free()
    assert not np.isnan(got).any(), "some outputs were never written"
    Wd = oracle.densify(Wb, d.mask, L.V)
    ref = oracle.conv_fused(Wd, Xb, bias=d.bias, residual=Rb, act=act, stride=L.stride).astype(np.float64)
    pre = oracle.conv_fused(Wd, Xb, bias=d.bias, residual=Rb, act=None, stride=L.stride)
    scale = min(float(np.max(np.abs(pre))), float(np.max(np.abs(ref))))
    bound = 2.0 ** -8 * np.abs(ref) + TOL * scale
    worst = float(np.max(np.abs(got - ref) - bound))
    assert worst <= 0.0, "%s %s: %.3g beyond the bound" % (L.name, info, worst)
    exact = np.mean(got == oracle.round_bf16(ref.astype(np.float32)))
    assert exact > 0.97, exact
    return info


@pytest.mark.parametrize("act", [None, "relu6"])
@pytest.mark.parametrize("V", [4, 8, 16])
def test_pointwise_16bit(V, act):
    L = workloads.Layer("m16_v%d" % V, 40, 60, 16, 16, N=3, V=V, sparsity=0.7, w_std=0.3)
    run_m16(L, 5500 + V, act=act, with_res=(act is not None))


@pytest.mark.parametrize("V", [4, 8, 16])
@pytest.mark.parametrize("Cin,sparsity", [(300, 0.5), (97, 0.0), (639, 0.9), (8, 0.3)])
def test_long_and_short_segments_16bit(V, Cin, sparsity):
    """Segments beyond the runs held in registers (150 and 97 kept columns), the widest tile (639
    channels, 160 KB), and groups shorter than one batch."""
    L = workloads.Layer("m16_seg", Cin, 2 * V + 3, 12, 12, N=2, V=V, sparsity=sparsity, w_std=0.1)
    run_m16(L, 5520 + Cin + V, act="relu", with_res=True, options={"group_slots": 1})


@pytest.mark.parametrize("H,W,stride", [(7, 7, 1), (9, 5, 1), (14, 14, 2), (1, 1, 1), (1, 33, 1), (13, 13, 2), (14, 14, 1), (6, 6, 1)])
def test_odd_images_and_strides_16bit(H, W, stride):
    L = workloads.Layer("m16_odd", 33, 19, H, W, stride=stride, N=6, V=4, sparsity=0.6, w_std=0.3)
    run_m16(L, 5540 + H + W, act="relu", with_res=True)
    L8 = workloads.Layer("m16_odd8", 33, 24, H, W, stride=stride, N=6, V=8, sparsity=0.6, w_std=0.3)
    run_m16(L8, 5560 + H + W)


@pytest.mark.parametrize("tiles,waves", [(0, 0), (3, 2), (16, 5), (1, 16)])
def test_group_tiles_and_wavefront_counts_16bit(tiles, waves):
    L = workloads.Layer("m16_gt", 128, 256, 14, 14, N=3, V=8, sparsity=0.85, w_std=0.1)
    info = run_m16(L, 5580, act="relu", options={"group_tiles": tiles, "waves": waves})
    if tiles:
        assert info["group_tiles"] == min(tiles, 32)


@pytest.mark.parametrize("V", [4, 8, 16])
@pytest.mark.parametrize("slots", [0, 2, 4])
def test_handles_with_several_groups_per_wavefront_16bit(V, slots):
    """Handles whose float32 layout interleaves the groups of a bundle (the default from 512 input
    channels on): the 16-bit layout gives every group a segment of its own again."""
    L = workloads.Layer("m16_gs%d_v%d" % (slots, V), 520, 5 * V + 2, 12, 12, N=3, V=V, sparsity=0.9, w_std=0.1)
    run_m16(L, 5570 + V + slots, act="relu", with_res=True, options={"group_slots": slots} if slots else None)
    Lu = workloads.Layer("m16_gsu%d_v%d" % (slots, V), 638, 3 * V, 7, 7, N=5, V=V, sparsity=0.8, w_std=0.1, mask_kind="zipf")
    run_m16(Lu, 5575 + V + slots, options={"group_slots": slots} if slots else None)


@pytest.mark.parametrize("V", [4, 8, 16])
@pytest.mark.parametrize("Cin,H,W", [(700, 14, 14), (1278, 7, 7), (1024, 5, 9)])
def test_wide_layers_one_pixel_per_lane_16bit(V, Cin, H, W):
    """More than 638 input channels: 64-pixel tiles of 128-byte rows, one pixel per lane (up to 1278)."""
    L = workloads.Layer("m16_wide%d_v%d" % (Cin, V), Cin, 3 * V + 1, H, W, N=5, V=V, sparsity=0.9, w_std=0.1)
    info = run_m16(L, 5610 + Cin + V, act="relu", with_res=True)
    assert info["pv"] == 1


@pytest.mark.parametrize("V", [4, 8, 16])
@pytest.mark.parametrize("H,W,stride", [(16, 16, 1), (14, 14, 1), (7, 7, 1), (9, 5, 1), (14, 14, 2)])
def test_one_pixel_per_lane_on_request_16bit(V, H, W, stride):
    L = workloads.Layer("m16_pv1_v%d" % V, 48, 2 * V + 3, H, W, stride=stride, N=7, V=V, sparsity=0.6, w_std=0.2)
    info = run_m16(L, 5630 + V + H + W, act="relu6", with_res=True, options={"pixels_per_lane": 1})
    assert info["pv"] == 1
    info = run_m16(L, 5630 + V + H + W, act="relu6", with_res=True, options={"pixels_per_lane": 2})
    assert info["pv"] == 2
    L5 = workloads.Layer("m16_pv1_gs_v%d" % V, 520, 2 * V, H, W, stride=stride, N=3, V=V, sparsity=0.9, w_std=0.1)
    run_m16(L5, 5650 + V + H + W, options={"pixels_per_lane": 1})


def test_in_place_residual_no_bias_and_device_built_handle_16bit():
    L = workloads.Layer("m16_inplace", 64, 64, 14, 14, N=4, V=8, sparsity=0.8, w_std=0.3)
    run_m16(L, 5590, act="relu", with_res=True, in_place=True, with_bias=False, on_device=True)


def test_mobilenet_shapes_16bit():
    for V in (8, 16):
        for (cin, cout, hw) in ((32, 64, 112), (64, 128, 56), (128, 128, 56), (128, 256, 28), (256, 256, 28), (256, 512, 14)):
            L = workloads.Layer("m16_mb_%d" % cin, cin, cout, hw, hw, N=2, V=V, sparsity=0.9, w_std=0.1)
            run_m16(L, 5600 + cin + V, act="relu")


@pytest.mark.parametrize("V", [8, 16])
def test_benchmark_layers_at_full_batch_16bit(V):
    """The 13 MobileNetV1-shaped pointwise layers at batch 32 and 90 % block sparsity, full tensors, in
    the launch configuration the 16-bit report times (default handles)."""
    import dataclasses
    for i, L0 in enumerate(workloads.mobilenet_v1_pointwise(32, 0.9)):
        run_m16(dataclasses.replace(L0, V=V), workloads.seed_for(2, i), act="relu")


def test_unsupported_layouts_and_rejected_arguments_16bit():
    import torch
    # 3x3 handles, more input channels than one 16-bit tile holds, chunked layouts and V < 4 are refused
    for L in (workloads.Layer("m16_3x3", 16, 8, 8, 8, k=3, N=1, V=4, sparsity=0.5),
              workloads.Layer("m16_wide", 1300, 16, 4, 4, N=1, V=4, sparsity=0.9),
              workloads.Layer("m16_chunk", 700, 8, 4, 4, N=1, V=2, sparsity=0.9),
              workloads.Layer("m16_v2", 16, 8, 4, 4, N=1, V=2, sparsity=0.5)):
        d = workloads.make_layer(L, 5700)
        packed = alcs.alcs_pack_weights(d.W, d.mask, L.V)
        with pytest.raises(alcs.AlcsError) as ei:
            packed.add_bf16_weights()
        assert ei.value.status == -2
        X = torch.zeros((L.N, L.Cin, L.H, L.W), dtype=torch.bfloat16, device="cuda")
        Y = torch.zeros((L.N, L.Cout, L.Ho, L.Wo), dtype=torch.bfloat16, device="cuda")
        with pytest.raises(alcs.AlcsError) as ei:
            alcs.alcs_sparse_conv_bf16_mfma(packed, X, None, None, Y)
        assert ei.value.status == -2
        packed.free()
    L = workloads.Layer("m16_rej", 16, 8, 8, 8, N=1, V=4, sparsity=0.5)
    d = workloads.make_layer(L, 5701)
    packed = alcs.alcs_pack_weights(d.W, d.mask, 4)
    X = torch.zeros((1, 16, 8, 8), dtype=torch.bfloat16, device="cuda")
    Y = torch.zeros((1, 8, 8, 8), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(alcs.AlcsError) as ei:                                  # no rounded weights yet
        alcs.alcs_sparse_conv_bf16_mfma(packed, X, None, None, Y)
    assert ei.value.status == -1
    packed.add_bf16_weights()
    with pytest.raises(alcs.AlcsError):
        alcs.alcs_sparse_conv_bf16_mfma(packed, X, None, None, Y, activation=9)
    with pytest.raises(ValueError):
        alcs.alcs_sparse_conv_bf16_mfma(packed, X.float(), None, None, Y)      # float32 tensor
    alcs.alcs_sparse_conv_bf16_mfma(packed, X[:0], None, None, Y[:0])          # empty batch
    torch.cuda.synchronize()
    packed.free()
