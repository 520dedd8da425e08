"""GPU parity of the depthwise 3x3 layer (alcs_depthwise_conv) and of the MobileNet block in one
kernel (alcs_dw_sparse_conv_fused: depthwise 3x3 + bias + activation feeding the sparse
pointwise convolution + bias + shortcut + activation) against the oracle, which runs the two
layers one after the other with the intermediate tensor rounded to fp32."""
import numpy as np
import pytest

import oracle
import paper_2109_00170_amd as alcs
import workloads
from gpu_util import TOL, assert_close_after_activation

pytestmark = pytest.mark.gpu

def dw_inputs(C, N, H, W, seed, x_scale=1.5):
    rng = np.random.default_rng(seed)
    D = (rng.standard_normal((C, 3, 3)) * 0.4).astype(np.float32)
    X = (rng.standard_normal((N, C, H, W)) * x_scale).astype(np.float32)
    b = rng.standard_normal(C).astype(np.float32)
    return D, X, b


@pytest.mark.parametrize("act", [None, "relu", "relu6"])
@pytest.mark.parametrize("stride", [1, 2])
@pytest.mark.parametrize("C,N,H,W", [(5, 3, 17, 16), (64, 2, 7, 7), (3, 1, 1, 1), (2, 2, 1, 9), (130, 1, 33, 2),
                                     (16, 2, 56, 56), (3, 2, 1, 4), (7, 1, 5, 8), (33, 3, 9, 20), (2, 1, 70, 4)])
def test_depthwise_layer(C, N, H, W, stride, act):
    import torch
    D, X, b = dw_inputs(C, N, H, W, 11 * C + H + stride)
    for bias in (None, b):
        Ho, Wo = oracle.out_size(H, 3, stride), oracle.out_size(W, 3, stride)
        Y = torch.full((N, C, Ho, Wo), float("nan"), dtype=torch.float32, device="cuda")
        alcs.alcs_depthwise_conv(torch.from_numpy(D).cuda(), torch.from_numpy(X).cuda(),
                                 None if bias is None else torch.from_numpy(bias).cuda(), Y, stride=stride,
                                 activation=act)
        torch.cuda.synchronize()
        got = Y.cpu().numpy()
        assert not np.isnan(got).any()
        ref = oracle.depthwise(D, X, bias=bias, stride=stride, act=act)
        pre = oracle.depthwise(D, X, bias=bias, stride=stride)
        assert_close_after_activation(got, ref, pre, "C=%d %dx%d s%d act=%s" % (C, H, W, stride, act))


def run_block(L, Hin, Win, dw_stride, seed, dw_act="relu", act=None, with_res=False, with_bias=True,
              dw_bias=True, workspace=False, expect_mode=1, pack_tuning=None, **tuning):
    """L describes the pointwise layer (its H x W is the depthwise layer's output)."""
    import torch
    assert (oracle.out_size(Hin, 3, dw_stride), oracle.out_size(Win, 3, dw_stride)) == (L.H, L.W)
    d = workloads.make_layer(L, seed, with_bias=with_bias)
    packed = alcs.alcs_pack_weights(d.W, d.mask, L.V, options=dict(pack_tuning or {}, **tuning))
    D, X, b1 = dw_inputs(L.Cin, L.N, Hin, Win, seed + 7)
    if not dw_bias:
        b1 = None
    rng = np.random.default_rng(seed + 1)
    R = (rng.standard_normal((L.N, L.Cout, L.H, L.W)) * 2).astype(np.float32) if with_res else None
    Y = torch.full((L.N, L.Cout, L.H, L.W), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.full((L.N, L.Cin, L.H, L.W), float("nan"), dtype=torch.float32, device="cuda") if workspace else None
    alcs.alcs_dw_sparse_conv_fused(
        packed, torch.from_numpy(D).cuda(), None if b1 is None else torch.from_numpy(b1).cuda(),
        torch.from_numpy(X).cuda(), None if d.bias is None else torch.from_numpy(d.bias).cuda(),
        None if R is None else torch.from_numpy(R).cuda(), Y, dw_stride=dw_stride, dw_activation=dw_act,
        activation=act, workspace=ws)
    torch.cuda.synchronize()
    info = alcs.alcs_last_launch()
    got = Y.cpu().numpy()
    packed.free()
    assert not np.isnan(got).any(), "some outputs were never written"
    Z = oracle.depthwise(D, X, bias=b1, stride=dw_stride, act=dw_act)
    ref = oracle.sparse_conv(d.W, d.mask, Z, L.V, bias=d.bias, residual=R, act=act)
    pre = oracle.sparse_conv(d.W, d.mask, Z, L.V, bias=d.bias, residual=R, act=None)
    assert_close_after_activation(got, ref, pre, "%s %s" % (L.name, info))
    if expect_mode is not None:
        assert info["mode"] == expect_mode, info
    if workspace and expect_mode == 1:
        assert bool(torch.isnan(ws).all()), "the fused kernel must not touch the workspace"
    if workspace and expect_mode is None:
        assert not bool(torch.isnan(ws).any()), "the two-layer path fills the workspace"
    return info


@pytest.mark.parametrize("dw_stride", [1, 2])
@pytest.mark.parametrize("V,pv", [(1, 1), (2, 2), (4, 1), (4, 2), (4, 4), (8, 4), (16, 1)])
def test_block_resident(V, pv, dw_stride):
    # pointwise tile axis: 3 images x 17 x 16 pixels (full tiles and a ragged one at every width)
    Hin, Win = (17, 16) if dw_stride == 1 else (33, 32)
    L = workloads.Layer("blk_v%d_pv%d" % (V, pv), 40, 60, 17, 16, N=3, V=V, sparsity=0.7, w_std=0.3)
    info = run_block(L, Hin, Win, dw_stride, 2000 + V + pv, pv=pv)
    assert info["pv"] == pv


@pytest.mark.parametrize("pv,waves", [(4, 1), (4, 3), (2, 1), (2, 3), (1, 1), (1, 5)])
def test_block_workgroups_smaller_than_the_tile(pv, waves):
    # fewer threads than tile pixels (several staging passes) and thread counts that are no
    # multiple of the tile width
    L = workloads.Layer("blk_small_wg", 10, 8, 20, 20, N=2, V=4, sparsity=0.5, w_std=0.3)
    info = run_block(L, 20, 20, 1, 2050 + pv + waves, pv=pv, waves=waves)
    assert info["pv"] == pv and info["waves"] == waves


@pytest.mark.parametrize("dw_stride", [1, 2])
@pytest.mark.parametrize("slots", [1, 2])
def test_block_taps_loaded_one_by_one(dw_stride, slots):
    # dw_own_taps: the stage that shares no taps between lanes must give the same block
    Cin = 64 if slots == 1 else 700
    L = workloads.Layer("blk_generic", Cin, 24, 14, 14, N=3, V=4, sparsity=0.8, w_std=0.2)
    run_block(L, 14 * dw_stride, 14 * dw_stride, dw_stride, 2080 + slots, dw_own_taps=1,
              pack_tuning={"group_slots": slots} if slots > 1 else None)


@pytest.mark.parametrize("dw_act,act,with_res", [(None, None, False), ("relu6", "relu6", False),
                                                 ("relu", None, True), ("relu6", "relu", True)])
def test_block_epilogues(dw_act, act, with_res):
    L = workloads.Layer("blk_epi", 48, 24, 14, 14, N=5, V=4, sparsity=0.8, w_std=0.3)
    run_block(L, 28, 28, 2, 2100, dw_act=dw_act, act=act, with_res=with_res)
    run_block(L, 14, 14, 1, 2101, dw_act=dw_act, act=act, with_res=with_res, with_bias=False, dw_bias=False)


@pytest.mark.parametrize("Hin,Win,dw_stride", [(7, 7, 1), (13, 13, 2), (1, 1, 1), (2, 3, 2), (1, 40, 1), (9, 5, 1)])
def test_block_odd_images(Hin, Win, dw_stride):
    # pixel counts that are no multiple of 4 (scalar stores), images smaller than the filter
    H, W = oracle.out_size(Hin, 3, dw_stride), oracle.out_size(Win, 3, dw_stride)
    L = workloads.Layer("blk_odd", 33, 19, H, W, N=6, V=4, sparsity=0.6, w_std=0.3)
    run_block(L, Hin, Win, dw_stride, 2200 + Hin)


@pytest.mark.parametrize("Cin,slots", [(700, 2), (1100, 4), (1100, 2)])
def test_block_several_groups_per_wavefront(Cin, slots):
    # wide inputs: 32- and 16-pixel tiles, a wavefront stages several channels at a time
    L = workloads.Layer("blk_gs%d" % slots, Cin, 72, 7, 7, N=9, V=4, sparsity=0.9, w_std=0.1)
    info = run_block(L, 14, 14, 2, 2300 + Cin, pack_tuning={"group_slots": slots})
    assert info["group_slots"] == slots


@pytest.mark.parametrize("Cin,hw,dw_stride,N", [(512, 14, 1, 32), (512, 7, 2, 120)])
def test_block_single_round_spreads_pixels_over_all_compute_units(Cin, hw, dw_stride, N):
    # workgroups that take fewer pixels than their tile holds (see the pointwise test of the same name)
    L = workloads.Layer("blk_narrow", Cin, 64, hw, hw, N=N, V=4, sparsity=0.9, w_std=0.1)
    full = run_block(L, hw * dw_stride, hw * dw_stride, dw_stride, 2400 + hw, full_tiles=1)
    spread = run_block(L, hw * dw_stride, hw * dw_stride, dw_stride, 2400 + hw)
    assert spread["workgroups"] > full["workgroups"], (full, spread)


@pytest.mark.parametrize("slots", [2, 4])
@pytest.mark.parametrize("hw,dw_stride", [(8, 1), (8, 2), (7, 1)])
@pytest.mark.parametrize("pv", [1, 2])
def test_block_several_groups_per_wavefront_pixels_per_lane(slots, hw, dw_stride, pv):
    # one or two pixels per lane: neighbouring pairs at 8x8, pixels half a tile apart at 7x7
    L = workloads.Layer("blk_gs%d_pv%d" % (slots, pv), 520, 40, hw, hw, N=7, V=4, sparsity=0.9, w_std=0.1)
    info = run_block(L, hw * dw_stride, hw * dw_stride, dw_stride, 2350 + slots + hw, pv=pv,
                     pack_tuning={"group_slots": slots})
    assert info["group_slots"] == slots and info["pv"] == pv


def test_block_mobilenet_shapes_small_batch():
    for (cin, cout, hw, s) in ((32, 64, 112, 1), (64, 128, 56, 2), (256, 512, 14, 2), (512, 512, 14, 1),
                               (1024, 1024, 7, 1)):
        L = workloads.Layer("blk_mb_%d" % cin, cin, cout, hw, hw, N=2, V=4, sparsity=0.9, w_std=0.1)
        run_block(L, hw * s, hw * s, s, 2400 + cin, dw_act="relu", act="relu")


def test_block_through_the_workspace_when_channels_are_chunked():
    import torch
    # V = 2 with more than 639 input channels is a chunked layout: the two layers run one after
    # the other; without a workspace the call is refused
    L = workloads.Layer("blk_chunk", 700, 20, 6, 6, N=2, V=2, sparsity=0.9, w_std=0.1)
    info = run_block(L, 11, 11, 2, 2500, workspace=True, expect_mode=2, act="relu")
    assert info["chunk_channels"] < 700
    with pytest.raises(alcs.AlcsError) as ei:
        run_block(L, 11, 11, 2, 2500, workspace=False, expect_mode=None)
    assert ei.value.status == -2 or "unsupported" in str(ei.value).lower()
    # a small layer whose groups are split over several workgroups per pixel tile goes through the
    # workspace for speed (two launches: the last one is the plain pointwise kernel, whose group
    # tiles show), unless told to stay in one kernel; without a workspace it is one kernel anyway
    L1 = workloads.Layer("blk_split", 64, 256, 7, 7, N=4, V=4, sparsity=0.8, w_std=0.2)
    info = run_block(L1, 7, 7, 1, 2502, workspace=True, expect_mode=None)
    assert info["group_tiles"] > 1
    info = run_block(L1, 7, 7, 1, 2502, workspace=True, expect_mode=1, dw_one_kernel=1)
    assert info["group_tiles"] > 1
    run_block(L1, 7, 7, 1, 2502, workspace=False, expect_mode=1)
    # a resident layout with one group tile leaves the workspace alone
    L2 = workloads.Layer("blk_ws_unused", 32, 16, 8, 8, N=2, V=4, sparsity=0.5, w_std=0.3)
    run_block(L2, 8, 8, 1, 2501, workspace=True, expect_mode=1)
    torch.cuda.synchronize()


def test_block_empty_batch_and_rejected_arguments():
    import torch
    L = workloads.Layer("blk_rej", 16, 8, 8, 8, N=1, V=4, sparsity=0.5)
    d = workloads.make_layer(L, 2600)
    packed = alcs.alcs_pack_weights(d.W, d.mask, L.V)
    D = torch.zeros((16, 3, 3), device="cuda")
    X = torch.zeros((1, 16, 8, 8), device="cuda")
    Y = torch.zeros((1, 8, 8, 8), device="cuda")
    lib = alcs.load_library()
    import ctypes
    P = lambda t: ctypes.c_void_p(t.data_ptr())
    call = lambda **kw: lib.alcs_dw_sparse_conv_fused(
        packed.handle, kw.get("D", P(D)), None, kw.get("s", 1), kw.get("a1", 0), P(X), None, None, P(Y), None,
        kw.get("N", 1), kw.get("Cin", 16), 8, 8, 8, kw.get("a2", 0), None)
    assert call() == 0
    assert call(N=0) == 0
    assert call(D=None) < 0
    assert call(s=3) < 0
    assert call(a1=7) < 0
    assert call(a2=-1) < 0
    assert call(Cin=12) < 0
    assert lib.alcs_depthwise_conv(P(D), P(X), None, P(X), 1, 16, 8, 8, 4, 0, None) < 0
    assert lib.alcs_depthwise_conv(P(D), P(X), None, P(X), 0, 16, 8, 8, 1, 0, None) == 0
    torch.cuda.synchronize()
    packed.free()
    # a 3x3 handle is not a pointwise layer
    L3 = workloads.Layer("blk_rej3", 16, 8, 8, 8, k=3, N=1, V=4, sparsity=0.5)
    d3 = workloads.make_layer(L3, 2601)
    p3 = alcs.alcs_pack_weights(d3.W, d3.mask, 4)
    assert lib.alcs_dw_sparse_conv_fused(p3.handle, P(D), None, 1, 0, P(X), None, None, P(Y), None, 1, 16, 8, 8, 8,
                                         0, None) < 0
    p3.free()
