"""GPU parity of alcs_sparse_conv_bf16 (X, residual and Y stored as bfloat16; weights, bias and
sums float32) against the oracle: the inputs are bfloat16 values held in float32 arrays, the
oracle evaluates the definition in double, and the kernel's output must be that value rounded
to bfloat16, give or take the float32 summation error (which can move a result sitting on a
rounding boundary to the neighbouring bfloat16 value)."""
import numpy as np
import pytest

import oracle
import paper_2109_00170_amd as alcs
import workloads
from gpu_util import TOL

pytestmark = pytest.mark.gpu

def run_bf16(L, seed, act=None, with_res=False, with_bias=True, in_place=False, pack_tuning=None, **tuning):
    import torch
    d = workloads.make_layer(L, seed, with_bias=with_bias)
    packed = alcs.alcs_pack_weights(d.W, d.mask, L.V, options=dict(pack_tuning or {}, **tuning))
    Xb = oracle.round_bf16(d.X)                                  # the tensor as stored: bfloat16 values
    rng = np.random.default_rng(seed + 1)
    Rb = oracle.round_bf16((rng.standard_normal((L.N, L.Cout, L.Ho, L.Wo)) * 2).astype(np.float32)) if with_res else None
    X = torch.from_numpy(Xb).cuda().to(torch.bfloat16)           # exact: the values are representable
    assert np.array_equal(X.float().cpu().numpy(), Xb)
    b = None if d.bias is None else torch.from_numpy(d.bias).cuda()
    if in_place:
        Y = torch.from_numpy(Rb).cuda().to(torch.bfloat16)
        R = Y
    else:
        Y = torch.full((L.N, L.Cout, L.Ho, L.Wo), float("nan"), dtype=torch.bfloat16, device="cuda")
        R = None if Rb is None else torch.from_numpy(Rb).cuda().to(torch.bfloat16)
    alcs.alcs_sparse_conv_bf16(packed, X, b, R, Y, stride=L.stride, activation=act)
    torch.cuda.synchronize()
    info = alcs.alcs_last_launch()
    got = Y.float().cpu().numpy()
    packed.free()
    assert not np.isnan(got).any(), "some outputs were never written"
    Wd = oracle.densify(d.W, d.mask, L.V)
    ref = oracle.conv_fused(Wd, Xb, bias=d.bias, residual=Rb, act=act, stride=L.stride).astype(np.float64)
    pre = oracle.conv_fused(Wd, Xb, bias=d.bias, residual=Rb, act=None, stride=L.stride)
    # the float32 bound is taken relative to max |ref| (the stated bound) and max |pre|, whichever is smaller
    scale = min(float(np.max(np.abs(pre))), float(np.max(np.abs(ref))))
    # half a bfloat16 unit of the element itself plus the float32 bound on the sum
    bound = 2.0 ** -8 * np.abs(ref) + TOL * scale
    worst = float(np.max(np.abs(got - ref) - bound))
    assert worst <= 0.0, "%s %s: %.3g beyond the bound" % (L.name, info, worst)
    # most elements are the oracle's value rounded to bfloat16 exactly
    exact = np.mean(got == oracle.round_bf16(ref.astype(np.float32)))
    assert exact > 0.97, exact
    return info


@pytest.mark.parametrize("act", [None, "relu6"])
@pytest.mark.parametrize("V,pv", [(1, 1), (2, 2), (4, 1), (4, 2), (4, 4), (8, 4), (16, 1)])
def test_resident_pointwise_bf16(V, pv, act):
    L = workloads.Layer("bf_v%d_pv%d" % (V, pv), 40, 60, 17, 16, N=3, V=V, sparsity=0.7, w_std=0.3)
    info = run_bf16(L, 3500 + V + pv, act=act, with_res=(act is not None), pv=pv)
    assert info["mode"] == 1 and info["pv"] == pv


@pytest.mark.parametrize("H,W,stride", [(7, 7, 1), (9, 5, 1), (14, 14, 2), (1, 1, 1), (1, 33, 1), (13, 13, 2)])
def test_odd_images_and_strides_bf16(H, W, stride):
    L = workloads.Layer("bf_odd", 33, 19, H, W, stride=stride, N=6, V=4, sparsity=0.6, w_std=0.3)
    run_bf16(L, 3520 + H, act="relu", with_res=True)


@pytest.mark.parametrize("Cin,slots", [(520, 0), (700, 2), (1100, 4), (1100, 2)])
def test_several_groups_per_wavefront_bf16(Cin, slots):
    L = workloads.Layer("bf_gs", Cin, 72, 7, 7, N=9, V=4, sparsity=0.9, w_std=0.1)
    info = run_bf16(L, 3540 + Cin, act=None, with_res=True, pack_tuning={"group_slots": slots} if slots else None)
    assert info["group_slots"] == (slots or 4)


@pytest.mark.parametrize("slots", [2, 4])
@pytest.mark.parametrize("pv", [1, 2])
def test_several_groups_per_wavefront_pixel_pairs_bf16(slots, pv):
    L = workloads.Layer("bf_gs_pv", 520, 72, 12, 12, N=5, V=4, sparsity=0.9, w_std=0.1)
    info = run_bf16(L, 3550 + slots + pv, act="relu", with_res=True, pack_tuning={"group_slots": slots}, pv=pv)
    assert info["group_slots"] == slots and info["pv"] == pv


def test_single_round_spreads_pixels_over_all_compute_units_bf16():
    L = workloads.Layer("bf_narrow", 512, 64, 14, 14, N=32, V=4, sparsity=0.9, w_std=0.1)
    full = run_bf16(L, 3570, act="relu", with_res=True, full_tiles=1)
    spread = run_bf16(L, 3570, act="relu", with_res=True)
    assert spread["workgroups"] > full["workgroups"], (full, spread)


def test_in_place_residual_and_no_bias_bf16():
    L = workloads.Layer("bf_inplace", 64, 64, 14, 14, N=4, V=4, sparsity=0.8, w_std=0.3)
    run_bf16(L, 3560, act="relu", with_res=True, in_place=True, with_bias=False)


def test_mobilenet_shapes_bf16():
    for (cin, cout, hw) in ((32, 64, 112), (128, 128, 56), (256, 512, 14), (512, 512, 14), (1024, 1024, 7)):
        L = workloads.Layer("bf_mb_%d" % cin, cin, cout, hw, hw, N=2, V=4, sparsity=0.9, w_std=0.1)
        run_bf16(L, 3580 + cin, act="relu")


def test_unsupported_layouts_and_rejected_arguments_bf16():
    import torch
    # a 3x3 handle and a chunked 1x1 layout are refused, not run wrongly
    for L in (workloads.Layer("bf_3x3", 16, 8, 8, 8, k=3, N=1, V=4, sparsity=0.5),
              workloads.Layer("bf_chunk", 700, 8, 4, 4, N=1, V=2, sparsity=0.9)):
        d = workloads.make_layer(L, 3600)
        packed = alcs.alcs_pack_weights(d.W, d.mask, L.V)
        X = torch.zeros((L.N, L.Cin, L.H, L.W), dtype=torch.bfloat16, device="cuda")
        Y = torch.zeros((L.N, L.Cout, L.Ho, L.Wo), dtype=torch.bfloat16, device="cuda")
        with pytest.raises(alcs.AlcsError) as ei:
            alcs.alcs_sparse_conv_bf16(packed, X, None, None, Y)
        assert ei.value.status == -2
        packed.free()
    L = workloads.Layer("bf_rej", 16, 8, 8, 8, N=1, V=4, sparsity=0.5)
    d = workloads.make_layer(L, 3601)
    packed = alcs.alcs_pack_weights(d.W, d.mask, 4)
    X = torch.zeros((1, 16, 8, 8), dtype=torch.bfloat16, device="cuda")
    Y = torch.zeros((1, 8, 8, 8), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(alcs.AlcsError):
        alcs.alcs_sparse_conv_bf16(packed, X, None, None, Y, activation=9)
    with pytest.raises(ValueError):
        alcs.alcs_sparse_conv_bf16(packed, X.float(), None, None, Y)         # float32 tensor
    alcs.alcs_sparse_conv_bf16(packed, X[:0], None, None, Y[:0])             # empty batch
    torch.cuda.synchronize()
    packed.free()
