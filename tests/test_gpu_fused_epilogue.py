"""GPU parity of alcs_sparse_conv_fused (convolution + bias + shortcut addition + ReLU /
ReLU6 in one kernel) against the oracle's definition, through every kernel family that
has an epilogue of its own: resident 1x1 with 1, 2 and 4 pixels per lane, several
groups per wavefront, chunked, persistent, 3x3 in every tile shape, FMA and MFMA forms."""
import numpy as np
import pytest

import oracle
import paper_2109_00170_amd as alcs
import workloads
from gpu_util import TOL, assert_close_after_activation, rel_err

pytestmark = pytest.mark.gpu

def run_fused(L, seed, act, with_res=True, in_place=False, with_bias=True, pack_tuning=None, **tuning):
    import torch
    d = workloads.make_layer(L, seed, with_bias=with_bias)
    rng = np.random.default_rng(seed + 1)
    R = (rng.standard_normal((L.N, L.Cout, L.Ho, L.Wo)) * 2).astype(np.float32) if with_res else None
    packed = alcs.alcs_pack_weights(d.W, d.mask, L.V, options=dict(pack_tuning or {}, **tuning))
    X = torch.from_numpy(d.X).cuda()
    b = None if d.bias is None else torch.from_numpy(d.bias).cuda()
    if in_place:
        Y = torch.from_numpy(R).cuda()
        Rd = Y
    else:
        Y = torch.full((L.N, L.Cout, L.Ho, L.Wo), float("nan"), dtype=torch.float32, device="cuda")
        Rd = None if R is None else torch.from_numpy(R).cuda()
    alcs.alcs_sparse_conv_fused(packed, X, b, Rd, Y, stride=L.stride, activation=act)
    torch.cuda.synchronize()
    info = alcs.alcs_last_launch()
    got = Y.cpu().numpy()
    packed.free()
    ref = oracle.sparse_conv(d.W, d.mask, d.X, L.V, bias=d.bias, stride=L.stride, residual=R, act=act)
    assert not np.isnan(got).any(), "some outputs were never written"
    # the stated bound (relative to max |ref|) and the one relative to the pre-activation values
    pre = oracle.sparse_conv(d.W, d.mask, d.X, L.V, bias=d.bias, stride=L.stride, residual=R, act=None)
    assert_close_after_activation(got, ref, pre, "%s %s act=%s" % (L.name, info, act))
    if act is not None:
        assert got.min() >= 0.0
    if act == "relu6":
        assert got.max() <= 6.0
    return info


@pytest.mark.parametrize("act", [None, "relu", "relu6"])
@pytest.mark.parametrize("V,pv", [(1, 1), (2, 2), (4, 1), (4, 2), (4, 4), (8, 4), (16, 1)])
def test_resident_pointwise(V, pv, act):
    # 17 x 16 pixels x 3 images: full tiles and a ragged one for every tile width; Cout = 60 is
    # ragged for V = 8 and 16
    L = workloads.Layer("fr_v%d_pv%d" % (V, pv), 40, 60, 17, 16, k=1, stride=1, N=3, V=V, sparsity=0.7,
                        w_std=0.3)
    info = run_fused(L, 1000 + V + pv, act, pv=pv)
    assert info["mode"] == 1 and info["pv"] == pv


@pytest.mark.parametrize("act", ["relu", "relu6"])
def test_in_place_residual_and_no_bias(act):
    L = workloads.Layer("fr_inplace", 64, 64, 14, 14, k=1, stride=1, N=4, V=4, sparsity=0.8, w_std=0.3)
    run_fused(L, 1010, act, in_place=True, with_bias=False)


def test_activation_only_and_residual_only():
    L = workloads.Layer("fr_parts", 48, 40, 12, 12, k=1, stride=1, N=2, V=4, sparsity=0.6, w_std=0.3)
    run_fused(L, 1020, "relu6", with_res=False)
    run_fused(L, 1021, None, with_res=True)


@pytest.mark.parametrize("Cin,gs", [(700, 2), (700, 4), (1400, 4)])
def test_several_groups_per_wavefront(Cin, gs):
    L = workloads.Layer("fr_gs%d" % gs, Cin, 72, 7, 7, k=1, stride=1, N=5, V=8, sparsity=0.9, w_std=0.1)
    info = run_fused(L, 1030 + gs, "relu6", pack_tuning={"group_slots": gs})
    assert info["group_slots"] == gs


def test_odd_pixel_count_and_stride2_pointwise():
    L = workloads.Layer("fr_odd", 33, 20, 9, 7, k=1, stride=1, N=3, V=4, sparsity=0.5, w_std=0.3)
    run_fused(L, 1040, "relu")
    L = workloads.Layer("fr_s2", 24, 36, 11, 9, k=1, stride=2, N=2, V=4, sparsity=0.5, w_std=0.3)
    run_fused(L, 1041, "relu6")


@pytest.mark.parametrize("V,pv", [(1, 1), (4, 2), (16, 4)])
def test_chunked_pointwise(V, pv):
    L = workloads.Layer("fr_chunk_v%d" % V, 100, 48, 16, 16, k=1, stride=1, N=2, V=V, sparsity=0.7, w_std=0.2)
    info = run_fused(L, 1050 + V, "relu6", pack_tuning={"chunk_channels": 32}, pv=pv)
    assert info["mode"] == 2


def test_persistent_pointwise():
    L = workloads.Layer("fr_stream", 24, 40, 212, 212, k=1, stride=1, N=3, V=4, sparsity=0.7, w_std=0.3)
    info = run_fused(L, 1060, "relu", path=4, pv=1)
    assert info["mode"] == 4


@pytest.mark.parametrize("stride", [1, 2])
@pytest.mark.parametrize("tile_width", [8, 16, 32])
@pytest.mark.parametrize("V", [2, 4, 16])
def test_conv3x3(V, stride, tile_width):
    L = workloads.Layer("fr_c3_v%d" % V, 40, 40, 13, 35, k=3, stride=stride, N=2, V=V, sparsity=0.75, w_std=0.1)
    info = run_fused(L, 1070 + V + stride + tile_width, "relu6", tile_width=tile_width)
    assert info["mode"] == 3


def test_identity_epilogue_is_bit_identical_to_the_plain_entry_point():
    import torch
    L = workloads.Layer("fr_same", 96, 64, 14, 14, k=1, stride=1, N=3, V=4, sparsity=0.8)
    d = workloads.make_layer(L, 1080, with_bias=True)
    packed = alcs.alcs_pack_weights(d.W, d.mask, L.V)
    X = torch.from_numpy(d.X).cuda()
    b = torch.from_numpy(d.bias).cuda()
    Y1 = torch.empty((3, 64, 14, 14), dtype=torch.float32, device="cuda")
    Y2 = torch.empty_like(Y1)
    alcs.alcs_sparse_conv(packed, X, b, Y1)
    alcs.alcs_sparse_conv_fused(packed, X, b, None, Y2, activation=None)
    torch.cuda.synchronize()
    assert torch.equal(Y1, Y2)
    packed.free()


def test_rejected_arguments():
    import ctypes
    import torch
    L = workloads.Layer("fr_rej", 16, 16, 8, 8, k=1, stride=1, N=2, V=4, sparsity=0.5)
    d = workloads.make_layer(L, 1090)
    packed = alcs.alcs_pack_weights(d.W, d.mask, L.V)
    X = torch.from_numpy(d.X).cuda()
    Y = torch.zeros((2, 16, 8, 8), dtype=torch.float32, device="cuda")
    R = torch.zeros_like(Y)
    lib = alcs.load_library()
    vp = ctypes.c_void_p

    def call(res_ptr, act):
        return lib.alcs_sparse_conv_fused(packed.handle, vp(X.data_ptr()), vp(None), vp(res_ptr), vp(Y.data_ptr()),
                                          2, 16, 16, 8, 8, 1, 1, act, vp(None))

    assert call(R.data_ptr(), 2) == 0
    assert call(R.data_ptr(), 3) == -1
    assert call(R.data_ptr(), -1) == -1
    assert call(R.data_ptr() + 4, 1) == -1       # residual not 16-byte aligned
    with pytest.raises(ValueError):
        alcs.alcs_sparse_conv_fused(packed, X, None, R[:1], Y)
    torch.cuda.synchronize()
    packed.free()
