"""Fully connected layers and batched matrix products through the same entry point: the paper's
latency model counts CONV and FC layers alike (Section 3.3), and an FC layer is the 1x1 case with a
1x1 image, the batch playing the pixel axis; [Cout, Cin] x [B, Cin, P] is the 1x1 case as it stands."""
import numpy as np
import pytest

import oracle
import paper_2109_00170_amd as alcs
import workloads
from gpu_util import TOL, assert_close_after_activation, rel_err

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("N,Cin,Cout,V", [(1, 1024, 1000, 4), (7, 1024, 1000, 16), (64, 2048, 1000, 4),
                                          (256, 1280, 1000, 8), (33, 512, 10, 2), (130, 4096, 100, 4)])
def test_fully_connected_layer(N, Cin, Cout, V):
    import torch
    L = workloads.Layer("fc_%d_%d" % (Cin, Cout), Cin, Cout, 1, 1, N=N, V=V, sparsity=0.8, w_std=0.05, x_dist="relu")
    d = workloads.make_layer(L, 3400 + N + Cin, with_bias=True)
    packed = alcs.alcs_pack_weights(d.W, d.mask, V)
    X = torch.from_numpy(d.X).cuda()
    b = torch.from_numpy(d.bias).cuda()
    Y = torch.full((N, Cout, 1, 1), float("nan"), dtype=torch.float32, device="cuda")
    alcs.alcs_sparse_conv_fused(packed, X, b, None, Y, activation="relu")
    torch.cuda.synchronize()
    got = Y.cpu().numpy()
    packed.free()
    assert not np.isnan(got).any()
    # the oracle's convolution on the same 1x1 layer (an FC layer is that layer on a 1x1 image)
    ref = oracle.sparse_conv(d.W, d.mask, d.X, V, bias=d.bias, act="relu")
    pre = oracle.sparse_conv(d.W, d.mask, d.X, V, bias=d.bias)
    assert_close_after_activation(got, ref, pre, "fc %d->%d N=%d" % (Cin, Cout, N))
    # and the matrix product written out, as a second opinion on the layer's meaning
    Wd = oracle.densify(d.W, d.mask, V).reshape(Cout, Cin).astype(np.float64)
    mm = np.maximum(d.X.reshape(N, Cin).astype(np.float64) @ Wd.T + d.bias, 0.0)
    assert float(np.max(np.abs(ref.reshape(N, Cout) - mm))) <= 1e-6 * float(np.max(np.abs(mm)))


def test_batched_matrix_product():
    import torch
    B, Cin, Cout, P, V = 5, 96, 72, 77, 4          # P odd: scalar loads and stores
    L = workloads.Layer("bmm", Cin, Cout, 1, P, N=B, V=V, sparsity=0.7, w_std=0.2, x_dist="uniform")
    d = workloads.make_layer(L, 3450)
    packed = alcs.alcs_pack_weights(d.W, d.mask, V)
    Y = torch.full((B, Cout, 1, P), float("nan"), dtype=torch.float32, device="cuda")
    alcs.alcs_sparse_conv(packed, torch.from_numpy(d.X).cuda(), None, Y)
    torch.cuda.synchronize()
    got = Y.cpu().numpy()
    packed.free()
    ref = oracle.sparse_conv(d.W, d.mask, d.X, V)
    assert rel_err(got, ref) <= TOL
    Wd = oracle.densify(d.W, d.mask, V).reshape(Cout, Cin).astype(np.float64)
    mm = np.einsum("oc,bcp->bop", Wd, d.X.reshape(B, Cin, P).astype(np.float64))
    assert float(np.max(np.abs(ref.reshape(B, Cout, P) - mm))) <= 1e-6 * float(np.max(np.abs(mm)))
