"""Fully connected layers and batched matrix products through the same entry point: the paper's
latency model counts CONV and FC layers alike (Section 3.3), and an FC layer is the 1x1 case with a
1x1 image, the batch playing the pixel axis; [Cout, Cin] x [B, Cin, P] is the 1x1 case as it stands."""
import numpy as np
import pytest

import oracle
import paper_2109_00170_amd as alcs
import workloads
from gpu_util import TOL

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
    got = Y.cpu().numpy().reshape(N, Cout)
    packed.free()
    assert not np.isnan(got).any()
    # the definition of an FC layer, written out: relu(X Wd^T + b) in double
    Wd = oracle.densify(d.W, d.mask, V).reshape(Cout, Cin).astype(np.float64)
    pre = d.X.reshape(N, Cin).astype(np.float64) @ Wd.T + d.bias
    err = float(np.max(np.abs(got - np.maximum(pre, 0.0))) / np.max(np.abs(pre)))
    assert err <= TOL, err


def test_batched_matrix_product():
    import torch
    B, Cin, Cout, P, V = 5, 96, 72, 77, 4          # P odd: scalar loads and stores
    L = workloads.Layer("bmm", Cin, Cout, 1, P, N=B, V=V, sparsity=0.7, w_std=0.2, x_dist="uniform")
    d = workloads.make_layer(L, 3450)
    packed = alcs.alcs_pack_weights(d.W, d.mask, V)
    Y = torch.full((B, Cout, 1, P), float("nan"), dtype=torch.float32, device="cuda")
    alcs.alcs_sparse_conv(packed, torch.from_numpy(d.X).cuda(), None, Y)
    torch.cuda.synchronize()
    got = Y.cpu().numpy().reshape(B, Cout, P)
    packed.free()
    Wd = oracle.densify(d.W, d.mask, V).reshape(Cout, Cin).astype(np.float64)
    ref = np.einsum("oc,bcp->bop", Wd, d.X.reshape(B, Cin, P).astype(np.float64))
    assert float(np.max(np.abs(got - ref)) / np.max(np.abs(ref))) <= TOL
