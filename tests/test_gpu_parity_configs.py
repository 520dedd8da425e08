"""GPU parity on the five benchmark configurations, in the launch configuration the
benchmark times (default tuning, full batch).

Every layer of every configuration is compared with the oracle element by element over the
whole output tensor at the stated batch: the multithreaded oracle needs 0.1 - 3 s per layer
(about 20 GMAC for the ResNet-50-shaped configuration, 28 for the sparsity sweep, 5 per
group size for the MobileNetV2-shaped one; budget: two minutes of oracle time for this file).
The small-batch runs of the same layers stay: they take different launch shapes.  Packing is
compared bit for bit in every case.  The bound is max |Y - Yref| / max |Yref| <= 1e-5, the
reference alone setting the scale.
"""
import dataclasses

import numpy as np
import pytest

import oracle
import paper_2109_00170_amd as alcs
import workloads
from gpu_util import TOL, oracle_ref, rel_err, run_sparse

pytestmark = pytest.mark.gpu


def full_check(L, seed, with_bias=False):
    d = workloads.make_layer(L, seed, with_bias=with_bias)
    got, info = run_sparse(d)
    assert not np.isnan(got).any(), "%s: some outputs were never written" % L.name
    ref = oracle_ref(d)
    err = rel_err(got, ref)
    assert err <= TOL, "%s %s rel err %.3g" % (L.name, info, err)
    # groups that keep nothing must reproduce the bias exactly, at any size
    if d.mask is not None:
        empty = np.nonzero(d.mask.reshape(L.G, -1).sum(axis=1) == 0)[0]
        for g in empty[:2]:
            ch = slice(g * L.V, min(L.Cout, (g + 1) * L.V))
            want = 0.0 if d.bias is None else d.bias[ch][None, :, None, None]
            assert np.array_equal(got[:, ch], np.broadcast_to(want, got[:, ch].shape).astype(np.float32))
    return info


# ----------------------------------------------------------------------------- config 2

@pytest.mark.parametrize("N,sparsity", [(1, None), (32, 0.9), (32, None)])
def test_config2_mobilenet_v1_pointwise(N, sparsity):
    for i, L in enumerate(workloads.mobilenet_v1_pointwise(N, sparsity)):
        full_check(L, workloads.seed_for(2, i))


# ----------------------------------------------------------------------------- config 3

def test_config3_resnet50_bottlenecks_small_batch_full_tensor():
    for i, L in enumerate(workloads.resnet50_bottlenecks(2)):
        info = full_check(L, workloads.seed_for(3, i))
        assert L.k != 3 or info["mode"] in (3, 7)


def test_config3_resnet50_bottlenecks_batch64_full_tensor():
    for i, L in enumerate(workloads.resnet50_bottlenecks(64)):
        info = full_check(L, workloads.seed_for(3, i))
        assert L.k != 3 or info["mode"] in (3, 7)


def test_config3_independent_pattern_per_tap():
    """The other reading of the 3x3 mask: every (c, r, s) position pruned on its own."""
    layers = [L for L in workloads.resnet50_bottlenecks(2) if L.k == 3]
    for j, L in enumerate((layers[0], [L for L in layers if L.stride == 2][1])):
        full_check(dataclasses.replace(L, tap_shared=False), workloads.seed_for(3, 90 + j))


# ----------------------------------------------------------------------------- config 4

@pytest.mark.parametrize("s", workloads.SWEEP_SPARSITIES)
def test_config4_sparsity_sweep(s):
    full_check(workloads.sweep_layer(s, N=8), workloads.seed_for(4, int(round(s * 100))))
    full_check(workloads.sweep_layer(s, N=256), workloads.seed_for(4, int(round(s * 100))))


def test_config4_sparsity_zero_equals_dense_conv():
    import torch
    L = workloads.sweep_layer(0.0, N=16)
    d = workloads.make_layer(L, workloads.seed_for(4, 0))
    a, _ = run_sparse(d)
    Wd = torch.from_numpy(d.W).cuda()
    X = torch.from_numpy(d.X).cuda()
    Y = torch.empty((L.N, L.Cout, L.Ho, L.Wo), dtype=torch.float32, device="cuda")
    alcs.alcs_dense_conv(Wd, X, None, Y)
    torch.cuda.synchronize()
    assert rel_err(a, Y.cpu().numpy()) <= TOL


# ----------------------------------------------------------------------------- config 5

@pytest.mark.parametrize("V", [1, 4, 8, 16])
def test_config5_mobilenet_v2_small_batch_full_tensor(V):
    for i, L in enumerate(workloads.mobilenet_v2_pointwise(2, V)):
        full_check(L, workloads.seed_for(5, 100 * V + i), with_bias=True)


@pytest.mark.parametrize("V", [1, 4, 8, 16])
def test_config5_mobilenet_v2_batch128_full_tensor(V):
    # all 18 layers for every group size (Cout = 24 with V = 16 is the ragged case)
    for i, L in enumerate(workloads.mobilenet_v2_pointwise(128, V)):
        full_check(L, workloads.seed_for(5, 100 * V + i), with_bias=True)
