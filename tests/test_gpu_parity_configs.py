"""GPU parity on the five benchmark configurations, in the launch configuration the
benchmark times (default tuning, full batch).

Where the oracle finishes the whole tensor in seconds it is compared element by
element; at the full batch of the larger configurations a few thousand output
elements per layer are recomputed one by one by the oracle (conv_at), after a
full-tensor comparison of the same layer at a small batch.  Packing is compared bit
for bit in every case.
"""
import dataclasses

import numpy as np
import pytest

import oracle
import paper_2109_00170_amd as alcs
import workloads
from gpu_util import TOL, oracle_ref, rel_err, run_sparse

pytestmark = pytest.mark.gpu

N_SAMPLES = 3000


def full_check(L, seed, with_bias=False):
    d = workloads.make_layer(L, seed, with_bias=with_bias)
    got, info = run_sparse(d)
    ref = oracle_ref(d)
    assert not np.isnan(got).any()
    err = rel_err(got, ref)
    assert err <= TOL, "%s %s rel err %.3g" % (L.name, info, err)
    return info


def sampled_check(L, seed, with_bias=False):
    """Full-size run; N_SAMPLES outputs are recomputed by the oracle from the definition."""
    import torch
    d = workloads.make_layer(L, seed, with_bias=with_bias)
    packed = alcs.alcs_pack_weights(d.W, d.mask, L.V)
    for got, want in zip(packed.export(), oracle.pack(d.W, d.mask, L.V)):
        assert got.tobytes() == want.tobytes()
    X = torch.from_numpy(d.X).cuda()
    b = None if d.bias is None else torch.from_numpy(d.bias).cuda()
    Y = torch.full((L.N, L.Cout, L.Ho, L.Wo), float("nan"), dtype=torch.float32, device="cuda")
    alcs.alcs_sparse_conv(packed, X, b, Y, stride=L.stride)
    torch.cuda.synchronize()
    info = alcs.alcs_last_launch()
    assert not bool(torch.isnan(Y).any()), "%s: some outputs were never written" % L.name
    ymax = float(Y.abs().max())
    rng = np.random.default_rng(seed + 77)
    idx = np.unique(np.concatenate([rng.integers(0, Y.numel(), size=N_SAMPLES),
                                    [0, Y.numel() - 1]]))          # include the corners
    got = Y.reshape(-1)[torch.from_numpy(idx).cuda()].cpu().numpy()
    Wd = oracle.densify(d.W, d.mask, L.V)
    ref = oracle.conv_at(Wd, d.X, idx, bias=d.bias, stride=L.stride)
    scale = max(ymax, float(np.max(np.abs(ref))), 1e-30)
    err = float(np.max(np.abs(got.astype(np.float64) - ref)) / scale)
    assert err <= TOL, "%s %s sampled rel err %.3g" % (L.name, info, err)
    # groups that keep nothing must reproduce the bias exactly, at any size
    if d.mask is not None:
        empty = np.nonzero(d.mask.reshape(L.G, -1).sum(axis=1) == 0)[0]
        for g in empty[:2]:
            ch = slice(g * L.V, min(L.Cout, (g + 1) * L.V))
            blk = Y[:, ch].cpu().numpy()
            want = 0.0 if d.bias is None else d.bias[ch][None, :, None, None]
            assert np.array_equal(blk, np.broadcast_to(want, blk.shape).astype(np.float32))
    packed.free()
    del X, Y
    torch.cuda.empty_cache()
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
        assert info["mode"] == (3 if L.k == 3 else info["mode"])


def test_config3_resnet50_bottlenecks_batch64_sampled():
    for i, L in enumerate(workloads.resnet50_bottlenecks(64)):
        sampled_check(L, workloads.seed_for(3, i))


def test_config3_independent_pattern_per_tap():
    """The other reading of the 3x3 mask: every (c, r, s) position pruned on its own."""
    layers = [L for L in workloads.resnet50_bottlenecks(2) if L.k == 3]
    for j, L in enumerate((layers[0], [L for L in layers if L.stride == 2][1])):
        full_check(dataclasses.replace(L, tap_shared=False), workloads.seed_for(3, 90 + j))


# ----------------------------------------------------------------------------- config 4

@pytest.mark.parametrize("s", workloads.SWEEP_SPARSITIES)
def test_config4_sparsity_sweep(s):
    full_check(workloads.sweep_layer(s, N=8), workloads.seed_for(4, int(round(s * 100))))
    sampled_check(workloads.sweep_layer(s, N=256), workloads.seed_for(4, int(round(s * 100))))


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
def test_config5_mobilenet_v2_batch128_sampled(V):
    layers = workloads.mobilenet_v2_pointwise(128, V)
    # V=4: every layer; other group sizes: the largest expansion, the ragged projection
    # (Cout=24 with V=16), the widest projection and a 7x7 layer
    pick = range(len(layers)) if V == 4 else [0, 3, 7, 16]
    for i in pick:
        sampled_check(layers[i], workloads.seed_for(5, 100 * V + i), with_bias=True)
