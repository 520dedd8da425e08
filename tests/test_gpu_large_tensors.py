"""Maximum sizes: input tensors with more than 2^31 elements (8.6 GB of fp32), so that every
element offset the kernels form has to be 64 bits wide.  A few thousand outputs are recomputed
one by one by the oracle (conv_at), among them the tensor's corners and elements whose
inputs lie beyond the 2^31-element mark; the all-dropped group must reproduce the bias."""
import numpy as np
import pytest

import oracle
import paper_2109_00170_amd as alcs
import workloads
from gpu_util import TOL

pytestmark = pytest.mark.gpu


def big_check(L, seed, entry):
    import torch
    free_b, _ = torch.cuda.mem_get_info()
    need = 4 * (L.N * L.Cin * L.H * L.W + 2 * L.N * L.Cout * L.Ho * L.Wo) + (1 << 30)
    if free_b < need:
        pytest.skip("needs %.1f GB of device memory" % (need / 1e9))
    assert L.N * L.Cin * L.H * L.W > 2 ** 31
    d = workloads.make_layer(L, seed, with_bias=True)
    d.mask[0] = 0                                   # group 0 keeps nothing: Y[:, 0:V] == bias
    packed = alcs.alcs_pack_weights(d.W, d.mask, L.V)
    X = torch.from_numpy(d.X).cuda()
    b = torch.from_numpy(d.bias).cuda()
    Y = torch.full((L.N, L.Cout, L.Ho, L.Wo), float("nan"), dtype=torch.float32, device="cuda")
    if entry == "sparse":
        alcs.alcs_sparse_conv(packed, X, b, Y, stride=L.stride)
    elif entry == "fused":
        alcs.alcs_sparse_conv_fused(packed, X, b, None, Y, stride=L.stride, activation=None)
    else:
        keep = np.repeat(d.mask, L.V, axis=0)[:L.Cout]
        Wd = torch.from_numpy(np.ascontiguousarray(d.W * keep, dtype=np.float32)).cuda()
        alcs.alcs_dense_conv(Wd, X, b, Y, stride=L.stride)
    torch.cuda.synchronize()
    assert not bool(torch.isnan(Y).any()), "some outputs were never written"
    rng = np.random.default_rng(seed)
    total = Y.numel()
    per_image = L.Cout * L.Ho * L.Wo
    idx = np.unique(np.concatenate([
        rng.integers(0, total, size=2000),
        rng.integers(total - per_image, total, size=1000),      # last image: inputs beyond 2^31 elements
        [0, total - 1, per_image - 1, per_image]]))
    got = Y.reshape(-1)[torch.from_numpy(idx).cuda()].cpu().numpy()
    ymax = float(Y.abs().max())
    blk = Y[:, :L.V].cpu().numpy()
    del Y, X
    torch.cuda.empty_cache()
    Wd_host = oracle.densify(d.W, d.mask, L.V)
    ref = oracle.conv_at(Wd_host, d.X, idx, bias=d.bias, stride=L.stride)
    err = float(np.max(np.abs(got.astype(np.float64) - ref)) / max(ymax, 1e-30))
    assert err <= TOL, "%s %s: sampled rel err %.3g" % (L.name, entry, err)
    if entry != "dense":
        want = np.broadcast_to(d.bias[:L.V][None, :, None, None], blk.shape)
        assert np.array_equal(blk, want.astype(np.float32))
    packed.free()


@pytest.mark.parametrize("entry", ["sparse", "fused", "dense"])
def test_pointwise_input_beyond_2_31_elements(entry):
    # 33 x 64 x 1024 x 1024 = 2.21e9 input elements (8.9 GB); 34.6e6 flattened output pixels
    L = workloads.Layer("big_pw", 64, 8, 1024, 1024, k=1, stride=1, N=33, V=4, sparsity=0.75, w_std=0.1)
    big_check(L, 8101, entry)


@pytest.mark.parametrize("entry", ["sparse", "dense"])
def test_conv3x3_input_beyond_2_31_elements(entry):
    # 9 x 64 x 2048 x 2048 = 2.42e9 input elements; stride 2 output 1024 x 1024
    L = workloads.Layer("big_c3", 64, 8, 2048, 2048, k=3, stride=2, N=9, V=4, sparsity=0.9, w_std=0.1)
    big_check(L, 8102, entry)
