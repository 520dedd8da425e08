"""Maximum sizes: input tensors with more than 2^31 elements (8.6 GB of fp32), so that every
element offset the kernels form has to be 64 bits wide.  A few thousand outputs are recomputed
one by one by the oracle (conv_at), among them the tensor's corners and elements whose
inputs lie beyond the 2^31-element mark; the all-dropped group must reproduce the bias."""
import numpy as np
import pytest

import oracle
import paper_2109_00170_amd as alcs
import workloads
from gpu_util import TOL, assert_close_after_activation

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
    blk = Y[:, :L.V].cpu().numpy()
    del Y, X
    torch.cuda.empty_cache()
    Wd_host = oracle.densify(d.W, d.mask, L.V)
    ref = oracle.conv_at(Wd_host, d.X, idx, bias=d.bias, stride=L.stride)
    # the scale comes from the oracle's values alone (the largest sampled reference output)
    err = float(np.max(np.abs(got.astype(np.float64) - ref)) / max(float(np.max(np.abs(ref))), 1e-30))
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


def test_depthwise_input_beyond_2_31_elements():
    """9 x 64 x 2048 x 2048 = 2.42e9 input elements (9.7 GB), stride 2: plane offsets need 64 bits.
    Four whole planes, among them the very last one, are recomputed by the oracle."""
    import torch
    N, C, H, W, stride = 9, 64, 2048, 2048, 2
    free_b, _ = torch.cuda.mem_get_info()
    need = 4 * N * C * (H * W + (H // 2) * (W // 2)) + (1 << 30)
    if free_b < need:
        pytest.skip("needs %.1f GB of device memory" % (need / 1e9))
    rng = np.random.default_rng(8103)
    D = (rng.standard_normal((C, 3, 3)) * 0.4).astype(np.float32)
    b = rng.standard_normal(C).astype(np.float32)
    X = torch.empty((N, C, H, W), dtype=torch.float32, device="cuda")
    planes = [(0, 0), (3, 17), (8, 0), (8, 63)]
    host = {}
    for n in range(N):                                 # filled image by image: no 9.7 GB host array
        X[n].normal_(0.0, 1.5)
    for (n, c) in planes:
        host[(n, c)] = X[n, c].cpu().numpy()
    Y = torch.full((N, C, H // 2, W // 2), float("nan"), dtype=torch.float32, device="cuda")
    alcs.alcs_depthwise_conv(torch.from_numpy(D).cuda(), X, torch.from_numpy(b).cuda(), Y, stride=stride,
                             activation="relu")
    torch.cuda.synchronize()
    assert not bool(torch.isnan(Y[8]).any()) and not bool(torch.isnan(Y[0]).any())
    for (n, c) in planes:
        ref = oracle.depthwise(D[c:c + 1], host[(n, c)][None, None], bias=b[c:c + 1], stride=stride, act="relu")[0, 0]
        pre = oracle.depthwise(D[c:c + 1], host[(n, c)][None, None], bias=b[c:c + 1], stride=stride)[0, 0]
        got = Y[n, c].cpu().numpy()
        assert_close_after_activation(got, ref, pre, "plane (%d, %d)" % (n, c))


def test_block_with_an_image_too_large_for_32_bit_tap_offsets():
    """1 x 64 x 4096 x 4096 (1.07e9 elements per image): the one-kernel block declines (its tap offsets
    are 32-bit) and the call runs the two layers through the workspace; without one it is refused.
    A band of output rows at the top, in the middle and at the bottom is recomputed by the oracle."""
    import torch
    N, Cin, Cout, H, W, s = 1, 64, 8, 4096, 4096, 2
    Ho, Wo = H // s, W // s
    free_b, _ = torch.cuda.mem_get_info()
    need = 4 * (Cin * H * W + Cin * Ho * Wo + Cout * Ho * Wo) + (1 << 30)
    if free_b < need:
        pytest.skip("needs %.1f GB of device memory" % (need / 1e9))
    L = workloads.Layer("big_blk", Cin, Cout, Ho, Wo, N=1, V=4, sparsity=0.75, w_std=0.1)
    d = workloads.make_layer(workloads.Layer("big_blk_w", Cin, Cout, 2, 2, N=1, V=4, sparsity=0.75, w_std=0.1), 8104,
                             with_bias=True)                       # weights, mask and bias only
    packed = alcs.alcs_pack_weights(d.W, d.mask, 4)
    rng = np.random.default_rng(8105)
    D = (rng.standard_normal((Cin, 3, 3)) * 0.4).astype(np.float32)
    b1 = rng.standard_normal(Cin).astype(np.float32)
    X = torch.empty((N, Cin, H, W), dtype=torch.float32, device="cuda").normal_(0.0, 1.5)
    Y = torch.full((N, Cout, Ho, Wo), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty((N, Cin, Ho, Wo), dtype=torch.float32, device="cuda")
    Dd, b1d, b2d = torch.from_numpy(D).cuda(), torch.from_numpy(b1).cuda(), torch.from_numpy(d.bias).cuda()
    with pytest.raises(alcs.AlcsError) as ei:
        alcs.alcs_dw_sparse_conv_fused(packed, Dd, b1d, X, b2d, None, Y, dw_stride=s, dw_activation="relu")
    assert ei.value.status == -2
    alcs.alcs_dw_sparse_conv_fused(packed, Dd, b1d, X, b2d, None, Y, dw_stride=s, dw_activation="relu",
                                   activation="relu", workspace=ws)
    torch.cuda.synchronize()
    assert not bool(torch.isnan(Y).any())
    for h0, h1 in ((0, 3), (1000, 1003), (Ho - 3, Ho)):
        # input rows 2*(h0-1) .. 2*h1 give output rows h0-1 .. h1 of which h0 .. h1-1 have their true
        # neighbours (the crop's own first and last output row see the crop's edge, except at the image's edge)
        r0, r1 = max(2 * (h0 - 1), 0), min(2 * h1 + 1, H)
        crop = X[:, :, r0:r1].cpu().numpy()
        Z = oracle.depthwise(D, crop, bias=b1, stride=s, act="relu")
        ref = oracle.sparse_conv(d.W, d.mask, Z, 4, bias=d.bias, act="relu")
        pre = oracle.sparse_conv(d.W, d.mask, Z, 4, bias=d.bias)
        first = h0 - r0 // 2                                 # crop-local index of output row h0
        got = Y[:, :, h0:h1].cpu().numpy()
        want = ref[:, :, first:first + (h1 - h0)]
        assert_close_after_activation(got, want, pre, "rows %d-%d" % (h0, h1))
    packed.free()


def test_bf16_pointwise_input_beyond_2_31_elements():
    """33 x 64 x 1024 x 1024 bfloat16 elements (4.4 GB): element offsets beyond 2^31 in the bfloat16
    build.  Sampled outputs (the last image among them) against the 1x1 definition written out in
    double on the gathered input columns."""
    import torch
    N, Cin, Cout, H, W, V = 33, 64, 8, 1024, 1024, 4
    free_b, _ = torch.cuda.mem_get_info()
    need = 2 * N * (Cin + Cout) * H * W + (1 << 30)
    if free_b < need:
        pytest.skip("needs %.1f GB of device memory" % (need / 1e9))
    assert N * Cin * H * W > 2 ** 31
    d = workloads.make_layer(workloads.Layer("big_bf_w", Cin, Cout, 2, 2, N=1, V=V, sparsity=0.75, w_std=0.1), 8106,
                             with_bias=True)
    packed = alcs.alcs_pack_weights(d.W, d.mask, V)
    X = torch.empty((N, Cin, H, W), dtype=torch.bfloat16, device="cuda")
    for n in range(N):
        X[n].normal_(0.0, 1.0)
    Y = torch.full((N, Cout, H, W), float("nan"), dtype=torch.bfloat16, device="cuda")
    alcs.alcs_sparse_conv_bf16(packed, X, torch.from_numpy(d.bias).cuda(), None, Y, activation="relu")
    torch.cuda.synchronize()
    assert not bool(torch.isnan(Y[N - 1]).any()) and not bool(torch.isnan(Y[0]).any())
    rng = np.random.default_rng(8107)
    ns = np.concatenate([rng.integers(0, N, 1500), np.full(500, N - 1), [0, N - 1]])
    ps = np.concatenate([rng.integers(0, H * W, 2000), [0, H * W - 1]])
    nt, pt = torch.from_numpy(ns).cuda(), torch.from_numpy(ps).cuda()
    cols = X.reshape(N, Cin, H * W)[nt, :, pt].float().cpu().numpy().astype(np.float64)        # [samples, Cin]
    got = Y.reshape(N, Cout, H * W)[nt, :, pt].float().cpu().numpy().astype(np.float64)       # [samples, Cout]
    Wd = oracle.densify(d.W, d.mask, V).reshape(Cout, Cin).astype(np.float64)
    pre = cols @ Wd.T + d.bias
    ref = np.maximum(pre, 0.0)
    bound = 2.0 ** -8 * np.abs(ref) + TOL * min(np.max(np.abs(pre)), np.max(np.abs(ref)))
    assert float(np.max(np.abs(got - ref) - bound)) <= 0.0
    packed.free()
