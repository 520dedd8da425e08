"""The storage format of Section 3.2.2 built on the GPU (alcs_pack_csr_device) against the
oracle's packer, bit for bit, and handles made from its arrays (alcs_pack_from_csr) against
handles packed on the host."""
import numpy as np
import pytest

import oracle
import paper_2109_00170_amd as alcs
import workloads
from gpu_util import TOL

pytestmark = pytest.mark.gpu


def random_layer(Cout, Cin, k, V, sparsity, seed):
    rng = np.random.default_rng(seed)
    W = rng.standard_normal((Cout, Cin, k, k)).astype(np.float32)
    W.reshape(-1)[rng.integers(0, W.size, 5)] = np.float32(-0.0)          # bit patterns must survive
    G = (Cout + V - 1) // V
    mask = workloads.mask_exact(G, Cin, k, sparsity, rng)
    return W, mask


@pytest.mark.parametrize("Cout,Cin,k,V,sparsity", [
    (8, 5, 1, 4, 0.5), (10, 3, 3, 4, 0.7), (7, 4, 1, 2, 0.3), (33, 2, 3, 16, 0.6), (5, 5, 1, 1, 0.5),
    (64, 300, 1, 8, 0.9), (256, 257, 1, 4, 0.8), (30, 64, 3, 4, 0.95), (128, 1030, 1, 4, 0.0),
    (16, 16, 1, 4, 1.0), (4100, 8, 1, 4, 0.5)])
def test_device_csr_bit_exact(Cout, Cin, k, V, sparsity):
    import torch
    W, mask = random_layer(Cout, Cin, k, V, sparsity, 3700 + Cout + Cin)
    want = oracle.pack(W, mask, V)
    got = alcs.alcs_pack_csr_device(torch.from_numpy(W).cuda(), torch.from_numpy(mask).cuda(), V)
    torch.cuda.synchronize()
    for g, w in zip(got, want):
        assert g.cpu().numpy().tobytes() == w.tobytes()
    if sparsity == 0.0:                     # no mask keeps everything
        got = alcs.alcs_pack_csr_device(torch.from_numpy(W).cuda(), None, V)
        for g, w in zip(got, want):
            assert g.cpu().numpy().tobytes() == w.tobytes()


def test_handle_from_device_arrays_equals_host_handle():
    import torch
    L = workloads.Layer("pk_dev", 96, 72, 12, 12, N=3, V=4, sparsity=0.8, w_std=0.2)
    d = workloads.make_layer(L, 3750, with_bias=True)
    host = alcs.alcs_pack_weights(d.W, d.mask, 4)
    dev = alcs.alcs_pack_on_device(torch.from_numpy(d.W).cuda(), torch.from_numpy(d.mask).cuda(), 4)
    assert dev.nnzb == host.nnzb and dev.selfcheck() == 0
    for a, b in zip(dev.export(), host.export()):
        assert a.tobytes() == b.tobytes()
    X = torch.from_numpy(d.X).cuda()
    b = torch.from_numpy(d.bias).cuda()
    Y1 = torch.empty((3, 72, 12, 12), device="cuda")
    Y2 = torch.empty_like(Y1)
    alcs.alcs_sparse_conv(host, X, b, Y1)
    alcs.alcs_sparse_conv(dev, X, b, Y2)
    torch.cuda.synchronize()
    assert torch.equal(Y1, Y2)
    ref = oracle.sparse_conv(d.W, d.mask, d.X, 4, bias=d.bias)
    assert float(np.max(np.abs(Y2.cpu().numpy() - ref)) / np.max(np.abs(ref))) <= TOL
    host.free()
    dev.free()


def test_projection_to_handle_without_the_weights_leaving_the_device():
    """scores -> projection -> flags on the device -> device CSR -> handle -> convolution."""
    import torch
    rng = np.random.default_rng(3760)
    W = (rng.standard_normal((64, 80, 1, 1)) * 0.2).astype(np.float32)
    Wd = torch.from_numpy(W).cuda()
    sc = alcs.alcs_block_scores(Wd, 4)
    k = np.arange(11) * 0.1 * W.size
    N, mask, _, _ = alcs.alcs_project_latency(sc.reshape(-1), [0, sc.numel()], [4], [(k, 5.0 + 0.01 * k)], 0.0,
                                              5.0 + 0.01 * 0.25 * W.size, 1e-6)
    packed = alcs.alcs_pack_on_device(Wd, mask, 4)
    assert packed.nnzb == N
    m = mask.cpu().numpy().reshape(16, 80, 1, 1)
    assert np.array_equal(m.reshape(-1), oracle.topn_mask(oracle.block_scores(W, 4).reshape(-1), N))
    X = rng.standard_normal((2, 80, 9, 9)).astype(np.float32)
    Y = torch.empty((2, 64, 9, 9), device="cuda")
    alcs.alcs_sparse_conv(packed, torch.from_numpy(X).cuda(), None, Y)
    torch.cuda.synchronize()
    ref = oracle.sparse_conv(W, m, X, 4)
    assert float(np.max(np.abs(Y.cpu().numpy() - ref)) / np.max(np.abs(ref))) <= TOL
    packed.free()


def test_rejected_arrays_and_capacity():
    import ctypes
    import torch
    W, mask = random_layer(8, 8, 1, 4, 0.5, 3770)
    rp, ci, va = oracle.pack(W, mask, 4)
    bad = ci.copy()
    if bad.size >= 2:
        first = int(rp[1])          # swap two columns of the first group that has at least two
        g = next(i for i in range(2) if rp[i + 1] - rp[i] >= 2)
        a = int(rp[g])
        bad[a], bad[a + 1] = bad[a + 1], bad[a]
        with pytest.raises(alcs.AlcsError):
            alcs.alcs_pack_from_csr(rp, bad, va, 8, 8, 1, 4)
    rp_bad = rp.copy()
    rp_bad[0] = 1
    with pytest.raises(alcs.AlcsError):
        alcs.alcs_pack_from_csr(rp_bad, ci, va, 8, 8, 1, 4)
    # too little room for the kept blocks: refused after the counting pass
    lib = alcs.load_library()
    Wd, md = torch.from_numpy(W).cuda(), torch.from_numpy(mask).cuda()
    rpd = torch.empty(3, dtype=torch.int32, device="cuda")
    cid = torch.empty(1, dtype=torch.int32, device="cuda")
    vad = torch.empty(4, dtype=torch.float32, device="cuda")
    P = lambda t: ctypes.c_void_p(t.data_ptr())
    nn = ctypes.c_longlong()
    rc = lib.alcs_pack_csr_device(P(Wd), P(md), 8, 8, 1, 4, P(rpd), P(cid), P(vad), ctypes.c_longlong(1),
                                  ctypes.byref(nn), None)
    assert rc < 0 and nn.value == int(rp[-1])
    torch.cuda.synchronize()
