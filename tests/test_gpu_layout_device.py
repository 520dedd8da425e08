"""The layout the kernels read, built on the GPU (alcs_pack_from_csr_device,
alcs_pack_weights_device), against the one the host packer builds: the same bytes (layout hash),
a green self-check, the canonical arrays of Section 3.2.2 bit for bit as the oracle packs them,
and the same convolution output bit for bit; the output is also held against the oracle."""
import numpy as np
import pytest

import oracle
import paper_2109_00170_amd as alcs
import workloads
from gpu_util import TOL

pytestmark = pytest.mark.gpu


def uneven_mask(G, Cin, k, sparsity, rng):
    """Groups of very different lengths: the keep probability varies tenfold over the groups."""
    p = (1.0 - sparsity) * rng.uniform(0.2, 2.0, size=(G, 1, 1, 1))
    return (rng.random((G, Cin, k, k)) < np.minimum(p, 1.0)).astype(np.uint8)


CASES = [
    # Cout, Cin, k, V, sparsity, options, even
    (72, 96, 1, 4, 0.8, None, True),            # one group per wavefront
    (30, 17, 1, 1, 0.5, None, True),
    (30, 17, 1, 2, 0.5, None, False),
    (64, 40, 1, 8, 0.7, None, True),
    (96, 33, 1, 16, 0.6, None, False),
    (70, 50, 1, 4, 0.6, None, True),            # Cout not a multiple of V
    (72, 520, 1, 4, 0.9, None, True),           # four groups per wavefront, parity-aware order
    (72, 520, 1, 4, 0.9, None, False),          # uneven groups: two per wavefront
    (72, 700, 1, 4, 0.9, {"group_slots": 2}, True),
    (74, 1100, 1, 4, 0.95, {"group_slots": 4}, False),   # last bundle not full
    (64, 512, 1, 8, 0.9, None, True),
    (40, 700, 1, 2, 0.9, None, True),           # chunks of 256 channels
    (40, 96, 1, 4, 0.8, {"chunk_channels": 32}, False),
    (24, 16, 3, 4, 0.7, None, True),            # 3x3: nine selector tables
    (20, 70, 3, 8, 0.9, None, False),
    (16, 16, 1, 4, 1.0, None, True),            # nothing kept
    (16, 24, 1, 4, 0.0, None, True),            # everything kept
    (1024, 512, 1, 4, 0.9, None, True),         # a MobileNet-sized layer
    (4400, 24, 1, 4, 0.5, None, False),         # 1100 segments: the scan of their starts takes two rounds
    (2000, 700, 1, 2, 0.9, None, True),         # 1000 groups x 3 chunks
    (300, 100, 3, 4, 0.8, None, False),         # 3x3, four chunks
]


@pytest.mark.parametrize("Cout,Cin,k,V,sparsity,options,even", CASES)
def test_device_layout_is_the_host_layout(Cout, Cin, k, V, sparsity, options, even):
    import torch
    rng = np.random.default_rng(4100 + Cout + Cin + V)
    W = (rng.standard_normal((Cout, Cin, k, k)) * 0.2).astype(np.float32)
    G = (Cout + V - 1) // V
    mask = workloads.mask_exact(G, Cin, k, sparsity, rng) if even else uneven_mask(G, Cin, k, sparsity, rng)
    host = alcs.alcs_pack_weights(W, mask, V, options=options)
    dev = alcs.alcs_pack_weights_device(torch.from_numpy(W).cuda(), torch.from_numpy(mask).cuda(), V, options=options)
    assert dev.on_device and dev.nnzb == host.nnzb
    # the convolution first, while the device-built handle has never been fetched to the host
    N, H = 3, 9
    X = rng.standard_normal((N, Cin, H, H)).astype(np.float32)
    Xd = torch.from_numpy(X).cuda()
    Y1 = torch.full((N, Cout, H, H), float("nan"), device="cuda")
    Y2 = torch.full((N, Cout, H, H), float("nan"), device="cuda")
    alcs.alcs_sparse_conv(host, Xd, None, Y1)
    info_host = alcs.alcs_last_launch()
    alcs.alcs_sparse_conv(dev, Xd, None, Y2)
    info_dev = alcs.alcs_last_launch()
    torch.cuda.synchronize()
    assert info_host == info_dev
    assert torch.equal(Y1, Y2)
    ref = oracle.sparse_conv(W, mask, X, V)
    scale = float(np.max(np.abs(ref)))
    assert float(np.max(np.abs(Y2.cpu().numpy() - ref))) <= TOL * scale
    # then the arrays
    assert dev.selfcheck() == 0
    assert dev.layout_hash() == host.layout_hash()
    for got, want in zip(dev.export(), oracle.pack(W, mask, V)):
        assert got.tobytes() == want.tobytes()
    assert dev.get_options() == host.get_options()
    host.free()
    dev.free()


def test_from_device_arrays_and_rejections():
    import torch
    rng = np.random.default_rng(4190)
    W = (rng.standard_normal((32, 40, 1, 1)) * 0.2).astype(np.float32)
    mask = workloads.mask_exact(8, 40, 1, 0.6, rng)
    rp, ci, va = oracle.pack(W, mask, 4)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    good = alcs.alcs_pack_from_csr_device(dev(rp), dev(ci), dev(va), 32, 40, 1, 4)
    host = alcs.alcs_pack_weights(W, mask, 4)
    assert good.layout_hash() == host.layout_hash() and good.selfcheck() == 0
    good.free()
    host.free()
    # not the canonical form: descending columns, a column beyond K, counts that do not add up,
    # a count beyond the arrays' length; every one refused by the checks on the device
    g = next(i for i in range(8) if rp[i + 1] - rp[i] >= 2)
    swapped = ci.copy()
    swapped[rp[g]], swapped[rp[g] + 1] = swapped[rp[g] + 1], swapped[rp[g]]
    beyond = ci.copy()
    beyond[-1] = 40
    down = rp.copy()
    down[3] = down[2] - 1
    first = rp.copy()
    first[0] = 1
    for r, c in ((rp, swapped), (rp, beyond), (down, ci), (first, ci)):
        with pytest.raises(alcs.AlcsError) as ei:
            alcs.alcs_pack_from_csr_device(dev(r), dev(c), dev(va), 32, 40, 1, 4)
        assert ei.value.status == -1
    with pytest.raises(alcs.AlcsError):
        alcs.alcs_pack_from_csr_device(dev(rp), dev(ci), dev(va), 32, 40, 1, 4, options={"measure_skip": 1})
    with pytest.raises(ValueError):
        alcs.alcs_pack_from_csr_device(dev(rp[:-1]), dev(ci), dev(va), 32, 40, 1, 4)
    torch.cuda.synchronize()


def test_set_options_and_reuse_of_a_device_built_handle():
    import torch
    L = workloads.Layer("ld_opts", 512, 64, 14, 14, N=4, V=4, sparsity=0.9, w_std=0.1)
    d = workloads.make_layer(L, 4195, with_bias=True)
    dev = alcs.alcs_pack_weights_device(torch.from_numpy(d.W).cuda(), torch.from_numpy(d.mask).cuda(), 4)
    X = torch.from_numpy(d.X).cuda()
    b = torch.from_numpy(d.bias).cuda()
    ref = oracle.sparse_conv(d.W, d.mask, d.X, 4, bias=d.bias)
    scale = float(np.max(np.abs(ref)))
    for opts in (None, {"pixels_per_lane": 1}, {"full_tiles": 1}):
        if opts:
            dev.set_options(opts)
        Y = torch.full((L.N, L.Cout, L.Ho, L.Wo), float("nan"), device="cuda")
        alcs.alcs_sparse_conv(dev, X, b, Y)
        torch.cuda.synchronize()
        assert float(np.max(np.abs(Y.cpu().numpy() - ref))) <= TOL * scale, opts
    dev.free()


def test_network_in_one_call_equals_layer_by_layer():
    import torch
    rng = np.random.default_rng(4198)
    shapes = [(64, 32, 1, 4), (128, 64, 1, 4), (72, 520, 1, 4), (24, 16, 3, 4), (40, 700, 1, 2), (64, 512, 1, 8), (16, 16, 1, 4)]
    Ws, masks, Vs = [], [], []
    for i, (co, ci, k, V) in enumerate(shapes):
        W = (rng.standard_normal((co, ci, k, k)) * 0.2).astype(np.float32)
        m = workloads.mask_exact((co + V - 1) // V, ci, k, 1.0 if i == 6 else 0.85, rng)
        Ws.append(W); masks.append(m); Vs.append(V)
    Wd = [torch.from_numpy(W).cuda() for W in Ws]
    md = [torch.from_numpy(m).cuda() for m in masks]
    md[1] = None                                            # everything kept
    masks[1] = np.ones_like(masks[1])
    need = alcs.alcs_pack_workspace_bytes(Wd, md, Vs)
    ws = torch.empty((need,), dtype=torch.uint8, device="cuda")
    for workspace in (ws, None):
        hs = alcs.alcs_pack_network_device(Wd, md, Vs, workspace=workspace)
        for h, W, m, V in zip(hs, Ws, masks, Vs):
            host = alcs.alcs_pack_weights(W, m, V)
            assert h.selfcheck() == 0 and h.layout_hash() == host.layout_hash()
            for got, want in zip(h.export(), oracle.pack(W, m, V)):
                assert got.tobytes() == want.tobytes()
            host.free()
            h.free()
    # too small a workspace, a layer the packer refuses: no handles, an error
    with pytest.raises(alcs.AlcsError) as ei:
        alcs.alcs_pack_network_device(Wd, md, Vs, workspace=ws[: need - 256])
    assert ei.value.status == -1
    with pytest.raises(alcs.AlcsError) as ei:
        alcs.alcs_pack_network_device(Wd, [None] * 7, [4, 4, 4, 4, 3, 8, 4])          # V = 3
    assert ei.value.status == -2
    torch.cuda.synchronize()


def test_more_groups_than_the_rank_kernel_takes_go_through_the_host():
    """20000 groups (V = 1): the device entry points fetch the arrays once and build the layout on the host."""
    import torch
    rng = np.random.default_rng(4199)
    Cout, Cin, V = 20000, 24, 1
    W = (rng.standard_normal((Cout, Cin, 1, 1)) * 0.2).astype(np.float32)
    mask = workloads.mask_exact(Cout, Cin, 1, 0.7, rng)
    host = alcs.alcs_pack_weights(W, mask, V)
    dev = alcs.alcs_pack_weights_device(torch.from_numpy(W).cuda(), torch.from_numpy(mask).cuda(), V)
    assert dev.layout_hash() == host.layout_hash() and dev.selfcheck() == 0
    rp, ci, va = oracle.pack(W, mask, V)
    dev2 = alcs.alcs_pack_from_csr_device(torch.from_numpy(rp).cuda(), torch.from_numpy(ci).cuda(), torch.from_numpy(va).cuda(),
                                          Cout, Cin, 1, V)
    assert dev2.layout_hash() == host.layout_hash()
    with pytest.raises(alcs.AlcsError) as ei:
        alcs.alcs_pack_network_device([torch.from_numpy(W).cuda()], [None], V)
    assert ei.value.status == -2
    X = rng.standard_normal((2, Cin, 3, 3)).astype(np.float32)
    Y = torch.empty((2, Cout, 3, 3), device="cuda")
    alcs.alcs_sparse_conv(dev, torch.from_numpy(X).cuda(), None, Y)
    torch.cuda.synchronize()
    ref = oracle.sparse_conv(W, mask, X, V)
    assert float(np.max(np.abs(Y.cpu().numpy() - ref))) <= TOL * float(np.max(np.abs(ref)))
    for h in (host, dev, dev2):
        h.free()
