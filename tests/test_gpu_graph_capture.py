"""The convolution entry points neither allocate nor synchronise, so a caller can record them into a
HIP graph: several layers are captured once and replayed with new inputs, with eager work and
synchronisations between the replays, and every replay must equal the eager result bit for bit."""
import numpy as np
import pytest

import oracle
import paper_2109_00170_amd as alcs
import workloads
from gpu_util import TOL, rel_err

pytestmark = pytest.mark.gpu


def test_captured_layers_replay_like_eager_launches():
    import torch
    layers = [
        workloads.Layer("g_pw", 96, 72, 14, 14, N=3, V=4, sparsity=0.8, w_std=0.2),
        workloads.Layer("g_pw512", 512, 64, 14, 14, N=4, V=4, sparsity=0.9, w_std=0.1),        # four groups per wavefront, 130 KB of LDS
        workloads.Layer("g_3x3", 24, 20, 19, 17, k=3, stride=2, N=2, V=4, sparsity=0.7, w_std=0.1),
        workloads.Layer("g_3x3ts", 32, 16, 28, 28, k=3, N=2, V=4, sparsity=0.7, w_std=0.1, tap_shared=True),
        workloads.Layer("g_m16", 64, 48, 16, 16, N=2, V=8, sparsity=0.7, w_std=0.2),
    ]
    data = [workloads.make_layer(L, 7000 + i, with_bias=True) for i, L in enumerate(layers)]
    packed = [alcs.alcs_pack_weights(d.W, d.mask, L.V) for d, L in zip(data, layers)]
    packed[4].add_bf16_weights()
    bias = [torch.from_numpy(d.bias).cuda() for d in data]
    dt = [torch.float32] * 4 + [torch.bfloat16]
    X = [torch.from_numpy(d.X).cuda().to(t) for d, t in zip(data, dt)]
    Y = [torch.zeros((L.N, L.Cout, L.Ho, L.Wo), dtype=t, device="cuda") for L, t in zip(layers, dt)]

    def launch_all():
        alcs.alcs_sparse_conv(packed[0], X[0], bias[0], Y[0])
        alcs.alcs_sparse_conv_fused(packed[1], X[1], bias[1], None, Y[1], activation="relu")
        alcs.alcs_sparse_conv(packed[2], X[2], bias[2], Y[2], stride=2)
        alcs.alcs_sparse_conv(packed[3], X[3], bias[3], Y[3])
        alcs.alcs_sparse_conv_bf16_mfma(packed[4], X[4], bias[4], None, Y[4], activation="relu6")

    launch_all()                                   # first use outside the capture (function attributes are set)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            launch_all()
    torch.cuda.synchronize()
    rng = np.random.default_rng(7100)
    for rep in range(4):
        for x in X:                                # new inputs in the captured buffers
            x.copy_(torch.from_numpy(rng.standard_normal(tuple(x.shape)).astype(np.float32)).cuda().to(x.dtype))
        for y in Y:
            y.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        got = [y.clone() for y in Y]
        for y in Y:
            y.fill_(float("nan"))
        launch_all()                               # the program's own eager work between replays
        torch.cuda.synchronize()
        for g, y, L in zip(got, Y, layers):
            assert not torch.isnan(g.float()).any(), (rep, L.name)
            assert torch.equal(g, y), (rep, L.name)
        # and the replay is right, not just repeatable: the first layer against the oracle
        ref = oracle.sparse_conv(data[0].W, data[0].mask, X[0].cpu().numpy(), 4, bias=data[0].bias)
        assert rel_err(got[0].cpu().numpy(), ref) <= TOL
    for p in packed:
        p.free()
