"""Helpers for the GPU parity tests: run a layer through the HIP library and the oracle."""
import numpy as np

import oracle
import paper_2109_00170_amd as alcs
import workloads

TOL = 1e-5   # max |err| / max |ref|, the bound the problem statement sets for fp32 outputs


def rel_err(got, ref):
    scale = float(np.max(np.abs(ref)))
    if scale == 0.0:
        return float(np.max(np.abs(got)))
    return float(np.max(np.abs(got.astype(np.float64) - ref.astype(np.float64))) / scale)


def run_sparse(d: workloads.LayerData, check_pack=True):
    """Pack on the library side, run alcs_sparse_conv on cuda:0, return (Y numpy, launch info)."""
    import torch
    L = d.layer
    packed = alcs.alcs_pack_weights(d.W, d.mask, L.V)
    assert packed.on_device
    if check_pack:
        for got, want in zip(packed.export(), oracle.pack(d.W, d.mask, L.V)):
            assert got.tobytes() == want.tobytes()
    X = torch.from_numpy(d.X).cuda()
    b = None if d.bias is None else torch.from_numpy(d.bias).cuda()
    Y = torch.full((L.N, L.Cout, L.Ho, L.Wo), float("nan"), dtype=torch.float32, device="cuda")
    alcs.alcs_sparse_conv(packed, X, b, Y, stride=L.stride)
    torch.cuda.synchronize()
    info = alcs.alcs_last_launch()
    out = Y.cpu().numpy()
    packed.free()
    return out, info


def run_dense(d: workloads.LayerData):
    import torch
    L = d.layer
    Wd = torch.from_numpy(oracle.densify(d.W, d.mask, L.V)).cuda()
    X = torch.from_numpy(d.X).cuda()
    b = None if d.bias is None else torch.from_numpy(d.bias).cuda()
    Y = torch.full((L.N, L.Cout, L.Ho, L.Wo), float("nan"), dtype=torch.float32, device="cuda")
    alcs.alcs_dense_conv(Wd, X, b, Y, stride=L.stride)
    torch.cuda.synchronize()
    return Y.cpu().numpy()


def oracle_ref(d: workloads.LayerData):
    L = d.layer
    return oracle.sparse_conv(d.W, d.mask, d.X, L.V, bias=d.bias, stride=L.stride)
