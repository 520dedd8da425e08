"""Helpers for the GPU parity tests: run a layer through the HIP library and the oracle."""
import numpy as np

import oracle
import paper_2109_00170_amd as alcs
import workloads

TOL = 1e-5   # max |err| / max |ref|, the bound the problem statement sets for fp32 outputs


def rel_err(got, ref):
    """max |got - ref| / max |ref| (the reference alone sets the scale), image by image so that
    tensors of several hundred MB need no float64 copies of themselves."""
    ref = np.asarray(ref)
    got = np.asarray(got)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    scale = float(np.max(np.abs(ref))) if ref.size else 0.0
    worst = 0.0
    if got.ndim >= 2 and got.size > (1 << 24):
        for g, r in zip(got, ref):
            worst = max(worst, float(np.max(np.abs(g.astype(np.float64) - r.astype(np.float64)))))
    elif got.size:
        worst = float(np.max(np.abs(got.astype(np.float64) - ref.astype(np.float64))))
    if scale == 0.0:
        return worst
    return worst / scale


def assert_close_after_activation(got, ref, pre, what):
    """Outputs behind a fused activation.  The stated bound is max |got - ref| <= TOL * max |ref|;
    the rounding error of the sum grows with the pre-activation values, which a clamp (ReLU6) cuts
    down in ``ref`` but not in the error, so the bound relative to max |pre| is the tighter claim
    about the arithmetic.  Both are asserted, and both ratios are returned."""
    err = float(np.max(np.abs(got.astype(np.float64) - ref.astype(np.float64)))) if got.size else 0.0
    s_ref = float(np.max(np.abs(ref))) if ref.size else 0.0
    s_pre = float(np.max(np.abs(pre))) if pre.size else 0.0
    assert err <= TOL * s_pre or err == 0.0, "%s: err %.3g, %.3g of max|pre|" % (what, err, err / max(s_pre, 1e-300))
    assert err <= TOL * s_ref or err == 0.0, "%s: err %.3g, %.3g of max|ref|" % (what, err, err / max(s_ref, 1e-300))
    return err / max(s_ref, 1e-300), err / max(s_pre, 1e-300)


def run_sparse(d: workloads.LayerData, check_pack=True, options=None):
    """Pack on the library side (with the handle's options, a dict, if any), run alcs_sparse_conv on
    cuda:0, return (Y numpy, launch info)."""
    import torch
    L = d.layer
    packed = alcs.alcs_pack_weights(d.W, d.mask, L.V, options=options or None)
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
