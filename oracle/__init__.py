"""ctypes front end of the CPU oracle (``alcs_oracle.c``).

Test infrastructure only: tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import this package; the product path never does, and
this package imports nothing from the HIP library.  Each function forwards to the C
routine of the same name; see the C file for the passage of the paper (Section
3.2.1 / 3.2.2 of arXiv 2109.00170) every routine follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "alcs_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP only for the (n, o) split)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
             "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.oracle_pack_count.restype = ctypes.c_int64
        lib.oracle_latency_estimate.restype = ctypes.c_double
        lib.oracle_network_latency.restype = ctypes.c_double
        _lib = lib
    return _lib


def _p(a, ct):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ct))


def _f32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def _check(rc, name):
    if rc != 0:
        raise ValueError("%s rejected its arguments (rc=%d)" % (name, rc))


def out_size(size: int, k: int, stride: int) -> int:
    return int(_load().oracle_out_size(int(size), int(k), int(stride)))


def n_groups(Cout: int, V: int) -> int:
    return (Cout + V - 1) // V


def max_threads() -> int:
    return int(_load().oracle_max_threads())


def densify(W, mask, V):
    """W [Cout,Cin,k,k] fp32, mask [G,Cin,k,k] uint8 or None -> W with dropped blocks zeroed."""
    W = _f32(W)
    Cout, Cin, k, k2 = W.shape
    assert k == k2
    if mask is not None:
        mask = np.ascontiguousarray(mask, dtype=np.uint8)
        assert mask.shape == (n_groups(Cout, V), Cin, k, k), mask.shape
    Wd = np.empty_like(W)
    _check(_load().oracle_densify(_p(W, ctypes.c_float), _p(mask, ctypes.c_uint8), Cout, Cin, k, V,
                                  _p(Wd, ctypes.c_float)), "oracle_densify")
    return Wd


def conv(Wd, X, bias=None, stride=1, nthreads=0):
    """Direct convolution of X [N,Cin,H,W] with dense-layout weights Wd [Cout,Cin,k,k]."""
    Wd, X, bias = _f32(Wd), _f32(X), _f32(bias)
    Cout, Cin, k, _ = Wd.shape
    N, Cin2, H, Wi = X.shape
    assert Cin == Cin2
    Ho, Wo = out_size(H, k, stride), out_size(Wi, k, stride)
    Y = np.empty((N, Cout, Ho, Wo), dtype=np.float32)
    _check(_load().oracle_conv(_p(Wd, ctypes.c_float), _p(X, ctypes.c_float),
                               _p(bias, ctypes.c_float), _p(Y, ctypes.c_float), N, Cin, Cout, H, Wi,
                               k, stride, int(nthreads)), "oracle_conv")
    return Y


ACTIVATIONS = {None: 0, "none": 0, "relu": 1, "relu6": 2}


def conv_fused(Wd, X, bias=None, residual=None, act=None, stride=1, nthreads=0):
    """act(conv(X) + bias + residual) with act in {None, "relu", "relu6"}; residual has Y's shape."""
    Wd, X, bias, residual = _f32(Wd), _f32(X), _f32(bias), _f32(residual)
    Cout, Cin, k, _ = Wd.shape
    N, Cin2, H, Wi = X.shape
    assert Cin == Cin2
    Ho, Wo = out_size(H, k, stride), out_size(Wi, k, stride)
    if residual is not None:
        assert residual.shape == (N, Cout, Ho, Wo)
    Y = np.empty((N, Cout, Ho, Wo), dtype=np.float32)
    _check(_load().oracle_conv_fused(_p(Wd, ctypes.c_float), _p(X, ctypes.c_float),
                                     _p(bias, ctypes.c_float), _p(residual, ctypes.c_float),
                                     _p(Y, ctypes.c_float), N, Cin, Cout, H, Wi, k, stride,
                                     ACTIVATIONS[act], int(nthreads)), "oracle_conv_fused")
    return Y


def depthwise(D, X, bias=None, stride=1, act=None):
    """Z = act(depthwise_conv(X; D) + bias): D is [C,k,k], one filter per channel."""
    D, X, bias = _f32(D), _f32(X), _f32(bias)
    C, k = D.shape[0], D.shape[1]
    if D.shape != (C, k, k) or X.ndim != 4 or X.shape[1] != C:
        raise ValueError("depthwise: D must be [C,k,k] and X [N,C,H,W]")
    N, _, H, Wi = X.shape
    Z = np.empty((N, C, out_size(H, k, stride), out_size(Wi, k, stride)), dtype=np.float32)
    _check(_load().oracle_depthwise(_p(D, ctypes.c_float), _p(X, ctypes.c_float), _p(bias, ctypes.c_float),
                                    _p(Z, ctypes.c_float), N, C, H, Wi, k, int(stride), ACTIVATIONS[act]),
           "oracle_depthwise")
    return Z


def conv_at(Wd, X, flat_idx, bias=None, stride=1):
    """The same sum for selected flat indices of Y[N,Cout,Ho,Wo]."""
    Wd, X, bias = _f32(Wd), _f32(X), _f32(bias)
    Cout, Cin, k, _ = Wd.shape
    N, _, H, Wi = X.shape
    idx = np.ascontiguousarray(flat_idx, dtype=np.int64)
    out = np.empty(idx.shape, dtype=np.float32)
    _check(_load().oracle_conv_at(_p(Wd, ctypes.c_float), _p(X, ctypes.c_float),
                                  _p(bias, ctypes.c_float), N, Cin, Cout, H, Wi, k, stride,
                                  _p(idx, ctypes.c_int64), ctypes.c_int64(idx.size),
                                  _p(out, ctypes.c_float)), "oracle_conv_at")
    return out


def pack(W, mask, V):
    """Grouped CSR (row_ptr [G+1] int32, col_idx [nnzb] int32, vals [nnzb,V] fp32)."""
    W = _f32(W)
    Cout, Cin, k, _ = W.shape
    G = n_groups(Cout, V)
    if mask is not None:
        mask = np.ascontiguousarray(mask, dtype=np.uint8)
        assert mask.shape == (G, Cin, k, k), mask.shape
    nnzb = int(_load().oracle_pack_count(_p(mask, ctypes.c_uint8), Cout, Cin, k, V))
    row_ptr = np.zeros(G + 1, dtype=np.int32)
    col_idx = np.zeros(max(nnzb, 1), dtype=np.int32)
    vals = np.zeros((max(nnzb, 1), V), dtype=np.float32)
    _check(_load().oracle_pack(_p(W, ctypes.c_float), _p(mask, ctypes.c_uint8), Cout, Cin, k, V,
                               _p(row_ptr, ctypes.c_int32), _p(col_idx, ctypes.c_int32),
                               _p(vals, ctypes.c_float)), "oracle_pack")
    return row_ptr, col_idx[:nnzb], vals[:nnzb]


def unpack(row_ptr, col_idx, vals, Cout, Cin, k, V):
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int32)
    col_idx = np.ascontiguousarray(col_idx, dtype=np.int32)
    vals = _f32(vals)
    Wd = np.empty((Cout, Cin, k, k), dtype=np.float32)
    _check(_load().oracle_unpack(_p(row_ptr, ctypes.c_int32), _p(col_idx, ctypes.c_int32),
                                 _p(vals, ctypes.c_float), Cout, Cin, k, V, _p(Wd, ctypes.c_float)),
           "oracle_unpack")
    return Wd


def im2col(X1, k, stride):
    X1 = _f32(X1)
    Cin, H, Wi = X1.shape
    P = out_size(H, k, stride) * out_size(Wi, k, stride)
    I = np.empty((Cin * k * k, P), dtype=np.float32)
    _check(_load().oracle_im2col(_p(X1, ctypes.c_float), Cin, H, Wi, k, stride, _p(I, ctypes.c_float)),
           "oracle_im2col")
    return I


def conv_csr(row_ptr, col_idx, vals, X, Cout, k, V, bias=None, stride=1):
    """Grouped-CSR times patch-matrix evaluator (the paper's algorithm order)."""
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int32)
    col_idx = np.ascontiguousarray(col_idx, dtype=np.int32)
    vals, X, bias = _f32(vals), _f32(X), _f32(bias)
    N, Cin, H, Wi = X.shape
    Ho, Wo = out_size(H, k, stride), out_size(Wi, k, stride)
    Y = np.empty((N, Cout, Ho, Wo), dtype=np.float32)
    scratch = np.empty(Cin * k * k * Ho * Wo, dtype=np.float32)
    accbuf = np.empty(V * Ho * Wo, dtype=np.float64)
    _check(_load().oracle_conv_csr(_p(row_ptr, ctypes.c_int32), _p(col_idx, ctypes.c_int32),
                                   _p(vals, ctypes.c_float), _p(X, ctypes.c_float),
                                   _p(bias, ctypes.c_float), _p(Y, ctypes.c_float), N, Cin, Cout, H,
                                   Wi, k, stride, V, _p(scratch, ctypes.c_float),
                                   _p(accbuf, ctypes.c_double)), "oracle_conv_csr")
    return Y


def sparse_conv(W, mask, X, V, bias=None, stride=1, nthreads=0, residual=None, act=None):
    """Definition of the hot path end to end: densify the pruned weights, then convolve
    (with the fused epilogue when a residual or an activation is given)."""
    if residual is None and ACTIVATIONS[act] == 0:
        return conv(densify(W, mask, V), X, bias=bias, stride=stride, nthreads=nthreads)
    return conv_fused(densify(W, mask, V), X, bias=bias, residual=residual, act=act, stride=stride,
                      nthreads=nthreads)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def latency_estimate(k, t, s) -> float:
    """Section 3.3, Eqs. (4)-(6): run time of a layer with ``s`` non-zero weights, from the
    run times ``t`` measured at ``k`` non-zero weights (``k`` strictly increasing)."""
    k, t = _f64(k), _f64(t)
    if k.ndim != 1 or k.shape != t.shape or k.size < 2 or not np.all(np.diff(k) > 0):
        raise ValueError("latency_estimate: need two or more strictly increasing knots")
    return float(_load().oracle_latency_estimate(_p(k, ctypes.c_double), _p(t, ctypes.c_double),
                                                 int(k.size), ctypes.c_double(float(s))))


def network_latency(tau, tables, nnz) -> float:
    """Section 3.3, Eq. (2): ``tau`` plus the estimate of every layer; ``tables`` is a list of
    (k, t) pairs, ``nnz`` the layers' numbers of non-zero weights."""
    if len(tables) != len(nnz):
        raise ValueError("network_latency: one table per layer")
    ks = [_f64(k) for k, _ in tables]
    ts = [_f64(t) for _, t in tables]
    for k, t in zip(ks, ts):
        if k.ndim != 1 or k.shape != t.shape or k.size < 2 or not np.all(np.diff(k) > 0):
            raise ValueError("network_latency: need two or more strictly increasing knots per layer")
    n = np.array([k.size for k in ks], dtype=np.int32)
    kk = _f64(np.concatenate(ks)) if ks else np.zeros(0)
    tt = _f64(np.concatenate(ts)) if ts else np.zeros(0)
    s = _f64(nnz)
    return float(_load().oracle_network_latency(ctypes.c_double(float(tau)), _p(kk, ctypes.c_double),
                                                _p(tt, ctypes.c_double), _p(n, ctypes.c_int), int(len(ks)),
                                                _p(s, ctypes.c_double)))


# ---------------------------------------------------------------------------------------------
# Projection onto the latency constraint (Section 3.4, Algorithm 1 of the paper): plain numpy.
# Test infrastructure like the rest of this package.

def block_scores(W, V) -> np.ndarray:
    """Algorithm 1, steps 1-2: the squared L2 norm of every block (the V weights of one group at
    one filter position; Section 3.2.1), the quantity the blocks are sorted by.  Returned as
    [G, Cin, k, k] float32.  Floating point decides the order, so the precision is part of the
    definition: float32, sum = 0, then for v = 0 .. V-1: sum = sum + w_v * w_v with the product
    and the sum each rounded to float32 (no fused multiply-add); rows beyond Cout in a ragged last
    group count as zero."""
    W = _f32(W)
    Cout, Cin, k, _ = W.shape
    G = n_groups(Cout, V)
    s = np.zeros((G, Cin, k, k), dtype=np.float32)
    for v in range(V):
        rows = np.arange(G) * V + v
        ok = rows < Cout
        w = np.zeros((G, Cin, k, k), dtype=np.float32)
        w[ok] = W[rows[ok]]
        s = (s + (w * w).astype(np.float32)).astype(np.float32)   # numpy float32 ops round once each
    return s


def topn_mask(scores, N) -> np.ndarray:
    """Algorithm 1, step 7: keep the N blocks with the largest score.  ``scores`` is the
    concatenation of all layers' block scores (1-D float32, non-negative).  Order: larger score
    first; among equal scores the block with the lower index first (the paper does not say; a
    total order makes the selection unique).  Scores are compared through their bit patterns,
    which orders non-negative floats (and puts NaN above infinity)."""
    s = np.ascontiguousarray(scores, dtype=np.float32).reshape(-1)
    n = s.size
    if not 0 <= N <= n:
        raise ValueError("N out of range")
    bits = s.view(np.uint32).astype(np.uint64)
    order = np.lexsort((np.arange(n, dtype=np.uint64), np.uint64(0xFFFFFFFF) - bits))  # primary: bits descending
    mask = np.zeros(n, dtype=np.uint8)
    mask[order[:N]] = 1
    return mask


def project_latency(scores_per_layer, V_per_layer, tables, tau, budget, eps):
    """Algorithm 1 (projection with bisection).  ``scores_per_layer``: one block-score array per
    layer (any shape); ``V_per_layer``: the layers' group sizes (a kept block is V non-zero
    weights); ``tables``: the layers' (k, t) latency tables; ``tau``, ``budget``, ``eps`` as in the
    algorithm.  Returns (N, masks_per_layer, t0, t1): the number of kept blocks, the keep / drop
    flag of every block (shaped like the scores) and the final latency bracket.

    Steps as printed: N0 = 0, N1 = number of blocks; t0 / t1 = latency with nothing / everything
    kept; while t1 - t0 > eps: N = (N0 + N1) / 2, t = T(top-N); t < budget moves (t0, N0) up,
    otherwise (t1, N1) down; the result keeps the (N0 + N1) / 2 largest blocks.  Halves are integer
    divisions, and the loop also ends when N1 - N0 <= 1 (the paper's loop would not end when one
    block changes the latency by more than eps)."""
    flat = [np.ascontiguousarray(s, dtype=np.float32).reshape(-1) for s in scores_per_layer]
    sizes = [f.size for f in flat]
    allscores = np.concatenate(flat) if flat else np.zeros(0, np.float32)
    starts = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)

    def latency(N):
        m = topn_mask(allscores, N)
        nnz = [float(int(m[starts[l]:starts[l + 1]].sum()) * int(V_per_layer[l])) for l in range(len(flat))]
        return network_latency(tau, tables, nnz), m

    N0, N1 = 0, int(allscores.size)
    t0, _ = latency(N0)
    t1, _ = latency(N1)
    while t1 - t0 > eps and N1 - N0 > 1:
        N = (N0 + N1) // 2
        t, _ = latency(N)
        if t < budget:
            t0, N0 = t, N
        else:
            t1, N1 = t, N
    N = (N0 + N1) // 2
    _, m = latency(N)
    masks = [m[starts[l]:starts[l + 1]].reshape(np.shape(scores_per_layer[l])) for l in range(len(flat))]
    return N, masks, t0, t1


def round_bf16(x) -> np.ndarray:
    """Round float32 values to bfloat16 (8 significant bits, round to nearest, ties to even) and
    return them as float32; NaN stays NaN.  For the tensors of the bfloat16 entry point."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32).astype(np.uint64)
    rounded = ((bits + 0x7FFF + ((bits >> 16) & 1)) >> 16) << 16
    out = (rounded & 0xFFFFFFFF).astype(np.uint32).view(np.float32).reshape(x.shape).copy()
    out[np.isnan(x)] = np.nan
    return out
