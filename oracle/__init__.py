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
