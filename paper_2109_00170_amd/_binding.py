"""Argument marshalling for the C ABI declared in include/alcs.h.  No arithmetic here."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.environ.get("ALCS_LIBRARY") or os.path.join(_HERE, "libalcs.so")
_lib = None

EXPORTS = [
    "alcs_strerror", "alcs_last_hip_error", "alcs_version", "alcs_pack_weights", "alcs_packed_info",
    "alcs_packed_on_device", "alcs_packed_export", "alcs_packed_selfcheck", "alcs_packed_free",
    "alcs_sparse_conv", "alcs_sparse_conv_timed", "alcs_sparse_conv_fused", "alcs_dense_conv",
    "alcs_pack_weights_opt", "alcs_packed_set_options", "alcs_packed_get_options",
    "alcs_depthwise_conv", "alcs_dw_sparse_conv_fused", "alcs_sparse_conv_bf16", "alcs_block_scores", "alcs_select_workspace_bytes",
    "alcs_topn_mask", "alcs_topn_mask_static", "alcs_project_latency", "alcs_pack_csr_device", "alcs_pack_from_csr",
    "alcs_pack_from_csr_device", "alcs_pack_weights_device", "alcs_packed_layout_hash",
    "alcs_pack_workspace_bytes", "alcs_pack_network_device", "alcs_packed_add_bf16_weights",
    "alcs_sparse_conv_bf16_mfma",
    "alcs_last_launch", "alcs_latency_estimate", "alcs_network_latency",
]


class Options(ctypes.Structure):
    """alcs_options of include/alcs.h: plain ints, 0 = automatic."""
    _fields_ = [(n, ctypes.c_int) for n in
                ("pixels_per_lane", "waves", "group_tiles", "path", "tile_width", "groups_per_wave",
                 "chunk_channels", "group_slots", "dw_own_taps", "dw_one_kernel", "full_tiles", "measure_skip")] + \
               [("reserved", ctypes.c_int * 4)]

    # short names used by tests and reports
    ALIASES = {"pv": "pixels_per_lane"}

    @classmethod
    def make(cls, options):
        """None, an Options, or a dict of field names (or aliases) to ints."""
        if options is None:
            return None
        if isinstance(options, cls):
            return options
        o = cls()
        for k, v in dict(options).items():
            k = cls.ALIASES.get(k, k)
            if k not in dict(cls._fields_) or k == "reserved":
                raise ValueError("unknown option %r" % k)
            setattr(o, k, int(v))
        return o


class AlcsError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = int(status)
        super().__init__("%s failed: %s (hip error %d)" % (where, alcs_strerror(status), _hip_err()))


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libalcs.so; raise ImportError if it has not been built (no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError("%s is missing: build it with `python -m paper_2109_00170_amd.build` "
                          "(or __graft_entry__.build())" % _LIB_PATH)
    # PyTorch ships its own HIP runtime (libamdhip64.so.7 under torch/lib).  It has to be
    # in the process before libalcs.so is loaded, so that both resolve to that one
    # runtime; otherwise two runtimes coexist and streams and the device cannot be shared.
    import torch  # noqa: F401
    lib = ctypes.CDLL(_LIB_PATH)
    vp, ci, cip = ctypes.c_void_p, ctypes.c_int, ctypes.POINTER(ctypes.c_int)
    lib.alcs_strerror.restype = ctypes.c_char_p
    lib.alcs_strerror.argtypes = [ci]
    lib.alcs_pack_weights.argtypes = [vp, vp, ci, ci, ci, ci, ctypes.POINTER(vp)]
    lib.alcs_packed_info.argtypes = [vp, cip, cip, ctypes.POINTER(ctypes.c_int64)]
    lib.alcs_packed_on_device.argtypes = [vp]
    lib.alcs_packed_export.argtypes = [vp, vp, vp, vp]
    lib.alcs_packed_selfcheck.argtypes = [vp]
    lib.alcs_packed_layout_hash.argtypes = [vp, vp]
    lib.alcs_packed_free.argtypes = [vp]
    lib.alcs_packed_free.restype = None
    lib.alcs_sparse_conv.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, vp]
    lib.alcs_sparse_conv_timed.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, vp, vp, vp]
    lib.alcs_sparse_conv_fused.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, ci, vp]
    lib.alcs_dense_conv.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, vp]
    lib.alcs_pack_weights_opt.argtypes = [vp, vp, ci, ci, ci, ci, vp, ctypes.POINTER(vp)]
    lib.alcs_packed_set_options.argtypes = [vp, vp]
    lib.alcs_packed_get_options.argtypes = [vp, vp]
    lib.alcs_last_launch.argtypes = [cip, ci]
    _lib = lib
    return lib


def _hip_err() -> int:
    return int(load_library().alcs_last_hip_error())


def alcs_strerror(status: int) -> str:
    return load_library().alcs_strerror(int(status)).decode()


def alcs_version() -> int:
    return int(load_library().alcs_version())


def out_size(size: int, kernel: int, stride: int) -> int:
    """Output extent for pad = (kernel-1)//2 (shape bookkeeping only)."""
    return (size + 2 * ((kernel - 1) // 2) - kernel) // stride + 1


class Packed:
    """Owner of an alcs_packed_t handle."""

    def __init__(self, handle, Cout, Cin, kernel, V):
        self._h = handle
        self.Cout, self.Cin, self.kernel, self.V = Cout, Cin, kernel, V
        G, K, nnzb = ctypes.c_int(), ctypes.c_int(), ctypes.c_int64()
        rc = load_library().alcs_packed_info(self._h, ctypes.byref(G), ctypes.byref(K), ctypes.byref(nnzb))
        if rc != 0:
            raise AlcsError(rc, "alcs_packed_info")
        self.G, self.K, self.nnzb = G.value, K.value, nnzb.value

    @property
    def handle(self):
        if self._h is None:
            raise ValueError("packed weights were freed")
        return self._h

    @property
    def on_device(self) -> bool:
        return load_library().alcs_packed_on_device(self.handle) == 1

    def export(self):
        """Canonical grouped CSR: (row_ptr [G+1] int32, col_idx [nnzb] int32, vals [nnzb,V] fp32)."""
        row_ptr = np.zeros(self.G + 1, dtype=np.int32)
        col_idx = np.zeros(max(self.nnzb, 1), dtype=np.int32)
        vals = np.zeros((max(self.nnzb, 1), self.V), dtype=np.float32)
        rc = load_library().alcs_packed_export(self.handle, row_ptr.ctypes.data, col_idx.ctypes.data,
                                               vals.ctypes.data)
        if rc != 0:
            raise AlcsError(rc, "alcs_packed_export")
        return row_ptr, col_idx[: self.nnzb], vals[: self.nnzb]

    def selfcheck(self) -> int:
        return int(load_library().alcs_packed_selfcheck(self.handle))

    def add_bf16_weights(self, stream=None) -> None:
        rc = load_library().alcs_packed_add_bf16_weights(self._h, _stream_ptr(stream))
        if rc != 0:
            raise AlcsError(rc, "alcs_packed_add_bf16_weights")

    def layout_hash(self) -> int:
        h = ctypes.c_ulonglong()
        rc = load_library().alcs_packed_layout_hash(self._h, ctypes.byref(h))
        if rc != 0:
            raise AlcsError(rc, "alcs_packed_layout_hash")
        return int(h.value)

    def set_options(self, options) -> None:
        """Replace the handle's launch options (dict or Options; None = all automatic)."""
        o = Options.make(options) or Options()
        rc = load_library().alcs_packed_set_options(self.handle, ctypes.byref(o))
        if rc != 0:
            raise AlcsError(rc, "alcs_packed_set_options")

    def get_options(self) -> dict:
        o = Options()
        rc = load_library().alcs_packed_get_options(self.handle, ctypes.byref(o))
        if rc != 0:
            raise AlcsError(rc, "alcs_packed_get_options")
        return {n: getattr(o, n) for n, _ in Options._fields_ if n != "reserved"}

    def free(self):
        if self._h is not None:
            load_library().alcs_packed_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def alcs_pack_weights(W: np.ndarray, mask: Optional[np.ndarray], V: int, options=None) -> Packed:
    """W [Cout,Cin,k,k] fp32 host array, mask [G,Cin,k,k] uint8 host array or None; options: None, a
    dict or an Options (then the call goes to alcs_pack_weights_opt)."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    if W.ndim != 4 or W.shape[2] != W.shape[3]:
        raise ValueError("W must be [Cout, Cin, k, k]")
    Cout, Cin, k, _ = W.shape
    mptr = None
    if mask is not None:
        mask = np.ascontiguousarray(mask, dtype=np.uint8)
        if mask.shape != ((Cout + V - 1) // V, Cin, k, k):
            raise ValueError("mask must be [ceil(Cout/V), Cin, k, k], got %r" % (mask.shape,))
        mptr = mask.ctypes.data
    out = ctypes.c_void_p()
    o = Options.make(options)
    if o is None:
        rc = load_library().alcs_pack_weights(W.ctypes.data, mptr, Cout, Cin, k, int(V), ctypes.byref(out))
    else:
        rc = load_library().alcs_pack_weights_opt(W.ctypes.data, mptr, Cout, Cin, k, int(V), ctypes.byref(o),
                                                  ctypes.byref(out))
    if rc != 0:
        raise AlcsError(rc, "alcs_pack_weights")
    return Packed(out, Cout, Cin, k, int(V))


def _stream_ptr(stream):
    if stream is None:
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if hasattr(stream, "cuda_stream"):
        return ctypes.c_void_p(stream.cuda_stream)
    return ctypes.c_void_p(int(stream))


def _dev_ptr(t, name, dtype_name="torch.float32"):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous() or str(t.dtype) != dtype_name:
        raise ValueError("%s must be a contiguous %s tensor on the GPU" % (name, dtype_name))
    return ctypes.c_void_p(t.data_ptr())


def alcs_sparse_conv(packed: Packed, X, bias, Y, stride: int = 1, stream=None, events=None) -> None:
    """Y[N,Cout,Ho,Wo] = sparse_conv(packed, X[N,Cin,H,W]) + bias; device tensors, async on stream.
    events = (start, stop) hipEvent_t handles (ints) routes the call to alcs_sparse_conv_timed."""
    N, Cin, H, W = X.shape
    k = packed.kernel
    exp = (N, packed.Cout, out_size(H, k, stride), out_size(W, k, stride))
    if tuple(Y.shape) != exp:
        raise ValueError("Y must have shape %r, got %r" % (exp, tuple(Y.shape)))
    lib = load_library()
    if events is None:
        rc = lib.alcs_sparse_conv(packed.handle, _dev_ptr(X, "X"), _dev_ptr(bias, "bias"), _dev_ptr(Y, "Y"),
                                  N, Cin, packed.Cout, H, W, k, int(stride), _stream_ptr(stream))
    else:
        rc = lib.alcs_sparse_conv_timed(packed.handle, _dev_ptr(X, "X"), _dev_ptr(bias, "bias"),
                                        _dev_ptr(Y, "Y"), N, Cin, packed.Cout, H, W, k, int(stride),
                                        _stream_ptr(stream), ctypes.c_void_p(events[0]),
                                        ctypes.c_void_p(events[1]))
    if rc != 0:
        raise AlcsError(rc, "alcs_sparse_conv")


ACTIVATIONS = {None: 0, "none": 0, "relu": 1, "relu6": 2}


def alcs_sparse_conv_fused(packed: Packed, X, bias, residual, Y, stride: int = 1, activation=None,
                           stream=None) -> None:
    """Y = act(sparse_conv(packed, X) + bias + residual); residual has Y's shape (or is None, or is Y);
    activation is None, "relu", "relu6" or an alcs_activation integer."""
    N, Cin, H, W = X.shape
    k = packed.kernel
    exp = (N, packed.Cout, out_size(H, k, stride), out_size(W, k, stride))
    if tuple(Y.shape) != exp:
        raise ValueError("Y must have shape %r, got %r" % (exp, tuple(Y.shape)))
    if residual is not None and tuple(residual.shape) != exp:
        raise ValueError("residual must have shape %r, got %r" % (exp, tuple(residual.shape)))
    act = activation if isinstance(activation, int) else ACTIVATIONS[activation]
    rc = load_library().alcs_sparse_conv_fused(packed.handle, _dev_ptr(X, "X"), _dev_ptr(bias, "bias"),
                                               _dev_ptr(residual, "residual"), _dev_ptr(Y, "Y"), N, Cin,
                                               packed.Cout, H, W, k, int(stride), int(act), _stream_ptr(stream))
    if rc != 0:
        raise AlcsError(rc, "alcs_sparse_conv_fused")


def alcs_sparse_conv_bf16(packed: Packed, X, bias, residual, Y, stride: int = 1, activation=None, stream=None,
                          mfma16: bool = False) -> None:
    """alcs_sparse_conv_fused on torch.bfloat16 tensors X, residual (or None) and Y; bias stays float32.
    mfma16 routes the call to alcs_sparse_conv_bf16_mfma (weights rounded to bfloat16 as well; the
    handle needs Packed.add_bf16_weights() first)."""
    N, Cin, H, W = X.shape
    k = packed.kernel
    exp = (N, packed.Cout, out_size(H, k, stride), out_size(W, k, stride))
    if tuple(Y.shape) != exp:
        raise ValueError("Y must have shape %r, got %r" % (exp, tuple(Y.shape)))
    if residual is not None and tuple(residual.shape) != exp:
        raise ValueError("residual must have shape %r, got %r" % (exp, tuple(residual.shape)))
    act = activation if isinstance(activation, int) else ACTIVATIONS[activation]
    bf = "torch.bfloat16"
    lib = load_library()
    fn, name = (lib.alcs_sparse_conv_bf16_mfma, "alcs_sparse_conv_bf16_mfma") if mfma16 else \
        (lib.alcs_sparse_conv_bf16, "alcs_sparse_conv_bf16")
    rc = fn(packed.handle, _dev_ptr(X, "X", bf), _dev_ptr(bias, "bias"), _dev_ptr(residual, "residual", bf),
            _dev_ptr(Y, "Y", bf), N, Cin, packed.Cout, H, W, k, int(stride), int(act), _stream_ptr(stream))
    if rc != 0:
        raise AlcsError(rc, name)


def alcs_sparse_conv_bf16_mfma(packed: Packed, X, bias, residual, Y, stride: int = 1, activation=None, stream=None) -> None:
    alcs_sparse_conv_bf16(packed, X, bias, residual, Y, stride=stride, activation=activation, stream=stream, mfma16=True)


class HipEvents:
    """A pool of raw hipEvent_t pairs from the HIP runtime that is already in the process
    (PyTorch's), for timing launches with alcs_sparse_conv_timed."""

    def __init__(self, n_pairs: int):
        import torch
        path = os.path.join(os.path.dirname(torch.__file__), "lib", "libamdhip64.so")
        self._hip = ctypes.CDLL(path)
        self._hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self._hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self._hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.pairs = []
        for _ in range(n_pairs):
            a, b = ctypes.c_void_p(), ctypes.c_void_p()
            if self._hip.hipEventCreate(ctypes.byref(a)) or self._hip.hipEventCreate(ctypes.byref(b)):
                raise RuntimeError("hipEventCreate failed")
            self.pairs.append((a.value, b.value))

    def elapsed_us(self, i: int) -> float:
        a, b = self.pairs[i]
        self._hip.hipEventSynchronize(ctypes.c_void_p(b))
        ms = ctypes.c_float()
        rc = self._hip.hipEventElapsedTime(ctypes.byref(ms), ctypes.c_void_p(a), ctypes.c_void_p(b))
        if rc:
            raise RuntimeError("hipEventElapsedTime failed (%d)" % rc)
        return ms.value * 1e3

    def close(self):
        for a, b in self.pairs:
            self._hip.hipEventDestroy(ctypes.c_void_p(a))
            self._hip.hipEventDestroy(ctypes.c_void_p(b))
        self.pairs = []


def alcs_dense_conv(W_dev, X, bias, Y, stride: int = 1, stream=None) -> None:
    """Dense reference: W_dev [Cout,Cin,k,k] on the device."""
    Cout, Cin, k, _ = W_dev.shape
    N, Cin2, H, W = X.shape
    if Cin != Cin2:
        raise ValueError("channel mismatch")
    exp = (N, Cout, out_size(H, k, stride), out_size(W, k, stride))
    if tuple(Y.shape) != exp:
        raise ValueError("Y must have shape %r, got %r" % (exp, tuple(Y.shape)))
    rc = load_library().alcs_dense_conv(_dev_ptr(W_dev, "W"), _dev_ptr(X, "X"), _dev_ptr(bias, "bias"),
                                        _dev_ptr(Y, "Y"), N, Cin, Cout, H, W, k, int(stride),
                                        _stream_ptr(stream))
    if rc != 0:
        raise AlcsError(rc, "alcs_dense_conv")


def _act(activation) -> int:
    return int(activation if isinstance(activation, int) else ACTIVATIONS[activation])


def alcs_depthwise_conv(D_dev, X, bias, Y, stride: int = 1, activation=None, stream=None) -> None:
    """Y = act(depthwise3x3(X; D_dev) + bias): D_dev [C,3,3] on the device."""
    N, C, H, W = X.shape
    if tuple(D_dev.shape) != (C, 3, 3):
        raise ValueError("depthwise weights must have shape %r" % ((C, 3, 3),))
    exp = (N, C, out_size(H, 3, stride), out_size(W, 3, stride))
    if tuple(Y.shape) != exp:
        raise ValueError("Y must have shape %r, got %r" % (exp, tuple(Y.shape)))
    rc = load_library().alcs_depthwise_conv(_dev_ptr(D_dev, "dw_weights"), _dev_ptr(X, "X"), _dev_ptr(bias, "bias"),
                                            _dev_ptr(Y, "Y"), N, C, H, W, int(stride), _act(activation),
                                            _stream_ptr(stream))
    if rc != 0:
        raise AlcsError(rc, "alcs_depthwise_conv")


def alcs_dw_sparse_conv_fused(packed: Packed, D_dev, dw_bias, X, bias, residual, Y, dw_stride: int = 1,
                              dw_activation=None, activation=None, workspace=None, stream=None) -> None:
    """Y = act(conv1x1(packed; dw_act(depthwise3x3(X; D_dev) + dw_bias)) + bias + residual) in one kernel;
    ``workspace`` ([N,Cin,Ho,Wo] or None) is used only by layouts the fused kernels do not cover."""
    N, Cin, H, W = X.shape
    if tuple(D_dev.shape) != (Cin, 3, 3):
        raise ValueError("depthwise weights must have shape %r" % ((Cin, 3, 3),))
    Ho, Wo = out_size(H, 3, dw_stride), out_size(W, 3, dw_stride)
    exp = (N, packed.Cout, Ho, Wo)
    if tuple(Y.shape) != exp:
        raise ValueError("Y must have shape %r, got %r" % (exp, tuple(Y.shape)))
    if residual is not None and tuple(residual.shape) != exp:
        raise ValueError("residual must have shape %r, got %r" % (exp, tuple(residual.shape)))
    if workspace is not None and tuple(workspace.shape) != (N, Cin, Ho, Wo):
        raise ValueError("workspace must have shape %r" % ((N, Cin, Ho, Wo),))
    rc = load_library().alcs_dw_sparse_conv_fused(
        packed.handle, _dev_ptr(D_dev, "dw_weights"), _dev_ptr(dw_bias, "dw_bias"), int(dw_stride),
        _act(dw_activation), _dev_ptr(X, "X"), _dev_ptr(bias, "bias"), _dev_ptr(residual, "residual"),
        _dev_ptr(Y, "Y"), _dev_ptr(workspace, "workspace"), N, Cin, packed.Cout, H, W, _act(activation),
        _stream_ptr(stream))
    if rc != 0:
        raise AlcsError(rc, "alcs_dw_sparse_conv_fused")


def alcs_last_launch() -> dict:
    buf = (ctypes.c_int * 10)()
    n = load_library().alcs_last_launch(buf, 10)
    keys = ["mode", "pv", "waves", "workgroups", "lds_bytes", "group_tiles", "chunk_channels", "path",
            "group_slots", "tile_width"]
    return {k: int(buf[i]) for i, k in enumerate(keys[:n])}


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def alcs_latency_estimate(k, t, s) -> float:
    """Run time of a layer with ``s`` non-zero weights from times ``t`` measured at ``k``."""
    k, t = _f64(k), _f64(t)
    if k.ndim != 1 or k.shape != t.shape:
        raise ValueError("k and t must be vectors of one length")
    out = ctypes.c_double()
    dp = ctypes.POINTER(ctypes.c_double)
    rc = load_library().alcs_latency_estimate(k.ctypes.data_as(dp), t.ctypes.data_as(dp), int(k.size),
                                              ctypes.c_double(float(s)), ctypes.byref(out))
    if rc != 0:
        raise AlcsError(rc, "alcs_latency_estimate")
    return float(out.value)


def alcs_network_latency(tau, tables, nnz) -> float:
    """``tau`` plus the estimates of all layers; ``tables`` = [(k, t), ...], ``nnz`` per layer."""
    if len(tables) != len(nnz):
        raise ValueError("one table per layer")
    ks = [_f64(k) for k, _ in tables]
    ts = [_f64(t) for _, t in tables]
    for k, t in zip(ks, ts):
        if k.ndim != 1 or k.shape != t.shape:
            raise ValueError("k and t must be vectors of one length")
    n = np.array([k.size for k in ks], dtype=np.int32)
    kk = _f64(np.concatenate(ks)) if ks else np.zeros(1)
    tt = _f64(np.concatenate(ts)) if ts else np.zeros(1)
    s = _f64(nnz) if len(nnz) else np.zeros(1)
    out = ctypes.c_double()
    dp = ctypes.POINTER(ctypes.c_double)
    rc = load_library().alcs_network_latency(ctypes.c_double(float(tau)), kk.ctypes.data_as(dp),
                                             tt.ctypes.data_as(dp), n.ctypes.data_as(ctypes.POINTER(ctypes.c_int)),
                                             int(len(ks)), s.ctypes.data_as(dp), ctypes.byref(out))
    if rc != 0:
        raise AlcsError(rc, "alcs_network_latency")
    return float(out.value)


def alcs_block_scores(W_dev, V: int, scores=None, stream=None):
    """Squared L2 norm of every block of V weights: W_dev [Cout,Cin,k,k] on the device ->
    float32 tensor [ceil(Cout/V), Cin, k, k] (allocated here unless ``scores`` is given)."""
    import torch
    Cout, Cin, k, _ = W_dev.shape
    G = (Cout + V - 1) // V
    if scores is None:
        scores = torch.empty((G, Cin, k, k), dtype=torch.float32, device=W_dev.device)
    if tuple(scores.shape) != (G, Cin, k, k):
        raise ValueError("scores must have shape %r" % ((G, Cin, k, k),))
    rc = load_library().alcs_block_scores(_dev_ptr(W_dev, "W"), Cout, Cin, k, int(V), _dev_ptr(scores, "scores"),
                                          _stream_ptr(stream))
    if rc != 0:
        raise AlcsError(rc, "alcs_block_scores")
    return scores


def _select_workspace(n_seg, device):
    import torch
    lib = load_library()
    lib.alcs_select_workspace_bytes.restype = ctypes.c_size_t
    nbytes = int(lib.alcs_select_workspace_bytes(int(n_seg)))
    return torch.empty(((nbytes + 7) // 8,), dtype=torch.int64, device=device)


def alcs_topn_mask(scores, N: int, seg_starts=None, want_mask: bool = True, stream=None):
    """Keep flags (uint8 tensor, or None) of the N largest entries of the 1-D float32 device tensor
    ``scores`` and the kept count per segment (numpy int64)."""
    import torch
    n = int(scores.numel())
    starts = np.ascontiguousarray([0, n] if seg_starts is None else seg_starts, dtype=np.int64)
    n_seg = int(starts.size) - 1
    ws = _select_workspace(n_seg, scores.device)
    mask = torch.empty((n,), dtype=torch.uint8, device=scores.device) if want_mask else None
    counts = np.zeros(n_seg, dtype=np.int64)
    llp = ctypes.POINTER(ctypes.c_longlong)
    rc = load_library().alcs_topn_mask(
        _dev_ptr(scores, "scores"), ctypes.c_longlong(n), ctypes.c_longlong(int(N)), starts.ctypes.data_as(llp), n_seg,
        None if mask is None else ctypes.c_void_p(mask.data_ptr()), counts.ctypes.data_as(llp),
        ctypes.c_void_p(ws.data_ptr()), _stream_ptr(stream))
    if rc != 0:
        raise AlcsError(rc, "alcs_topn_mask")
    return mask, counts


def alcs_topn_mask_static(scores, N: int, seg_starts=None, mask=None, stream=None):
    """alcs_topn_mask through the entry point that allocates nothing: ``mask`` is a caller-made uint8
    device tensor of scores.numel() entries (or None for counts only); returns the kept count per
    segment (numpy int64)."""
    n = int(scores.numel())
    starts = np.ascontiguousarray([0, n] if seg_starts is None else seg_starts, dtype=np.int64)
    n_seg = int(starts.size) - 1
    if mask is not None and int(mask.numel()) != n:
        raise ValueError("mask must have %d entries" % n)
    counts = np.zeros(n_seg, dtype=np.int64)
    llp = ctypes.POINTER(ctypes.c_longlong)
    rc = load_library().alcs_topn_mask_static(
        _dev_ptr(scores, "scores"), ctypes.c_longlong(n), ctypes.c_longlong(int(N)), starts.ctypes.data_as(llp), n_seg,
        _dev_ptr(mask, "mask", "torch.uint8"), counts.ctypes.data_as(llp), _stream_ptr(stream))
    if rc != 0:
        raise AlcsError(rc, "alcs_topn_mask_static")
    return counts


def alcs_project_latency(scores, seg_starts, V_per_layer, tables, tau, budget, eps, want_mask: bool = True,
                         stream=None):
    """Algorithm 1 on the device tensor ``scores`` (all layers back to back): returns
    (N, mask uint8 tensor or None, t0, t1)."""
    import torch
    starts = np.ascontiguousarray(seg_starts, dtype=np.int64)
    L = int(starts.size) - 1
    if len(V_per_layer) != L or len(tables) != L:
        raise ValueError("one group size and one table per layer")
    Vs = np.ascontiguousarray(V_per_layer, dtype=np.int32)
    ks = [_f64(k) for k, _ in tables]
    ts = [_f64(t) for _, t in tables]
    nn = np.array([k.size for k in ks], dtype=np.int32)
    kk, tt = _f64(np.concatenate(ks)), _f64(np.concatenate(ts))
    n = int(scores.numel())
    ws = _select_workspace(L, scores.device)
    mask = torch.empty((n,), dtype=torch.uint8, device=scores.device) if want_mask else None
    N_out = ctypes.c_longlong()
    t0, t1 = ctypes.c_double(), ctypes.c_double()
    dp, ip = ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int)
    rc = load_library().alcs_project_latency(
        _dev_ptr(scores, "scores"), starts.ctypes.data_as(ctypes.POINTER(ctypes.c_longlong)), Vs.ctypes.data_as(ip), L,
        ctypes.c_double(float(tau)), kk.ctypes.data_as(dp), tt.ctypes.data_as(dp), nn.ctypes.data_as(ip),
        ctypes.c_double(float(budget)), ctypes.c_double(float(eps)),
        None if mask is None else ctypes.c_void_p(mask.data_ptr()), ctypes.byref(N_out), ctypes.byref(t0),
        ctypes.byref(t1), ctypes.c_void_p(ws.data_ptr()), _stream_ptr(stream))
    if rc != 0:
        raise AlcsError(rc, "alcs_project_latency")
    return int(N_out.value), mask, float(t0.value), float(t1.value)


def alcs_pack_csr_device(W_dev, mask_dev, V: int, stream=None):
    """The grouped CSR of Section 3.2.2 built on the device: returns (row_ptr int32 [G+1],
    col_idx int32 [nnzb], vals float32 [nnzb*V]) as device tensors.  mask_dev: uint8 device tensor
    [G,Cin,k,k] (or flat) or None."""
    import torch
    Cout, Cin, k, _ = W_dev.shape
    G = (Cout + V - 1) // V
    if mask_dev is not None and mask_dev.numel() != G * Cin * k * k:
        raise ValueError("mask must have %d entries" % (G * Cin * k * k))
    lib = load_library()
    row_ptr = torch.empty((G + 1,), dtype=torch.int32, device=W_dev.device)
    nnzb = ctypes.c_longlong()
    mp = _dev_ptr(mask_dev, "mask", "torch.uint8")
    args = (_dev_ptr(W_dev, "W"), mp, Cout, Cin, k, int(V), _dev_ptr(row_ptr, "row_ptr", "torch.int32"))
    rc = lib.alcs_pack_csr_device(*args, None, None, ctypes.c_longlong(0), ctypes.byref(nnzb), _stream_ptr(stream))
    if rc != 0:
        raise AlcsError(rc, "alcs_pack_csr_device")
    n = int(nnzb.value)
    col_idx = torch.empty((n,), dtype=torch.int32, device=W_dev.device)
    vals = torch.empty((n * V,), dtype=torch.float32, device=W_dev.device)
    if n:
        rc = lib.alcs_pack_csr_device(*args, _dev_ptr(col_idx, "col_idx", "torch.int32"), _dev_ptr(vals, "vals"),
                                      ctypes.c_longlong(n), ctypes.byref(nnzb), _stream_ptr(stream))
        if rc != 0:
            raise AlcsError(rc, "alcs_pack_csr_device")
    return row_ptr, col_idx, vals


def alcs_pack_from_csr(row_ptr, col_idx, vals, Cout: int, Cin: int, kernel: int, V: int) -> Packed:
    """A handle from the canonical arrays (numpy, host)."""
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int32)
    col_idx = np.ascontiguousarray(col_idx, dtype=np.int32)
    vals = np.ascontiguousarray(vals, dtype=np.float32)
    G = (Cout + V - 1) // V
    if row_ptr.size != G + 1 or col_idx.size != int(row_ptr[-1]) or vals.size != col_idx.size * V:
        raise ValueError("array sizes do not fit the layer")
    out = ctypes.c_void_p()
    vp = ctypes.c_void_p
    rc = load_library().alcs_pack_from_csr(vp(row_ptr.ctypes.data), vp(col_idx.ctypes.data) if col_idx.size else None,
                                           vp(vals.ctypes.data) if vals.size else None, int(Cout), int(Cin), int(kernel),
                                           int(V), ctypes.byref(out))
    if rc != 0:
        raise AlcsError(rc, "alcs_pack_from_csr")
    return Packed(out, Cout, Cin, kernel, int(V))


def alcs_pack_from_csr_device(row_ptr, col_idx, vals, Cout: int, Cin: int, kernel: int, V: int, options=None,
                              stream=None) -> Packed:
    """A handle from canonical arrays that are device tensors (int32, int32, float32); the layout
    the kernels read is built on the device."""
    G = (Cout + V - 1) // V
    if row_ptr.numel() != G + 1 or vals.numel() != col_idx.numel() * V:
        raise ValueError("array sizes do not fit the layer")
    out = ctypes.c_void_p()
    opt = Options.make(options)
    rc = load_library().alcs_pack_from_csr_device(
        _dev_ptr(row_ptr, "row_ptr", "torch.int32"), _dev_ptr(col_idx, "col_idx", "torch.int32") if col_idx.numel() else None,
        _dev_ptr(vals, "vals") if vals.numel() else None, int(Cout), int(Cin), int(kernel), int(V),
        None if opt is None else ctypes.byref(opt), _stream_ptr(stream), ctypes.byref(out))
    if rc != 0:
        raise AlcsError(rc, "alcs_pack_from_csr_device")
    return Packed(out, Cout, Cin, kernel, int(V))


def alcs_pack_weights_device(W_dev, mask_dev, V: int, options=None, stream=None) -> Packed:
    """Device weights [Cout,Cin,k,k] and device flags (uint8 [G,Cin,k,k] or None) -> handle; arrays
    and layout are built by kernels, the host reads back a few scalars."""
    Cout, Cin, k, _ = W_dev.shape
    G = (Cout + V - 1) // V
    if mask_dev is not None and mask_dev.numel() != G * Cin * k * k:
        raise ValueError("mask must have %d entries" % (G * Cin * k * k))
    out = ctypes.c_void_p()
    opt = Options.make(options)
    rc = load_library().alcs_pack_weights_device(
        _dev_ptr(W_dev, "W"), _dev_ptr(mask_dev, "mask", "torch.uint8"), int(Cout), int(Cin), int(k), int(V),
        None if opt is None else ctypes.byref(opt), _stream_ptr(stream), ctypes.byref(out))
    if rc != 0:
        raise AlcsError(rc, "alcs_pack_weights_device")
    return Packed(out, Cout, Cin, k, int(V))


class LayerDesc(ctypes.Structure):
    """alcs_layer_desc of include/alcs.h."""
    _fields_ = [("W_dev", ctypes.c_void_p), ("mask_dev", ctypes.c_void_p), ("Cout", ctypes.c_int), ("Cin", ctypes.c_int),
                ("kernel", ctypes.c_int), ("V", ctypes.c_int), ("options", ctypes.c_void_p)]


def _layer_descs(Ws, masks, Vs, options):
    n = len(Ws)
    Vs = [int(Vs)] * n if np.isscalar(Vs) else [int(v) for v in Vs]
    opts = [Options.make(o) for o in (options if isinstance(options, (list, tuple)) else [options] * n)]
    descs = (LayerDesc * n)()
    for i, (W, m) in enumerate(zip(Ws, masks)):
        Cout, Cin, k, _ = W.shape
        G = (Cout + Vs[i] - 1) // Vs[i]
        if m is not None and m.numel() != G * Cin * k * k:
            raise ValueError("mask %d must have %d entries" % (i, G * Cin * k * k))
        wp, mp = _dev_ptr(W, "W"), _dev_ptr(m, "mask", "torch.uint8")
        descs[i] = LayerDesc(wp.value, None if mp is None else mp.value, Cout, Cin, k, Vs[i],
                             None if opts[i] is None else ctypes.addressof(opts[i]))
    return descs, opts, Vs


def alcs_pack_workspace_bytes(Ws, masks, Vs, options=None) -> int:
    descs, _keep, _ = _layer_descs(Ws, masks, Vs, options)
    lib = load_library()
    lib.alcs_pack_workspace_bytes.restype = ctypes.c_longlong
    n = int(lib.alcs_pack_workspace_bytes(descs, len(Ws)))
    if n < 0:
        raise AlcsError(n, "alcs_pack_workspace_bytes")
    return n


def alcs_pack_network_device(Ws, masks, Vs, options=None, workspace=None, stream=None):
    """Handles for a list of layers (device weights [Cout,Cin,k,k], device flags or None each) in one
    call; workspace: a uint8 device tensor of alcs_pack_workspace_bytes bytes, or None."""
    descs, _keep, Vs = _layer_descs(Ws, masks, Vs, options)
    n = len(Ws)
    out = (ctypes.c_void_p * n)()
    ws_ptr, ws_bytes = None, 0
    if workspace is not None:
        ws_ptr, ws_bytes = _dev_ptr(workspace, "workspace", "torch.uint8"), workspace.numel()
    rc = load_library().alcs_pack_network_device(descs, n, ws_ptr, ctypes.c_longlong(ws_bytes), _stream_ptr(stream), out)
    if rc != 0:
        raise AlcsError(rc, "alcs_pack_network_device")
    return [Packed(ctypes.c_void_p(out[i]), W.shape[0], W.shape[1], W.shape[2], Vs[i]) for i, W in enumerate(Ws)]


def alcs_pack_on_device(W_dev, mask_dev, V: int, options=None) -> Packed:
    """Device weights and flags -> handle without the host seeing weights, flags or layout."""
    return alcs_pack_weights_device(W_dev, mask_dev, V, options=options)
