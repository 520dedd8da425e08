"""Host logic of the library, without a GPU: the packer against the oracle (bit exact),
the tuned layout's self-check, argument validation, and the exported symbols."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2109_00170_amd as alcs
from paper_2109_00170_amd import _binding
import workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "alcs.h")).read()
    declared = set(re.findall(r"\b(alcs_[a-z0-9_]+)\s*\(", header))
    declared -= {"alcs_status"}
    assert declared == set(_binding.EXPORTS), declared ^ set(_binding.EXPORTS)
    lib = alcs.load_library()
    for name in declared:
        assert getattr(lib, name) is not None
    assert alcs.alcs_version() >= 100
    assert "INVALID" in alcs.alcs_strerror(-1) and alcs.alcs_strerror(0) == "ALCS_OK"


CASES = [(64, 64, 1, 4, 0.5), (10, 7, 3, 4, 0.4), (24, 96, 1, 16, 0.15), (33, 20, 1, 8, 0.3),
         (7, 5, 3, 1, 0.5), (6, 9, 1, 2, 0.5), (40, 1100, 1, 4, 0.1), (16, 70, 3, 4, 0.2),
         (512, 512, 1, 4, 0.1)]


@pytest.mark.parametrize("Cout,Cin,k,V,density", CASES)
def test_pack_is_bit_exact_against_oracle(Cout, Cin, k, V, density):
    rng = np.random.default_rng(Cout * 7 + Cin * 3 + k + V)
    G = oracle.n_groups(Cout, V)
    W = rng.standard_normal((Cout, Cin, k, k)).astype(np.float32)
    W.reshape(-1)[::97] = -0.0
    mask = (rng.random((G, Cin, k, k)) < density).astype(np.uint8)
    p = alcs.alcs_pack_weights(W, mask, V)
    assert (p.G, p.K, p.nnzb) == (G, Cin * k * k, int(mask.sum()))
    for got, want in zip(p.export(), oracle.pack(W, mask, V)):
        assert got.dtype == want.dtype and got.tobytes() == want.tobytes()
    assert p.selfcheck() == 0
    p.free()


def test_pack_without_mask_and_with_empty_mask():
    rng = np.random.default_rng(1)
    W = rng.standard_normal((8, 6, 3, 3)).astype(np.float32)
    p = alcs.alcs_pack_weights(W, None, 4)
    for got, want in zip(p.export(), oracle.pack(W, None, 4)):
        assert got.tobytes() == want.tobytes()
    assert p.selfcheck() == 0
    p0 = alcs.alcs_pack_weights(W, np.zeros((2, 6, 3, 3), np.uint8), 4)
    assert p0.nnzb == 0 and p0.export()[0].tolist() == [0, 0, 0] and p0.selfcheck() == 0


def test_zipf_masks_pack_and_selfcheck():
    for V in (1, 4, 8, 16):
        L = workloads.mobilenet_v2_pointwise(1, V)[7]
        d = workloads.make_layer(workloads.Layer(**{**L.__dict__, "H": 4, "W": 4}), 5)
        p = alcs.alcs_pack_weights(d.W, d.mask, V)
        for got, want in zip(p.export(), oracle.pack(d.W, d.mask, V)):
            assert got.tobytes() == want.tobytes()
        assert p.selfcheck() == 0


def test_argument_validation_on_the_host():
    lib = alcs.load_library()
    W = np.zeros((8, 4, 1, 1), np.float32)
    out = ctypes.c_void_p()
    E_INVALID, E_UNSUPPORTED, E_NO_DEVICE = -1, -2, -5
    assert lib.alcs_pack_weights(None, None, 8, 4, 1, 4, ctypes.byref(out)) == E_INVALID
    assert lib.alcs_pack_weights(W.ctypes.data, None, 8, 4, 1, 4, None) == E_INVALID
    assert lib.alcs_pack_weights(W.ctypes.data, None, 0, 4, 1, 4, ctypes.byref(out)) == E_INVALID
    assert lib.alcs_pack_weights(W.ctypes.data, None, 8, 4, 2, 4, ctypes.byref(out)) == E_UNSUPPORTED
    assert lib.alcs_pack_weights(W.ctypes.data, None, 8, 4, 5, 4, ctypes.byref(out)) == E_UNSUPPORTED
    assert lib.alcs_pack_weights(W.ctypes.data, None, 8, 4, 1, 3, ctypes.byref(out)) == E_UNSUPPORTED
    assert out.value is None
    assert lib.alcs_packed_info(None, None, None, None) == E_INVALID
    assert lib.alcs_packed_export(None, None, None, None) == E_INVALID
    assert lib.alcs_packed_selfcheck(None) == E_INVALID
    lib.alcs_packed_free(None)
    p = alcs.alcs_pack_weights(W, None, 4)
    x = ctypes.c_void_p(0x1000)
    # shape mismatch with the handle is reported before anything touches a device
    assert lib.alcs_sparse_conv(p.handle, x, None, x, 1, 5, 8, 4, 4, 1, 1, None) == E_INVALID
    assert lib.alcs_sparse_conv(p.handle, x, None, x, 1, 4, 9, 4, 4, 1, 1, None) == E_INVALID
    assert lib.alcs_sparse_conv(p.handle, x, None, x, 1, 4, 8, 4, 4, 3, 1, None) == E_INVALID
    assert lib.alcs_sparse_conv(p.handle, x, None, x, 1, 4, 8, 4, 4, 1, 3, None) == E_UNSUPPORTED
    assert lib.alcs_sparse_conv(p.handle, None, None, x, 1, 4, 8, 4, 4, 1, 1, None) == E_INVALID
    assert lib.alcs_sparse_conv(p.handle, x, None, ctypes.c_void_p(0x1004), 1, 4, 8, 4, 4, 1, 1, None) == E_INVALID
    assert lib.alcs_sparse_conv(None, x, None, x, 1, 4, 8, 4, 4, 1, 1, None) == E_INVALID
    assert lib.alcs_sparse_conv(p.handle, x, None, x, 0, 4, 8, 4, 4, 1, 1, None) == 0   # N == 0: no-op
    if not p.on_device:
        assert lib.alcs_sparse_conv(p.handle, x, None, x, 1, 4, 8, 4, 4, 1, 1, None) == E_NO_DEVICE
    assert lib.alcs_dense_conv(None, x, None, x, 1, 4, 8, 4, 4, 1, 1, None) == E_INVALID
    assert lib.alcs_dense_conv(x, x, None, x, 1, 4, 8, 4, 4, 2, 1, None) == E_UNSUPPORTED
    assert lib.alcs_dense_conv(x, x, None, x, 0, 4, 8, 4, 4, 1, 1, None) == 0
    # options: negative fields, reserved fields and the measurement-only field are refused
    for bad in ({"waves": -1}, {"measure_skip": 1}):
        with pytest.raises(alcs.AlcsError) as e:
            alcs.alcs_pack_weights(np.zeros((8, 4, 1, 1), np.float32), None, 4, options=bad)
        assert e.value.status == E_INVALID
    o = alcs.Options()
    o.reserved[2] = 1
    with pytest.raises(alcs.AlcsError):
        alcs.alcs_pack_weights(np.zeros((8, 4, 1, 1), np.float32), None, 4, options=o)
    with pytest.raises(ValueError):
        alcs.alcs_pack_weights(np.zeros((8, 4, 1, 1), np.float32), None, 4, options={"no_such_option": 1})


def test_chunked_layouts_selfcheck_for_every_chunk_size():
    rng = np.random.default_rng(3)
    W = rng.standard_normal((20, 37, 1, 1)).astype(np.float32)
    mask = (rng.random((5, 37, 1, 1)) < 0.3).astype(np.uint8)
    for kc in (1, 5, 8, 36, 37, 64):
        p = alcs.alcs_pack_weights(W, mask, 4, options={"chunk_channels": kc})
        assert p.selfcheck() == 0
        for got, want in zip(p.export(), oracle.pack(W, mask, 4)):
            assert got.tobytes() == want.tobytes()


@pytest.mark.parametrize("gs", [1, 2, 4])
@pytest.mark.parametrize("V,Cout", [(4, 44), (8, 40), (16, 50)])
def test_group_slot_layouts_selfcheck(gs, V, Cout):
    """Bundles of 1, 2 or 4 groups per wavefront, including a last bundle that is not full."""
    rng = np.random.default_rng(gs * 10 + V)
    G = oracle.n_groups(Cout, V)
    W = rng.standard_normal((Cout, 70, 1, 1)).astype(np.float32)
    mask = (rng.random((G, 70, 1, 1)) < 0.35).astype(np.uint8)
    mask[1] = 0          # an empty group ends up in the last bundle
    p = alcs.alcs_pack_weights(W, mask, V, options={"group_slots": gs})
    assert p.selfcheck() == 0
    for got, want in zip(p.export(), oracle.pack(W, mask, V)):
        assert got.tobytes() == want.tobytes()


@pytest.mark.parametrize("Cin", [640, 1280, 2048, 2560])
def test_wide_inputs_pack_and_selfcheck(Cin):
    rng = np.random.default_rng(Cin)
    W = rng.standard_normal((24, Cin, 1, 1)).astype(np.float32)
    mask = (rng.random((6, Cin, 1, 1)) < 0.1).astype(np.uint8)
    p = alcs.alcs_pack_weights(W, mask, 4)
    assert p.selfcheck() == 0
    for got, want in zip(p.export(), oracle.pack(W, mask, 4)):
        assert got.tobytes() == want.tobytes()


def test_python_binding_rejects_bad_mask_shape():
    W = np.zeros((8, 4, 1, 1), np.float32)
    with pytest.raises(ValueError):
        alcs.alcs_pack_weights(W, np.ones((3, 4, 1, 1), np.uint8), 4)
    with pytest.raises(alcs.AlcsError):
        alcs.alcs_pack_weights(W, None, 5)


def test_handle_from_canonical_arrays_equals_handle_from_weights():
    import workloads
    rng = np.random.default_rng(77)
    for (Cout, Cin, k, V, sp) in [(10, 6, 3, 4, 0.6), (8, 700, 1, 2, 0.9), (33, 5, 1, 16, 0.3), (4, 4, 1, 4, 1.0)]:
        W = rng.standard_normal((Cout, Cin, k, k)).astype(np.float32)
        mask = workloads.mask_exact((Cout + V - 1) // V, Cin, k, sp, rng)
        rp, ci, va = oracle.pack(W, mask, V)
        a = alcs.alcs_pack_from_csr(rp, ci, va, Cout, Cin, k, V)
        b = alcs.alcs_pack_weights(W, mask, V)
        assert a.nnzb == b.nnzb and a.selfcheck() == 0
        for x, y in zip(a.export(), b.export()):
            assert x.tobytes() == y.tobytes()
        a.free()
        b.free()
    # arrays that are not the canonical form are refused
    W = rng.standard_normal((8, 8, 1, 1)).astype(np.float32)
    rp, ci, va = oracle.pack(W, np.ones((2, 8, 1, 1), np.uint8), 4)
    bad = ci.copy()
    bad[0], bad[1] = bad[1], bad[0]
    with pytest.raises(alcs.AlcsError):
        alcs.alcs_pack_from_csr(rp, bad, va, 8, 8, 1, 4)
    bad = ci.copy()
    bad[3] = 8
    with pytest.raises(alcs.AlcsError):
        alcs.alcs_pack_from_csr(rp, bad, va, 8, 8, 1, 4)
