"""Pins for the oracle's grouped-CSR packing (Section 3.2.2, "Storage format").

Every expected value here comes from the paper's prose example, from a closed
form, or from an explicit construction in the test; none is produced by the oracle
itself or by the HIP library.
"""
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "storage_format_example.txt")


def _read_golden():
    V = K = count = None
    kept = []
    with open(GOLDEN) as f:
        for line in f:
            t = line.split()
            if not t or t[0].startswith("#"):
                continue
            if t[0] == "group_size":
                V = int(t[1])
            elif t[0] == "num_columns":
                K = int(t[1])
            elif t[0] == "count":
                count = int(t[1])
            elif t[0] == "kept":
                kept.append((int(t[3]), [float(x) for x in t[5:]]))
    return V, K, count, kept


def test_paper_storage_format_example():
    """The group of the paper's figure: count 3, offsets 1 and 3 are absolute
    0-based positions (a delta encoding would give 2 for the second), values are
    stored one V-vector per kept column, top row first."""
    V, K, count, kept = _read_golden()
    W = np.zeros((V, K, 1, 1), dtype=np.float32)
    mask = np.zeros((1, K, 1, 1), dtype=np.uint8)
    for off, vals in kept:
        mask[0, off, 0, 0] = 1
        W[:, off, 0, 0] = vals
    row_ptr, col_idx, vals = oracle.pack(W, mask, V)
    assert row_ptr.tolist() == [0, count] == [0, 3]
    assert col_idx[:2].tolist() == [1, 3]               # the two offsets the paper prints
    assert vals.reshape(-1)[:4].tolist() == [1.0, 3.0, 2.0, 1.0]
    assert col_idx.tolist() == [k[0] for k in kept]
    assert vals.tolist() == [k[1] for k in kept]


def _rand_case(rng, Cout, Cin, k, V, density):
    G = oracle.n_groups(Cout, V)
    W = rng.standard_normal((Cout, Cin, k, k)).astype(np.float32)
    mask = (rng.random((G, Cin, k, k)) < density).astype(np.uint8)
    return W, mask


@pytest.mark.parametrize("Cout,Cin,k,V", [(8, 5, 1, 4), (6, 7, 3, 2), (5, 3, 3, 4), (24, 9, 1, 16),
                                          (7, 4, 1, 1), (16, 16, 3, 8)])
def test_pack_invariants_and_round_trip(Cout, Cin, k, V):
    rng = np.random.default_rng(7 + Cout * 131 + Cin * 17 + k + V)
    W, mask = _rand_case(rng, Cout, Cin, k, V, 0.4)
    G, K = oracle.n_groups(Cout, V), Cin * k * k
    row_ptr, col_idx, vals = oracle.pack(W, mask, V)
    assert row_ptr[0] == 0 and np.all(np.diff(row_ptr) >= 0)
    assert row_ptr[G] == int(mask.sum()) == len(col_idx) == len(vals)
    flat_mask = mask.reshape(G, K)
    for g in range(G):
        cols = col_idx[row_ptr[g]:row_ptr[g + 1]]
        # strictly ascending, inside the row, and exactly the kept positions
        assert np.array_equal(cols, np.nonzero(flat_mask[g])[0])
    # expected dense matrix built by hand: W where the group's flag is set, else 0
    keep = np.repeat(flat_mask, V, axis=0)[:Cout].astype(bool)
    expect = np.where(keep, W.reshape(Cout, K), np.float32(0)).reshape(W.shape)
    got = oracle.unpack(row_ptr, col_idx, vals, Cout, Cin, k, V)
    assert got.tobytes() == expect.tobytes()            # bit for bit
    assert oracle.densify(W, mask, V).tobytes() == expect.tobytes()


def test_values_are_column_vectors_top_row_first():
    V, Cin = 4, 3
    W = np.arange(8 * Cin, dtype=np.float32).reshape(8, Cin, 1, 1) + 1
    mask = np.array([[0, 1, 1], [1, 0, 0]], dtype=np.uint8).reshape(2, Cin, 1, 1)
    row_ptr, col_idx, vals = oracle.pack(W, mask, V)
    assert row_ptr.tolist() == [0, 2, 3]
    assert col_idx.tolist() == [1, 2, 0]
    assert vals.tolist() == [[2, 5, 8, 11], [3, 6, 9, 12], [13, 16, 19, 22]]


def test_column_order_is_c_then_r_then_s():
    Cin, k, V = 2, 3, 1
    W = np.zeros((1, Cin, k, k), dtype=np.float32)
    mask = np.zeros((1, Cin, k, k), dtype=np.uint8)
    for (c, r, s) in [(1, 2, 0), (0, 1, 2), (1, 0, 1)]:
        mask[0, c, r, s] = 1
        W[0, c, r, s] = 100 * c + 10 * r + s
    _, col_idx, vals = oracle.pack(W, mask, V)
    assert col_idx.tolist() == [0 * 9 + 1 * 3 + 2, 1 * 9 + 0 * 3 + 1, 1 * 9 + 2 * 3 + 0]
    assert vals.reshape(-1).tolist() == [12.0, 101.0, 120.0]


def test_all_kept_and_all_dropped():
    rng = np.random.default_rng(3)
    W = rng.standard_normal((8, 6, 3, 3)).astype(np.float32)
    G, K = 2, 54
    for m in (None, np.ones((G, 6, 3, 3), np.uint8)):
        row_ptr, col_idx, vals = oracle.pack(W, m, 4)
        assert row_ptr.tolist() == [0, K, 2 * K]
        assert col_idx.tolist() == list(range(K)) * 2
        assert np.array_equal(vals[:K], W.reshape(8, K)[:4].T)
    row_ptr, col_idx, vals = oracle.pack(W, np.zeros((G, 6, 3, 3), np.uint8), 4)
    assert row_ptr.tolist() == [0, 0, 0] and len(col_idx) == 0 and len(vals) == 0


def test_mask_rules_not_the_values():
    """A kept block of zeros is stored; a dropped block of non-zeros is not."""
    W = np.array([[0.0, 5.0], [0.0, 6.0]], dtype=np.float32).reshape(2, 2, 1, 1)
    mask = np.array([[1, 0]], dtype=np.uint8).reshape(1, 2, 1, 1)
    row_ptr, col_idx, vals = oracle.pack(W, mask, 2)
    assert row_ptr.tolist() == [0, 1] and col_idx.tolist() == [0]
    assert vals.tolist() == [[0.0, 0.0]]
    assert oracle.densify(W, mask, 2).reshape(-1).tolist() == [0.0, 0.0, 0.0, 0.0]


def test_ragged_last_group_padded_with_positive_zero():
    V, Cout, Cin = 4, 6, 3
    W = -np.ones((Cout, Cin, 1, 1), dtype=np.float32)
    row_ptr, col_idx, vals = oracle.pack(W, None, V)
    assert row_ptr.tolist() == [0, 3, 6]
    last = vals[3:]
    assert np.all(last[:, :2] == -1.0)
    assert last[:, 2:].tobytes() == np.zeros((3, 2), np.float32).tobytes()  # +0.0f, not -0.0f
    back = oracle.unpack(row_ptr, col_idx, vals, Cout, Cin, 1, V)
    assert back.tobytes() == W.tobytes()


def test_negative_zero_and_nan_bits_survive():
    W = np.array([[-0.0, np.nan], [np.inf, 1e-42]], dtype=np.float32).reshape(2, 2, 1, 1)
    row_ptr, col_idx, vals = oracle.pack(W, None, 2)
    assert vals.tobytes() == np.ascontiguousarray(W.reshape(2, 2).T).tobytes()
