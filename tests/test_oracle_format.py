"""Pins for the oracle's brick builder (Section 3.2): closed-form worked
examples, invariants the paper states, a round trip, and a second, naive
builder written independently in this file."""
import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

import oracle
from paper_2504_06443_amd import workloads as W

PAD = 0xFFFFFFFF


def naive_builder(A: W.CSR):
    """Dict-of-sets reference, no sorting tricks: follows Section 3.2 literally."""
    P = (A.M + 15) // 16
    panel_ptr, brick_cols, brick_mask, valptr, packed = [0], [], [], [0], []
    for p in range(P):
        cells = {}
        for i in range(16 * p, min(A.M, 16 * p + 16)):
            for e in range(A.rowptr[i], A.rowptr[i + 1]):
                cells[(i - 16 * p, int(A.colind[e]))] = float(A.vals[e])
        active = sorted({c for (_, c) in cells})
        nb = (len(active) + 3) // 4
        for b in range(nb):
            cols = active[4 * b:4 * b + 4]
            mask = 0
            vals = []
            for r in range(16):               # row-major inside the brick
                for c, col in enumerate(cols):
                    if (r, col) in cells:
                        mask |= 1 << (4 * r + c)
                        vals.append(cells[(r, col)])
            brick_cols += cols + [PAD] * (4 - len(cols))
            brick_mask.append(mask)
            packed += vals
            valptr.append(len(packed))
        panel_ptr.append(panel_ptr[-1] + nb)
    return dict(panel_ptr=np.array(panel_ptr, np.uint32), brick_cols=np.array(brick_cols, np.uint32),
                brick_mask=np.array(brick_mask, np.uint64), brick_valptr=np.array(valptr, np.uint32),
                vals=np.array(packed, np.float32))


def assert_same_format(a, b):
    for k in ("panel_ptr", "brick_cols", "brick_mask", "brick_valptr", "vals"):
        assert a[k].dtype == b[k].dtype, k
        assert np.array_equal(a[k].view(np.uint8), b[k].view(np.uint8)), k


def check_invariants(A: W.CSR, f):
    nb = len(f["brick_mask"])
    P = (A.M + 15) // 16
    assert len(f["panel_ptr"]) == P + 1 and f["panel_ptr"][0] == 0 and f["panel_ptr"][-1] == nb
    pops = np.array([bin(int(m)).count("1") for m in f["brick_mask"]], dtype=np.int64)
    assert pops.sum() == A.nnz == int(f["brick_valptr"][-1])
    assert np.array_equal(np.diff(f["brick_valptr"].astype(np.int64)), pops)
    assert (pops > 0).all()                       # no empty brick is stored
    cols = f["brick_cols"].reshape(nb, 4)
    for p in range(P):
        b0, b1 = int(f["panel_ptr"][p]), int(f["panel_ptr"][p + 1])
        flat = cols[b0:b1].ravel()
        real = flat[flat != PAD]
        assert (np.diff(real.astype(np.int64)) > 0).all()       # ascending, distinct
        assert len(real) == int(f["ncols"][p])
        assert (flat[:len(real)] != PAD).all()                  # pads only at the tail
        assert b1 - b0 == (len(real) + 3) // 4
    # every real brick column holds at least one non-zero (Section 6.4), pads hold none
    for b in range(nb):
        m = int(f["brick_mask"][b])
        for c in range(4):
            colbits = sum((m >> (4 * r + c)) & 1 for r in range(16))
            assert (colbits >= 1) == (cols[b, c] != PAD)


def test_identity16_closed_form():
    A = W.csr_from_coo(16, 16, np.arange(16), np.arange(16), np.arange(1, 17, dtype=np.float32))
    f = oracle.build_bricks(16, A.rowptr, A.colind, A.vals)
    assert f["panel_ptr"].tolist() == [0, 4]
    assert f["brick_cols"].tolist() == list(range(16))
    # brick b holds rows/cols 4b..4b+3 on its diagonal: bits (4b+c)*4 + c
    assert [int(m) for m in f["brick_mask"]] == [0x8421 << (16 * b) for b in range(4)]
    assert f["brick_valptr"].tolist() == [0, 4, 8, 12, 16]
    assert f["vals"].tolist() == [float(v) for v in range(1, 17)]


def test_dense_16x4_closed_form():
    rows, cols = np.divmod(np.arange(64), 4)
    vals = np.arange(64, dtype=np.float32)
    A = W.csr_from_coo(16, 4, rows, cols, vals)
    f = oracle.build_bricks(16, A.rowptr, A.colind, A.vals)
    assert f["panel_ptr"].tolist() == [0, 1]
    assert int(f["brick_mask"][0]) == 0xFFFFFFFFFFFFFFFF
    assert f["vals"].tolist() == vals.tolist()        # row-major inside the brick
    assert f["brick_cols"].tolist() == [0, 1, 2, 3]


@pytest.mark.parametrize("i,j", [(0, 0), (5, 9), (15, 2), (21, 30), (31, 0)])
def test_single_entry_closed_form(i, j):
    A = W.csr_from_coo(32, 31, [i], [j], np.array([3.5], np.float32))
    f = oracle.build_bricks(32, A.rowptr, A.colind, A.vals)
    p = i // 16
    assert f["panel_ptr"].tolist() == ([0, 1, 1] if p == 0 else [0, 0, 1])
    assert f["brick_cols"].tolist() == [j, PAD, PAD, PAD]
    assert int(f["brick_mask"][0]) == 1 << (4 * (i % 16))
    assert f["vals"].tolist() == [3.5]


def test_dense_column_closed_form():
    A = W.csr_from_coo(16, 10, np.arange(16), np.full(16, 7), np.arange(16, dtype=np.float32))
    f = oracle.build_bricks(16, A.rowptr, A.colind, A.vals)
    assert int(f["brick_mask"][0]) == 0x1111111111111111
    assert f["brick_cols"].tolist() == [7, PAD, PAD, PAD]
    assert f["vals"].tolist() == [float(r) for r in range(16)]


def test_column_compaction_and_row_major_order():
    """Two rows sharing far-apart columns: compaction packs them into one brick and
    the values come out row by row, not column by column."""
    #        col: 3   50  51  900
    # row 2:      a       b
    # row 9:          c       d
    # row 2 again col 900: e
    rows = [2, 2, 9, 9, 2]
    cols = [3, 51, 50, 900, 900]
    vals = np.array([1, 2, 3, 4, 5], np.float32)
    A = W.csr_from_coo(16, 1000, rows, cols, vals)
    f = oracle.build_bricks(16, A.rowptr, A.colind, A.vals)
    assert f["brick_cols"].tolist() == [3, 50, 51, 900]
    bits = [4 * 2 + 0, 4 * 2 + 2, 4 * 2 + 3, 4 * 9 + 1, 4 * 9 + 3]
    assert int(f["brick_mask"][0]) == sum(1 << b for b in bits)
    assert f["vals"].tolist() == [1.0, 2.0, 5.0, 3.0, 4.0]


def test_five_columns_make_a_padded_second_brick():
    A = W.csr_from_coo(16, 100, [0, 0, 0, 0, 0], [10, 20, 30, 40, 50], np.arange(5, dtype=np.float32))
    f = oracle.build_bricks(16, A.rowptr, A.colind, A.vals)
    assert f["panel_ptr"].tolist() == [0, 2]
    assert f["brick_cols"].tolist() == [10, 20, 30, 40, 50, PAD, PAD, PAD]
    assert [int(m) for m in f["brick_mask"]] == [0xF, 0x1]
    assert f["brick_valptr"].tolist() == [0, 4, 5]


@pytest.mark.parametrize("maker", [
    lambda: W.uniform_random(50, 37, 0.1, 1, empty_row_frac=0.2),
    lambda: W.uniform_random(16, 64, 0.5, 2),
    lambda: W.uniform_random(97, 5, 0.3, 3),
    lambda: W.uniform_random(33, 200, 0.02, 4),
    lambda: W.tiny_banded(M=300, seed=5),
    lambda: W.clustered_blocks(200, 3, 30, seed=6),
    lambda: W.brick_sweep(0.2, M=128, target_nnz=900, seed=7),
    lambda: W.power_law(M=400, target_nnz=None, cap=200, seed=8),
])
def test_matches_naive_builder_roundtrip_and_invariants(maker):
    A = maker()
    f = oracle.build_bricks(A.M, A.rowptr, A.colind, A.vals)
    assert_same_format(f, naive_builder(A))
    check_invariants(A, f)
    rp, ci, v = oracle.bricks_to_csr(A.M, f)
    assert np.array_equal(rp, A.rowptr) and np.array_equal(ci, A.colind)
    assert np.array_equal(v.view(np.uint32), A.vals.view(np.uint32))


def test_explicit_zeros_and_negative_zero_survive_round_trip():
    vals = np.array([0.0, -0.0, 1.0], np.float32)
    A = W.csr_from_coo(20, 9, [1, 1, 18], [2, 5, 5], vals)
    f = oracle.build_bricks(A.M, A.rowptr, A.colind, A.vals)
    rp, ci, v = oracle.bricks_to_csr(A.M, f)
    assert np.array_equal(v.view(np.uint32), A.vals.view(np.uint32))
    assert int(f["brick_valptr"][-1]) == 3


def test_empty_matrices():
    for M in (0, 1, 16, 40):
        A = W.csr_from_coo(M, 8, [], [])
        f = oracle.build_bricks(M, A.rowptr, A.colind, A.vals)
        assert f["panel_ptr"].tolist() == [0] * ((M + 15) // 16 + 1)
        assert len(f["brick_mask"]) == 0 and f["brick_valptr"].tolist() == [0]


@settings(max_examples=60, deadline=None)
@given(st.integers(1, 40), st.integers(1, 40), st.floats(0.01, 0.6), st.integers(0, 10**6))
def test_hypothesis_against_naive(M, K, density, seed):
    A = W.uniform_random(M, K, density, seed)
    f = oracle.build_bricks(A.M, A.rowptr, A.colind, A.vals)
    assert_same_format(f, naive_builder(A))
    rp, ci, v = oracle.bricks_to_csr(A.M, f)
    assert np.array_equal(rp, A.rowptr) and np.array_equal(ci, A.colind) and np.array_equal(v, A.vals)
