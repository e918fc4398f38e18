"""Pins for the oracle's synergy model (Section 4, Eq. 4; Section 6.4, Table 1)
and for the load-balance arithmetic (Section 5, Eq. 6-7)."""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2504_06443_amd import workloads as W


def read_rows(path):
    with open(path) as fh:
        return [ln.split() for ln in fh if ln.strip() and not ln.startswith("#")]


def synergy_of(A, N=128):
    f = oracle.build_bricks(A.M, A.rowptr, A.colind, A.vals)
    return oracle.synergy(A.M, A.K, N, A.rowptr, A.colind, f), f


def column_matrix(nrows_filled):
    """One panel, one active column with `nrows_filled` entries: alpha = n/64."""
    return W.csr_from_coo(16, 8, np.arange(nrows_filled), np.full(nrows_filled, 3),
                          np.ones(nrows_filled, np.float32))


def full_cols_matrix(ncols_full, extra):
    """One brick with `ncols_full` complete columns plus `extra` entries in the next."""
    rows = list(np.tile(np.arange(16), ncols_full)) + list(range(extra))
    cols = list(np.repeat(np.arange(ncols_full), 16)) + [ncols_full] * extra
    return W.csr_from_coo(16, 8, rows, cols, np.ones(len(rows), np.float32))


def test_table1_ranges(golden_dir):
    table = read_rows(os.path.join(golden_dir, "synergy_table1.txt"))
    names = [r[0] for r in table]
    assert names == list(oracle.SYNERGY_NAMES)
    # a single brick with n stored elements has alpha = n/64 for every n in 1..64
    for n in range(1, 65):
        full, extra = divmod(n, 16)
        A = column_matrix(n) if n <= 16 else full_cols_matrix(full, extra)
        s, f = synergy_of(A)
        if len(f["brick_mask"]) != 1:
            continue
        alpha = Fraction(n, 64)
        assert s["alpha_brick"] == float(alpha)
        expect = None
        for k, (name, lo, hi, hi_incl) in enumerate(table):
            lo, hi = Fraction(lo), Fraction(hi)
            if alpha >= lo and (alpha < hi or (int(hi_incl) and alpha == hi)):
                expect = k
        assert s["synergy_class"] == expect, (n, alpha)


def test_boundaries_are_inclusive_below():
    # alpha = 8/64 exactly -> Medium; 7/64 -> Low; 16/64 exactly -> High; 15/64 -> Medium
    assert synergy_of(column_matrix(8))[0]["synergy_class"] == 1
    assert synergy_of(column_matrix(7))[0]["synergy_class"] == 0
    assert synergy_of(column_matrix(16))[0]["synergy_class"] == 2
    assert synergy_of(column_matrix(15))[0]["synergy_class"] == 1


def test_oi_closed_form(golden_dir):
    for alpha, oi in read_rows(os.path.join(golden_dir, "oi_shmem.txt")):
        n = int(round(float(alpha) * 64))
        full, extra = divmod(n, 16)
        A = column_matrix(n) if n <= 16 else full_cols_matrix(full, extra)
        s, _ = synergy_of(A)
        assert s["alpha_brick"] == float(alpha)
        assert s["oi_shmem"] == float(oi)


def test_identity16_low_synergy_oi32():
    A = W.csr_from_coo(16, 16, np.arange(16), np.arange(16), np.ones(16, np.float32))
    s, _ = synergy_of(A)
    assert s["n_bricks"] == 4 and s["alpha_brick"] == 1 / 16 and s["oi_shmem"] == 32.0
    assert s["synergy_class"] == 0 and s["alpha_col"] == 1 / 16
    assert s["panels_by_class"] == [1, 0, 0] and s["bricks_by_class"] == [4, 0, 0]
    hist = [0] * 65
    hist[4] = 4
    assert s["brick_pop_hist"] == hist


def test_counts_against_independent_numpy():
    A = W.uniform_random(100, 60, 0.08, 5, empty_row_frac=0.3)
    s, f = synergy_of(A, N=32)
    P = 7
    assert (s["M"], s["K"], s["nnz"], s["n_panels"]) == (100, 60, A.nnz, P)
    assert s["n_distinct_cols"] == len(np.unique(A.colind))
    per_panel_cols = [len(np.unique(A.colind[A.rowptr[16 * p]:A.rowptr[min(100, 16 * p + 16)]]))
                      for p in range(P)]
    assert s["n_active_cols"] == sum(per_panel_cols)
    nb_p = [(c + 3) // 4 for c in per_panel_cols]
    assert s["n_bricks"] == sum(nb_p)
    assert s["n_nonempty_panels"] == sum(1 for b in nb_p if b)
    assert sum(s["panels_by_class"]) == s["n_nonempty_panels"]
    assert sum(s["bricks_by_class"]) == s["n_bricks"] and sum(s["nnz_by_class"]) == A.nnz
    assert sum(s["brick_pop_hist"]) == s["n_bricks"]
    assert sum(k * c for k, c in enumerate(s["brick_pop_hist"])) == A.nnz
    # bytes model, retyped from its statement: A = 4 nnz + 28 nb + 4 + 4 (P+1)
    a_bytes = 4 * A.nnz + 28 * s["n_bricks"] + 4 + 4 * (P + 1)
    assert s["bytes_min"] == a_bytes + 4 * 32 * s["n_distinct_cols"] + 4 * 32 * 100
    assert s["bytes_noreuse"] == a_bytes + 4 * 32 * s["n_active_cols"] + 4 * 32 * 100
    assert s["roof_gflops_hbm"] == pytest.approx(2 * A.nnz * 32 / s["bytes_min"] * 8e12 / 1e9, rel=1e-12)
    assert s["roof_gflops_mfma"] == pytest.approx(s["alpha_brick"] * 157.3e12 / 1e9, rel=1e-12)
    assert 1 / 16 <= s["alpha_col"] <= 1 and 1 / 64 <= s["alpha_brick"] <= 1
    assert s["alpha_col"] >= s["alpha_brick"]        # padding only lowers the brick figure


def test_bytes_model_hand_counted(golden_dir):
    """bytes_min / bytes_noreuse and both HBM operational intensities against integers counted
    by hand for a two-panel matrix (derivation in the golden file)."""
    g = dict((k, int(v)) for k, v in read_rows(os.path.join(golden_dir, "bytes_model_example.txt")))
    rows = [0, 3, 5, 16, 17, 18, 19, 20]
    cols = [1, 1, 6, 1, 2, 3, 4, 5]
    A = W.csr_from_coo(32, 8, rows, cols, np.ones(8, np.float32))
    s, _ = synergy_of(A, N=4)
    for k in ("nnz", "n_bricks", "n_active_cols", "n_distinct_cols"):
        assert s[k] == g[k], k
    assert s["bytes_min"] == g["bytes_min"] and s["bytes_noreuse"] == g["bytes_noreuse"]
    assert s["oi_hbm_min"] == pytest.approx(g["flops"] / g["bytes_min"], rel=1e-15)
    assert s["oi_hbm_noreuse"] == pytest.approx(g["flops"] / g["bytes_noreuse"], rel=1e-15)
    assert s["oi_hbm_noreuse"] < s["oi_hbm_min"]
    # a matrix whose panels share no column has nothing to reuse: both models coincide
    B = W.csr_from_coo(32, 8, [0, 1, 16, 17], [0, 1, 2, 3], np.ones(4, np.float32))
    t, _ = synergy_of(B, N=4)
    assert t["bytes_noreuse"] == t["bytes_min"] and t["oi_hbm_noreuse"] == t["oi_hbm_min"]


def test_per_panel_classes_mixed():
    # panel 0: dense 16x4 (High); panel 1: one entry (Low); panel 2: empty; panel 3: 8 in a column (Medium)
    rows = list(np.repeat(np.arange(16), 4)) + [20] + list(48 + np.arange(8))
    cols = list(np.tile(np.arange(4), 16)) + [1] + [2] * 8
    A = W.csr_from_coo(64, 4, rows, cols, np.ones(len(rows), np.float32))
    s, _ = synergy_of(A)
    assert s["panels_by_class"] == [1, 1, 1] and s["n_nonempty_panels"] == 3 and s["n_panels"] == 4
    assert s["nnz_by_class"] == [1, 8, 64]


def test_empty_matrix_has_no_class():
    A = W.csr_from_coo(32, 8, [], [])
    s, _ = synergy_of(A)
    assert s["synergy_class"] == -1 and s["alpha_brick"] == 0.0 and s["n_bricks"] == 0


# ------------------------------------------------------------------ Section 5
def test_paper_worked_example(golden_dir):
    g = dict((k, int(v)) for k, v in read_rows(os.path.join(golden_dir, "load_balance_example.txt")))
    # a block is four bricks: give panel 0 ten blocks' worth of bricks, the others one
    bricks = [4 * g["heavy_panel_blocks"]] + [4 * g["other_panel_blocks"]] * (g["panels"] - 1)
    parts, waves = oracle.partition_counts(bricks, g["panels"], g["sms"], g["resident_per_sm"])
    assert waves == g["waves"]
    assert parts[0] == g["parts_heavy"] and set(parts[1:]) == {g["parts_other"]}


def test_uniform_panels_never_split():
    for waves_cfg in ((10, 1), (1000, 8)):
        parts, _ = oracle.partition_counts([12] * 500, 500, *waves_cfg)
        assert set(parts) == {1}


def rounding_rows(golden_dir):
    out = []
    for name, blocks, ratio, nearest, from2, others in read_rows(
            os.path.join(golden_dir, "load_balance_rounding.txt")):
        out.append((name, [int(b) for b in blocks.split(",")], Fraction(ratio), int(nearest),
                    int(from2), int(others)))
    return out


def test_rounding_of_eq7_hand_worked(golden_dir):
    """Both readings of Eq. 7's rounding against examples worked by hand (one wave of work)."""
    rows = rounding_rows(golden_dir)
    assert len(rows) >= 8
    for name, blocks, ratio, nearest, from2, others in rows:
        bricks = [4 * b for b in blocks]
        P = len(blocks)
        assert Fraction(blocks[0] * P, sum(blocks)) == ratio, name      # the fixture's own arithmetic
        for policy, want in (("nearest", nearest), ("from2", from2)):
            parts, waves = oracle.partition_counts(bricks, P, 1000, 1, policy=policy)
            assert waves == 1
            assert parts[0] == want, (name, policy)
            assert set(parts[1:]) == {others}, (name, policy)


def test_more_waves_divide_the_ratio():
    """Eq. 7 divides the load by the number of waves: the panel of example a (ratio 32/3 in
    one wave) gets round(32/3 / 2) = 5 parts with two waves of work, 32/9 -> 4 with three,
    and 1 once the waves reach the ratio."""
    bricks = [4 * 30] + [4] * 15
    for items_per_capacity, want in ((1, 11), (2, 5), (3, 4), (8, 1), (11, 1)):
        for policy in ("nearest", "from2"):
            parts, waves = oracle.partition_counts(bricks, 16 * items_per_capacity, 16, 1, policy=policy)
            assert waves == items_per_capacity
            expect = want
            if policy == "from2" and Fraction(32, 3) / items_per_capacity < 2:
                expect = 1
            assert parts[0] == expect, (items_per_capacity, policy)


def test_split_follows_eq6_eq7_exact_fractions():
    bricks = [400, 8, 8, 8, 40, 0, 8, 8]
    P = len(bricks)
    for items, cus, res in ((8, 4, 1), (8, 2, 1), (64, 4, 2), (8, 256, 8)):
        for policy in ("from2", "nearest"):
            parts, waves = oracle.partition_counts(bricks, items, cus, res, policy=policy)
            blocks = [Fraction(-(-b // 4)) for b in bricks]
            avg = sum(blocks) / P
            w = max(1, -(-items // (cus * res)))
            assert waves == w
            for p in range(P):
                ratio = blocks[p] / avg / w                     # Eq. 6 then Eq. 7
                nearest = max(1, int((ratio + Fraction(1, 2)) // 1))   # nearest, halves up
                expect = 1 if (policy == "from2" and ratio < 2) else nearest
                assert parts[p] == expect


def test_ranges_tile_the_panel_once():
    for nb in (0, 1, 3, 4, 5, 17, 400, 965):
        for parts in (1, 2, 3, 7, 50):
            rs = oracle.partition_ranges(nb, parts)
            assert rs[0][0] == 0 and rs[-1][1] == nb
            for (a, b), (c, d) in zip(rs, rs[1:]):
                assert b == c and d > c
            assert all(lo % 4 == 0 for lo, _ in rs)         # cuts fall on block boundaries
