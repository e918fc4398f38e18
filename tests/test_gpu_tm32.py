"""32-row panels on the GPU (Section 4, Eq. 5): the format built by the library from its 16-row
format equals the oracle's bit for bit, and the 32-row kernel's product meets the same bound as
the 16-row one."""
import numpy as np
import pytest

import oracle
from paper_2504_06443_amd import workloads as W
from test_gpu_parity import TOL, check_c, make_plan, run_product

pytestmark = pytest.mark.gpu

TM32_KEYS = ("sp_ptr", "sp_merged", "bc_cols", "bc_brick", "br_row", "br_mask", "br_valptr", "vals")

CASES = {
    "ragged": lambda: W.uniform_random(203, 157, 0.05, 1, empty_row_frac=0.2),
    "dense": lambda: W.uniform_random(70, 40, 0.6, 2),
    "one_row": lambda: W.uniform_random(1, 300, 0.3, 3),
    "seventeen_rows": lambda: W.uniform_random(17, 90, 0.2, 4),
    "blocks": lambda: W.clustered_blocks(2000, 5, 60, seed=6),
    "paired": lambda: W.paired_panels(3000, cols_per_group=60, half_width=200, seed=7),
    "paired_wide": lambda: W.paired_panels(1500, cols_per_group=240, half_width=600, row_fill=0.3, seed=9),
    "powerlaw": lambda: W.power_law(M=1500, target_nnz=None, cap=600, seed=8),
    "empty": lambda: W.csr_from_coo(50, 20, [], []),
    "single_bottom": lambda: W.csr_from_coo(40, 33, [37], [32], np.array([2.5], np.float32)),
}


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2504_06443_amd import binding
    return binding


def assert_tm32_equal(got, ref):
    for k in ("n_super_panels", "n_brick_cols", "n_bricks", "n_merged"):
        pass
    assert got["n_super_panels"] == ref["Q"] and got["n_brick_cols"] == ref["nbc"]
    assert got["n_bricks"] == ref["nbr"] and got["n_merged"] == ref["n_merged"]
    for k in TM32_KEYS:
        assert got[k].dtype == ref[k].dtype and got[k].shape == ref[k].shape, k
        assert np.array_equal(got[k].view(np.uint8), ref[k].view(np.uint8)), k


@pytest.mark.parametrize("name", list(CASES))
def test_format_bit_exact_and_product(gpu, name):
    A = CASES[name]()
    plan = make_plan(gpu, A)
    for num, den in ((6, 5), (2, 1), (0, 1)):
        print(f"tm32 case {name} threshold {num}/{den}: M={A.M} nnz={A.nnz}", flush=True)
        gpu.spmm_plan_set_panel_height(plan, 32, num, den)
        ref = oracle.build_tm32(A.M, A.rowptr, A.colind, A.vals, num=num, den=den)
        assert_tm32_equal(gpu.spmm_plan_tm32_export(plan), ref)
        for N in (128, 4, 32, 64, 96, 260):
            B = W.dense_b(A.K, N, 77)
            Cref, S = oracle.spmm_f64(A.rowptr, A.colind, A.vals, B)
            Cg = run_product(gpu, plan, A, B, route=gpu.ROUTE_MFMA)
            assert not np.isnan(Cg).any(), "every element of C must be written"
            check_c(Cg, Cref, S)
    # back to 16-row panels: the same product, from the other kernel
    gpu.spmm_plan_set_panel_height(plan, 16)
    B = W.dense_b(A.K, 64, 5)
    Cref, S = oracle.spmm_f64(A.rowptr, A.colind, A.vals, B)
    check_c(run_product(gpu, plan, A, B, route=gpu.ROUTE_MFMA), Cref, S)


def test_integer_values_are_exact_on_32_row_panels(gpu):
    A = W.paired_panels(700, cols_per_group=50, half_width=150, seed=3)
    A.vals = np.random.default_rng(1).integers(1, 8, size=A.nnz).astype(np.float32)
    plan = make_plan(gpu, A)
    gpu.spmm_plan_set_panel_height(plan, 32)
    assert gpu.spmm_plan_tm32_sizes(plan)["n_merged"] > 0
    for N in (16, 32, 64, 128, 200):
        B = np.random.default_rng(5).integers(-8, 9, size=(A.K, N)).astype(np.float32)
        Cref = oracle.spmm_f64(A.rowptr, A.colind, A.vals, B, want_abs=False)
        Cg = run_product(gpu, plan, A, B, route=gpu.ROUTE_MFMA)
        assert np.array_equal(Cg.astype(np.float64), Cref), N


def test_update_values_reaches_the_32_row_copy(gpu):
    import torch
    A = W.paired_panels(2000, cols_per_group=60, half_width=200, seed=11)
    plan = make_plan(gpu, A)
    gpu.spmm_plan_set_panel_height(plan, 32)
    new_vals = np.random.default_rng(2).uniform(-1, 1, A.nnz).astype(np.float32)
    gpu.spmm_plan_update_values(plan, torch.from_numpy(new_vals).cuda())
    torch.cuda.synchronize()
    ref = oracle.build_tm32(A.M, A.rowptr, A.colind, new_vals)
    assert_tm32_equal(gpu.spmm_plan_tm32_export(plan), ref)
    B = W.dense_b(A.K, 128, 3)
    Cref, S = oracle.spmm_f64(A.rowptr, A.colind, new_vals, B)
    check_c(run_product(gpu, plan, W.CSR(A.M, A.K, A.rowptr, A.colind, new_vals), B, route=gpu.ROUTE_MFMA), Cref, S)


def test_paired_workload_full_size(gpu):
    """The input on which the 32-row kernel is measured: both halves of every 32-row group share
    their active columns at Medium density.  Format bit-exact, every element of C."""
    import torch
    from test_gpu_fullsize import compare_all
    A = W.paired_panels(262144, cols_per_group=240, half_width=1024, row_fill=0.19, seed=1006)
    N = 128
    plan = make_plan(gpu, A)
    gpu.spmm_plan_set_panel_height(plan, 32)
    ref = oracle.build_tm32(A.M, A.rowptr, A.colind, A.vals)
    assert_tm32_equal(gpu.spmm_plan_tm32_export(plan), ref)
    assert ref["beta"] > 1.9 and ref["n_merged"] == ref["Q"]
    B = W.dense_b(A.K, N, 4242)
    Cref, S = oracle.spmm_f64(A.rowptr, A.colind, A.vals, B)
    Bd = torch.from_numpy(B).cuda()
    for rows in (32, 16):
        gpu.spmm_plan_set_panel_height(plan, rows)
        Cd = torch.full((A.M, N), float("nan"), dtype=torch.float32, device="cuda")
        gpu.spmm_exec(plan, Bd, Cd)
        torch.cuda.synchronize()
        worst = compare_all(Cd, Cref, S, f"paired {rows}-row panels")
        print(f"paired workload, {rows}-row panels: all elements within {worst:.2e}", flush=True)
    with pytest.raises(gpu.SpmmError):
        gpu.spmm_plan_set_panel_height(plan, 24)
