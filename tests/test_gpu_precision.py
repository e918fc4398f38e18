"""Opt-in split-bf16 arithmetic of the MFMA brick kernel (the counterpart of the paper's TF32
rounding of FP32 inputs, Section 2 "Background") against the fp64 oracle.

Bounds (per element, relative to sum|a.b|).  bf16 carries 8 significant bits, so rounding to
nearest leaves at most 2^-8 of a number and two terms leave at most 2^-16.  Three products of
two terms per input (a1 b1 + a1 b2 + a2 b1) drop a2 b2 and the two representation residuals,
each at most 2^-16 |a.b|: 3 x 2^-16 = 4.6e-5, tested as 5e-5.  Six products of three terms
drop terms of at most 2^-24 |a.b|: the 1e-5 of the FP32 path.  Small-integer data is exact in bf16, so there the result must be
the oracle's bit for bit, which separates operand-layout mistakes from rounding."""
import numpy as np
import pytest

import oracle
from paper_2504_06443_amd import workloads as W
from test_gpu_parity import SMALL, make_plan, run_product

pytestmark = pytest.mark.gpu

TOLERANCE = {"bf16x3": 5e-5, "bf16x6": 1e-5}


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2504_06443_amd import binding
    return binding


def worst_error(Cg, Cref, S):
    Cg = Cg.astype(np.float64)
    zero = S == 0
    assert not Cg[zero].any(), "entries with no contributing product must be exactly 0"
    return float((np.abs(Cg - Cref)[~zero] / S[~zero]).max()) if (~zero).any() else 0.0


@pytest.mark.parametrize("mode", ["bf16x3", "bf16x6"])
@pytest.mark.parametrize("N", [16, 32, 64, 128, 256, 4, 36, 200])
def test_integer_data_is_exact(gpu, mode, N):
    A = W.uniform_random(333, 211, 0.08, 21, integer_values=True)
    B = np.random.default_rng(5).integers(-8, 9, size=(A.K, N)).astype(np.float32)
    Cref = oracle.spmm_f64(A.rowptr, A.colind, A.vals, B, want_abs=False)
    plan = make_plan(gpu, A)
    gpu.spmm_plan_set_precision(plan, gpu.PRECISIONS[mode])
    for split in (1, 2, 3):
        print(f"exact case {mode} N={N} split={split}", flush=True)
        Cg = run_product(gpu, plan, A, B, route=gpu.ROUTE_MFMA, split=split)
        assert np.array_equal(Cg.astype(np.float64), Cref), (mode, N, split)


@pytest.mark.parametrize("mode", ["bf16x3", "bf16x6"])
@pytest.mark.parametrize("name", list(SMALL))
def test_small_shapes_within_bound(gpu, mode, name):
    A = SMALL[name]()
    plan = make_plan(gpu, A)
    gpu.spmm_plan_set_precision(plan, gpu.PRECISIONS[mode])
    for N in (1, 7, 16, 33, 64, 100, 128, 130, 260):
        B = W.dense_b(A.K, N, 77)
        Cref, S = oracle.spmm_f64(A.rowptr, A.colind, A.vals, B)
        for route in (gpu.ROUTE_AUTO, gpu.ROUTE_CLASS):
            print(f"case {name} {mode} N={N} route={route}", flush=True)
            Cg = run_product(gpu, plan, A, B, route=route)
            assert not np.isnan(Cg).any()
            assert worst_error(Cg, Cref, S) <= TOLERANCE[mode], (name, N, route)


@pytest.mark.parametrize("mode", ["bf16x3", "bf16x6"])
def test_wide_dynamic_range(gpu, mode):
    """Values spread over 2^-40 .. 2^40: bf16 keeps FP32's exponent range, so the split needs
    no scaling; the bound is relative to sum|a.b| all the same."""
    A = W.clustered_blocks(3000, 6, 90, seed=9)
    rng = np.random.default_rng(3)
    A.vals = (A.vals * np.exp2(rng.integers(-40, 41, size=A.nnz))).astype(np.float32)
    B = (W.dense_b(A.K, 128, 4) * np.exp2(rng.integers(-40, 41, size=(A.K, 1)))).astype(np.float32)
    Cref, S = oracle.spmm_f64(A.rowptr, A.colind, A.vals, B)
    plan = make_plan(gpu, A)
    gpu.spmm_plan_set_precision(plan, gpu.PRECISIONS[mode])
    Cg = run_product(gpu, plan, A, B)
    assert np.isfinite(Cg).all()
    assert worst_error(Cg, Cref, S) <= TOLERANCE[mode]


def test_modes_differ_from_fp32_only_within_their_bounds(gpu):
    """All three arithmetic modes on one Medium-synergy input: each within its own bound, the
    six-product mode about as close to the oracle as FP32."""
    import torch
    A = W.clustered_blocks(20000, 10, 256, seed=12)
    N = 128
    B = W.dense_b(A.K, N, 13)
    Cref, S = oracle.spmm_f64(A.rowptr, A.colind, A.vals, B)
    plan = make_plan(gpu, A)
    errs = {}
    for mode in ("fp32", "bf16x3", "bf16x6"):
        gpu.spmm_plan_set_precision(plan, gpu.PRECISIONS[mode])
        errs[mode] = worst_error(run_product(gpu, plan, A, B), Cref, S)
    print("max error / sum|a.b| per mode:", errs, flush=True)
    assert errs["fp32"] <= 1e-5 and errs["bf16x3"] <= 5e-5 and errs["bf16x6"] <= 1e-5
    assert errs["bf16x6"] <= 4 * max(errs["fp32"], 1e-7)
    with pytest.raises(gpu.SpmmError):
        gpu.spmm_plan_set_precision(plan, 7)
