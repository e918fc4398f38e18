"""Large N with the decoded bricks of a panel shared by the wavefronts of one workgroup
(Section 3.3): the product equals the oracle's to the FP32 bound and is bit-identical to the
one-wavefront-per-tile kernel's, on widths that take the 4-wavefront variant, the 2-wavefront
variant, a masked tail tile, and widths the variant does not serve."""
import numpy as np
import pytest

import oracle
from paper_2504_06443_amd import workloads as W
from test_gpu_parity import SMALL, check_c, make_plan, run_product

pytestmark = pytest.mark.gpu

# 512, 1024: four wavefronts; 256, 768: two; 500: four with a masked tail; 260: three tiles and
# 384: three tiles (not served: must fall back to the ordinary kernel); 128: below the threshold
WIDTHS = (512, 256, 768, 1024, 500, 260, 384, 128)


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2504_06443_amd import binding
    return binding


@pytest.mark.parametrize("name", list(SMALL))
def test_shared_decode_matches_oracle_and_plain_kernel(gpu, name):
    A = SMALL[name]()
    plan = make_plan(gpu, A)
    for N in WIDTHS:
        print(f"wide case {name}: M={A.M} K={A.K} nnz={A.nnz} N={N}", flush=True)
        B = W.dense_b(A.K, N, 31)
        Cref, S = oracle.spmm_f64(A.rowptr, A.colind, A.vals, B)
        gpu.spmm_plan_set_tile_sharing(plan, gpu.SHARE_NONE)
        C_plain = run_product(gpu, plan, A, B, route=gpu.ROUTE_MFMA)
        gpu.spmm_plan_set_tile_sharing(plan, gpu.SHARE_WORKGROUP)
        C_wide = run_product(gpu, plan, A, B, route=gpu.ROUTE_MFMA)
        assert not np.isnan(C_wide).any(), "every element of C must be written"
        check_c(C_wide, Cref, S)
        assert np.array_equal(C_wide.view(np.uint32), C_plain.view(np.uint32)), N


@pytest.mark.parametrize("split", [0, 3])
def test_shared_decode_with_split_panels(gpu, split):
    """Heavy panels split along K (Eq. 6-7, or forced) write partial tiles that the merge sums."""
    A = W.power_law(M=6000, target_nnz=None, cap=2000, seed=12)
    plan = make_plan(gpu, A)
    gpu.spmm_plan_set_tile_sharing(plan, gpu.SHARE_WORKGROUP)
    for N in (512, 256):
        print(f"wide split case: split={split} N={N} nnz={A.nnz}", flush=True)
        B = W.dense_b(A.K, N, 32)
        Cref, S = oracle.spmm_f64(A.rowptr, A.colind, A.vals, B)
        Cg = run_product(gpu, plan, A, B, route=gpu.ROUTE_MFMA, split=split)
        assert not np.isnan(Cg).any()
        check_c(Cg, Cref, S)
        if split == 3:
            assert gpu.spmm_plan_worklist(plan, N)["n_split_panels"] > 0


def test_shared_decode_exact_on_integers(gpu):
    A = W.clustered_blocks(3000, 6, 80, seed=14)
    A.vals = np.random.default_rng(2).integers(1, 8, size=A.nnz).astype(np.float32)
    plan = make_plan(gpu, A)
    gpu.spmm_plan_set_tile_sharing(plan, gpu.SHARE_WORKGROUP)
    for N in (256, 512):
        B = np.random.default_rng(6).integers(-8, 9, size=(A.K, N)).astype(np.float32)
        Cref = oracle.spmm_f64(A.rowptr, A.colind, A.vals, B, want_abs=False)
        Cg = run_product(gpu, plan, A, B, route=gpu.ROUTE_MFMA)
        assert np.array_equal(Cg.astype(np.float64), Cref), N


def test_unknown_mode_is_rejected(gpu):
    A = SMALL["single"]()
    plan = make_plan(gpu, A)
    with pytest.raises(gpu.SpmmError):
        gpu.spmm_plan_set_tile_sharing(plan, 7)
