"""GPU parity at the benchmark's full sizes, in the launch configuration
bench.py times (automatic routing and splitting).  The format and the synergy
counts are compared bit for bit with the CPU oracle, and every element of C is
compared with the oracle's fp64 product: |C - C_ref| <= 1e-5 * sum|a.b|, exactly
zero where that sum is zero.  Only the cases whose B exceeds 4 GiB fall back to
sampled rows."""
import numpy as np
import pytest

import oracle
from paper_2504_06443_amd import workloads as W
from test_gpu_parity import (FMT_KEYS, INT_KEYS, TOL, assert_format_equal, make_plan)

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(1200)]

ROUTES = {"auto": 0, "mfma": 1, "valu": 2, "class": 3}


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2504_06443_amd import binding
    return binding


def compare_all(Cd, Cref, S, tag):
    """Every element of the device result against the oracle, in row chunks.  Returns the
    largest |C - C_ref| / sum|a.b|."""
    M = Cref.shape[0]
    worst = 0.0
    step = 1 << 16
    for r0 in range(0, M, step):
        r1 = min(M, r0 + step)
        Cg = Cd[r0:r1].cpu().numpy().astype(np.float64)
        assert np.isfinite(Cg).all(), f"{tag}: every element of C must be written (rows {r0}..{r1})"
        s = S[r0:r1]
        zero = s == 0
        assert not Cg[zero].any(), f"{tag}: rows {r0}..{r1}: non-zero where no product contributes"
        err = np.abs(Cg - Cref[r0:r1])
        np.divide(err, s, out=err, where=~zero)
        err[zero] = 0.0
        w = float(err.max()) if err.size else 0.0
        if w > TOL:
            i, j = np.unravel_index(int(err.argmax()), err.shape)
            raise AssertionError(f"{tag}: C[{r0 + i},{j}] off by {w:.3e} x sum|a.b|")
        worst = max(worst, w)
    return worst


def check_full(gpu, A, N, tag, check_format=True, routes=("auto",), plan=None):
    import torch
    print(f"{tag}: M={A.M} nnz={A.nnz} N={N}", flush=True)
    if plan is None:
        plan = make_plan(gpu, A)
    if check_format:
        ref = oracle.build_bricks(A.M, A.rowptr, A.colind, A.vals)
        assert_format_equal(gpu.spmm_plan_export(plan), ref)
        got, exp = gpu.spmm_synergy(plan, N), oracle.synergy(A.M, A.K, N, A.rowptr, A.colind, ref)
        for k in INT_KEYS:
            assert got[k] == exp[k], k
        print(f"{tag}: format and counts bit-exact, alpha={got['alpha_brick']:.3f}", flush=True)
    B = W.dense_b(A.K, N, 4242)
    Bd = torch.from_numpy(B).cuda()
    Cref, S = oracle.spmm_f64(A.rowptr, A.colind, A.vals, B)
    for route in routes:
        gpu.spmm_plan_set_route(plan, ROUTES[route])
        Cd = torch.full((A.M, N), float("nan"), dtype=torch.float32, device="cuda")
        gpu.spmm_exec(plan, Bd, Cd)
        torch.cuda.synchronize()
        worst = compare_all(Cd, Cref, S, f"{tag} N={N} {route}")
        print(f"{tag} N={N} {route}: all {A.M}x{N} elements within {worst:.2e} x sum|a.b|", flush=True)
        del Cd
    return plan


def test_config2_clustered(gpu):
    A, Ns = W.config(2)
    check_full(gpu, A, Ns[0], "config2", routes=("auto", "valu"))


def test_config3_powerlaw(gpu):
    A, Ns = W.config(3)
    plan = check_full(gpu, A, Ns[0], "config3", routes=("auto", "class"))
    # the literal rounding of Eq. 7 splits more panels; same product
    gpu.spmm_plan_set_split(plan, gpu.SPLIT_EQ7_NEAREST)
    check_full(gpu, A, Ns[0], "config3 nearest-split", check_format=False, routes=("auto",), plan=plan)


@pytest.mark.parametrize("fill", [0.05, 0.1, 0.2, 0.4, 0.8])
def test_config5_sweep(gpu, fill):
    """The whole grid of the synergy sweep: five fills x six widths on the brick kernel,
    three of the widths on the CSR kernel as well."""
    A, Ns = W.config(5, fill=fill)
    plan = None
    for N in Ns:
        routes = ("mfma", "valu") if N in (16, 128, 512) else ("mfma",)
        plan = check_full(gpu, A, N, f"config5 f={fill}", check_format=(N == Ns[0]), routes=routes,
                          plan=plan)


def test_scattered_sweep_takes_the_sort_path(gpu):
    """Random 16x4 cells over 262144 columns, 244 entries per panel: too scattered for the
    plan's bitmap path, well filled enough for its per-panel sort.  Format bit-exact."""
    A = W.brick_sweep(0.4, M=1 << 18, target_nnz=4_000_000, seed=77)
    check_full(gpu, A, 64, "scattered sweep", check_format=True, routes=("mfma",))


@pytest.mark.parametrize("fill", [0.8, 0.4])
def test_million_row_sweep(gpu, fill):
    """The scaled-up sweep (M = K = 2^20, 32 M entries, B and C of 512 MB each: beyond the
    256 MB Infinity Cache) on which the HBM-roofline figure is quoted: format bit-exact and
    every element of C, in the configuration bench.py times."""
    A = W.brick_sweep(fill, M=1 << 20, target_nnz=32_000_000, seed=1005)
    check_full(gpu, A, 128, f"sweepxl f={fill}", check_format=True, routes=("auto",))


def test_config4_fem(gpu):
    A, Ns = W.config(4)
    plan = None
    for N in Ns:
        plan = check_full(gpu, A, N, "config4", check_format=(N == Ns[0]), plan=plan)


@pytest.mark.parametrize("K,N", [(1 << 21, 520), ((1 << 20) - 1, 1024)],
                         ids=["above_4gib", "just_below_4gib"])
def test_b_around_4gib(gpu, K, N):
    """B of 4.4 GB: byte offsets into B no longer fit 32 bits, which must switch the
    library to its 64-bit addressing kernel.  B of 4 GiB minus one row: the 32-bit
    offsets of the fast kernel come within 4 KB of wrapping.  Rows at both ends of B
    are referenced."""
    import torch
    M = 4096
    rng = np.random.default_rng(7)
    per_row = 24
    rows = np.repeat(np.arange(M), per_row)
    cols = np.concatenate([rng.integers(0, K, size=M * per_row - 64),
                           np.arange(K - 32, K), np.arange(0, 32)])
    A = W.csr_from_coo(M, K, rows, cols, rng.uniform(-1, 1, size=rows.size).astype(np.float32))
    assert (4 * K * N >= 1 << 32) == (N == 520)
    gen = torch.Generator(device="cuda").manual_seed(11)
    Bd = torch.randn((K, N), generator=gen, device="cuda", dtype=torch.float32)
    plan = make_plan(gpu, A)
    for route in (gpu.ROUTE_AUTO, gpu.ROUTE_VALU):
        gpu.spmm_plan_set_route(plan, route)
        Cd = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
        gpu.spmm_exec(plan, Bd, Cd)
        torch.cuda.synchronize()
        assert not torch.isnan(Cd).any().item()
        sample = np.unique(np.concatenate([rng.integers(0, M, 64), [0, M - 1]]))
        # the oracle only needs the B rows these sampled rows touch: remap columns to a small B
        ent = np.concatenate([np.arange(A.rowptr[i], A.rowptr[i + 1]) for i in sample])
        used, inv = np.unique(A.colind[ent], return_inverse=True)
        Bsmall = Bd[torch.from_numpy(used.astype(np.int64)).cuda()].cpu().numpy()
        rp = np.zeros(len(sample) + 1, np.int32)
        rp[1:] = np.cumsum([A.rowptr[i + 1] - A.rowptr[i] for i in sample])
        Cref, S = oracle.spmm_f64(rp, inv.astype(np.int32), A.vals[ent], Bsmall)
        Cg = Cd[torch.from_numpy(sample).cuda()].cpu().numpy().astype(np.float64)
        assert (np.abs(Cg - Cref) / S).max() <= TOL, route
