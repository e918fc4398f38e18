"""GPU parity at the benchmark's full sizes, in the launch configuration
bench.py times (automatic routing and splitting).  The format and the synergy
counts are compared bit for bit with the CPU oracle; C is compared on sampled
rows the oracle computes one by one, and on a whole-matrix property
(C x = A (B x) for a random x, evaluated by the oracle in fp64)."""
import numpy as np
import pytest

import oracle
from paper_2504_06443_amd import workloads as W
from test_gpu_parity import (FMT_KEYS, INT_KEYS, TOL, assert_format_equal, make_plan)

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2504_06443_amd import binding
    return binding


def check_full(gpu, A, N, tag, check_format=True, routes=("auto",)):
    import torch
    print(f"{tag}: M={A.M} nnz={A.nnz} N={N}", flush=True)
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
    rng = np.random.default_rng(99)
    rows = np.unique(np.concatenate([rng.integers(0, A.M, 3000), np.arange(0, 48),
                                     np.arange(A.M - 48, A.M),
                                     np.argsort(np.diff(A.rowptr))[-32:]]))   # heaviest rows too
    Cref, S = oracle.spmm_rows_f64(rows, A.rowptr, A.colind, A.vals, B)
    x = rng.standard_normal(N)
    y_ref, y_abs = oracle.spmm_f64(A.rowptr, A.colind, A.vals,
                                   (B.astype(np.float64) @ x).astype(np.float32)[:, None])
    for route in routes:
        gpu.spmm_plan_set_route(plan, {"auto": 0, "mfma": 1, "valu": 2, "class": 3}[route])
        Cd = torch.full((A.M, N), float("nan"), dtype=torch.float32, device="cuda")
        gpu.spmm_exec(plan, Bd, Cd)
        torch.cuda.synchronize()
        assert not torch.isnan(Cd).any().item(), "every element of C must be written"
        Cg = Cd[torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
        zero = S == 0
        assert not Cg[zero].any()
        worst = (np.abs(Cg - Cref)[~zero] / S[~zero]).max()
        assert worst <= TOL, f"{tag} {route}: sampled rows error {worst:.3e}"
        # whole-matrix property; B x was rounded to fp32 for the oracle, so allow that much
        y = (Cd.double() @ torch.from_numpy(x).cuda()).cpu().numpy()
        scale = Cd.abs().double().matmul(torch.from_numpy(np.abs(x)).cuda()).cpu().numpy() + 1e-30
        assert (np.abs(y - y_ref[:, 0]) / scale).max() < 1e-4, f"{tag} {route}: C x != A (B x)"
        print(f"{tag} {route}: max sampled error {worst:.2e}", flush=True)


def test_config2_clustered(gpu):
    A, Ns = W.config(2)
    check_full(gpu, A, Ns[0], "config2", routes=("auto", "valu"))


def test_config3_powerlaw(gpu):
    A, Ns = W.config(3)
    check_full(gpu, A, Ns[0], "config3", routes=("auto", "class"))


@pytest.mark.parametrize("fill", [0.05, 0.2, 0.8])
def test_config5_sweep(gpu, fill):
    A, Ns = W.config(5, fill=fill)
    for N in (16, 128, 512):
        check_full(gpu, A, N, f"config5 f={fill}", check_format=(N == 16), routes=("mfma", "valu"))


def test_scattered_sweep_takes_the_sort_path(gpu):
    """Random 16x4 cells over 262144 columns, 244 entries per panel: too scattered for the
    plan's bitmap path, well filled enough for its per-panel sort.  Format bit-exact."""
    A = W.brick_sweep(0.4, M=1 << 18, target_nnz=4_000_000, seed=77)
    check_full(gpu, A, 64, "scattered sweep", check_format=True, routes=("mfma",))


def test_config4_fem(gpu):
    A, Ns = W.config(4)
    for N in Ns:
        check_full(gpu, A, N, "config4", check_format=(N == Ns[0]))


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
