"""spmm_exec_noalloc: the entry point for callers that cannot allocate device memory.

Its output must equal spmm_exec's bit for bit (same kernels, same work list, deterministic
merge) on two calls in a row, the second with a smaller input, while the free device memory
does not change; sizes beyond the static scratch are rejected with SPMM_ELIMIT."""
import ctypes

import numpy as np
import pytest

import oracle
from paper_2504_06443_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2504_06443_amd import binding
    return binding


def _plan(gpu, A):
    import torch
    return gpu.spmm_plan(A.M, A.K, torch.from_numpy(A.rowptr).cuda(),
                         torch.from_numpy(A.colind).cuda(), torch.from_numpy(A.vals).cuda())


def _raw_noalloc(gpu, plan, Bd, Cd):
    """Through the C ABI itself: raw pointers, current stream."""
    import torch
    st = gpu._lib.spmm_exec_noalloc(plan._h, ctypes.c_void_p(Bd.data_ptr()), Bd.shape[1],
                                    ctypes.c_void_p(Cd.data_ptr()),
                                    ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    return st


def test_noalloc_equals_exec_twice_second_smaller(gpu):
    import torch
    # first input: heavy panels split by Eq. 6-7 and by force, Low-class panels on the CSR
    # kernel, so the static scratch carries work items, merge items, CSR panels and partial tiles
    big = W.power_law(M=6000, target_nnz=None, cap=2500, alpha=1.5, seed=71)
    small = W.clustered_blocks(1500, 6, 90, seed=72)
    cases = [(big, 128, gpu.ROUTE_MFMA, 0), (small, 48, gpu.ROUTE_CLASS, 3)]
    plans, Bs, refs, outs = [], [], [], []
    for A, N, route, split in cases:
        plan = _plan(gpu, A)
        gpu.spmm_plan_set_route(plan, route)
        gpu.spmm_plan_set_split(plan, split)
        Bd = torch.from_numpy(W.dense_b(A.K, N, 5)).cuda()
        refs.append(gpu.spmm_exec(plan, Bd).clone())          # the existing entry point
        outs.append(torch.full((A.M, N), float("nan"), dtype=torch.float32, device="cuda"))
        plans.append(plan)
        Bs.append(Bd)
    wl = gpu.spmm_plan_worklist(plans[0], 128)
    assert wl["n_split_panels"] > 0, "the first case must use partial tiles"
    # two calls in a row, the second on the smaller input; then the first again (the scratch
    # now holds the other list and must be refilled), then a repeat (nothing is copied).
    # Every call gets its own output so that nothing but the entry point runs between the two
    # readings of the free device memory (PyTorch's own allocator may grow when it compares).
    order = (0, 1, 0, 0, 1)
    results = [torch.full_like(outs[k], float("nan")) for k in order]
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    for out, k in zip(results, order):
        print(f"noalloc call on case {k}: M={cases[k][0].M} N={cases[k][1]}", flush=True)
        assert _raw_noalloc(gpu, plans[k], Bs[k], out) == gpu.SPMM_OK, gpu.spmm_last_error()
        torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert free1 == free0, "spmm_exec_noalloc must not allocate device memory"
    for out, k in zip(results, order):
        assert torch.equal(out, refs[k]), f"case {k}: differs from spmm_exec"
        outs[k] = out
    # and against the oracle, to the same bar as every other product
    A, N = cases[1][0], cases[1][1]
    Cref, S = oracle.spmm_f64(A.rowptr, A.colind, A.vals, Bs[1].cpu().numpy())
    Cg = outs[1].cpu().numpy().astype(np.float64)
    assert not Cg[S == 0].any()
    assert (np.abs(Cg - Cref)[S > 0] / S[S > 0]).max() <= 1e-5


def test_noalloc_first_use_of_a_new_width_allocates_nothing(gpu):
    """No earlier spmm_exec for this N: the work list is built on the host and lives in the
    static scratch, so even the first call leaves the free device memory unchanged."""
    import torch
    A = W.power_law(M=3000, target_nnz=None, cap=1200, alpha=1.6, seed=73)
    plan = _plan(gpu, A)
    gpu.spmm_plan_set_route(plan, gpu.ROUTE_MFMA)
    gpu.spmm_plan_set_split(plan, 2)
    N = 96
    Bd = torch.from_numpy(W.dense_b(A.K, N, 6)).cuda()
    Cd = torch.full((A.M, N), float("nan"), dtype=torch.float32, device="cuda")
    ref = torch.empty_like(Cd)
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    assert _raw_noalloc(gpu, plan, Bd, Cd) == gpu.SPMM_OK, gpu.spmm_last_error()
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert free1 == free0
    gpu.spmm_exec(plan, Bd, ref)
    torch.cuda.synchronize()
    assert torch.equal(Cd, ref)


def test_noalloc_rejects_sizes_beyond_the_scratch(gpu):
    import torch
    # every panel split in two at N = 4096: 2 x 16 x 4096 x 4 B = 512 KiB of partial tiles per
    # panel, 125 panels -> 62 MiB, beyond the 32 MiB array
    A = W.uniform_random(2000, 600, 0.1, 74)
    plan = _plan(gpu, A)
    gpu.spmm_plan_set_route(plan, gpu.ROUTE_MFMA)
    gpu.spmm_plan_set_split(plan, 2)
    N = 4096
    Bd = torch.zeros((A.K, N), device="cuda")
    Cd = torch.full((A.M, N), 7.0, dtype=torch.float32, device="cuda")
    assert _raw_noalloc(gpu, plan, Bd, Cd) == gpu.SPMM_ELIMIT
    assert "scratch" in gpu.spmm_last_error()
    torch.cuda.synchronize()
    assert bool((Cd == 7.0).all()), "a rejected call must not touch C"
    # the allocating entry point still serves that size
    gpu.spmm_exec(plan, Bd, Cd)
    torch.cuda.synchronize()
    assert not bool(Cd.any())


def test_noalloc_follows_the_plan_options(gpu):
    """The opt-in modes (split-bf16 arithmetic, tile sharing for wide N, 32-row panels) go through
    the same launcher, so the allocation-free entry point must give what spmm_exec gives."""
    import torch
    A = W.paired_panels(3000, cols_per_group=120, half_width=400, seed=73)
    Bd = torch.from_numpy(W.dense_b(A.K, 256, 6)).cuda()
    plan = _plan(gpu, A)
    settings = [
        ("bf16x3", lambda: gpu.spmm_plan_set_precision(plan, gpu.PRECISIONS["bf16x3"])),
        ("fp32", lambda: gpu.spmm_plan_set_precision(plan, gpu.PRECISIONS["fp32"])),
        ("tile sharing", lambda: gpu.spmm_plan_set_tile_sharing(plan, gpu.SHARE_WORKGROUP)),
        ("32-row panels", lambda: gpu.spmm_plan_set_panel_height(plan, 32)),
    ]
    for name, apply in settings:
        apply()
        ref = gpu.spmm_exec(plan, Bd).clone()
        out = torch.full_like(ref, float("nan"))
        print(f"noalloc with {name}", flush=True)
        assert _raw_noalloc(gpu, plan, Bd, out) == gpu.SPMM_OK, gpu.spmm_last_error()
        torch.cuda.synchronize()
        assert torch.equal(out, ref), name
