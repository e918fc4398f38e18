"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the
same seeded inputs.  Format, masks and synergy counts bit-exact; C within
1e-5 of sum|a.b| per element, and exactly zero where that sum is zero."""
import numpy as np
import pytest

import oracle
from paper_2504_06443_amd import workloads as W

pytestmark = pytest.mark.gpu

TOL = 1e-5
FMT_KEYS = ("panel_ptr", "brick_cols", "brick_mask", "brick_valptr", "vals")
INT_KEYS = ("M", "K", "nnz", "n_panels", "n_nonempty_panels", "n_bricks", "n_active_cols",
            "n_distinct_cols", "panels_by_class", "bricks_by_class", "nnz_by_class",
            "brick_pop_hist", "synergy_class")
FP_KEYS = ("alpha_brick", "alpha_col", "beta", "oi_shmem", "bytes_min", "bytes_noreuse",
           "oi_hbm_min", "oi_hbm_noreuse", "roof_gflops_hbm", "roof_gflops_mfma")


@pytest.fixture(scope="module")
def gpu():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2504_06443_amd import binding
    return binding


def to_dev(A):
    import torch
    return (torch.from_numpy(A.rowptr).cuda(), torch.from_numpy(A.colind).cuda(),
            torch.from_numpy(A.vals).cuda())


def make_plan(gpu, A):
    rp, ci, v = to_dev(A)
    return gpu.spmm_plan(A.M, A.K, rp, ci, v)


def assert_format_equal(got, ref):
    for k in FMT_KEYS:
        assert got[k].dtype == ref[k].dtype and got[k].shape == ref[k].shape, k
        assert np.array_equal(got[k].view(np.uint8), ref[k].view(np.uint8)), k


def check_c(Cg, Cref, S):
    Cg = Cg.astype(np.float64)
    zero = S == 0
    assert not Cg[zero].any(), "entries with no contributing product must be exactly 0"
    err = np.abs(Cg - Cref)
    worst = (err[~zero] / S[~zero]).max() if (~zero).any() else 0.0
    assert worst <= TOL, f"max |C-Cref| / sum|ab| = {worst:.3e}"
    return worst


def run_product(gpu, plan, A, B, route=None, split=None):
    import torch
    if route is not None:
        gpu.spmm_plan_set_route(plan, route)
    if split is not None:
        gpu.spmm_plan_set_split(plan, split)
    Bd = torch.from_numpy(B).cuda()
    Cd = torch.full((A.M, B.shape[1]), float("nan"), dtype=torch.float32, device="cuda")
    gpu.spmm_exec(plan, Bd, Cd)
    torch.cuda.synchronize()
    return Cd.cpu().numpy()


SMALL = {
    "uniform_ragged": lambda: W.uniform_random(203, 157, 0.05, 1, empty_row_frac=0.2),
    "dense_small": lambda: W.uniform_random(48, 40, 0.6, 2),
    "one_row": lambda: W.uniform_random(1, 300, 0.3, 3),
    "tall_skinny": lambda: W.uniform_random(1000, 5, 0.3, 4),
    "banded": lambda: W.tiny_banded(M=1500, seed=5),
    "blocks": lambda: W.clustered_blocks(2000, 5, 60, seed=6),
    "powerlaw": lambda: W.power_law(M=3000, target_nnz=None, cap=500, seed=7),
    "sweep_high": lambda: W.brick_sweep(0.8, M=1024, target_nnz=30000, seed=8),
    "sweep_low": lambda: W.brick_sweep(0.05, M=1024, target_nnz=30000, seed=9),
    "empty": lambda: W.csr_from_coo(50, 20, [], []),
    "single": lambda: W.csr_from_coo(40, 33, [37], [32], np.array([2.5], np.float32)),
}


@pytest.mark.parametrize("name", list(SMALL))
def test_format_and_counts_bit_exact(gpu, name):
    A = SMALL[name]()
    print(f"case {name}: M={A.M} K={A.K} nnz={A.nnz}", flush=True)
    plan = make_plan(gpu, A)
    ref = oracle.build_bricks(A.M, A.rowptr, A.colind, A.vals)
    assert_format_equal(gpu.spmm_plan_export(plan), ref)
    for N in (1, 128):
        got = gpu.spmm_synergy(plan, N)
        exp = oracle.synergy(A.M, A.K, N, A.rowptr, A.colind, ref)
        for k in INT_KEYS:
            assert got[k] == exp[k], (k, got[k], exp[k])
        for k in FP_KEYS:
            assert got[k] == pytest.approx(exp[k], rel=1e-12, abs=0), k


@pytest.mark.parametrize("name", list(SMALL))
@pytest.mark.parametrize("N", [1, 7, 16, 33, 64, 100, 128, 130, 260])
def test_product_all_routes(gpu, name, N):
    A = SMALL[name]()
    B = W.dense_b(A.K, N, 77)
    Cref, S = oracle.spmm_f64(A.rowptr, A.colind, A.vals, B)
    plan = make_plan(gpu, A)
    for route in (gpu.ROUTE_AUTO, gpu.ROUTE_CLASS, gpu.ROUTE_VALU):
        print(f"case {name} N={N} route={route}", flush=True)
        Cg = run_product(gpu, plan, A, B, route=route)
        assert not np.isnan(Cg).any(), "every element of C must be written"
        check_c(Cg, Cref, S)


@pytest.mark.parametrize("N", [16, 32, 64, 128, 200])
def test_integer_values_are_exact(gpu, N):
    """Small-integer A and B: every partial sum is exact in fp32, so the result
    must equal the fp64 oracle bit for bit -- isolates indexing from rounding."""
    A = W.uniform_random(333, 211, 0.08, 21, integer_values=True)
    B = np.random.default_rng(5).integers(-8, 9, size=(A.K, N)).astype(np.float32)
    Cref = oracle.spmm_f64(A.rowptr, A.colind, A.vals, B, want_abs=False)
    plan = make_plan(gpu, A)
    for route in (gpu.ROUTE_MFMA, gpu.ROUTE_VALU):
        for split in (1, 2, 3):
            Cg = run_product(gpu, plan, A, B, route=route, split=split)
            assert np.array_equal(Cg.astype(np.float64), Cref), (route, split)


@pytest.mark.parametrize("N", [4, 16, 32, 64, 100, 128, 256, 300, 512, 520, 1024, 6])
def test_csr_kernel_rows_side_by_side_and_long_rows(gpu, N):
    """The CSR path puts several rows into one wavefront (64 / lanes-per-row of them) and gives
    rows above 256 entries a workgroup of their own: rows of 0, 1, 255, 256, 257, 1000 and 2999
    entries next to ordinary ones, a ragged last panel, at widths on both sides of every
    lanes-per-row step; also under the class routing, where only Low-synergy panels go there."""
    rng = np.random.default_rng(4)
    M, K = 203, 3000
    lens = rng.integers(0, 40, size=M)
    lens[[3, 17, 18, 50, 64, 130, 202]] = [255, 256, 257, 1000, 2999, 1, 0]
    rows = np.repeat(np.arange(M), lens)
    cols = np.concatenate([rng.choice(K, size=l, replace=False) for l in lens])
    A = W.csr_from_coo(M, K, rows, cols, rng.uniform(-1, 1, size=rows.size).astype(np.float32))
    assert np.array_equal(np.diff(A.rowptr), lens)
    B = W.dense_b(K, N, 8)
    Cref, S = oracle.spmm_f64(A.rowptr, A.colind, A.vals, B)
    plan = make_plan(gpu, A)
    for route in (gpu.ROUTE_VALU, gpu.ROUTE_CLASS):
        print(f"csr rows case N={N} route={route}", flush=True)
        Cg = run_product(gpu, plan, A, B, route=route)
        assert not np.isnan(Cg).any(), "every element of C must be written"
        check_c(Cg, Cref, S)
    C1 = run_product(gpu, plan, A, B, route=gpu.ROUTE_VALU)
    C2 = run_product(gpu, plan, A, B, route=gpu.ROUTE_VALU)
    assert np.array_equal(C1, C2), "the long-row reduction must be reproducible"


def test_identity_and_permutation(gpu):
    n, N = 1000, 64
    B = W.dense_b(n, N, 3)
    eye = W.csr_from_coo(n, n, np.arange(n), np.arange(n), np.ones(n, np.float32))
    perm = np.random.default_rng(1).permutation(n)
    pm = W.csr_from_coo(n, n, np.arange(n), perm, np.ones(n, np.float32))
    for route in (gpu.ROUTE_MFMA, gpu.ROUTE_VALU):
        assert np.array_equal(run_product(gpu, make_plan(gpu, eye), eye, B, route=route), B)
        assert np.array_equal(run_product(gpu, make_plan(gpu, pm), pm, B, route=route), B[perm])


@pytest.mark.parametrize("split", [0, 2, 3, 5])
@pytest.mark.parametrize("N", [32, 128, 150])
def test_split_panels_merge(gpu, split, N):
    """Heavy panels split along K (Section 5): parts tile the panel, the merged
    result matches the oracle and is reproducible run to run."""
    A = W.power_law(M=2000, target_nnz=None, cap=1500, alpha=1.5, seed=31)
    B = W.dense_b(A.K, N, 32)
    Cref, S = oracle.spmm_f64(A.rowptr, A.colind, A.vals, B)
    plan = make_plan(gpu, A)
    C1 = run_product(gpu, plan, A, B, route=gpu.ROUTE_MFMA, split=split)
    check_c(C1, Cref, S)
    wl = gpu.spmm_plan_worklist(plan, N)
    fmt = gpu.spmm_plan_export(plan)
    if split > 1:
        assert wl["n_split_panels"] > 0
    seen = {}
    for panel, b0, b1, part, nparts in wl["items"]:
        seen.setdefault(panel, []).append((part, b0, b1, nparts))
    for panel, lst in seen.items():
        lst.sort()
        assert [x[0] for x in lst] == list(range(lst[0][3]))
        assert lst[0][1] == fmt["panel_ptr"][panel] and lst[-1][2] == fmt["panel_ptr"][panel + 1]
        for (_, _, e, _), (_, s, _, _) in zip(lst, lst[1:]):
            assert e == s
    C2 = run_product(gpu, plan, A, B)
    assert np.array_equal(C1, C2)


@pytest.mark.parametrize("policy", ["from2", "nearest"])
@pytest.mark.parametrize("M,N", [(4000, 128), (120000, 32), (120000, 512)])
def test_auto_split_matches_oracle_partition(gpu, policy, M, N):
    """The library's Eq. 6-7 split equals the oracle's, under both rounding policies, with
    num_waves = ceil(panels x column tiles / (CUs x resident wavefronts per CU)) formed here
    from the device's CU count as PyTorch reports it and the kernel occupancy the library
    states (one, two and several waves of work)."""
    import torch
    A = W.power_law(M=M, target_nnz=None, cap=2000, alpha=1.6, seed=41)
    plan = make_plan(gpu, A)
    gpu.spmm_plan_set_route(plan, gpu.ROUTE_MFMA)
    gpu.spmm_plan_set_split(plan, gpu.SPLIT_EQ7_FROM2 if policy == "from2" else gpu.SPLIT_EQ7_NEAREST)
    wl = gpu.spmm_plan_worklist(plan, N)
    fmt = gpu.spmm_plan_export(plan)
    nb_p = np.diff(fmt["panel_ptr"].astype(np.int64))
    panels = list(range(len(nb_p)))   # this route sends every panel, empty ones too, to the brick kernel
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    assert wl["num_cus"] == cus
    # 4 SIMDs per CU with at most 8 resident wavefronts each; the kernels run 4-wave workgroups
    assert wl["resident_waves_per_cu"] in range(4, 33, 4)
    items = len(panels) * -(-N // wl["n_tile"])
    want_waves = max(1, -(-items // (cus * wl["resident_waves_per_cu"])))
    assert wl["num_waves"] == want_waves
    parts, waves = oracle.partition_counts([int(nb_p[p]) for p in panels], items, cus,
                                           wl["resident_waves_per_cu"], policy=policy)
    assert waves == want_waves
    got = {}
    for panel, b0, b1, part, nparts in wl["items"]:
        got.setdefault(panel, []).append((int(b0), int(b1)))
    for p, want in zip(panels, parts):
        base = int(fmt["panel_ptr"][p])
        # the library's own floor on top of Eq. 6-7: a part keeps at least 4 blocks (16 bricks)
        want = min(want, max(1, -(-int(nb_p[p]) // 4) // 4))
        expect = [(base + lo, base + hi) for lo, hi in oracle.partition_ranges(int(nb_p[p]), want)]
        assert sorted(got[p]) == expect, p
    if M == 4000:
        assert wl["n_split_panels"] > 0
        B = W.dense_b(A.K, N, 42)
        Cref, S = oracle.spmm_f64(A.rowptr, A.colind, A.vals, B)
        check_c(run_product(gpu, plan, A, B), Cref, S)


def test_invalid_csr_is_rejected(gpu):
    import torch
    good = W.uniform_random(40, 30, 0.2, 1)
    cases = {}
    rp = good.rowptr.copy(); rp[5], rp[6] = rp[6], rp[5] + 0
    if rp[5] > rp[6]:
        cases["rowptr_not_monotone"] = (rp, good.colind, good.vals)
    rp2 = good.rowptr.copy(); rp2[0] = 1
    cases["rowptr_start"] = (rp2, good.colind, good.vals)
    ci = good.colind.copy(); ci[3] = 30
    cases["col_out_of_range"] = (good.rowptr, ci, good.vals)
    ci2 = good.colind.copy(); ci2[0] = -1
    cases["col_negative"] = (good.rowptr, ci2, good.vals)
    row = int(np.argmax(np.diff(good.rowptr) >= 2))
    s = good.rowptr[row]
    ci3 = good.colind.copy(); ci3[s], ci3[s + 1] = ci3[s + 1], ci3[s]
    cases["unsorted_row"] = (good.rowptr, ci3, good.vals)
    ci4 = good.colind.copy(); ci4[s + 1] = ci4[s]
    cases["duplicate"] = (good.rowptr, ci4, good.vals)
    for name, (rp_, ci_, v_) in cases.items():
        print("invalid case", name, flush=True)
        with pytest.raises(gpu.SpmmError) as e:
            gpu.spmm_plan(40, 30, torch.from_numpy(rp_).cuda(), torch.from_numpy(ci_).cuda(),
                          torch.from_numpy(v_).cuda())
        assert e.value.code == gpu.SPMM_EFORMAT, name
    # and a valid plan still works afterwards
    plan = make_plan(gpu, good)
    assert gpu.spmm_plan_sizes(plan)["nnz"] == good.nnz


def test_invalid_rows_on_the_bitmap_path_are_rejected(gpu):
    """Band-like matrices take the plan's per-panel bitmap path.  A panel whose only row is
    stored in descending order, or holds a column beyond K before a small one, has an inverted
    column span (last column of every row below the first column of some row): no bitmap is
    built for it, and it must still be rejected, not silently dropped."""
    import torch
    base = W.tiny_banded(M=640, seed=3)           # bitmap path: narrow spans, many entries

    def with_panel_replaced(panel, cols):
        keep = (np.repeat(np.arange(base.M), np.diff(base.rowptr)) // 16) != panel
        rows = np.repeat(np.arange(base.M), np.diff(base.rowptr))[keep]
        rp = np.zeros(base.M + 1, np.int64)
        np.add.at(rp, rows + 1, 1)
        rp[16 * panel + 1] += len(cols)
        rp = np.cumsum(rp).astype(np.int32)
        ci = np.concatenate([base.colind[keep][:rp[16 * panel]], np.asarray(cols, np.int32),
                             base.colind[keep][rp[16 * panel]:]]).astype(np.int32)
        return rp, ci, np.ones(len(ci), np.float32)

    cases = {
        "single_descending_row": with_panel_replaced(5, [7, 3]),
        "single_row_out_of_range_then_small": with_panel_replaced(9, [base.K + 5, 2]),
        "negative_then_valid": with_panel_replaced(0, [4, -1]),
        "last_panel_descending": with_panel_replaced(39, [600, 599, 598]),
    }
    # all 16 rows of a panel descending
    rp, ci, v = with_panel_replaced(7, [])
    rows16 = []
    for r in range(16):
        rows16.append([200 + r + 2, 200 + r])
    rp2 = rp.astype(np.int64).copy()
    add = np.zeros(base.M + 1, np.int64)
    for r in range(16):
        add[16 * 7 + r + 1:] += 2
    at = int(rp[16 * 7])
    cases["sixteen_descending_rows"] = ((rp2 + add).astype(np.int32),
                                        np.concatenate([ci[:at], np.asarray(rows16, np.int32).ravel(),
                                                        ci[at:]]).astype(np.int32),
                                        np.ones(len(ci) + 32, np.float32))
    for name, (rp_, ci_, v_) in cases.items():
        print("invalid bitmap-path case", name, flush=True)
        assert rp_[-1] == len(ci_) == len(v_)
        with pytest.raises(gpu.SpmmError) as e:
            gpu.spmm_plan(base.M, base.K, torch.from_numpy(rp_).cuda(), torch.from_numpy(ci_).cuda(),
                          torch.from_numpy(v_).cuda())
        assert e.value.code == gpu.SPMM_EFORMAT, name
    with pytest.raises(ValueError):     # the binding checks the array lengths before the call
        gpu.spmm_plan(base.M, base.K, torch.from_numpy(base.rowptr[:-1].copy()).cuda(),
                      torch.from_numpy(base.colind).cuda(), torch.from_numpy(base.vals).cuda())
    with pytest.raises(ValueError):
        gpu.spmm_plan(base.M, base.K, torch.from_numpy(base.rowptr).cuda(),
                      torch.from_numpy(base.colind).cuda(), torch.from_numpy(base.vals[:-1].copy()).cuda())
    plan = make_plan(gpu, base)          # the untouched matrix still plans
    assert gpu.spmm_plan_sizes(plan)["nnz"] == base.nnz


def test_degenerate_sizes(gpu):
    import torch
    # M = 0
    A = W.csr_from_coo(0, 10, [], [])
    plan = make_plan(gpu, A)
    Cd = gpu.spmm_exec(plan, torch.zeros((10, 8), device="cuda"))
    assert tuple(Cd.shape) == (0, 8)
    # N = 0
    A = W.uniform_random(20, 10, 0.3, 1)
    plan = make_plan(gpu, A)
    Cd = gpu.spmm_exec(plan, torch.zeros((10, 0), device="cuda"))
    assert tuple(Cd.shape) == (20, 0)
    # explicit zeros are kept and give exact zeros
    A = W.csr_from_coo(20, 9, [1, 1, 18], [2, 5, 5], np.array([0.0, -0.0, 1.0], np.float32))
    plan = make_plan(gpu, A)
    ref = oracle.build_bricks(A.M, A.rowptr, A.colind, A.vals)
    assert_format_equal(gpu.spmm_plan_export(plan), ref)
    B = W.dense_b(9, 16, 1)
    Cg = run_product(gpu, plan, A, B, route=gpu.ROUTE_MFMA)
    assert not Cg[1].any() and np.array_equal(Cg[18], B[5])


def test_config1_tiny_banded_full(gpu):
    A, Ns = W.config(1)
    plan = make_plan(gpu, A)
    ref = oracle.build_bricks(A.M, A.rowptr, A.colind, A.vals)
    assert_format_equal(gpu.spmm_plan_export(plan), ref)
    for N in Ns + [128]:
        B = W.dense_b(A.K, N, 1001)
        Cref, S = oracle.spmm_f64(A.rowptr, A.colind, A.vals, B)
        for route in (gpu.ROUTE_AUTO, gpu.ROUTE_CLASS, gpu.ROUTE_VALU):
            check_c(run_product(gpu, plan, A, B, route=route), Cref, S)


def test_exec_on_side_stream_and_graph_replay(gpu):
    """spmm_exec only enqueues work once an N's work list is cached: it can run on a
    non-default stream and be captured in a HIP graph; every replay must reproduce
    the eager result bit for bit (also for a matrix with split panels and both kernels)."""
    import torch
    # upper half: dense 3x3 blocks (Medium class -> MFMA kernel, split in two by force);
    # lower half: scattered power-law rows (Low class -> CSR kernel)
    top = W.clustered_blocks(1536, 6, 90, seed=50)
    low = W.power_law(M=1500, target_nnz=None, cap=300, seed=51)
    rows = np.concatenate([np.repeat(np.arange(top.M), np.diff(top.rowptr)),
                           top.M + np.repeat(np.arange(low.M), np.diff(low.rowptr))])
    cols = np.concatenate([top.colind, low.colind])
    A = W.csr_from_coo(top.M + low.M, max(top.K, low.K), rows, cols,
                       np.concatenate([top.vals, low.vals]))
    N = 128
    plan = make_plan(gpu, A)
    gpu.spmm_plan_set_route(plan, gpu.ROUTE_CLASS)
    gpu.spmm_plan_set_split(plan, 2)
    B1 = torch.from_numpy(W.dense_b(A.K, N, 1)).cuda()
    B2 = torch.from_numpy(W.dense_b(A.K, N, 2)).cuda()
    eager1 = gpu.spmm_exec(plan, B1).clone()          # also caches the work list for N
    eager2 = gpu.spmm_exec(plan, B2).clone()
    torch.cuda.synchronize()
    wl = gpu.spmm_plan_worklist(plan, N)
    assert wl["n_split_panels"] > 0 and wl["n_valu_panels"] > 0 and wl["n_mfma_items"] > 0

    side = torch.cuda.Stream()
    Bs = B1.clone()
    Cs = torch.empty_like(eager1)
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        gpu.spmm_exec(plan, Bs, Cs)                   # uses the current (side) stream
    side.synchronize()
    assert torch.equal(Cs, eager1)

    graph = torch.cuda.CUDAGraph()
    Cs.zero_()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        gpu.spmm_exec(plan, Bs, Cs)
    for k, (src, expect) in enumerate([(B1, eager1), (B2, eager2), (B1, eager1), (B2, eager2)]):
        Bs.copy_(src)
        Cs.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(Cs, expect), f"replay {k}"


def test_routes_send_the_expected_panels_to_the_csr_kernel(gpu):
    """AUTO keeps every panel on the brick kernel; CLASS is the paper's rule (Table 1: panels with
    fewer than 8 stored elements per brick on average go to the CSR kernel).  The expected panel
    sets come from the oracle's format; the product is checked on both routes."""
    top = W.clustered_blocks(1536, 6, 90, seed=50)                     # Medium panels
    low = W.power_law(M=1500, target_nnz=None, cap=300, seed=51)        # Low panels, some empty
    rows = np.concatenate([np.repeat(np.arange(top.M), np.diff(top.rowptr)),
                           top.M + np.repeat(np.arange(low.M), np.diff(low.rowptr))])
    A = W.csr_from_coo(top.M + low.M, max(top.K, low.K), rows,
                       np.concatenate([top.colind, low.colind]), np.concatenate([top.vals, low.vals]))
    ref = oracle.build_bricks(A.M, A.rowptr, A.colind, A.vals)
    P = len(ref["panel_ptr"]) - 1
    nb_p = np.diff(ref["panel_ptr"].astype(np.int64))
    nnz_p = np.diff(A.rowptr[np.minimum(np.arange(P + 1) * 16, A.M)].astype(np.int64))
    low_panels = np.nonzero((nb_p > 0) & (nnz_p < 8 * nb_p))[0]
    assert len(low_panels) > 10 and (nnz_p[nb_p > 0] >= 8 * nb_p[nb_p > 0]).sum() > 10
    plan = make_plan(gpu, A)
    gpu.spmm_plan_set_route(plan, gpu.ROUTE_AUTO)
    for N in (16, 32, 33, 64, 128, 512):
        assert gpu.spmm_plan_worklist(plan, N)["n_valu_panels"] == 0, N
    gpu.spmm_plan_set_route(plan, gpu.ROUTE_CLASS)
    for N in (16, 128):
        wl = gpu.spmm_plan_worklist(plan, N)
        got = set(wl["valu_panels"].tolist())
        assert set(low_panels.tolist()) <= got, N                      # every Low panel
        assert all(nb_p[p] == 0 or nnz_p[p] < 8 * nb_p[p] for p in got), N   # and only Low or empty ones
    for route in (gpu.ROUTE_AUTO, gpu.ROUTE_CLASS):
        for N in (32, 64):
            B = W.dense_b(A.K, N, 3)
            Cref, S = oracle.spmm_f64(A.rowptr, A.colind, A.vals, B)
            check_c(run_product(gpu, plan, A, B, route=route), Cref, S)


def test_gather_calibration_runs(gpu):
    """The measurement aid reads only inside the buffer it is given and leaves the sink alone."""
    import torch
    buf = torch.ones(1 << 20, dtype=torch.float32, device="cuda")      # 4 MiB = 8192 rows
    sink = torch.zeros(256, dtype=torch.float32, device="cuda")
    gpu.spmm_calibrate_gather(buf, 8192, 64, 1024, sink)
    torch.cuda.synchronize()
    assert not sink.any()
    with pytest.raises(ValueError):
        gpu.spmm_calibrate_gather(buf, 16384, 64, 1024, sink)             # buffer too small
    with pytest.raises(gpu.SpmmError):
        gpu.spmm_calibrate_gather(buf, 8192, 60, 1024, sink)              # loads not a multiple of 8


def test_error_paths_on_device(gpu):
    import ctypes
    import torch
    A = W.uniform_random(40, 30, 0.2, 1)
    plan = make_plan(gpu, A)
    B = torch.zeros((30, 8), device="cuda")
    C = torch.zeros((40, 8), device="cuda")
    lib = gpu._lib
    assert lib.spmm_exec(plan._h, ctypes.c_void_p(B.data_ptr()), -1, ctypes.c_void_p(C.data_ptr()), None) == gpu.SPMM_EINVAL
    assert lib.spmm_exec(plan._h, ctypes.c_void_p(B.data_ptr()), 8, None, None) == gpu.SPMM_EINVAL
    assert lib.spmm_exec(plan._h, None, 8, ctypes.c_void_p(C.data_ptr()), None) == gpu.SPMM_EINVAL
    assert "NULL" in gpu.spmm_last_error()
    assert lib.spmm_plan_set_route(plan._h, 7) == gpu.SPMM_EINVAL
    assert lib.spmm_plan_set_split(plan._h, -2) == gpu.SPMM_EINVAL
    assert lib.spmm_plan_set_split(plan._h, gpu.SPLIT_EQ7_NEAREST) == gpu.SPMM_OK
    assert lib.spmm_plan_set_split(plan._h, gpu.SPLIT_EQ7_FROM2) == gpu.SPMM_OK
    with pytest.raises(ValueError):
        gpu.spmm_exec(plan, torch.zeros((31, 8), device="cuda"))
    # nnz that disagrees with rowptr[M]
    rp, ci, v = to_dev(A)
    out = ctypes.c_void_p()
    st = lib.spmm_plan(A.M, A.K, A.nnz - 1, ctypes.c_void_p(rp.data_ptr()), ctypes.c_void_p(ci.data_ptr()),
                       ctypes.c_void_p(v.data_ptr()), None, ctypes.byref(out))
    assert st == gpu.SPMM_EFORMAT and not out.value
    # the plan is still usable
    gpu.spmm_exec(plan, B, C)
    torch.cuda.synchronize()


@pytest.mark.parametrize("name", ["uniform_ragged", "blocks", "powerlaw", "sweep_high", "empty",
                                  "single"])
def test_update_values_keeps_pattern_and_replaces_values(gpu, name):
    """Value-only update (Section 6, pre-processing overheads: one pattern, many products):
    afterwards the exported format equals the oracle's format of the new matrix bit for bit,
    and every route multiplies with the new values."""
    import torch
    A = SMALL[name]()
    plan = make_plan(gpu, A)
    rng = np.random.default_rng(123)
    new_vals = rng.uniform(-1, 1, A.nnz).astype(np.float32)
    if A.nnz > 3:
        new_vals[::3] = 0.0            # zeros stay stored entries
    gpu.spmm_plan_update_values(plan, torch.from_numpy(new_vals).cuda())
    torch.cuda.synchronize()
    ref = oracle.build_bricks(A.M, A.rowptr, A.colind, new_vals)
    assert_format_equal(gpu.spmm_plan_export(plan), ref)
    N = 48
    B = W.dense_b(A.K, N, 9)
    Cref, S = oracle.spmm_f64(A.rowptr, A.colind, new_vals, B)
    A2 = W.CSR(A.M, A.K, A.rowptr, A.colind, new_vals)
    for route in (gpu.ROUTE_AUTO, gpu.ROUTE_CLASS, gpu.ROUTE_VALU):
        check_c(run_product(gpu, plan, A2, B, route=route), Cref, S)
    with pytest.raises(ValueError):
        gpu.spmm_plan_update_values(plan, torch.zeros(A.nnz + 1, device="cuda"))


def test_plan_paths_for_wide_panels(gpu):
    """The plan has two per-panel paths (a bitmap of the panel's column span in LDS; a sort of
    the panel's entries in LDS) and a search-based one.  Cases: a span beyond the largest bitmap
    and a scattered matrix whose bitmaps would dwarf its entry lists (both sorted); one panel
    with a 700k-column span and many entries (bitmap, LDS allocation above the default limit);
    the same with more bricks than LDS holds beside that bitmap (starts on the bitmap path,
    finishes search-based); a span beyond the bitmap with more entries in one panel than the
    sort holds (search-based from the start).  All must give the oracle's format, counts and
    product."""
    rng = np.random.default_rng(77)

    def scattered(K, M, n):
        rows = rng.integers(0, M, n)
        cols = np.concatenate([rng.integers(0, 50, n // 3), rng.integers(K - 50, K, n // 3),
                               rng.integers(0, K, n - 2 * (n // 3))])
        return W.csr_from_coo(M, K, rows, cols, rng.uniform(-1, 1, n).astype(np.float32))

    def shared_columns(K, ncols):   # one panel, every row stores the same ncols columns
        cols = np.sort(rng.choice(K, size=ncols, replace=False))
        cols[0], cols[-1] = 0, K - 1
        rows = np.repeat(np.arange(16), ncols)
        return W.csr_from_coo(16, K, rows, np.tile(cols, 16),
                              rng.uniform(-1, 1, 16 * ncols).astype(np.float32))

    cases = {"beyond_bitmap": scattered(1_300_000, 70, 900),            # sorted per panel
             "scattered_cost_rule": scattered(700_000, 70, 900),       # sorted per panel
             "large_lds": shared_columns(700_000, 300),                # bitmap, large LDS
             "late_fallback": shared_columns(700_000, 2400),           # bitmap, then searches
             "search_path": shared_columns(1_300_000, 600),            # searches from the start
             "sort_wide_keys": scattered(3_000_000, 70, 900)}          # sorted, 64-bit keys
    for name, A in cases.items():
        print(f"wide panel case {name}: K={A.K} nnz={A.nnz}", flush=True)
        plan = make_plan(gpu, A)
        ref = oracle.build_bricks(A.M, A.rowptr, A.colind, A.vals)
        assert_format_equal(gpu.spmm_plan_export(plan), ref)
        got = gpu.spmm_synergy(plan, 8)
        exp = oracle.synergy(A.M, A.K, 8, A.rowptr, A.colind, ref)
        for k in INT_KEYS:
            assert got[k] == exp[k], (k, got[k], exp[k])
        B = W.dense_b(A.K, 4, 5)
        Cref, S = oracle.spmm_f64(A.rowptr, A.colind, A.vals, B)
        for route in (gpu.ROUTE_AUTO, gpu.ROUTE_VALU):
            check_c(run_product(gpu, plan, A, B, route=route), Cref, S)


@pytest.mark.parametrize("seed", range(24))
def test_random_shapes(gpu, seed):
    """Seeded random shapes, densities and widths (ragged last panel, empty rows, rows
    longer than a chunk, N off the vector width): format and counts bit-exact, product
    within tolerance on the brick kernel, the class-routed mix and the CSR kernel."""
    rng = np.random.default_rng(1000 + seed)
    M = int(rng.integers(1, 400))
    K = int(rng.integers(1, 3000))
    density = float(rng.choice([0.002, 0.02, 0.1, 0.5]))
    N = int(rng.choice([1, 3, 4, 8, 17, 32, 48, 64, 96, 128, 132, 256, 300]))
    A = W.uniform_random(M, K, density, 7000 + seed, empty_row_frac=float(rng.choice([0.0, 0.3])))
    print(f"random case seed={seed}: M={M} K={K} nnz={A.nnz} N={N}", flush=True)
    plan = make_plan(gpu, A)
    ref = oracle.build_bricks(A.M, A.rowptr, A.colind, A.vals)
    assert_format_equal(gpu.spmm_plan_export(plan), ref)
    got = gpu.spmm_synergy(plan, N)
    exp = oracle.synergy(A.M, A.K, N, A.rowptr, A.colind, ref)
    for k in INT_KEYS:
        assert got[k] == exp[k], (k, got[k], exp[k])
    B = W.dense_b(A.K, N, seed)
    Cref, S = oracle.spmm_f64(A.rowptr, A.colind, A.vals, B)
    for route, split in ((gpu.ROUTE_MFMA, 0), (gpu.ROUTE_MFMA, 2), (gpu.ROUTE_CLASS, 0),
                         (gpu.ROUTE_VALU, 0)):
        Cg = run_product(gpu, plan, A, B, route=route, split=split)
        assert not np.isnan(Cg).any()
        check_c(Cg, Cref, S)


def test_plans_release_their_memory(gpu):
    """Creating, using and destroying plans in a loop (all three plan paths, work lists with
    split panels) must not accumulate device memory."""
    import torch
    mats = [W.clustered_blocks(3000, 6, 90, seed=1), W.power_law(M=2000, target_nnz=None, cap=800, seed=2),
            W.brick_sweep(0.4, M=4096, target_nnz=120_000, seed=3)]
    def cycle():
        for A in mats:
            plan = make_plan(gpu, A)
            B = torch.zeros((A.K, 32), device="cuda")
            gpu.spmm_plan_set_split(plan, 2)
            gpu.spmm_exec(plan, B)
            gpu.spmm_plan_set_split(plan, 0)
            gpu.spmm_exec(plan, B)
            torch.cuda.synchronize()
            plan.destroy()
            del B
    cycle()
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    free0, _ = torch.cuda.mem_get_info()
    for _ in range(30):
        cycle()
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    free1, _ = torch.cuda.mem_get_info()
    assert free0 - free1 < 8 << 20, f"device memory shrank by {(free0 - free1) >> 20} MiB over 90 plans"


def test_heavy_first_order_gives_the_same_product(gpu):
    """The sorted schedule that Section 5 discusses and rejects: same product bit for bit
    (each work item computes the same tile; only the dispatch order changes), work items
    in descending size."""
    A = W.power_law(M=3000, target_nnz=None, cap=900, alpha=1.7, seed=61)
    B = W.dense_b(A.K, 96, 62)
    Cref, S = oracle.spmm_f64(A.rowptr, A.colind, A.vals, B)
    plan = make_plan(gpu, A)
    C_panel = run_product(gpu, plan, A, B, route=gpu.ROUTE_MFMA)
    gpu.spmm_plan_set_order(plan, gpu.ORDER_HEAVY_FIRST)
    C_heavy = run_product(gpu, plan, A, B, route=gpu.ROUTE_MFMA)
    check_c(C_heavy, Cref, S)
    assert np.array_equal(C_panel, C_heavy)
    sizes = [int(b1) - int(b0) for _, b0, b1, _, _ in gpu.spmm_plan_worklist(plan, 96)["items"]]
    assert sizes == sorted(sizes, reverse=True) and len(set(sizes)) > 3
    with pytest.raises(gpu.SpmmError):
        gpu.spmm_plan_set_order(plan, 5)
