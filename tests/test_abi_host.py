"""CPU-only checks of the C-ABI library: it loads without a GPU, exports every
symbol the header declares, and its host-side arithmetic (Eq. 6-7 of Section 5)
agrees with the oracle's and with the paper's worked example."""
import os
import re

import numpy as np
import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def binding():
    from paper_2504_06443_amd import binding as b
    return b


def declared_functions():
    text = open(os.path.join(ROOT, "include", "spmm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(spmm_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(binding):
    names = declared_functions()
    assert "spmm_plan" in names and "spmm_exec" in names and "spmm_synergy" in names
    for n in names:
        assert hasattr(binding._lib, n), n
    assert sorted(binding.EXPORTED) == names


def test_struct_layout_matches_header(binding):
    import ctypes
    # 8 + 3*3 + 65 int64, 2 int32, 10 doubles
    assert ctypes.sizeof(binding._Synergy) == 8 * (8 + 9 + 65) + 8 + 8 * 10
    assert ctypes.sizeof(binding._WorkItem) == 20
    assert ctypes.sizeof(binding._WorklistInfo) == 48


def test_partition_paper_example(binding, golden_dir):
    g = {}
    for ln in open(os.path.join(golden_dir, "load_balance_example.txt")):
        if ln.strip() and not ln.startswith("#"):
            k, v = ln.split()
            g[k] = int(v)
    bricks = [4 * g["heavy_panel_blocks"]] + [4 * g["other_panel_blocks"]] * (g["panels"] - 1)
    parts, waves = binding.spmm_partition_counts(bricks, g["panels"], g["sms"], g["resident_per_sm"])
    assert waves == g["waves"]
    assert parts[0] == g["parts_heavy"] and set(parts[1:].tolist()) == {g["parts_other"]}


def test_partition_rounding_examples(binding, golden_dir):
    """The hand-worked rounding examples of Eq. 7 through the C ABI, both policies."""
    n = 0
    for ln in open(os.path.join(golden_dir, "load_balance_rounding.txt")):
        if not ln.strip() or ln.startswith("#"):
            continue
        name, blocks, _, nearest, from2, others = ln.split()
        bricks = [4 * int(b) for b in blocks.split(",")]
        for policy, want in ((binding.SPLIT_EQ7_NEAREST, int(nearest)), (binding.SPLIT_EQ7_FROM2, int(from2))):
            parts, waves = binding.spmm_partition_counts(bricks, len(bricks), 1000, 1, policy)
            assert waves == 1 and parts[0] == want, (name, policy)
            assert set(parts[1:].tolist()) == {int(others)}, (name, policy)
        n += 1
    assert n >= 8


@pytest.mark.parametrize("seed", range(5))
def test_partition_matches_oracle(binding, seed):
    rng = np.random.default_rng(seed)
    P = int(rng.integers(1, 400))
    bricks = rng.zipf(1.6, size=P).clip(max=5000).astype(np.uint32)
    bricks[rng.random(P) < 0.1] = 0
    for items, cus, res in ((P, 256, 8), (P, 4, 1), (3 * P, 16, 2)):
        for policy, name in ((binding.SPLIT_EQ7_FROM2, "from2"), (binding.SPLIT_EQ7_NEAREST, "nearest")):
            parts, waves = binding.spmm_partition_counts(bricks, items, cus, res, policy)
            eparts, ewaves = oracle.partition_counts(bricks.tolist(), items, cus, res, policy=name)
            assert waves == ewaves and parts.tolist() == eparts


def test_partition_rejects_bad_arguments(binding):
    with pytest.raises(binding.SpmmError) as e:
        binding.spmm_partition_counts([1, 2], 2, 0, 1)
    assert e.value.code == binding.SPMM_EINVAL
    assert "bad argument" in binding.spmm_last_error()
    with pytest.raises(binding.SpmmError):
        binding.spmm_partition_counts([1, 2], 2, 1, 1, policy=5)


def test_null_plan_is_an_error_not_a_crash(binding):
    import ctypes
    assert binding._lib.spmm_exec(None, None, 4, None, None) == binding.SPMM_EINVAL
    assert binding._lib.spmm_exec_noalloc(None, None, 4, None, None) == binding.SPMM_EINVAL
    assert binding._lib.spmm_synergy(None, 4, None) == binding.SPMM_EINVAL
    assert binding._lib.spmm_plan_sizes(None, None) == binding.SPMM_EINVAL
    assert binding._lib.spmm_plan_update_values(None, None, None) == binding.SPMM_EINVAL
    assert binding._lib.spmm_plan_set_order(None, 0) == binding.SPMM_EINVAL
    assert binding._lib.spmm_plan_set_precision(None, 0) == binding.SPMM_EINVAL
    assert binding._lib.spmm_plan_set_tile_sharing(None, 0) == binding.SPMM_EINVAL
    assert binding._lib.spmm_plan_set_panel_height(None, 32, 6, 5, None) == binding.SPMM_EINVAL
    assert binding._lib.spmm_plan_tm32_sizes(None, None) == binding.SPMM_EINVAL
    # the measurement aid checks its sizes before it touches the GPU
    assert binding._lib.spmm_calibrate_gather(None, 1024, 8, 4, None, None) == binding.SPMM_EINVAL
    fake = ctypes.c_void_p(4096)   # never dereferenced: the size rules fail first
    assert binding._lib.spmm_calibrate_gather(fake, 1000, 8, 4, fake, None) == binding.SPMM_EINVAL
    assert binding._lib.spmm_calibrate_gather(fake, 1024, 7, 4, fake, None) == binding.SPMM_EINVAL
    assert binding._lib.spmm_calibrate_gather(fake, 1024, 8, 3, fake, None) == binding.SPMM_EINVAL
    binding._lib.spmm_plan_destroy(None)
    out = ctypes.c_void_p()
    assert binding._lib.spmm_plan(-1, 1, 0, None, None, None, None, ctypes.byref(out)) == binding.SPMM_EINVAL
    assert binding._lib.spmm_plan(1, 1, 2**31, None, None, None, None, ctypes.byref(out)) in (
        binding.SPMM_EINVAL, binding.SPMM_ELIMIT)
