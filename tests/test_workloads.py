"""The seeded input generators shared by the tests, the bench and the smoke check: determinism, the prefix
property of the value arrays, and the shape of the irregular offset arrays."""
import numpy as np
import pytest

from paper_1811_09736_amd import workloads


def test_inputs_are_deterministic_and_nested():
    a = workloads.make_input(100000, "uniform_pm1", 7)
    assert a.dtype == np.float16 and a.flags["C_CONTIGUOUS"]
    assert np.array_equal(a, workloads.make_input(100000, "uniform_pm1", 7))
    assert np.array_equal(a[:5000], workloads.make_input(5000, "uniform_pm1", 7))          # a prefix of any longer draw
    assert not np.array_equal(a, workloads.make_input(100000, "uniform_pm1", 8))
    assert workloads.sha256(a) == workloads.sha256(a.copy())
    assert np.all(np.abs(a.astype(np.float64)) <= 1.0)
    ints = workloads.make_input(50000, "int4", (3, 1)).astype(np.float64)
    assert np.all(ints == np.rint(ints)) and ints.min() == -4 and ints.max() == 4
    sub = workloads.make_input(1000, "subnormal", 1).astype(np.float64)
    assert np.all(np.abs(sub) < 2.0 ** -14) and np.any(sub != 0)
    with pytest.raises(ValueError):
        workloads.make_input(8, "cauchy", 0)


@pytest.mark.parametrize("recipe,mean_lo,mean_hi", [("uniform16", 15, 17), ("uniform1024", 980, 1070),
                                                     ("lognormal256", 1000, 4000), ("few7", 1 << 16, 1 << 18)])
def test_offsets_cover_the_array(recipe, mean_lo, mean_hi):
    n = 1 << 20
    off = workloads.make_offsets(n, recipe, 5)
    assert off.dtype == np.uint64 and off[0] == 0 and off[-1] == n
    lens = np.diff(off.astype(np.int64))
    assert np.all(lens >= 0)                                          # non-decreasing; empty segments allowed
    assert mean_lo <= lens.mean() <= mean_hi
    assert np.array_equal(off, workloads.make_offsets(n, recipe, 5))
    assert not np.array_equal(off, workloads.make_offsets(n, recipe, 6))
    if recipe == "few7":
        assert lens.size == 7
    if recipe == "uniform16":
        assert lens.min() == 0 and lens.max() == 32
    if recipe == "lognormal256":                                      # heavy tail: most segments short, most elements in long ones
        assert np.median(lens) < 400 and lens[lens > 4096].sum() > n // 4
    with pytest.raises(ValueError):
        workloads.make_offsets(n, "zipf3", 0)


def test_configurations_and_their_bytes():
    cfgs = list(workloads.configs())
    assert len(cfgs) == 1 + 5 + 2 + 1 + 16
    assert all(w.n % w.seg_len == 0 for w in cfgs)
    assert {w.n for w in cfgs} == {1 << 20, 1 << 24, 1 << 28}
    assert workloads.algorithmic_bytes("segmented_reduce", 1 << 28, 256) == (1 << 29, 1 << 22)
    assert workloads.algorithmic_bytes("scan", 1 << 28, 1 << 28) == (1 << 29, 1 << 30)
