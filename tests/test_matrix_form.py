"""The paper's matrix-product algorithms (oracle/matrix_form.py) must reproduce the plain
definition (oracle/tcr_oracle.c) for every tiling the paper describes.  This pins the
readings of the garbled passages (row- vs column-major, which of U / L carries the
diagonal, the G matrix, the block-level scan)."""
import numpy as np
import pytest

from oracle import matrix_form as mf
from paper_1811_09736_amd import workloads


def _data(n, seed=21, dist="int8"):
    # integer-valued input: every summation order is exact in binary64, so equality is exact
    x = workloads.make_input(n, dist, seed)
    return x, x.astype(np.float64)


def test_constant_matrices_match_the_displayed_ones():
    # Section 4: P has a first row of ones.  Section 5 displays U with a full first row and a
    # single one in the last row (upper triangular with diagonal), L with a zero first row and
    # a last row of ones except the diagonal (strictly lower).
    assert mf.P[0].tolist() == [1.0] * 16 and not mf.P[1:].any()
    assert mf.U[0].tolist() == [1.0] * 16 and mf.U[15].tolist() == [0.0] * 15 + [1.0]
    assert mf.L[0].tolist() == [0.0] * 16 and mf.L[15].tolist() == [1.0] * 15 + [0.0]
    assert np.array_equal(mf.U, mf.L.T + np.eye(16))


def test_tile_products_against_hand_written_loops():
    # the displayed identities of Section 5, checked entry by entry with explicit loops
    rng = np.random.default_rng(3)
    v = rng.integers(-9, 9, 256).astype(np.float64)
    a = mf.load_tile(v, 0)
    assert all(a[r, c] == v[16 * r + c] for r in range(16) for c in range(16))      # row-major
    ac = mf.load_tile(v, 0, "colmajor")
    assert all(ac[r, c] == v[16 * c + r] for r in range(16) for c in range(16))
    au, la = a @ mf.U, mf.L @ a
    g = la @ mf.ONES
    for r in range(16):
        for c in range(16):
            assert au[r, c] == sum(a[r, :c + 1])                 # inclusive scan of each row
            assert la[r, c] == sum(a[:r, c])                     # exclusive scan of each column
            assert g[r, c] == sum(v[:16 * r])                    # everything before row r
            assert (g + au)[r, c] == sum(v[:16 * r + c + 1])     # Scan(V) read in row-major order
    pa = mf.P @ ac
    assert all(pa[0, c] == sum(v[16 * c: 16 * c + 16]) for c in range(16)) and not pa[1:].any()
    assert (pa @ mf.P.T)[0, 0] == v.sum() and np.count_nonzero(pa @ mf.P.T) <= 1


def test_reduction_16_and_256(oracle):
    x, xd = _data(256 * 6)
    assert np.array_equal(mf.reduction_16(xd), oracle.segmented_reduce(x, 16))
    assert np.array_equal(mf.reduction_256(xd), oracle.segmented_reduce(x, 256))


@pytest.mark.parametrize("seg", [256, 512, 1024, 4096])
def test_reduction_256n(oracle, seg):
    x, xd = _data(8192)
    assert np.array_equal(mf.reduction_256n(xd, seg), oracle.segmented_reduce(x, seg))


@pytest.mark.parametrize("seg", [16, 32, 48, 64, 240])
def test_reduction_16n_strided(oracle, seg):
    x, xd = _data(16 * seg * 3)
    assert np.array_equal(mf.reduction_16n_strided(xd, seg), oracle.segmented_reduce(x, seg))


@pytest.mark.parametrize("seg,wpb", [(1024, 1), (1024, 4), (4096, 2), (4096, 16), (8192, 8)])
def test_block_reduction(oracle, seg, wpb):
    x, xd = _data(2 * 8192)
    assert np.array_equal(mf.block_reduction_256n(xd, seg, wpb), oracle.segmented_reduce(x, seg))


def test_grid_reduction(oracle):
    x, xd = _data(1 << 17)
    for block_len in (1024, 4096, 1 << 15):
        assert mf.grid_reduction(xd, block_len) == oracle.reduce(x)


def test_scan_16(oracle):
    x, xd = _data(256 * 5)
    assert np.array_equal(mf.scan_16(xd), oracle.segmented_scan(x, 16))


@pytest.mark.parametrize("seg", [256, 512, 2048])
def test_scan_256n(oracle, seg):
    x, xd = _data(4096)
    assert np.array_equal(mf.scan_256n(xd, seg), oracle.segmented_scan(x, seg))


@pytest.mark.parametrize("seg", [16, 32, 64, 112])
def test_scan_16n(oracle, seg):
    x, xd = _data(16 * seg * 2)
    assert np.array_equal(mf.scan_16n(xd, seg), oracle.segmented_scan(x, seg))


@pytest.mark.parametrize("seg,wpb", [(256, 1), (1024, 4), (4096, 4), (4096, 16), (2048, 8), (6144, 3)])
def test_block_scan(oracle, seg, wpb):
    x, xd = _data(3 * 4096)
    assert np.array_equal(mf.block_scan_256n(xd, seg, wpb), oracle.segmented_scan(x, seg))


def test_grid_scan(oracle):
    x, xd = _data(1 << 15)
    for block_len in (1024, 4096):
        assert np.array_equal(mf.grid_scan(xd, block_len), oracle.scan(x))


def test_real_valued_agreement_is_rounding_only(oracle):
    # on real-valued data the two differ only by the order of binary64 additions
    x = workloads.make_input(8192, "uniform_pm1", 1)
    xd = x.astype(np.float64)
    ref = oracle.segmented_scan(x, 2048)
    assert np.max(np.abs(mf.scan_256n(xd, 2048) - ref)) <= 2048 * 2.0 ** -52
    assert np.max(np.abs(mf.block_scan_256n(xd, 2048, 4) - ref)) <= 2048 * 2.0 ** -52
    assert np.max(np.abs(mf.reduction_256n(xd, 2048) - oracle.segmented_reduce(x, 2048))) <= 2048 * 2.0 ** -52


def test_swapped_triangles_would_be_caught(oracle):
    # the reading printed in the closing sentence of the derivation (U lower, L upper) does not
    # give a scan: planting it here shows the comparison above can tell the two apart
    x, xd = _data(256)
    a = mf.load_tile(xd, 0)
    u_bad = np.tril(np.ones((16, 16)))
    l_bad = np.triu(np.ones((16, 16)), 1)
    wrong = (l_bad @ a) @ mf.ONES + a @ u_bad
    assert not np.array_equal(wrong.reshape(-1), oracle.scan(x))
    # and the column-major index formula printed for the scan tile does not either
    a_cm = mf.load_tile(xd, 0, "colmajor")
    wrong2 = (mf.L @ a_cm) @ mf.ONES + a_cm @ mf.U
    assert not np.array_equal(wrong2.reshape(-1), oracle.scan(x))
