"""Regular segments of 3 to 30 elements that are no power of two, or 4 or 8 (packed_rows_reduce_kernel: rows of m whole segments,
m * seg_len even and at most 32, one product per 16 rows with a masked constant matrix): tcr_segmented_reduce and
tcr_segmented_moments against the oracle.

Integer-valued inputs must match exactly; real-valued ones within |y - ref| <= 1e-3 * max(|ref|, rho), rho = the
root of the segment's sum of squares (for the sums of squares, whose terms are all positive: plain relative error).
A wavefront takes 16 * U rows (U = 8 or 4 by the row width, the other one as the alternative of the tuning table), a
workgroup four wavefronts: the segment counts below leave a ragged last row, a ragged last tile, a ragged last
wavefront and a ragged last workgroup, and fill each exactly.
"""
import numpy as np
import pytest
import torch

from paper_1811_09736_amd import workloads

pytestmark = pytest.mark.gpu

LENGTHS = [3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15, 18, 20, 22, 24, 26, 28, 30]
PACKED, PACKED_ALT, ROWS, TILES = 4, 5, 0, 1


def per_row(seg):
    m = 32 // seg
    return m - 1 if seg % 2 and m % 2 else m


@pytest.fixture(scope="module")
def tcr():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1811_09736_amd import binding
    binding.set_variant("reset")
    binding.tuning_import("")
    yield binding
    binding.tuning_import("")
    binding.set_variant("reset")
    binding.check_device_flags()


def _counts(seg):
    m = per_row(seg)
    wave8, wave4 = 16 * 8 * m, 16 * 4 * m                     # segments per wavefront with either shape
    counts = {2, 3, m - 1, m, m + 1, 16 * m - 1, 16 * m, 16 * m + 1, wave4 - 1, wave4 + 1, wave8, wave8 + m + 1,
              4 * wave8 - 1, 4 * wave8, 4 * wave8 + 1, 9 * wave8 + 5}
    return sorted(c for c in counts if c >= 2)               # (one segment is the full reduction: another kernel)


@pytest.mark.parametrize("choice", [PACKED, PACKED_ALT])
@pytest.mark.parametrize("seg", LENGTHS)
def test_sums_and_moments_are_exact_on_integers(tcr, oracle, seg, choice):
    tcr.tuning_import(f"reduce_any:{seg.bit_length() - 1}={choice};")
    try:
        for nseg in _counts(seg):
            x = workloads.make_input(seg * nseg, "int8" if nseg % 2 else "int4", seg + nseg)
            xd = torch.from_numpy(x).cuda()
            assert tcr.kernel_name(tcr.OP_SEGMENTED_REDUCE, x.size, seg) == "packed_rows_reduce_kernel"
            got = tcr.segmented_reduce(xd, seg).cpu().numpy().astype(np.float64)
            ref = oracle.segmented_reduce(x, seg)
            bad = np.flatnonzero(got != ref)
            assert bad.size == 0, f"L={seg} nseg={nseg}: segment {bad[0]}: {got[bad[0]]} != {ref[bad[0]]}"
            a, q = tcr.segmented_moments(xd, seg)
            ra, rq = oracle.segmented_moments(x, seg)
            assert np.array_equal(a.cpu().numpy().astype(np.float64), ra), f"L={seg} nseg={nseg}: sums"
            assert np.array_equal(q.cpu().numpy().astype(np.float64), rq), f"L={seg} nseg={nseg}: squares"
    finally:
        tcr.tuning_import("")


def test_it_is_the_default_for_its_lengths_and_for_no_other(tcr):
    for seg in range(1, 40):
        name = tcr.kernel_name(tcr.OP_SEGMENTED_REDUCE, seg * 1000, seg)
        assert (name == "packed_rows_reduce_kernel") == (seg in LENGTHS), (seg, name)


@pytest.mark.parametrize("dist", ["uniform_pm1", "normal", "uniform_01"])
@pytest.mark.parametrize("seg", [3, 7, 9, 12, 15, 18, 24, 30])
def test_real_valued_inputs(tcr, oracle, seg, dist):
    nseg = 100003
    x = workloads.make_input(seg * nseg, dist, seg)
    xd = torch.from_numpy(x).cuda()
    ra, rq = oracle.segmented_moments(x, seg)
    rho = np.sqrt(rq)
    got = tcr.segmented_reduce(xd, seg).cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - ra) <= 1e-3 * np.maximum(np.abs(ra), rho)), f"L={seg} {dist}"
    a, q = tcr.segmented_moments(xd, seg)
    assert np.all(np.abs(a.cpu().numpy().astype(np.float64) - ra) <= 1e-3 * np.maximum(np.abs(ra), rho)), f"L={seg} {dist}"
    assert np.all(np.abs(q.cpu().numpy().astype(np.float64) - rq) <= 1e-3 * rq), f"L={seg} {dist}: squares"


@pytest.mark.parametrize("seg", [6, 11, 24])
def test_views_at_other_alignments(tcr, oracle, seg):
    # 4-byte aligned views keep the kernel (its rows start on 4-byte boundaries); 2-byte aligned ones go to the
    # kernels that lay their tiles out from the 16-byte boundary below the first element
    nseg = 16 * 8 * 4 * per_row(seg) + 7
    x = workloads.make_input(seg * nseg + 8, "int8", seg)
    for lead in (2, 6, 1, 3):
        xd = torch.from_numpy(x).cuda()[lead:lead + seg * nseg]
        xs = x[lead:lead + seg * nseg].copy()
        assert np.array_equal(tcr.segmented_reduce(xd, seg).cpu().numpy().astype(np.float64), oracle.segmented_reduce(xs, seg))
        a, q = tcr.segmented_moments(xd, seg)
        ra, rq = oracle.segmented_moments(xs, seg)
        assert np.array_equal(a.cpu().numpy().astype(np.float64), ra) and np.array_equal(q.cpu().numpy().astype(np.float64), rq)
    # results that are not 16-byte aligned: single stores
    xd = torch.from_numpy(x).cuda()[:seg * nseg]
    out = torch.zeros(nseg + 1, dtype=torch.float32, device="cuda")
    tcr.segmented_reduce(xd, seg, out=out[1:])
    assert np.array_equal(out[1:].cpu().numpy().astype(np.float64), oracle.segmented_reduce(x[:seg * nseg].copy(), seg))
    assert float(out[0]) == 0.0


def test_the_earlier_kernels_stay_available(tcr, oracle):
    x = workloads.make_input(12 * 40001, "int8", 9)
    xd = torch.from_numpy(x).cuda()
    ref = oracle.segmented_reduce(x, 12)
    tcr.set_variant("untuned_reduce", "tiles")
    try:
        assert tcr.kernel_name(tcr.OP_SEGMENTED_REDUCE, x.size, 12).startswith("irregular_reduce_kernel<regular>")
        assert np.array_equal(tcr.segmented_reduce(xd, 12).cpu().numpy().astype(np.float64), ref)
    finally:
        tcr.set_variant("reset")
    tcr.tuning_import(f"reduce_any:3={TILES};")
    try:
        assert tcr.kernel_name(tcr.OP_SEGMENTED_REDUCE, x.size, 12).startswith("irregular_reduce_kernel<regular>")
        assert np.array_equal(tcr.segmented_reduce(xd, 12).cpu().numpy().astype(np.float64), ref)
    finally:
        tcr.tuning_import("")
    assert np.array_equal(tcr.segmented_reduce(xd, 12).cpu().numpy().astype(np.float64), ref)
    # 4 and 8 elements: whole segments inside a lane's eight elements, one thread per segment for the moments
    for seg in (4, 8):
        m = x.size // seg * seg
        ref, (ra, rq) = oracle.segmented_reduce(x[:m], seg), oracle.segmented_moments(x[:m], seg)
        tcr.set_variant("untuned_reduce", "tiles")
        try:
            assert tcr.kernel_name(tcr.OP_SEGMENTED_REDUCE, m, seg) == "tiny_reduce_kernel"
            assert np.array_equal(tcr.segmented_reduce(xd[:m], seg).cpu().numpy().astype(np.float64), ref)
            a, q = tcr.segmented_moments(xd[:m], seg)
            assert np.array_equal(a.cpu().numpy().astype(np.float64), ra) and np.array_equal(q.cpu().numpy().astype(np.float64), rq)
        finally:
            tcr.set_variant("reset")


@pytest.mark.parametrize("seg", [5, 12, 30])
def test_at_bench_size(tcr, oracle, seg):
    n = (1 << 28) // seg * seg
    x = workloads.make_input(n, "int4", seg)
    xd = torch.from_numpy(x).cuda()
    got = tcr.segmented_reduce(xd, seg).cpu().numpy().astype(np.float64)
    assert np.array_equal(got, oracle.segmented_reduce(x, seg))
