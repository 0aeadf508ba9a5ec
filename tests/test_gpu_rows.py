"""Regular segments of a length that is no power of two, from 17 elements on (rows_reduce_kernel: masked row
products, whole segments per workgroup; below 32 elements a row of 32 holds two boundaries and, between them, a
whole segment): tcr_segmented_reduce and tcr_segmented_moments against the oracle.

Integer-valued inputs must match exactly; real-valued ones within |y - ref| <= 1e-3 * max(|ref|, rho), rho = the
root of the segment's sum of squares (for the sums of squares, whose terms are all positive: plain relative error).
A workgroup takes as many whole segments as fit into 16320 elements, on rows of 32 elements of the array: the
lengths and counts below put segment ends on, next to and far from row ends, fill a workgroup exactly, leave
ragged last workgroups, and the views that start at element 1, 3 or 7 shift everything against the rows.
"""
import numpy as np
import pytest
import torch

from paper_1811_09736_amd import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tcr():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1811_09736_amd import binding
    binding.set_variant("reset")
    yield binding
    binding.set_variant("reset")
    binding.check_device_flags()


LENGTHS = [17, 18, 19, 21, 23, 24, 25, 27, 29, 30, 31, 33, 35, 48, 63, 65, 96, 97, 100, 127, 129, 196, 255, 257, 480, 511, 513, 784, 999, 1000, 1001, 2040,
           3000, 4097, 5440, 8159, 8160]


def _counts(seg):
    per_group = 16320 // seg
    return sorted({1, 2, per_group, per_group + 1, 3 * per_group - 1, 3 * per_group, 7 * per_group + 2})


@pytest.mark.parametrize("seg", LENGTHS)
def test_sums_and_moments_are_exact_on_integers(tcr, oracle, seg):
    for nseg in _counts(seg):
        n = seg * nseg
        for lead in (0, 1, 3, 7):
            x = workloads.make_input(n + lead, "int4", seg + nseg)
            xd = torch.from_numpy(x).cuda()[lead:]
            xs = x[lead:].copy()
            if nseg > 1:          # (even lengths up to 30: only the views that are not 4-byte aligned come here)
                want = "packed_rows_reduce_kernel" if seg <= 30 and seg % 2 == 0 else "rows_reduce_kernel"
                assert tcr.kernel_name(tcr.OP_SEGMENTED_REDUCE, n, seg) == want
            got = tcr.segmented_reduce(xd, seg).cpu().numpy().astype(np.float64)
            ref = oracle.segmented_reduce(xs, seg)
            bad = np.flatnonzero(got != ref)
            assert bad.size == 0, f"L={seg} nseg={nseg} lead={lead}: segment {bad[0]}: {got[bad[0]]} != {ref[bad[0]]}"
            if nseg > 1 and lead == 0 and seg <= 30 and seg % 2 == 0:        # the masked rows of the array, by the tuning table
                tcr.tuning_import("reduce_any:4=0;")
                try:
                    assert tcr.kernel_name(tcr.OP_SEGMENTED_REDUCE, n, seg) == "rows_reduce_kernel"
                    got = tcr.segmented_reduce(xd, seg).cpu().numpy().astype(np.float64)
                finally:
                    tcr.tuning_import("")
                assert np.array_equal(got, ref), f"L={seg} nseg={nseg}: rows_reduce_kernel"
            a, q = tcr.segmented_moments(xd, seg)
            ra, rq = oracle.segmented_moments(xs, seg)
            assert np.array_equal(a.cpu().numpy().astype(np.float64), ra), f"L={seg} nseg={nseg} lead={lead}: sums"
            assert np.array_equal(q.cpu().numpy().astype(np.float64), rq), f"L={seg} nseg={nseg} lead={lead}: squares"


@pytest.mark.parametrize("dist", ["uniform_pm1", "normal", "uniform_01"])
@pytest.mark.parametrize("seg", [17, 24, 31, 33, 100, 196, 999, 3001, 8160])
def test_real_valued_inputs(tcr, oracle, seg, dist):
    nseg = 5 * (16320 // seg) + 3
    x = workloads.make_input(seg * nseg, dist, seg)
    xd = torch.from_numpy(x).cuda()
    ra, rq = oracle.segmented_moments(x, seg)
    rho = np.sqrt(rq)
    got = tcr.segmented_reduce(xd, seg).cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - ra) <= 1e-3 * np.maximum(np.abs(ra), rho)), f"L={seg} {dist}"
    a, q = tcr.segmented_moments(xd, seg)
    assert np.all(np.abs(a.cpu().numpy().astype(np.float64) - ra) <= 1e-3 * np.maximum(np.abs(ra), rho)), f"L={seg} {dist}"
    assert np.all(np.abs(q.cpu().numpy().astype(np.float64) - rq) <= 1e-3 * rq), f"L={seg} {dist}: squares"


def test_large_values_next_to_small_ones_do_not_mix(tcr, oracle):
    # every piece of a row is summed on its own (masked operands), so a segment of tiny values between
    # segments of huge ones keeps its full precision: exact here, since each segment's sum is exact in binary32
    seg, nseg = 100, 999
    x = np.empty(seg * nseg, dtype=np.float16)
    x.reshape(nseg, seg)[0::2] = np.float16(2048.0)
    x.reshape(nseg, seg)[1::2] = np.float16(2.0 ** -14)
    got = tcr.segmented_reduce(torch.from_numpy(x).cuda(), seg).cpu().numpy().astype(np.float64)
    assert np.array_equal(got, oracle.segmented_reduce(x, seg))


@pytest.mark.parametrize("seg", [64, 256, 4096, 100])
def test_views_that_are_not_16_byte_aligned(tcr, oracle, seg):
    # powers of two as well: the tuned kernels need aligned 128-bit loads, this one lays its rows out from the
    # 16-byte boundary below the first element
    nseg = 3 * (16320 // seg) + 1
    x = workloads.make_input(seg * nseg + 5, "int8", seg)
    for lead in (1, 5):
        xd = torch.from_numpy(x).cuda()[lead:lead + seg * nseg]
        ref = oracle.segmented_reduce(x[lead:lead + seg * nseg].copy(), seg)
        assert np.array_equal(tcr.segmented_reduce(xd, seg).cpu().numpy().astype(np.float64), ref)


def test_fixed_tiles_stay_available_as_the_measured_alternative(tcr, oracle):
    x = workloads.make_input(100 * 4001, "int8", 9)
    xd = torch.from_numpy(x).cuda()
    ref = oracle.segmented_reduce(x, 100)
    tcr.set_variant("untuned_reduce", "tiles")
    try:
        assert tcr.kernel_name(tcr.OP_SEGMENTED_REDUCE, x.size, 100).startswith("irregular_reduce_kernel<regular>")
        assert np.array_equal(tcr.segmented_reduce(xd, 100).cpu().numpy().astype(np.float64), ref)
    finally:
        tcr.set_variant("reset")
    assert np.array_equal(tcr.segmented_reduce(xd, 100).cpu().numpy().astype(np.float64), ref)


def test_at_bench_size(tcr, oracle):
    # the launch configuration bench.py times: n = 2^28 (rounded down to whole segments), every result compared
    n28 = 1 << 28
    x = workloads.make_input(n28, "uniform_01", 4)
    xd = torch.from_numpy(x).cuda()
    for seg in (100, 196):
        n = (n28 // seg) * seg
        ra, rq = oracle.segmented_moments(x[:n], seg)
        got = tcr.segmented_reduce(xd[:n], seg).cpu().numpy().astype(np.float64)
        assert np.max(np.abs(got - ra) / ra) <= 1e-3
        a, q = tcr.segmented_moments(xd[:n], seg)
        assert np.max(np.abs(a.cpu().numpy().astype(np.float64) - ra) / ra) <= 1e-3
        assert np.max(np.abs(q.cpu().numpy().astype(np.float64) - rq) / rq) <= 1e-3
