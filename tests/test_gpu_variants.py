"""Scan variants (exclusive, binary16 output) through tcr_segmented_scan_ex / tcr_scan_ex against the oracle.

Exclusive: the oracle's own exclusive scan.  Binary16 output: the oracle's binary64 value rounded to binary16
(numpy, round to nearest even, overflow to infinity).  Integer-valued inputs must match exactly -- the binary32
sum is exact, so its rounding equals the rounding of the exact value.  For real-valued inputs the binary32 sum
carries a few ulps of error, which can tip a value that lies next to a rounding boundary to the neighbouring
binary16 number, so the bar is one binary16 spacing.
"""
import numpy as np
import pytest
import torch

from paper_1811_09736_amd import workloads

pytestmark = pytest.mark.gpu

EXCL, F16 = 1, 2


@pytest.fixture(scope="module")
def tcr():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1811_09736_amd import binding
    binding.set_variant("reset")
    yield binding
    binding.set_variant("reset")
    binding.check_device_flags()


def reference(oracle, x, seg, flags):
    ref = oracle.segmented_scan_exclusive(x, seg) if flags & EXCL else oracle.segmented_scan(x, seg)
    return ref


def scan_rho(x, seg, flags):
    """rho of the tolerance rule |y - ref| <= 1e-3 * max(|ref|, rho) for every scan output: the root of the sum
    of squares of the inputs the output adds up -- for the exclusive scan the elements IN FRONT of k (so the
    scale of the first output of a segment is 0: it must be exactly 0)."""
    sq = np.cumsum((x.astype(np.float64) ** 2).reshape(-1, seg), axis=1)
    if flags & EXCL:
        sq = np.concatenate([np.zeros((sq.shape[0], 1)), sq[:, :-1]], axis=1)
    return np.sqrt(sq).reshape(-1)


def check(got, ref, flags, exact, what, rho=None):
    g = got.cpu().numpy()
    if flags & F16:
        assert g.dtype == np.float16
        with np.errstate(over="ignore"):
            want = ref.astype(np.float16)
        if exact:
            same = (g == want) | (np.isinf(g) & np.isinf(want) & (np.sign(g) == np.sign(want)))
            assert same.all(), f"{what}: first mismatch at {np.flatnonzero(~same)[0]}"
        else:
            fin = np.isfinite(want) & (np.abs(ref) < 65504.0 * (1 - 2.0 ** -10))
            g64 = g[fin].astype(np.float64)
            spacing = np.maximum(2.0 ** (np.floor(np.log2(np.maximum(np.abs(ref[fin]), 2.0 ** -14))) - 10), 2.0 ** -24)
            # one binary16 spacing for the rounding of the result; where the output is small against the
            # inputs it adds up (zero-mean data near a zero crossing) the binary32 sum in front of that
            # rounding has the rho part of the binary32 rule on top
            slack = 1e-3 * np.where(rho[fin] > np.abs(ref[fin]), rho[fin], 0.0)
            assert np.all(np.abs(g64 - ref[fin]) <= spacing + slack), what
    else:
        g64 = g.astype(np.float64)
        if exact:
            assert np.array_equal(g64, ref), f"{what}: first mismatch at {np.flatnonzero(g64 != ref)[0]}"
        else:
            assert np.all(np.abs(g64 - ref) <= 1e-3 * np.maximum(np.abs(ref), rho)), what


SEGS = [16, 32, 64, 256, 512, 1024, 4096, 8192, 16384, 32768, 1 << 16, 1 << 17, 1 << 20]
GENERIC = [1, 3, 24, 97, 100, 1000, 4097]


@pytest.mark.parametrize("flags", [EXCL, F16, EXCL | F16])
@pytest.mark.parametrize("seg", SEGS + GENERIC)
def test_variants_exact(tcr, oracle, seg, flags):
    nseg = 3 if seg >= 8192 else (3 * 8192 // seg + 3)
    n = seg * nseg
    x = workloads.make_input(n, "int4", 500 + seg % 89)
    xd = torch.from_numpy(x).cuda()
    got = tcr.segmented_scan_ex(xd, seg, flags)
    check(got, reference(oracle, x, seg, flags), flags, True, f"L={seg} flags={flags}")


@pytest.mark.parametrize("flags", [EXCL, F16, EXCL | F16])
@pytest.mark.parametrize("dist", ["uniform_01", "uniform_pm1"])
@pytest.mark.parametrize("seg", [16, 256, 2048, 16384, 1 << 17, 100, 3000, 3584, 3 << 16])
def test_variants_real(tcr, oracle, seg, flags, dist):
    # seg_len 16 .. 2048: no carry between workgroups; 16384: tiles by ticket; 2^17, 3 * 2^16: the chain;
    # 100, 3000: fixed tiles with the segment starts marked; 3584: one workgroup per segment.
    # uniform_pm1 is zero-mean: outputs cross zero, the rho part of the rule decides there.
    nseg = 3 if seg >= 8192 else (3 * 8192 // seg + 3)
    n = seg * nseg
    x = workloads.make_input(n, dist, 4)
    xd = torch.from_numpy(x).cuda()
    got = tcr.segmented_scan_ex(xd, seg, flags)
    ref = reference(oracle, x, seg, flags)
    check(got, ref, flags, False, f"L={seg} flags={flags} {dist}", scan_rho(x, seg, flags))
    if flags & EXCL:
        assert not got[::seg].any(), "the first output of every segment of an exclusive scan is exactly 0"


@pytest.mark.parametrize("flags", [EXCL, F16, EXCL | F16])
@pytest.mark.parametrize("n", [1, 7, 513, 8193, 100003, (1 << 21) + 9])
def test_full_scan_variants(tcr, oracle, n, flags):
    x = workloads.make_input(n, "int4", n % 777)
    xd = torch.from_numpy(x).cuda()
    got = tcr.scan_ex(xd, flags)
    check(got, reference(oracle, x, n, flags), flags, True, f"full n={n} flags={flags}")


def test_flags_zero_is_the_plain_scan(tcr):
    x = torch.from_numpy(workloads.make_input(1 << 16, "int8", 1)).cuda()
    assert torch.equal(tcr.segmented_scan_ex(x, 256, 0), tcr.segmented_scan(x, 256))
    assert torch.equal(tcr.scan_ex(x, 0), tcr.scan(x))


def test_exclusive_plus_input_is_inclusive(tcr):
    x = torch.from_numpy(workloads.make_input(1 << 20, "int8", 2)).cuda()
    for seg in (64, 4096, 1 << 18, 1 << 20):
        inc = tcr.segmented_scan(x, seg)
        exc = tcr.segmented_scan_ex(x, seg, EXCL)
        assert torch.equal(exc + x.float(), inc)
        assert not exc[::seg].any()


def test_dpp_formulation_has_no_tuned_variant_kernels(tcr):
    x = torch.from_numpy(workloads.make_input(1 << 12, "int4", 3)).cuda()
    tcr.set_variant("formulation", "dpp")
    try:
        with pytest.raises(tcr.TcrError) as e:
            tcr.segmented_scan_ex(x, 256, EXCL)
        assert e.value.status == tcr.ERR_UNSUPPORTED
        assert torch.equal(tcr.segmented_scan_ex(x, 256, 0), tcr.segmented_scan(x, 256))
        tcr.segmented_scan_ex(x[:4095], 3, EXCL)   # untuned lengths take every flag
    finally:
        tcr.set_variant("reset")


# ------------------------------------------------------------------ irregular segments

def _random_offsets(n, nseg, seed):
    rng = np.random.default_rng(seed)
    cuts = np.sort(rng.integers(0, n + 1, nseg - 1))
    return np.concatenate([[0], cuts, [n]]).astype(np.int64)


@pytest.mark.parametrize("n,nseg", [(1000, 7), (100003, 400), (1 << 20, 5000), (1 << 20, 3)])
def test_irregular_segments(tcr, oracle, n, nseg):
    x = workloads.make_input(n, "int8", n % 321)
    off = _random_offsets(n, nseg, nseg)
    off[nseg // 2 + 1] = off[nseg // 2]                      # at least one empty segment
    xd = torch.from_numpy(x).cuda()
    od = torch.from_numpy(off).cuda()
    red = tcr.irregular_reduce(xd, od).cpu().numpy().astype(np.float64)
    assert np.array_equal(red, oracle.irregular_reduce(x, off))
    scan = tcr.irregular_scan(xd, od).cpu().numpy().astype(np.float64)
    assert np.array_equal(scan, oracle.irregular_scan(x, off))
    y = workloads.make_input(n, "uniform_pm1", 5)
    yd = torch.from_numpy(y).cuda()
    got = tcr.irregular_scan(yd, od).cpu().numpy().astype(np.float64)
    ref = oracle.irregular_scan(y, off)
    # rho: root of the sum of squares since the start of the element's segment
    sq = np.concatenate([[0.0], np.cumsum(y.astype(np.float64) ** 2)])
    start_of = np.repeat(off[:-1], np.diff(off))
    rho = np.sqrt(np.maximum(sq[1:] - sq[start_of], 0.0))
    assert np.all(np.abs(got - ref) <= 1e-3 * np.maximum(np.abs(ref), rho))


def test_irregular_partial_cover_and_uniform(tcr, oracle):
    x = workloads.make_input(4096 + 3, "int4", 1)
    xd = torch.from_numpy(x).cuda()
    off = np.array([5, 5, 130, 1000, 4000], dtype=np.int64)   # does not cover the input; x[5:] is only 2-byte aligned
    od = torch.from_numpy(off).cuda()
    out = torch.full((x.size,), -1.0, dtype=torch.float32, device="cuda")
    tcr.irregular_scan(xd, od, out=out)
    got = out.cpu().numpy().astype(np.float64)
    ref = oracle.irregular_scan(x, off)
    assert np.array_equal(got[5:4000], ref[5:4000])
    assert np.all(got[:5] == -1.0) and np.all(got[4000:] == -1.0)          # untouched outside the segments
    reg = torch.arange(0, 4097, 256, dtype=torch.int64, device="cuda")
    assert torch.equal(tcr.irregular_reduce(xd, reg), tcr.segmented_reduce(xd[:4096].clone(), 256))
    assert tcr.irregular_reduce(xd, torch.zeros(1, dtype=torch.int64, device="cuda")).numel() == 0


def test_irregular_behind_unaligned_pointers(tcr, oracle):
    # a view that starts at element 1 is only 2-byte (input) / 4-byte (output) aligned: the element-wise
    # kernels run instead of the ones that read whole 8-element groups
    x = workloads.make_input(20001, "int8", 77)
    xd = torch.from_numpy(x).cuda()[1:]
    off = _random_offsets(20000, 40, 9)
    od = torch.from_numpy(off).cuda()
    out = torch.zeros(20001, dtype=torch.float32, device="cuda")[1:]
    tcr.irregular_scan(xd, od, out=out)
    assert np.array_equal(out.cpu().numpy().astype(np.float64), oracle.irregular_scan(x[1:].copy(), off))
    red = tcr.irregular_reduce(xd, od).cpu().numpy().astype(np.float64)
    assert np.array_equal(red, oracle.irregular_reduce(x[1:].copy(), off))


def _segment_kernel_by_default(seg):
    # one workgroup per segment where the segments start on 128-byte boundaries and fill four fifths of the
    # workgroup's share (2, 3, 4, 6, 8, 12 or 16 tiles of 512 elements)
    if seg % 64 or seg <= 512 or seg > 8192:
        return False
    t = -(-seg // 512)
    share = t if t <= 4 else 6 if t <= 6 else 8 if t <= 8 else 12 if t <= 12 else 16
    return 5 * seg >= 4 * share * 512


@pytest.mark.parametrize("seg", [256 + 8, 511, 513, 520, 1000, 1280, 1536, 3000, 3584, 8000, 8192 - 64, 8200, 3001, 40000, 65528, 100003])
@pytest.mark.parametrize("flags", [0, 1, 2, 3])
def test_other_segment_lengths_take_every_flag(tcr, oracle, seg, flags):
    # by default: one workgroup per segment where that is known to win, else fixed tiles of the array with the
    # segment starts marked; every multiple of 8 above one tile is also run through the kernel with one workgroup
    # per segment
    nseg = max(3, (200000 // seg) | 1)
    x = workloads.make_input(seg * nseg, "int4", seg % 89)
    xd = torch.from_numpy(x).cuda()
    want = "scan_segment_kernel" if _segment_kernel_by_default(seg) else "irregular_scan_kernel<regular>"
    assert tcr.kernel_name(tcr.OP_SEGMENTED_SCAN, x.size, seg) == want
    ref = oracle.segmented_scan_exclusive(x, seg) if flags & 1 else oracle.segmented_scan(x, seg)
    if flags & 2:
        ref = ref.astype(np.float16).astype(np.float64)            # integer sums: one correct rounding
    got = tcr.segmented_scan_ex(xd, seg, flags).cpu().numpy().astype(np.float64)
    assert np.array_equal(got, ref)
    if seg % 8 == 0 and seg > 512 and want != "scan_segment_kernel":
        tcr.tuning_import(f"scan_any:{seg.bit_length() - 1}=2;")
        try:
            assert tcr.kernel_name(tcr.OP_SEGMENTED_SCAN, x.size, seg) == "scan_segment_kernel"
            got = tcr.segmented_scan_ex(xd, seg, flags).cpu().numpy().astype(np.float64)
        finally:
            tcr.tuning_import("")
        assert np.array_equal(got, ref)
    assert np.array_equal(tcr.segmented_reduce(xd, seg).cpu().numpy().astype(np.float64), oracle.segmented_reduce(x, seg))


# ------------------------------------------------------------------ first two moments

@pytest.mark.parametrize("seg", [1, 5, 8, 12, 16, 32, 49, 64, 96, 97, 128, 196, 200, 256, 300, 512, 784, 999, 1000, 3136, 4096, 3001, 1 << 16, (1 << 17) + 8, 3 << 18, 1 << 21])
def test_segmented_moments(tcr, oracle, seg):
    nseg = max(2, (1 << 21) // seg) | 1 if seg < (1 << 20) else 2
    n = seg * nseg
    x = workloads.make_input(n, "int4", seg % 97)                      # |x| <= 4: sums of squares stay below 2^24
    xd = torch.from_numpy(x).cuda()
    a, q = tcr.segmented_moments(xd, seg)
    ra, rq = oracle.segmented_moments(x, seg)
    assert np.max(rq) < 2 ** 24
    assert np.array_equal(a.cpu().numpy().astype(np.float64), ra)
    assert np.array_equal(q.cpu().numpy().astype(np.float64), rq)
    assert torch.equal(a, tcr.segmented_reduce(xd, seg))              # the first moment is the reduction
    y = workloads.make_input(n, "normal", 7)
    a, q = tcr.segmented_moments(torch.from_numpy(y).cuda(), seg)
    ra, rq = oracle.segmented_moments(y, seg)
    got_q = q.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got_q - rq) <= 1e-3 * rq)                     # all terms positive: plain relative error
    rho = np.sqrt(rq)
    assert np.all(np.abs(a.cpu().numpy().astype(np.float64) - ra) <= 1e-3 * np.maximum(np.abs(ra), rho))


def test_full_moments_and_errors(tcr, oracle):
    x = workloads.make_input((1 << 22) + 8, "int4", 5)
    xd = torch.from_numpy(x).cuda()
    a, q = tcr.segmented_moments(xd, x.size)                           # one segment: pieces + second kernel
    ra, rq = oracle.segmented_moments(x, x.size)
    assert float(a.cpu()[0]) == ra[0] and float(q.cpu()[0]) == rq[0]
    with pytest.raises(tcr.TcrError):
        tcr.segmented_moments(xd, 7)                                   # 7 does not divide n
    with pytest.raises(tcr.TcrError):
        tcr.segmented_moments(xd, 0)
    tcr.check_device_flags()
