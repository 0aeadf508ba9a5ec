"""Irregular segments (tcr_irregular_reduce / tcr_irregular_scan) on 16-byte aligned arrays: the kernels that cut
the work by elements.  Every case compares the whole output with the oracle's plain per-segment loops.

Integer-valued inputs must match exactly.  Real-valued inputs: |y - ref| <= 1e-3 * max(|ref|, rho), rho = the
root of the sum of squares over the same prefix (scan) or segment (reduce) -- the bar of the regular tests.
The tile is 32768 elements for the scan and 16384 for the reduction; the sizes below span several tiles with a
ragged tail, and the offsets put segment starts on, next to and far from tile and wavefront boundaries.
"""
import numpy as np
import pytest
import torch

from paper_1811_09736_amd import workloads

pytestmark = pytest.mark.gpu

SCAN_TILE, REDUCE_TILE = 32768, 16384


@pytest.fixture(scope="module")
def tcr():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1811_09736_amd import binding
    binding.set_variant("reset")
    yield binding
    binding.set_variant("reset")
    binding.check_device_flags()


def _rho(x, off):
    """Per element: root of the sum of squares since the start of its segment; per segment: over the segment."""
    sq = np.concatenate([[0.0], np.cumsum(x.astype(np.float64) ** 2)])
    off = np.asarray(off, dtype=np.int64)
    lens = np.diff(off)
    start_of = np.repeat(off[:-1], lens)
    k = np.arange(off[0], off[-1])
    rho_scan = np.zeros(x.size)
    rho_scan[off[0]:off[-1]] = np.sqrt(np.maximum(sq[k + 1] - sq[start_of], 0.0))
    rho_red = np.sqrt(np.maximum(sq[off[1:]] - sq[off[:-1]], 0.0))
    return rho_scan, rho_red


def _run(tcr, oracle, x, off, exact, what):
    off = np.asarray(off, dtype=np.int64)
    xd = torch.from_numpy(x).cuda()
    od = torch.from_numpy(off).cuda()
    ref_red = oracle.irregular_reduce(x, off)
    ref_scan = oracle.irregular_scan(x, off)
    out = torch.full((x.size,), -3.0, dtype=torch.float32, device="cuda")
    tcr.irregular_scan(xd, od, out=out)
    red = tcr.irregular_reduce(xd, od)
    torch.cuda.synchronize()
    tcr.check_device_flags()
    scan = out.cpu().numpy().astype(np.float64)
    red = red.cpu().numpy().astype(np.float64)
    lo, hi = int(off[0]), int(off[-1])
    assert np.all(scan[:lo] == -3.0) and np.all(scan[hi:] == -3.0), f"{what}: wrote outside the segments"
    if exact:
        bad = np.flatnonzero(scan[lo:hi] != ref_scan[lo:hi])
        assert bad.size == 0, f"{what}: scan differs first at {lo + bad[0]}: {scan[lo + bad[0]]} != {ref_scan[lo + bad[0]]}"
        bad = np.flatnonzero(red != ref_red)
        assert bad.size == 0, f"{what}: reduce differs first at segment {bad[0]}: {red[bad[0]]} != {ref_red[bad[0]]}"
    else:
        rho_scan, rho_red = _rho(x, off)
        assert np.all(np.abs(scan - ref_scan)[lo:hi] <= 1e-3 * np.maximum(np.abs(ref_scan), rho_scan)[lo:hi]), what
        assert np.all(np.abs(red - ref_red) <= 1e-3 * np.maximum(np.abs(ref_red), rho_red)), what


@pytest.mark.parametrize("recipe", ["uniform1", "uniform16", "uniform300", "uniform1024", "uniform20000",
                                    "lognormal64", "lognormal256", "few2", "few7", "few40"])
@pytest.mark.parametrize("n", [3 * SCAN_TILE + 1234, 1 << 20, 40000 - 3])
def test_length_mixes(tcr, oracle, recipe, n):
    off = workloads.make_offsets(n, recipe, (n % 1000, 7)).view(np.int64)
    _run(tcr, oracle, workloads.make_input(n, "int8", 11), off, True, f"{recipe} n={n} int8")
    _run(tcr, oracle, workloads.make_input(n, "uniform_pm1", 12), off, False, f"{recipe} n={n} uniform_pm1")


@pytest.mark.parametrize("seg", [8192, 16384, 32768, 65536, 3 * 16384, 100000, 1])
def test_regular_offsets_match_the_segmented_calls(tcr, oracle, seg):
    # starts exactly on tile and wavefront boundaries; also checked against the regular entry points
    n = (5 * SCAN_TILE // seg) * seg if seg > 1 else 70000
    x = workloads.make_input(n, "int8", 3)
    off = np.arange(0, n + 1, seg, dtype=np.int64)
    _run(tcr, oracle, x, off, True, f"regular {seg}")
    xd, od = torch.from_numpy(x).cuda(), torch.from_numpy(off).cuda()
    assert torch.equal(tcr.irregular_reduce(xd, od), tcr.segmented_reduce(xd, seg))
    assert torch.equal(tcr.irregular_scan(xd, od), tcr.segmented_scan(xd, seg))


def test_single_segment_is_the_full_operation(tcr, oracle):
    n = 7 * SCAN_TILE + 8 * 37
    x = workloads.make_input(n, "int4", 5)
    _run(tcr, oracle, x, [0, n], True, "one segment")
    xd = torch.from_numpy(x).cuda()
    od = torch.tensor([0, n], dtype=torch.int64, device="cuda")
    assert torch.equal(tcr.irregular_scan(xd, od), tcr.scan(xd))
    assert torch.equal(tcr.irregular_reduce(xd, od), tcr.reduce(xd))


@pytest.mark.parametrize("lo,hi", [(0, 5), (5, 5), (SCAN_TILE - 1, SCAN_TILE + 1), (REDUCE_TILE, 2 * REDUCE_TILE),
                                   (3, 4 * SCAN_TILE - 3), (2 * SCAN_TILE + 17, 2 * SCAN_TILE + 17)])
def test_partial_cover(tcr, oracle, lo, hi):
    # elements in front of offsets[0] and behind offsets[nseg] belong to no segment and must stay untouched
    n = 4 * SCAN_TILE + 100
    x = workloads.make_input(n, "int8", 21)
    mid = np.sort(np.random.default_rng(lo + hi).integers(lo, hi, 9, endpoint=True))
    _run(tcr, oracle, x, np.concatenate([[lo], mid, [hi]]), True, f"cover [{lo}, {hi})")


def test_runs_of_empty_segments(tcr, oracle):
    # many entries of offsets on one position: at 0, on a tile boundary, inside a tile and at n
    n = 2 * SCAN_TILE + 512
    x = workloads.make_input(n, "int8", 22)
    off = np.concatenate([np.zeros(700, np.int64), [5], np.full(1500, REDUCE_TILE, np.int64), [REDUCE_TILE + 9],
                          np.full(3000, SCAN_TILE + 100, np.int64), np.full(900, n, np.int64)])
    _run(tcr, oracle, x, off, True, "runs of empty segments")
    xd = torch.from_numpy(x).cuda()
    empties = torch.full((5000,), 77, dtype=torch.int64, device="cuda")
    assert torch.count_nonzero(tcr.irregular_reduce(xd, empties)).item() == 0


def test_no_elements(tcr):
    x = torch.empty(0, dtype=torch.float16, device="cuda")
    od = torch.zeros(9, dtype=torch.int64, device="cuda")
    red = tcr.irregular_reduce(x, od, out=torch.full((8,), 5.0, dtype=torch.float32, device="cuda"))
    assert torch.count_nonzero(red).item() == 0
    assert tcr.irregular_scan(x, od).numel() == 0


def test_carry_over_many_tiles_next_to_tiny_segments(tcr, oracle):
    # long segments of ones between stretches of short segments, 2000 of which hold multiples of 2^-24 only:
    # a carry that leaks across a segment start swamps the tiny sums behind it, and every sum stays exact
    n = 40 * SCAN_TILE
    rng = np.random.default_rng(8)
    x = workloads.make_input(n, "int1", 30)
    x[: 12 * SCAN_TILE] = np.float16(1.0)
    lens = np.concatenate([[9 * SCAN_TILE + 5], rng.integers(0, 40, 5000), [17 * SCAN_TILE + 3], rng.integers(0, 3000, 40)])
    off = np.concatenate([[0], np.cumsum(lens)])
    off = np.concatenate([off[off < n], [n]])
    tiny = slice(int(off[1]), int(off[2001]))
    x[tiny] = workloads.make_input(tiny.stop - tiny.start, "subnormal", 4)
    assert np.abs(oracle.irregular_scan(x, off)).max() < 2.0 ** 24
    _run(tcr, oracle, x, off, True, "long and short segments mixed")


def test_repeated_launches_share_the_workspace(tcr, oracle):
    n = 6 * SCAN_TILE
    x = workloads.make_input(n, "int8", 40)
    xd = torch.from_numpy(x).cuda()
    for seed in range(6):
        off = workloads.make_offsets(n, ("few5", "uniform4000", "lognormal256")[seed % 3], seed).view(np.int64)
        od = torch.from_numpy(off).cuda()
        red = tcr.irregular_reduce(xd, od)
        scan = tcr.irregular_scan(xd, od)
        full = tcr.scan(xd)                                        # a chained regular scan in between
        assert np.array_equal(red.cpu().numpy().astype(np.float64), oracle.irregular_reduce(x, off))
        assert np.array_equal(scan.cpu().numpy().astype(np.float64), oracle.irregular_scan(x, off))
        assert np.array_equal(full.cpu().numpy().astype(np.float64), oracle.scan(x))
    tcr.check_device_flags()


def test_caller_supplied_workspace(tcr, oracle):
    n = 40 * SCAN_TILE + 16
    x = workloads.make_input(n, "int8", 41)
    off = workloads.make_offsets(n, "lognormal256", 3).view(np.int64)
    xd, od = torch.from_numpy(x).cuda(), torch.from_numpy(off).cuda()
    need = max(tcr.workspace_bytes(tcr.OP_IRREGULAR_REDUCE, n, 0), tcr.workspace_bytes(tcr.OP_IRREGULAR_SCAN, n, 0))
    buf = torch.empty(need, dtype=torch.uint8, device="cuda")
    try:
        tcr.set_workspace(buf)
        for _ in range(2):
            assert np.array_equal(tcr.irregular_reduce(xd, od).cpu().numpy().astype(np.float64), oracle.irregular_reduce(x, off))
            assert np.array_equal(tcr.irregular_scan(xd, od).cpu().numpy().astype(np.float64), oracle.irregular_scan(x, off))
        tcr.set_workspace(buf[:1024])                                # room for 32 tiles: too small for either
        with pytest.raises(tcr.TcrError) as err:
            tcr.irregular_reduce(xd, od)
        assert err.value.status == tcr.ERR_WORKSPACE
        with pytest.raises(tcr.TcrError) as err:
            tcr.irregular_scan(xd, od)
        assert err.value.status == tcr.ERR_WORKSPACE
    finally:
        tcr.set_workspace(None)
    assert np.array_equal(tcr.irregular_reduce(xd, od).cpu().numpy().astype(np.float64), oracle.irregular_reduce(x, off))


def test_capture_and_replay(tcr, oracle):
    # recorded once the workspace exists; offsets and data change between replays (same number of segments)
    n = 5 * SCAN_TILE + 8
    nseg = 3000
    side = torch.cuda.Stream()
    xd = torch.empty(n, dtype=torch.float16, device="cuda")
    od = torch.empty(nseg + 1, dtype=torch.int64, device="cuda")
    red = torch.empty(nseg, dtype=torch.float32, device="cuda")
    scan = torch.empty(n, dtype=torch.float32, device="cuda")

    def cuts(k):
        c = np.sort(np.random.default_rng(k).integers(0, n, nseg - 1, endpoint=True))
        return np.concatenate([[0], c, [n]]).astype(np.int64)

    def calls():
        tcr.irregular_reduce(xd, od, out=red)
        tcr.irregular_scan(xd, od, out=scan)

    xd.copy_(torch.from_numpy(workloads.make_input(n, "int8", 50)).cuda())
    od.copy_(torch.from_numpy(cuts(0)).cuda())
    with torch.cuda.stream(side):
        calls()                                                      # eager once: the stream's workspace exists now
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        calls()
    for k in (1, 2, 3):
        x = workloads.make_input(n, "int8", 50 + k)
        off = cuts(k)
        xd.copy_(torch.from_numpy(x).cuda())
        od.copy_(torch.from_numpy(off).cuda())
        red.fill_(float("nan"))
        scan.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(red.cpu().numpy().astype(np.float64), oracle.irregular_reduce(x, off))
        assert np.array_equal(scan.cpu().numpy().astype(np.float64), oracle.irregular_scan(x, off))
        with torch.cuda.stream(side):                                # eager calls share the device-managed counters
            got = tcr.irregular_scan(xd, od)
        side.synchronize()
        assert np.array_equal(got.cpu().numpy().astype(np.float64), oracle.irregular_scan(x, off))
    tcr.check_device_flags(side)


@pytest.mark.parametrize("flags", [1, 2, 3])
@pytest.mark.parametrize("recipe", ["uniform16", "lognormal256", "few5"])
def test_scan_flags(tcr, oracle, recipe, flags):
    # exclusive and binary16 output (integer sums: one correct rounding), partial cover
    n = 5 * SCAN_TILE + 24
    x = workloads.make_input(n, "int4", 60)
    off = workloads.make_offsets(n - 40, recipe, flags).view(np.int64) + 16
    xd, od = torch.from_numpy(x).cuda(), torch.from_numpy(off).cuda()
    out = torch.full((n,), -3.0, dtype=torch.float16 if flags & 2 else torch.float32, device="cuda")
    tcr.irregular_scan_ex(xd, od, flags, out=out)
    got = out.cpu().numpy().astype(np.float64)
    ref = oracle.irregular_scan_exclusive(x, off) if flags & 1 else oracle.irregular_scan(x, off)
    if flags & 2:
        ref = ref.astype(np.float16).astype(np.float64)
    lo, hi = int(off[0]), int(off[-1])
    assert np.array_equal(got[lo:hi], ref[lo:hi])
    assert np.all(got[:lo] == -3.0) and np.all(got[hi:] == -3.0)
    assert torch.equal(tcr.irregular_scan_ex(xd, od, 0), tcr.irregular_scan(xd, od))


@pytest.mark.parametrize("in_shift,out_shift", [(1, 1), (3, 3), (7, 7), (5, 1), (0, 2), (4, 0), (6, 6)])
def test_unaligned_arrays(tcr, oracle, in_shift, out_shift):
    # views that start in_shift / out_shift elements into 16-byte aligned buffers: the tiles start at the aligned
    # boundary below `in`; equal shifts keep 128-bit stores, different ones store results one by one
    n = 3 * SCAN_TILE + 100
    base = workloads.make_input(n + 8, "int8", 70 + in_shift)
    x = base[in_shift:in_shift + n].copy()
    xd = torch.from_numpy(base).cuda()[in_shift:in_shift + n]
    assert xd.data_ptr() % 16 == (2 * in_shift) % 16
    for recipe in ("uniform16", "lognormal256", "few3"):
        off = workloads.make_offsets(n, recipe, in_shift).view(np.int64)
        od = torch.from_numpy(off).cuda()
        red = tcr.irregular_reduce(xd, od).cpu().numpy().astype(np.float64)
        assert np.array_equal(red, oracle.irregular_reduce(x, off)), recipe
        for flags in (0, 1, 2):
            dtype = torch.float16 if flags & 2 else torch.float32
            buf = torch.full((n + 16,), -3.0, dtype=dtype, device="cuda")
            out = buf[out_shift:out_shift + n]
            tcr.irregular_scan_ex(xd, od, flags, out=out)
            ref = oracle.irregular_scan_exclusive(x, off) if flags & 1 else oracle.irregular_scan(x, off)
            if flags & 2:
                ref = ref.astype(np.float16).astype(np.float64)
            got = buf.cpu().numpy().astype(np.float64)
            assert np.array_equal(got[out_shift:out_shift + n], ref), f"{recipe} flags={flags}"
            assert np.all(got[:out_shift] == -3.0) and np.all(got[out_shift + n:] == -3.0), f"{recipe} flags={flags}: wrote outside"
    # a partial cover behind an unaligned pointer
    off = np.array([3, 3, 40, SCAN_TILE + 5, n - 9], dtype=np.int64)
    od = torch.from_numpy(off).cuda()
    assert np.array_equal(tcr.irregular_reduce(xd, od).cpu().numpy().astype(np.float64), oracle.irregular_reduce(x, off))
    buf = torch.full((n + 16,), -3.0, dtype=torch.float32, device="cuda")
    tcr.irregular_scan(xd, od, out=buf[out_shift:out_shift + n])
    got = buf.cpu().numpy().astype(np.float64)[out_shift:out_shift + n]
    assert np.array_equal(got[3:n - 9], oracle.irregular_scan(x, off)[3:n - 9])
    assert np.all(got[:3] == -3.0) and np.all(got[n - 9:] == -3.0)


@pytest.mark.parametrize("seg", [1, 5, 16, 64, 100, 256, 1000, 4096, 32768, 40000, 1 << 17])
@pytest.mark.parametrize("in_shift,out_shift", [(1, 1), (5, 2), (0, 3), (4, 4)])
def test_regular_calls_behind_unaligned_pointers(tcr, oracle, seg, in_shift, out_shift):
    # the regular entry points accept views that are not 16-byte aligned: the tiled kernels run them
    nseg = max(3, (150000 // seg) | 1)
    n = seg * nseg
    base = workloads.make_input(n + 8, "int4", 80 + seg % 13)
    x = base[in_shift:in_shift + n].copy()
    xd = torch.from_numpy(base).cuda()[in_shift:in_shift + n]
    red = tcr.segmented_reduce(xd, seg).cpu().numpy().astype(np.float64)
    assert np.array_equal(red, oracle.segmented_reduce(x, seg))
    if in_shift:
        a, q = tcr.segmented_moments(xd, seg)
        ra, rq = oracle.segmented_moments(x, seg)
        assert np.array_equal(a.cpu().numpy().astype(np.float64), ra) and np.array_equal(q.cpu().numpy().astype(np.float64), rq)
        assert float(tcr.reduce(xd).cpu()[0]) == oracle.reduce(x)
    for flags in (0, 1, 3):
        dtype = torch.float16 if flags & 2 else torch.float32
        buf = torch.full((n + 16,), -3.0, dtype=dtype, device="cuda")
        tcr.segmented_scan_ex(xd, seg, flags, out=buf[out_shift:out_shift + n])
        ref = oracle.segmented_scan_exclusive(x, seg) if flags & 1 else oracle.segmented_scan(x, seg)
        if flags & 2:
            ref = ref.astype(np.float16).astype(np.float64)
        got = buf.cpu().numpy().astype(np.float64)
        assert np.array_equal(got[out_shift:out_shift + n], ref), f"flags={flags}"
        assert np.all(got[:out_shift] == -3.0) and np.all(got[out_shift + n:] == -3.0), f"flags={flags}: wrote outside"
    full = torch.full((n + 16,), -3.0, dtype=torch.float32, device="cuda")
    tcr.scan(xd, out=full[out_shift:out_shift + n])
    assert np.array_equal(full.cpu().numpy().astype(np.float64)[out_shift:out_shift + n], oracle.scan(x))


@pytest.mark.parametrize("recipe", ["uniform1", "uniform16", "uniform300", "lognormal256", "few5"])
@pytest.mark.parametrize("in_shift", [0, 3])
def test_irregular_moments(tcr, oracle, recipe, in_shift):
    n = 4 * SCAN_TILE + 200
    base = workloads.make_input(n + 8, "int1", 90)                 # |x| <= 1: the sums of squares stay below 2^24
    x = base[in_shift:in_shift + n].copy()
    xd = torch.from_numpy(base).cuda()[in_shift:in_shift + n]
    off = workloads.make_offsets(n - 50, recipe, 9).view(np.int64) + 20
    od = torch.from_numpy(off).cuda()
    a, q = tcr.irregular_moments(xd, od)
    ra, rq = oracle.irregular_moments(x, off)
    assert np.array_equal(a.cpu().numpy().astype(np.float64), ra) and np.array_equal(q.cpu().numpy().astype(np.float64), rq)
    assert torch.equal(a, tcr.irregular_reduce(xd, od))
    y = workloads.make_input(n, "normal", 7)
    a, q = tcr.irregular_moments(torch.from_numpy(y).cuda(), od)
    ra, rq = oracle.irregular_moments(y, off)
    assert np.all(np.abs(q.cpu().numpy().astype(np.float64) - rq) <= 1e-3 * rq)
    assert np.all(np.abs(a.cpu().numpy().astype(np.float64) - ra) <= 1e-3 * np.maximum(np.abs(ra), np.sqrt(rq)))


# ------------------------------------------------------------------ long segments: the two-kernel scan

@pytest.mark.parametrize("recipe", ["uniform16", "uniform1024", "uniform20000", "lognormal256", "few2", "few7", "few40"])
@pytest.mark.parametrize("n", [9 * SCAN_TILE + 1234, (1 << 20) + 8, 3 * SCAN_TILE - 3])
def test_two_kernel_scan_on_every_mix(tcr, oracle, recipe, n):
    # forced: the pipelined chain for the tiles without a segment start, a second kernel for the others -- also
    # on mixes where every tile holds starts and the chain has nothing to store
    off = workloads.make_offsets(n, recipe, (n % 1000, 9)).view(np.int64)
    tcr.set_variant("irregular_scan", "chain")
    try:
        _run(tcr, oracle, workloads.make_input(n, "int8", 15), off, True, f"chain {recipe} n={n} int8")
        _run(tcr, oracle, workloads.make_input(n, "uniform_pm1", 16), off, False, f"chain {recipe} n={n} uniform_pm1")
    finally:
        tcr.set_variant("reset")


@pytest.mark.parametrize("flags", [0, 1, 2, 3])
def test_two_kernel_scan_is_chosen_for_few_long_segments(tcr, oracle, flags):
    # 40 tiles, 7 segments: fewer segments than a quarter of the tiles; partial cover, starts on and next to tile
    # boundaries, an empty segment, every scan mode
    n = 40 * SCAN_TILE + 4000
    x = workloads.make_input(n, "int4", 17)
    off = np.array([5, SCAN_TILE, SCAN_TILE, 3 * SCAN_TILE + 1, 11 * SCAN_TILE - 1, 11 * SCAN_TILE + 8, 30 * SCAN_TILE + 777, n - 9], dtype=np.int64)
    xd, od = torch.from_numpy(x).cuda(), torch.from_numpy(off).cuda()
    fill = -3.0
    out = torch.full((n,), fill, dtype=torch.float16 if flags & 2 else torch.float32, device="cuda")
    tcr.irregular_scan_ex(xd, od, flags, out=out)
    got = out.cpu().numpy().astype(np.float64)
    ref = oracle.irregular_scan_exclusive(x, off) if flags & 1 else oracle.irregular_scan(x, off)
    if flags & 2:
        ref = ref.astype(np.float16).astype(np.float64)
    lo, hi = int(off[0]), int(off[-1])
    assert np.array_equal(got[lo:hi], ref[lo:hi])
    assert np.all(got[:lo] == fill) and np.all(got[hi:] == fill), "wrote outside the segments"
    # and the single-kernel form on the same input
    tcr.set_variant("irregular_scan", "single")
    try:
        out2 = torch.full_like(out, fill)
        tcr.irregular_scan_ex(xd, od, flags, out=out2)
    finally:
        tcr.set_variant("reset")
    assert torch.equal(out, out2)
    tcr.check_device_flags()
