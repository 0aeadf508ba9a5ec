"""Auto-tuner (Section 6 of the paper tunes algorithm, wavefronts per workgroup and coarsening per
segment size): every launch shape the tuner may choose gives the oracle's result, and tcr_autotune
leaves a valid choice behind."""
import numpy as np
import pytest
import torch

from paper_1811_09736_amd import workloads

pytestmark = pytest.mark.gpu

N = 1 << 22


@pytest.fixture(scope="module")
def tcr():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1811_09736_amd import binding
    binding.set_variant("reset")
    binding.tuning_import("")
    yield binding
    binding.tuning_import("")
    binding.check_device_flags()


@pytest.fixture(scope="module")
def data():
    x = workloads.make_input(N + 512 * 37 + 5, "int8", 11)          # integer valued: every shape must be bit exact
    return x, torch.from_numpy(x).cuda()


SCAN_SHAPE_TILES = [1024, 2048, 4096, 8192, 16384, 32768, 65536, 16384, 32768, 65536, 32768, 32768]
SCAN_SHAPE_TICKET = [False] * 7 + [True] * 5
SCAN_SHAPE_PERSISTENT = [False] * 10 + [True] * 2


@pytest.mark.parametrize("log2_seg", [10, 12, 14, 15, 16, 18, 20])
@pytest.mark.parametrize("shape", range(12))
def test_every_scan_shape_matches_oracle(tcr, oracle, data, log2_seg, shape):
    seg = 1 << log2_seg
    if not SCAN_SHAPE_TICKET[shape] and SCAN_SHAPE_TILES[shape] < seg:
        pytest.skip("a share without carry must hold the whole segment")
    if SCAN_SHAPE_PERSISTENT[shape] and SCAN_SHAPE_TILES[shape] > seg:
        pytest.skip("the pipelined shapes are for segments longer than a share")
    x, xd = data
    tcr.tuning_import(f"scan:{log2_seg}={shape};")
    try:
        got = tcr.segmented_scan(xd[:N], seg).cpu().numpy().astype(np.float64)
    finally:
        tcr.tuning_import("")
    assert np.array_equal(got, oracle.segmented_scan(x[:N], seg))
    tcr.check_device_flags()


@pytest.mark.parametrize("drop", [0, 5, 1549, 18949, 58949])
@pytest.mark.parametrize("shape", [7, 8, 9, 10, 11])
def test_every_full_scan_shape_matches_oracle(tcr, oracle, data, shape, drop):
    # ragged n: not a multiple of 8 (the pipelined shapes then fall back), a multiple of 8 inside a
    # wavefront's share, and a last tile that holds only a few wavefront shares
    x, xd = data
    x, xd = x[:x.size - drop], xd[:xd.numel() - drop]
    tcr.tuning_import(f"scan:41={shape};")
    try:
        if shape >= 10:
            assert (tcr.kernel_name(tcr.OP_SCAN, x.size, x.size) == "scan_chain_kernel<mfma>") == (x.size % 8 == 0)
        got = tcr.scan(xd).cpu().numpy().astype(np.float64)
    finally:
        tcr.tuning_import("")
    ref = oracle.scan(x)
    assert np.max(np.abs(ref)) < 2 ** 24
    assert np.array_equal(got, ref)
    tcr.check_device_flags()


@pytest.mark.parametrize("log2_seg", [10, 13, 14, 16, 17, 20])
@pytest.mark.parametrize("shape", range(4))
def test_every_reduce_shape_matches_oracle(tcr, oracle, data, log2_seg, shape):
    seg = 1 << log2_seg
    x, xd = data
    tcr.tuning_import(f"reduce:{log2_seg}={shape};")                     # ids beyond the candidate list fall back to 0
    try:
        got = tcr.segmented_reduce(xd[:N], seg).cpu().numpy().astype(np.float64)
    finally:
        tcr.tuning_import("")
    assert np.array_equal(got, oracle.segmented_reduce(x[:N], seg))


@pytest.mark.parametrize("shape", range(4))
def test_every_full_reduce_shape_matches_oracle(tcr, oracle, data, shape):
    x, xd = data
    tcr.tuning_import(f"reduce:41={shape};")
    try:
        got = float(tcr.reduce(xd).cpu())
    finally:
        tcr.tuning_import("")
    assert got == oracle.reduce(x)


# ------------------------------------------------------------------ the wider search space

@pytest.mark.parametrize("form", [0, 32])
@pytest.mark.parametrize("shape", range(4))
@pytest.mark.parametrize("log2_seg", [4, 5, 6, 9])
def test_every_small_segment_shape_and_formulation_matches_oracle(tcr, oracle, data, log2_seg, shape, form):
    seg = 1 << log2_seg
    x, xd = data
    n = N + 512 * 37                                           # a ragged last workgroup for every shape
    tcr.tuning_import(f"scan:{log2_seg}={shape + form};reduce:{log2_seg}={shape + form};")
    try:
        want = "dpp" if form else "mfma"
        assert tcr.kernel_name(tcr.OP_SEGMENTED_SCAN, n, seg) == f"scan_small_kernel<{want}>"
        assert tcr.kernel_name(tcr.OP_SEGMENTED_REDUCE, n, seg) == f"reduce_small_kernel<{want}>"
        scan = tcr.segmented_scan(xd[:n], seg).cpu().numpy().astype(np.float64)
        red = tcr.segmented_reduce(xd[:n], seg).cpu().numpy().astype(np.float64)
        excl = tcr.segmented_scan_ex(xd[:n], seg, 1).cpu().numpy().astype(np.float64)     # the other modes stay on the matrix cores
    finally:
        tcr.tuning_import("")
    assert np.array_equal(scan, oracle.segmented_scan(x[:n], seg))
    assert np.array_equal(red, oracle.segmented_reduce(x[:n], seg))
    assert np.array_equal(excl, oracle.segmented_scan_exclusive(x[:n], seg))


@pytest.mark.parametrize("value", [12, 13, 32 + 12, 32 + 13, 32 + 7, 32 + 9, 32 + 10, 32 + 11])
@pytest.mark.parametrize("log2_seg", [17, 20, 41])
def test_carry_strategies_and_formulations_as_tuned_choices(tcr, oracle, data, log2_seg, value):
    x, xd = data
    seg = N if log2_seg == 41 else 1 << log2_seg
    tcr.tuning_import(f"scan:{log2_seg}={value};reduce:{log2_seg}={32 if value >= 32 else 0};")
    try:
        name = tcr.kernel_name(tcr.OP_SEGMENTED_SCAN, N, seg)
        assert ("dpp" in name) == (value >= 32)
        if value % 32 == 12:
            assert name.startswith("reduce_span_kernel+scan_partials_kernel+")
        if value % 32 == 13:
            assert name.endswith("+uniform_add_kernel")
        scan = tcr.segmented_scan(xd[:N], seg).cpu().numpy().astype(np.float64)
        red = tcr.segmented_reduce(xd[:N], seg).cpu().numpy().astype(np.float64)
        f16 = tcr.segmented_scan_ex(xd[:N], seg, 2).cpu().numpy().astype(np.float64)    # no three-kernel form: falls back
    finally:
        tcr.tuning_import("")
    ref = oracle.segmented_scan(x[:N], seg)
    assert np.array_equal(scan, ref)
    assert np.array_equal(red, oracle.segmented_reduce(x[:N], seg))
    assert np.array_equal(f16, ref.astype(np.float16).astype(np.float64))
    tcr.check_device_flags()


@pytest.mark.parametrize("choice", range(6))
@pytest.mark.parametrize("seg", [12, 24, 100, 520, 999, 3000, 3001, 40000, 3 << 16, 100003])
def test_every_kernel_for_other_lengths_matches_oracle(tcr, oracle, seg, choice):
    nseg = max(3, (300000 // seg) | 1)
    x = workloads.make_input(seg * nseg, "int4", seg % 89)
    xd = torch.from_numpy(x).cuda()
    cls = seg.bit_length() - 1
    tcr.tuning_import(f"scan_any:{cls}={choice % 4};reduce_any:{cls}={choice};")          # (four kernels for scans, six for reductions)
    try:
        names = (tcr.kernel_name(tcr.OP_SEGMENTED_SCAN, x.size, seg), tcr.kernel_name(tcr.OP_SEGMENTED_REDUCE, x.size, seg))
        scan = tcr.segmented_scan(xd, seg).cpu().numpy().astype(np.float64)
        red = tcr.segmented_reduce(xd, seg).cpu().numpy().astype(np.float64)
        excl16 = tcr.segmented_scan_ex(xd, seg, 3).cpu().numpy().astype(np.float64)
    finally:
        tcr.tuning_import("")
    assert np.array_equal(scan, oracle.segmented_scan(x, seg)), names
    assert np.array_equal(red, oracle.segmented_reduce(x, seg)), names
    assert np.array_equal(excl16, oracle.segmented_scan_exclusive(x, seg).astype(np.float16).astype(np.float64)), names
    tcr.check_device_flags()


@pytest.mark.parametrize("recipe", ["uniform16", "lognormal256", "few7"])
@pytest.mark.parametrize("reduce_shape,scan_shape", [(0, 0), (1, 1), (2, 1)])
def test_every_irregular_tile_shape_matches_oracle(tcr, oracle, recipe, reduce_shape, scan_shape):
    n = (1 << 20) + 4321
    x = workloads.make_input(n, "int8", 13)
    off = workloads.make_offsets(n, recipe, 3).view(np.int64)
    xd, od = torch.from_numpy(x).cuda(), torch.from_numpy(off).cuda()
    tcr.tuning_import(f"irregular:0={reduce_shape};irregular:1={scan_shape};")
    try:
        red = tcr.irregular_reduce(xd, od).cpu().numpy().astype(np.float64)
        scan = tcr.irregular_scan(xd, od).cpu().numpy().astype(np.float64)
        a, q = tcr.irregular_moments(xd, od)
        excl = tcr.irregular_scan_ex(xd, od, 1).cpu().numpy().astype(np.float64)
    finally:
        tcr.tuning_import("")
    assert np.array_equal(red, oracle.irregular_reduce(x, off))
    lo, hi = int(off[0]), int(off[-1])
    assert np.array_equal(scan[lo:hi], oracle.irregular_scan(x, off)[lo:hi])
    assert np.array_equal(excl[lo:hi], oracle.irregular_scan_exclusive(x, off)[lo:hi])
    ra, rq = oracle.irregular_moments(x, off)
    assert np.array_equal(a.cpu().numpy().astype(np.float64), ra) and np.array_equal(q.cpu().numpy().astype(np.float64), rq)
    tcr.check_device_flags()


def test_autotune_searches_every_class(tcr, oracle, data):
    x, xd = data
    out = torch.empty(N, dtype=torch.float32, device="cuda")
    off = workloads.make_offsets(N, "lognormal256", 3).view(np.int64)
    od = torch.from_numpy(off).cuda()
    n100 = (N // 100) * 100
    n3k = (N // 3000) * 3000
    try:
        tcr.autotune(tcr.OP_SEGMENTED_SCAN, xd[:N], out, 64)
        tcr.autotune(tcr.OP_SEGMENTED_REDUCE, xd[:N], out, 64)
        tcr.autotune(tcr.OP_SEGMENTED_SCAN, xd[:n100], out, 100)
        tcr.autotune(tcr.OP_SEGMENTED_REDUCE, xd[:n100], out, 100)
        tcr.autotune(tcr.OP_SEGMENTED_SCAN, xd[:n3k], out, 3000)
        n6 = (N // 6) * 6
        tcr.autotune(tcr.OP_SEGMENTED_REDUCE, xd[:n6], out, 6)
        tcr.autotune_irregular(tcr.OP_IRREGULAR_REDUCE, xd[:N], od, out)
        tcr.autotune_irregular(tcr.OP_IRREGULAR_SCAN, xd[:N], od, out)
        tcr.autotune(tcr.OP_SEGMENTED_SCAN, xd[:N], out, 4)              # a single kernel: no entry
        table = dict(item.split("=") for item in tcr.tuning_export().split(";") if item)
        assert set(table) == {"scan:6", "reduce:6", "scan_any:6", "reduce_any:6", "reduce_any:2", "scan_any:11", "irregular:0", "irregular:1"}
        assert int(table["reduce_any:2"]) in (1, 2, 4, 5)                # rows of whole segments or tiles, two shapes each
        assert np.array_equal(tcr.segmented_reduce(xd[:n6], 6).cpu().numpy().astype(np.float64), oracle.segmented_reduce(x[:n6], 6))
        assert int(table["scan:6"]) % 32 in range(4) and int(table["reduce:6"]) % 32 in range(4)
        assert int(table["reduce_any:6"]) in (0, 1, 2)                   # rows or tiles; the masked tiles start at 256
        assert int(table["scan_any:11"]) in (0, 1, 2)                    # tiles or one workgroup per segment
        assert np.array_equal(tcr.segmented_scan(xd[:N], 64).cpu().numpy().astype(np.float64), oracle.segmented_scan(x[:N], 64))
        assert np.array_equal(tcr.segmented_reduce(xd[:N], 64).cpu().numpy().astype(np.float64), oracle.segmented_reduce(x[:N], 64))
        assert np.array_equal(tcr.segmented_scan(xd[:n100], 100).cpu().numpy().astype(np.float64), oracle.segmented_scan(x[:n100], 100))
        assert np.array_equal(tcr.segmented_reduce(xd[:n100], 100).cpu().numpy().astype(np.float64), oracle.segmented_reduce(x[:n100], 100))
        assert np.array_equal(tcr.segmented_scan(xd[:n3k], 3000).cpu().numpy().astype(np.float64), oracle.segmented_scan(x[:n3k], 3000))
        assert np.array_equal(tcr.irregular_reduce(xd[:N], od).cpu().numpy().astype(np.float64), oracle.irregular_reduce(x[:N], off))
        assert np.array_equal(tcr.irregular_scan(xd[:N], od).cpu().numpy().astype(np.float64), oracle.irregular_scan(x[:N], off))
        tcr.check_device_flags()
    finally:
        tcr.tuning_import("")


def test_autotune_picks_valid_shapes_and_results_stay_exact(tcr, oracle, data):
    x, xd = data
    out = torch.empty(N, dtype=torch.float32, device="cuda")
    try:
        tcr.autotune(tcr.OP_SEGMENTED_SCAN, xd[:N], out, 1 << 14)
        tcr.autotune(tcr.OP_SEGMENTED_REDUCE, xd[:N], out, 1 << 14)
        tcr.autotune(tcr.OP_SCAN, xd[:N], out, 0)
        tcr.autotune(tcr.OP_REDUCE, xd[:N], out, 0)
        tcr.autotune(tcr.OP_SEGMENTED_SCAN, xd[:N], out, 8)              # a single kernel: no entry
        table = dict(item.split("=") for item in tcr.tuning_export().split(";") if item)
        assert set(table) == {"scan:14", "reduce:14", "scan:41", "reduce:41"}
        assert int(table["scan:14"]) % 32 in range(4, 10)                # shares that hold a 16384-element segment
        assert int(table["scan:41"]) % 32 in (7, 8, 9, 10, 11, 12, 13)
        assert np.array_equal(tcr.segmented_scan(xd[:N], 1 << 14).cpu().numpy().astype(np.float64),
                              oracle.segmented_scan(x[:N], 1 << 14))
        assert np.array_equal(tcr.segmented_reduce(xd[:N], 1 << 14).cpu().numpy().astype(np.float64),
                              oracle.segmented_reduce(x[:N], 1 << 14))
        assert np.array_equal(tcr.scan(xd[:N]).cpu().numpy().astype(np.float64), oracle.scan(x[:N]))
        assert float(tcr.reduce(xd[:N]).cpu()) == oracle.reduce(x[:N])
        tcr.check_device_flags()
    finally:
        tcr.tuning_import("")
