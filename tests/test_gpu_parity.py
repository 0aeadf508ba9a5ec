"""Parity of the HIP library (through its C ABI) with the CPU oracle, element by element.

Bar: integer-valued inputs -> the binary32 outputs equal the oracle's binary64 values
exactly; real-valued inputs -> |y - ref| <= 1e-3 * max(|ref|, rho) per output, where rho is
the root-sum-square of the inputs that output adds up (the natural scale of a zero-mean sum;
for the smallest outputs of zero-mean data a pure relative error is unbounded).
"""
import numpy as np
import pytest
import torch

from paper_1811_09736_amd import workloads

pytestmark = pytest.mark.gpu

REL_TOL = 1e-3


@pytest.fixture(scope="module")
def tcr():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1811_09736_amd import binding      # fails loudly if libtcr.so is missing
    binding.set_variant("reset")
    yield binding
    binding.set_variant("reset")
    binding.check_device_flags()


@pytest.fixture(params=["mfma", "dpp"])
def form(request, tcr):
    tcr.set_variant("formulation", request.param)
    yield request.param
    tcr.set_variant("reset")


def dev(x: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(x).cuda()


def assert_exact(got: torch.Tensor, ref: np.ndarray, what: str):
    g = got.cpu().numpy().astype(np.float64)
    if not np.array_equal(g, ref):
        bad = np.flatnonzero(g != ref)
        raise AssertionError(f"{what}: {bad.size} mismatches, first at {bad[0]}: got {g[bad[0]]!r} want {ref[bad[0]]!r}")


def assert_close_scan(got: torch.Tensor, ref: np.ndarray, x: np.ndarray, seg: int, what: str):
    g = got.cpu().numpy().astype(np.float64)
    x64 = x.astype(np.float64)
    rho = np.sqrt(np.cumsum((x64 * x64).reshape(-1, seg), axis=1)).reshape(-1)
    tol = REL_TOL * np.maximum(np.abs(ref), rho)
    err = np.abs(g - ref)
    if not np.all(err <= tol):
        bad = int(np.argmax(err - tol))
        raise AssertionError(f"{what}: worst at {bad}: got {g[bad]!r} want {ref[bad]!r} tol {tol[bad]!r}")


def assert_close_reduce(got: torch.Tensor, ref: np.ndarray, x: np.ndarray, seg: int, what: str):
    g = got.cpu().numpy().astype(np.float64)
    x64 = x.astype(np.float64)
    rho = np.sqrt((x64 * x64).reshape(-1, seg).sum(axis=1))
    tol = REL_TOL * np.maximum(np.abs(ref), rho)
    err = np.abs(g - ref)
    if not np.all(err <= tol):
        bad = int(np.argmax(err - tol))
        raise AssertionError(f"{what}: worst at segment {bad}: got {g[bad]!r} want {ref[bad]!r} tol {tol[bad]!r}")


def ragged_n(seg: int) -> int:
    """A few workgroup shares (8192 elements each) plus a tail that fills neither a workgroup nor,
    for short segments, a 512-element tile."""
    whole = 3 * 8192
    tail_segments = 3 if seg <= 512 else 1
    return (whole // seg + tail_segments) * seg if seg <= 8192 else 3 * seg


SMALL_SEGS = [16, 32, 64, 128, 256, 512]
LONG_SEGS = [1024, 2048, 4096, 8192, 16384, 32768, 1 << 16, 1 << 17, 1 << 18, 1 << 20, 1 << 21]


# ------------------------------------------------------------------ segmented, moderate sizes

@pytest.mark.parametrize("seg", SMALL_SEGS + LONG_SEGS)
def test_segmented_exact(tcr, oracle, form, seg):
    n = ragged_n(seg)
    x = workloads.make_input(n, "int8", 40 + seg % 97)
    xd = dev(x)
    assert_exact(tcr.segmented_scan(xd, seg), oracle.segmented_scan(x, seg), f"scan L={seg} n={n} {form}")
    assert_exact(tcr.segmented_reduce(xd, seg), oracle.segmented_reduce(x, seg), f"reduce L={seg} n={n} {form}")


@pytest.mark.parametrize("seg", SMALL_SEGS + LONG_SEGS)
@pytest.mark.parametrize("dist", ["uniform_pm1", "uniform_01"])
def test_segmented_real(tcr, oracle, form, seg, dist):
    n = ragged_n(seg)
    x = workloads.make_input(n, dist, 7)
    xd = dev(x)
    assert_close_scan(tcr.segmented_scan(xd, seg), oracle.segmented_scan(x, seg), x, seg, f"scan L={seg} {dist} {form}")
    assert_close_reduce(tcr.segmented_reduce(xd, seg), oracle.segmented_reduce(x, seg), x, seg,
                        f"reduce L={seg} {dist} {form}")


@pytest.mark.parametrize("seg", [16, 64, 512, 1024, 1 << 15])
def test_single_segment_and_tiny_inputs(tcr, oracle, form, seg):
    for nseg in (1, 2, 5):
        x = workloads.make_input(seg * nseg, "int4", nseg)
        xd = dev(x)
        assert_exact(tcr.segmented_scan(xd, seg), oracle.segmented_scan(x, seg), f"scan L={seg} x{nseg}")
        assert_exact(tcr.segmented_reduce(xd, seg), oracle.segmented_reduce(x, seg), f"reduce L={seg} x{nseg}")


# ------------------------------------------------------------------ segment lengths without a tuned path

GENERIC_SEGS = [1, 2, 3, 4, 5, 7, 8, 12, 15, 17, 24, 48, 96, 97, 100, 127, 129, 255, 257, 264, 511, 513, 520, 1000, 1536,
                3000, 4097, 10000, 3 << 15]


@pytest.mark.parametrize("seg", GENERIC_SEGS)
def test_any_segment_length(tcr, oracle, seg):
    nseg = max(3, (40000 // seg) | 1)                 # odd counts: segments start at odd offsets for odd seg
    n = seg * nseg
    x = workloads.make_input(n, "int8", 300 + seg % 91)
    xd = dev(x)
    assert_exact(tcr.segmented_scan(xd, seg), oracle.segmented_scan(x, seg), f"scan L={seg} n={n}")
    assert_exact(tcr.segmented_reduce(xd, seg), oracle.segmented_reduce(x, seg), f"reduce L={seg} n={n}")
    y = workloads.make_input(n, "uniform_pm1", 17)
    yd = dev(y)
    assert_close_scan(tcr.segmented_scan(yd, seg), oracle.segmented_scan(y, seg), y, seg, f"scan L={seg} real")
    assert_close_reduce(tcr.segmented_reduce(yd, seg), oracle.segmented_reduce(y, seg), y, seg, f"reduce L={seg} real")


# ------------------------------------------------------------------ full operations, any n

FULL_NS = [1, 2, 7, 8, 9, 15, 16, 17, 511, 512, 513, 1000, 4095, 8191, 8192, 8193, 16384, 16385,
           100003, (1 << 20) + 5, 3 * (1 << 20) - 1]


@pytest.mark.parametrize("n", FULL_NS)
def test_full_exact_any_n(tcr, oracle, form, n):
    x = workloads.make_input(n, "int4", n % 1000)
    xd = dev(x)
    assert_exact(tcr.scan(xd), oracle.scan(x), f"scan n={n} {form}")
    assert float(tcr.reduce(xd).cpu()[0]) == oracle.reduce(x), f"reduce n={n} {form}"
    # the segmented entry points with one segment are the full operations
    assert_exact(tcr.segmented_scan(xd, n), oracle.scan(x), f"segmented_scan L=n={n}")
    assert float(tcr.segmented_reduce(xd, n).cpu()[0]) == oracle.reduce(x)


@pytest.mark.parametrize("n", [1000, 8193, 100003, (1 << 20) + 5])
def test_full_real_any_n(tcr, oracle, form, n):
    x = workloads.make_input(n, "normal", 2)
    xd = dev(x)
    assert_close_scan(tcr.scan(xd), oracle.scan(x), x, n, f"scan n={n} {form}")
    assert_close_reduce(tcr.reduce(xd), np.array([oracle.reduce(x)]), x, n, f"reduce n={n} {form}")


def test_empty_inputs(tcr):
    e = torch.empty(0, dtype=torch.float16, device="cuda")
    assert tcr.scan(e).numel() == 0
    assert tcr.segmented_scan(e, 16).numel() == 0
    assert tcr.segmented_reduce(e, 16).numel() == 0
    out = torch.full((1,), 7.0, dtype=torch.float32, device="cuda")
    tcr.reduce(e, out=out)
    assert float(out.cpu()[0]) == 0.0


# ------------------------------------------------------------------ closed forms and invariants on the device

@pytest.mark.parametrize("seg", [16, 256, 4096, 1 << 16, 1 << 22])
def test_all_ones_closed_form(tcr, form, seg):
    n = max(seg, 1 << 18)
    xd = torch.ones(n, dtype=torch.float16, device="cuda")
    scan = tcr.segmented_scan(xd, seg).cpu().numpy()
    assert np.array_equal(scan, (np.arange(n) % seg + 1).astype(np.float32))      # < 2^24: exact in binary32
    assert np.array_equal(tcr.segmented_reduce(xd, seg).cpu().numpy(), np.full(n // seg, float(seg), np.float32))


@pytest.mark.parametrize("m", [16, 512, 2048])
def test_ramp_closed_form(tcr, form, m):
    ramp = np.arange(1, m + 1, dtype=np.float64)
    x = np.tile(ramp, 24).astype(np.float16)
    xd = dev(x)
    assert np.array_equal(tcr.segmented_reduce(xd, m).cpu().numpy().astype(np.float64), np.full(24, m * (m + 1) / 2.0))
    assert np.array_equal(tcr.segmented_scan(xd, m).cpu().numpy().astype(np.float64), np.tile(ramp * (ramp + 1) / 2, 24))


@pytest.mark.parametrize("seg", [16, 128, 512, 2048, 1 << 15])
def test_subnormal_inputs_are_not_flushed(tcr, oracle, form, seg):
    # sums of binary16 subnormals are small multiples of 2^-24: exact in binary32 unless inputs are flushed to zero
    n = ragged_n(seg)
    x = workloads.make_input(n, "subnormal", 9)
    xd = dev(x)
    assert_exact(tcr.segmented_scan(xd, seg), oracle.segmented_scan(x, seg), f"subnormal scan L={seg}")
    assert_exact(tcr.segmented_reduce(xd, seg), oracle.segmented_reduce(x, seg), f"subnormal reduce L={seg}")


@pytest.mark.parametrize("seg", [64, 1024, 1 << 17])
def test_last_scan_element_is_the_reduction(tcr, form, seg):
    x = workloads.make_input(4 * max(seg, 8192), "int8", 12)
    xd = dev(x)
    scan = tcr.segmented_scan(xd, seg)
    red = tcr.segmented_reduce(xd, seg)
    assert torch.equal(scan[seg - 1:: seg], red)
    # first differences give back the input
    d = torch.diff(scan.view(-1, seg), dim=1)
    assert torch.equal(d, xd.view(-1, seg)[:, 1:].float())


# ------------------------------------------------------------------ cross-workgroup carry

@pytest.mark.parametrize("carry", ["lookback", "reduce_then_scan", "scan_then_propagate"])
def test_carry_strategies_agree_with_oracle(tcr, oracle, form, carry):
    tcr.set_variant("scan_carry", carry)
    for n, seg in (((1 << 21) + 12345, None), (1 << 21, 1 << 16), (3 << 19, 1 << 19)):
        x = workloads.make_input(n, "int8", 77)
        xd = dev(x)
        if seg is None:
            assert_exact(tcr.scan(xd), oracle.scan(x), f"scan n={n} {carry} {form}")
        else:
            assert_exact(tcr.segmented_scan(xd, seg), oracle.segmented_scan(x, seg), f"scan L={seg} {carry} {form}")


def test_lookback_repeated_launches(tcr, oracle):
    # many back-to-back launches reuse the descriptor table through its epoch tag and the running
    # ticket counter; any early or lost carry shows up as a wrong integer
    n = (1 << 22) + 777
    x = workloads.make_input(n, "int8", 5)
    xd = dev(x)
    ref = torch.from_numpy(oracle.scan(x).astype(np.float32)).cuda()
    outs = [torch.empty(n, dtype=torch.float32, device="cuda") for _ in range(4)]
    for it in range(100):
        tcr.scan(xd, out=outs[it % 4])
        if it % 4 == 3:
            for o in outs:
                assert torch.equal(o, ref), f"iteration {it}"
    # interleave a differently shaped problem on the same stream
    y = workloads.make_input(1 << 20, "int4", 6)
    yd = dev(y)
    yref = oracle.segmented_scan(y, 1 << 18)
    for it in range(10):
        a = tcr.segmented_scan(yd, 1 << 18)
        b = tcr.scan(xd)
        assert_exact(a, yref, "interleaved segmented scan")
        assert torch.equal(b, ref)
    tcr.check_device_flags()


# tile counts of the persistent chain (32768-element tiles, one workgroup per compute unit, three tiles in
# flight per workgroup): fewer tiles than pipeline stages, a ragged last tile that holds a few or nearly all
# wavefront shares, exactly / one more than / far more tiles than workgroups
CHAIN_NS = [8, 4096 + 8, 32768 - 8, 32768, 32768 + 8, 65536, 3 * 32768 + 40, 255 * 32768, 256 * 32768 + 8,
            257 * 32768, 300 * 32768 - 32760, 700 * 32768 + 512 * 9]


@pytest.mark.parametrize("n", CHAIN_NS)
def test_pipelined_chain_tile_counts(tcr, oracle, n):
    tcr.set_variant("reset")
    assert tcr.kernel_name(tcr.OP_SCAN, n, n) in ("scan_chain_kernel<mfma>", "scan_block_kernel<mfma,nocarry>")
    x = workloads.make_input(n, "int4", n % 997)
    xd = dev(x)
    ref = oracle.scan(x)
    assert np.max(np.abs(ref)) < 2 ** 24
    assert_exact(tcr.scan(xd), ref, f"scan n={n}")
    assert_exact(tcr.scan_ex(xd, tcr.SCAN_EXCLUSIVE), ref - x.astype(np.float64), f"exclusive scan n={n}")
    tcr.check_device_flags()


@pytest.mark.parametrize("seg", [1 << 15, 1 << 16, 1 << 19])
def test_pipelined_chain_segmented(tcr, oracle, seg):
    # more tiles than workgroups, segments of 1, 2 and 16 tiles: the carry restarts at every segment
    tcr.set_variant("reset")
    n = max(300 * 32768 // seg, 3) * seg
    assert tcr.kernel_name(tcr.OP_SEGMENTED_SCAN, n, seg) == "scan_chain_kernel<mfma>"
    x = workloads.make_input(n, "int8", seg % 991)
    xd = dev(x)
    assert_exact(tcr.segmented_scan(xd, seg), oracle.segmented_scan(x, seg), f"segmented scan L={seg}")
    y = workloads.make_input(n, "uniform_pm1", 17)
    assert_close_scan(tcr.segmented_scan(dev(y), seg), oracle.segmented_scan(y, seg), y, seg, f"scan L={seg} real")
    tcr.check_device_flags()


@pytest.mark.parametrize("seg", [65536 + 8, 100000, 3 << 16, (3 << 20) + 4096, 1000000])
def test_long_segments_of_any_length(tcr, oracle, seg):
    # no power of two: the chain runs on a per-segment tile grid whose last tile overhangs the segment's end;
    # reductions add 65536-element pieces of every segment
    tcr.set_variant("reset")
    nseg = max(3, (9 << 20) // seg)
    n = seg * nseg
    assert tcr.kernel_name(tcr.OP_SEGMENTED_SCAN, n, seg) == "scan_chain_kernel<mfma>"
    x = workloads.make_input(n, "int8", seg % 983)
    xd = dev(x)
    ref = oracle.segmented_scan(x, seg)
    assert_exact(tcr.segmented_scan(xd, seg), ref, f"scan L={seg}")
    assert_exact(tcr.segmented_scan_ex(xd, seg, tcr.SCAN_EXCLUSIVE), ref - x.astype(np.float64), f"exclusive scan L={seg}")
    got16 = tcr.segmented_scan_ex(xd, seg, tcr.OUT_F16).cpu().numpy().astype(np.float64)
    assert np.array_equal(got16, ref.astype(np.float16).astype(np.float64))
    assert_exact(tcr.segmented_reduce(xd, seg), oracle.segmented_reduce(x, seg), f"reduce L={seg}")
    y = workloads.make_input(n, "uniform_pm1", 19)
    yd = dev(y)
    assert_close_scan(tcr.segmented_scan(yd, seg), oracle.segmented_scan(y, seg), y, seg, f"scan L={seg} real")
    assert_close_reduce(tcr.segmented_reduce(yd, seg), oracle.segmented_reduce(y, seg), y, seg, f"reduce L={seg} real")
    tcr.check_device_flags()


def test_pipelined_chain_repeated_launches(tcr, oracle):
    # back-to-back launches share the aggregate table (epoch tag) and the running ticket counter, of which
    # every launch draws tiles + 3 * workgroups; a lost or early carry shows up as a wrong integer
    tcr.set_variant("reset")
    n = (1 << 22) + 776
    assert tcr.kernel_name(tcr.OP_SCAN, n, n) == "scan_chain_kernel<mfma>"
    x = workloads.make_input(n, "int8", 5)
    xd = dev(x)
    ref = torch.from_numpy(oracle.scan(x).astype(np.float32)).cuda()
    y = workloads.make_input(1 << 21, "int4", 6)
    yd = dev(y)
    yref = torch.from_numpy(oracle.segmented_scan(y, 1 << 17).astype(np.float32)).cuda()
    outs = [torch.empty(n, dtype=torch.float32, device="cuda") for _ in range(4)]
    youts = [torch.empty(1 << 21, dtype=torch.float32, device="cuda") for _ in range(4)]
    for it in range(200):
        tcr.scan(xd, out=outs[it % 4])
        tcr.segmented_scan(yd, 1 << 17, out=youts[it % 4])
        if it % 4 == 3:
            for o in outs:
                assert torch.equal(o, ref), f"iteration {it}"
            for o in youts:
                assert torch.equal(o, yref), f"iteration {it}"
    # alternate with the look-back kernels on the same table (n not a multiple of 8)
    for it in range(10):
        a = tcr.scan(xd[: n - 3])
        b = tcr.scan(xd)
        assert torch.equal(a, ref[: n - 3]) and torch.equal(b, ref)
    tcr.check_device_flags()


def test_non_default_stream(tcr, oracle):
    x = workloads.make_input((1 << 20) + 24, "int8", 8)
    xd = dev(x)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        scan = tcr.scan(xd, stream=s)
        red = tcr.segmented_reduce(xd[: 1 << 20], 1 << 18, stream=s)
    s.synchronize()
    assert_exact(scan, oracle.scan(x), "scan on a side stream")
    assert_exact(red, oracle.segmented_reduce(np.ascontiguousarray(x[: 1 << 20]), 1 << 18), "reduce on a side stream")
    tcr.check_device_flags(s)


# ------------------------------------------------------------------ C ABI error paths on a live device

def test_errors_on_device(tcr):
    x = torch.zeros(4096 + 8, dtype=torch.float16, device="cuda")
    out = torch.zeros(4096 + 8, dtype=torch.float32, device="cuda")
    raw = tcr.raw()
    assert raw.tcr_segmented_scan(x.data_ptr(), out.data_ptr(), 4096, 48, None) == tcr.ERR_INVALID_ARG   # 48 does not divide 4096
    assert raw.tcr_segmented_scan(x.data_ptr() + 1, out.data_ptr(), 4096, 16, None) == tcr.ERR_INVALID_ARG   # odd address
    assert raw.tcr_scan(x.data_ptr(), out.data_ptr() + 2, 4096, None) == tcr.ERR_INVALID_ARG                 # floats at 2 mod 4
    assert raw.tcr_segmented_scan(x.data_ptr() + 2, out.data_ptr(), 4096, 16, None) == tcr.OK                # natural alignment
    assert raw.tcr_scan(x.data_ptr(), out.data_ptr() + 4, 4096, None) == tcr.OK
    with pytest.raises(TypeError):
        tcr.scan(x.float())
    with pytest.raises(tcr.TcrError):
        tcr.segmented_reduce(x[:4096], 100)
    torch.cuda.synchronize()


# ------------------------------------------------------------------ workspace life cycle and concurrency

def test_two_streams_run_chained_scans_concurrently(tcr, oracle):
    # each (device, stream) pair owns its look-back table and ticket counter, so chained scans issued on two
    # streams at the same time must not disturb each other
    n = (1 << 22) + 4096
    x = workloads.make_input(n, "int8", 21)
    y = workloads.make_input(n, "int4", 22)
    xd, yd = dev(x), dev(y)
    xref = torch.from_numpy(oracle.scan(x).astype(np.float32)).cuda()
    yref = torch.from_numpy(oracle.segmented_scan(y[: 1 << 22], 1 << 20).astype(np.float32)).cuda()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    outs1 = [torch.empty(n, dtype=torch.float32, device="cuda") for _ in range(3)]
    outs2 = [torch.empty(1 << 22, dtype=torch.float32, device="cuda") for _ in range(3)]
    for it in range(60):
        tcr.scan(xd, out=outs1[it % 3], stream=s1)
        tcr.segmented_scan(yd[: 1 << 22], 1 << 20, out=outs2[it % 3], stream=s2)
    s1.synchronize()
    s2.synchronize()
    for o in outs1:
        assert torch.equal(o, xref)
    for o in outs2:
        assert torch.equal(o, yref)
    tcr.check_device_flags(s1)
    tcr.check_device_flags(s2)


def test_workspace_grows_shrinks_and_survives_release(tcr, oracle):
    small = workloads.make_input((1 << 18) + 8, "int8", 31)
    large = workloads.make_input((1 << 24) + 8, "int8", 32)
    sd, ld = dev(small), dev(large)
    sref, lref = oracle.scan(small), oracle.scan(large)
    for _ in range(2):
        assert_exact(tcr.scan(sd), sref, "small before growth")
        assert_exact(tcr.scan(ld), lref, "large (table grows)")
        assert_exact(tcr.scan(sd), sref, "small after growth")
        assert float(tcr.reduce(ld).cpu()[0]) == oracle.reduce(large)
        torch.cuda.synchronize()
        tcr.release()                                   # next round starts from a released library
    tcr.check_device_flags()


def test_streams_that_come_and_go_release_their_workspaces(tcr, oracle):
    # one library-owned workspace per (device, stream): a caller that creates streams freely drops each one's
    x = workloads.make_input((1 << 19) + 8, "int8", 33)
    xd = dev(x)
    ref = oracle.scan(x)
    out = torch.empty(x.size, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    for _ in range(8):
        st = torch.cuda.Stream()
        tcr.scan(xd, out=out, stream=st)
        st.synchronize()
        assert_exact(out, ref, "scan on a fresh stream")
        tcr.release_stream(st)
        tcr.release_stream(st)                          # nothing left: a no-op
    tcr.scan(xd, out=out)                               # the default stream's workspace is untouched
    assert_exact(out, ref, "default stream afterwards")
    tcr.check_device_flags()


@pytest.mark.parametrize("finish", ["fused", "second_kernel"])
def test_long_reductions_both_finishes(tcr, oracle, form, finish):
    # device-level reduction: the last workgroup adds the partials (one kernel) or a second kernel does
    tcr.set_variant("reduce_finish", finish)
    x = workloads.make_input((1 << 23) + 12345, "int8", 41)
    xd = dev(x)
    for n in (100003, 1 << 20, (1 << 22) + 8, x.size):
        assert float(tcr.reduce(xd[:n]).cpu()[0]) == oracle.reduce(x[:n]), f"reduce n={n}"
    for seg in (1 << 19, 1 << 20, 1 << 22):
        m = (1 << 23) // seg * seg
        assert_exact(tcr.segmented_reduce(xd[:m], seg), oracle.segmented_reduce(x[:m], seg), f"reduce L={seg}")
    # the running counter is shared with the scans' tile tickets on the same stream
    ref = oracle.scan(x[: 1 << 22])
    for it in range(20):
        r = tcr.reduce(xd)
        sc = tcr.scan(xd[: 1 << 22])
        assert float(r.cpu()[0]) == oracle.reduce(x)
        if it % 5 == 0:
            assert_exact(sc, ref, "scan between fused reductions")
    tcr.check_device_flags()


def test_caller_supplied_workspace(tcr, oracle):
    n = (1 << 22) + 4096
    x = workloads.make_input(n, "int8", 31)
    xd = dev(x)
    ref_scan = oracle.scan(x)
    need = tcr.workspace_bytes(tcr.OP_SCAN, n, n)
    buf = torch.full((need,), 0xA5, dtype=torch.uint8, device="cuda")      # arbitrary contents
    tcr.check_device_flags()
    try:
        tcr.set_workspace(buf)
        for _ in range(3):
            assert_exact(tcr.scan(xd), ref_scan, "chained scan, caller workspace")
        tcr.tuning_import("scan:41=9;")                                     # the look-back kernel on the same buffer
        assert_exact(tcr.scan(xd), ref_scan, "look-back scan, caller workspace")
        tcr.tuning_import("")
        assert float(tcr.reduce(xd).cpu()[0]) == oracle.reduce(x)
        assert_exact(tcr.segmented_reduce(xd[: 1 << 22], 1 << 21), oracle.segmented_reduce(x[: 1 << 22], 1 << 21),
                     "long-segment reduce, caller workspace")
        for strategy in ("reduce_then_scan", "scan_then_propagate"):
            tcr.set_variant("scan_carry", strategy)
            assert_exact(tcr.scan(xd), ref_scan, f"{strategy}, caller workspace")
        tcr.set_variant("reset")
        s2 = torch.cuda.Stream()                                            # any stream uses the one buffer
        torch.cuda.synchronize()
        out = torch.empty(n, dtype=torch.float32, device="cuda")
        tcr.scan(xd, out=out, stream=s2)
        s2.synchronize()
        assert_exact(out, ref_scan, "other stream, caller workspace")
        tcr.check_device_flags()
        # a buffer that is too small: calls that need more fail without allocating, others still run
        tcr.set_workspace(buf[:1024])
        with pytest.raises(tcr.TcrError) as e:
            tcr.scan(xd)
        assert e.value.status == tcr.ERR_WORKSPACE
        assert_exact(tcr.segmented_scan(xd[: 1 << 20], 256), oracle.segmented_scan(x[: 1 << 20], 256), "no workspace needed")
        with pytest.raises(tcr.TcrError):
            tcr.set_workspace(buf[1:2049])                                  # misaligned
        with pytest.raises(tcr.TcrError):
            tcr.set_workspace(buf[:256])                                    # too small to hold anything
    finally:
        tcr.set_variant("reset")
        tcr.tuning_import("")
        tcr.set_workspace(None)
    assert_exact(tcr.scan(xd), ref_scan, "library workspace again")
    tcr.check_device_flags()


def test_caller_workspace_of_exactly_the_documented_size_serves_the_tiled_kernels(tcr, oracle):
    # regular calls that land on the fixed tiles of the irregular kernels: reductions of 5 .. 15 elements that are
    # no power of two, and views that are not 16-byte aligned (the tiles start at the boundary below them)
    n = 24 * 30011                                       # (a multiple of 12 as well)
    x = workloads.make_input(n + 1, "int8", 41)
    xd = dev(x)
    cases = [("segmented_reduce seg_len 12", tcr.OP_SEGMENTED_REDUCE, n, 12, lambda: tcr.segmented_reduce(xd[:n], 12),
              lambda: oracle.segmented_reduce(x[:n], 12)),
             ("segmented_reduce seg_len 16 behind x[1:]", tcr.OP_SEGMENTED_REDUCE, n - 8, 16,
              lambda: tcr.segmented_reduce(xd[1:n - 7], 16), lambda: oracle.segmented_reduce(x[1:n - 7].copy(), 16)),
             ("reduce behind x[1:]", tcr.OP_REDUCE, n, 0, lambda: tcr.reduce(xd[1:]), lambda: np.array([oracle.reduce(x[1:].copy())])),
             ("segmented_scan seg_len 24 behind x[1:]", tcr.OP_SEGMENTED_SCAN, n, 24,
              lambda: tcr.segmented_scan(xd[1:], 24), lambda: oracle.segmented_scan(x[1:].copy(), 24)),
             ("segmented_moments seg_len 12", tcr.OP_SEGMENTED_MOMENTS, n, 12, lambda: tcr.segmented_moments(xd[:n], 12)[1],
              lambda: oracle.segmented_moments(x[:n], 12)[1])]
    try:
        for what, op, nn, seg, run, ref in cases:
            need = tcr.workspace_bytes(op, nn, seg)
            buf = torch.full((need,), 0x5A, dtype=torch.uint8, device="cuda")
            tcr.set_workspace(buf)
            assert_exact(run(), ref(), what + ", caller workspace of tcr_workspace_bytes")
            torch.cuda.synchronize()
            tcr.set_workspace(None)
    finally:
        tcr.set_workspace(None)
    tcr.check_device_flags()


def test_outputs_do_not_depend_on_previous_contents(tcr, oracle):
    x = workloads.make_input((1 << 20) + 24, "int8", 33)
    xd = dev(x)
    ref = oracle.scan(x)
    out = torch.full((x.size,), float("nan"), dtype=torch.float32, device="cuda")
    tcr.scan(xd, out=out)
    assert_exact(out, ref, "scan into a NaN-filled buffer")
    red = torch.full((1 << 8,), float("nan"), dtype=torch.float32, device="cuda")
    tcr.segmented_reduce(xd[: 1 << 20], 1 << 12, out=red)
    assert_exact(red, oracle.segmented_reduce(np.ascontiguousarray(x[: 1 << 20]), 1 << 12), "reduce into NaNs")
