"""The five evaluation configurations at their full sizes, in the launch configuration that
bench.py times (default variant), checked against the CPU oracle on every output element.

Integer-valued configurations (3b, 4) must match bit for bit; the others must satisfy
|y - ref| <= 1e-3 * max(|ref|, rho) with rho = sqrt(sum of squares of the inputs the output
adds up).  For the non-negative inputs of configuration 5, |ref| >= rho always, so the rule is
a plain relative error of 1e-3 there.
"""
import numpy as np
import pytest
import torch

from paper_1811_09736_amd import workloads

pytestmark = pytest.mark.gpu

REL_TOL = 1e-3
CHUNK = 1 << 24

_cache = {}


def _input(n, dist, seed):
    key = (n, dist, str(seed))
    if key not in _cache:
        _cache.clear()                                   # one 512 MiB input (and its device copy) at a time
        x = workloads.make_input(n, dist, seed)
        _cache[key] = (x, torch.from_numpy(x).cuda())
    return _cache[key]


@pytest.fixture(scope="module")
def tcr():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1811_09736_amd import binding
    binding.set_variant("reset")
    yield binding
    _cache.clear()
    binding.check_device_flags()


def _compare(got: torch.Tensor, ref: np.ndarray, x: np.ndarray, seg: int, is_scan: bool, exact: bool,
             nonneg: bool, what: str):
    g32 = got.cpu().numpy()
    worst = 0.0
    for lo in range(0, ref.size, CHUNK):
        hi = min(lo + CHUNK, ref.size)
        g = g32[lo:hi].astype(np.float64)
        r = ref[lo:hi]
        if exact:
            if not np.array_equal(g, r):
                bad = lo + int(np.flatnonzero(g != r)[0])
                raise AssertionError(f"{what}: first mismatch at {bad}: got {g32[bad]!r} want {ref[bad]!r}")
            continue
        if nonneg:
            scale = np.abs(r)
        elif is_scan:
            # chunk boundaries are multiples of seg or lie inside one long segment
            if seg <= CHUNK:
                xs = x[lo:hi].astype(np.float64)
                rho = np.sqrt(np.cumsum((xs * xs).reshape(-1, seg), axis=1)).reshape(-1)
            else:
                first = lo - lo % seg
                xs = x[first:hi].astype(np.float64)
                rho = np.sqrt(np.cumsum(xs * xs))[lo - first:]
            scale = np.maximum(np.abs(r), rho)
        else:
            xs = x[lo * seg:hi * seg].astype(np.float64)
            scale = np.maximum(np.abs(r), np.sqrt((xs * xs).reshape(-1, seg).sum(axis=1)))
        err = np.abs(g - r)
        tol = REL_TOL * scale
        if not np.all(err <= tol):
            bad = int(np.argmax(err - tol))
            raise AssertionError(f"{what}: worst at {lo + bad}: got {g[bad]!r} want {r[bad]!r} tol {tol[bad]!r}")
        nz = scale > 0
        if nz.any():
            worst = max(worst, float(np.max(err[nz] / scale[nz])))
    if not exact:
        print(f"  {what}: max error / scale = {worst:.3e}", flush=True)
    return worst


CONFIGS = list(workloads.configs())


@pytest.mark.parametrize("w", CONFIGS, ids=[w.name for w in CONFIGS])
def test_config(tcr, oracle, w):
    x, xd = _input(w.n, w.dist, w.seed)
    nonneg = w.dist == "uniform_01"
    if w.op == "segmented_reduce":
        got = tcr.segmented_reduce(xd, w.seg_len)
        ref = oracle.segmented_reduce(x, w.seg_len)
        worst = _compare(got, ref, x, w.seg_len, False, w.exact, nonneg, w.name)
    elif w.op == "segmented_scan":
        got = tcr.segmented_scan(xd, w.seg_len)
        ref = oracle.segmented_scan(x, w.seg_len)
        worst = _compare(got, ref, x, w.seg_len, True, w.exact, nonneg, w.name)
    elif w.op == "reduce":
        got = tcr.reduce(xd)
        ref = np.array([oracle.reduce(x)])
        if w.exact:
            assert abs(ref[0]) < 2 ** 24                      # any binary32 summation order is then exact
        _compare(got, ref, x, w.n, False, w.exact, nonneg, w.name)
    else:
        got = tcr.scan(xd)
        ref = oracle.scan(x)
        if w.exact:
            assert np.max(np.abs(ref)) < 2 ** 24
        _compare(got, ref, x, w.n, True, w.exact, nonneg, w.name)
        # the carry crossed workgroups: many tiles, and the last element is the grand total
        assert float(got[-1].cpu()) == float(np.float32(ref[-1])) or not w.exact
    if nonneg and w.op.startswith("segmented"):
        # second, tighter gate for non-negative data, derived from the arithmetic: an output passes through at
        # most 32 (in-row adds of a product) + 15 (row carries) + 8 + 16 (tile and wavefront carries) binary32
        # roundings, plus -- scan -- the cross-workgroup chain: per 32768-element workgroup share of its segment
        # at most twelve (a ten-level tree over the up to 256 aggregates since the workgroup's previous share,
        # adding that share's prefix, adding the own total), or -- reduce -- one per tile chained through the
        # accumulator; every partial sum is bounded by the output itself, so the relative error is at most that
        # count times 2^-24.
        roundings = 71 + (12 * (w.seg_len // 32768) if w.op == "segmented_scan" else w.seg_len // 512)
        assert worst <= roundings * 2.0 ** -24, (w.name, worst)
    tcr.check_device_flags()


def test_config4_integer_variants_both_carry_strategies(tcr, oracle):
    """Configuration 4 again under the reduce-then-scan carry and the DPP formulation."""
    w = [c for c in CONFIGS if c.name.startswith("cfg4")][0]
    x, xd = _input(w.n, w.dist, w.seed)
    ref = oracle.scan(x)
    try:
        for key, val in (("scan_carry", "reduce_then_scan"), ("scan_carry", "scan_then_propagate"), ("formulation", "dpp")):
            tcr.set_variant("reset")
            tcr.set_variant(key, val)
            _compare(tcr.scan(xd), ref, x, w.n, True, True, False, f"cfg4 {key}={val}")
    finally:
        tcr.set_variant("reset")


@pytest.mark.parametrize("recipe", ["uniform16", "lognormal256", "few7"])
def test_irregular_mixes_at_bench_size(tcr, oracle, recipe):
    # the three offset arrays bench.py times, over the input of configuration 5 (non-negative: plain relative
    # error), every output element against the oracle
    n = 1 << 28
    x, xd = _input(n, "uniform_01", 4)
    off = workloads.make_offsets(n, recipe, 5).view(np.int64)
    od = torch.from_numpy(off).cuda()
    nseg = off.size - 1
    red = tcr.irregular_reduce(xd, od).cpu().numpy().astype(np.float64)
    ref = oracle.irregular_reduce(x, off)
    err = np.abs(red - ref)
    assert np.all(err <= REL_TOL * np.abs(ref)), f"{recipe}: reduce, worst segment {int(np.argmax(err - REL_TOL * np.abs(ref)))}"
    print(f"  {recipe}: {nseg} segments, reduce max relative error {np.max(err[ref > 0] / ref[ref > 0]):.3e}", flush=True)
    del red, ref, err
    got = tcr.irregular_scan(xd, od).cpu().numpy()
    ref = oracle.irregular_scan(x, off)
    worst = 0.0
    for lo in range(0, n, CHUNK):
        r = ref[lo:lo + CHUNK]
        e = np.abs(got[lo:lo + CHUNK].astype(np.float64) - r)
        if not np.all(e <= REL_TOL * np.abs(r)):
            bad = lo + int(np.argmax(e - REL_TOL * np.abs(r)))
            raise AssertionError(f"{recipe}: scan, worst at {bad}: got {got[bad]!r} want {ref[bad]!r}")
        nz = r > 0
        worst = max(worst, float(np.max(e[nz] / r[nz])))
    print(f"  {recipe}: scan max relative error {worst:.3e}", flush=True)
    tcr.check_device_flags()
