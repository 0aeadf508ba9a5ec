"""Beyond 2^31 elements: byte offsets no longer fit 32 bits, the pipelined chain runs 65568 tiles and rebases
its range-checked buffer resources per tile.  The input is a period-7 integer pattern whose periods sum to
zero, so every prefix is a small integer with a closed form; every output is compared with that closed form
(computed with integer index arithmetic on the device, in chunks) and sampled outputs with the oracle."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

N = (1 << 31) + (1 << 20)
PATTERN = np.array([3, -1, -2, 2, -3, 0, 1], dtype=np.float16)           # sums to zero
CHUNK = 1 << 27


@pytest.fixture(scope="module")
def tcr():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    if torch.cuda.get_device_properties(0).total_memory < 40 * (1 << 30):
        pytest.skip("needs 40 GiB of device memory")
    from paper_1811_09736_amd import binding
    binding.set_variant("reset")
    binding.tuning_import("")
    yield binding
    binding.release()
    torch.cuda.empty_cache()


@pytest.fixture(scope="module")
def data():
    x = np.tile(PATTERN, N // 7 + 1)[:N].copy()
    return x, torch.from_numpy(x).cuda()


def _prefix_table(device):
    return torch.tensor(np.concatenate([[0.0], np.cumsum(PATTERN.astype(np.float64))[:-1], [0.0]])[:8],
                        dtype=torch.float32, device=device)


def _expected_scan_chunk(lo, hi, seg, device):
    """Inclusive scan restarted every `seg` elements, positions lo .. hi-1: P(k) - P(start - 1) with
    P(k) = sum of the pattern's first (k mod 7) + 1 entries (whole periods add nothing)."""
    incl = torch.tensor(np.cumsum(PATTERN.astype(np.float64)), dtype=torch.float32, device=device)
    k = torch.arange(lo, hi, dtype=torch.int64, device=device)
    start = k - k % seg
    before = torch.where(start % 7 == 0, torch.zeros((), device=device), incl[(start - 1) % 7])
    return incl[k % 7] - before


@pytest.mark.parametrize("seg", [1 << 20, N])
def test_scan_beyond_2_31_elements(tcr, oracle, data, seg):
    x, xd = data
    print(f"  scan n={N} seg={seg} kernel={tcr.kernel_name(tcr.OP_SEGMENTED_SCAN, N, seg)}", flush=True)
    out = tcr.segmented_scan(xd, seg)
    for lo in range(0, N, CHUNK):
        hi = min(lo + CHUNK, N)
        want = _expected_scan_chunk(lo, hi, seg, xd.device)
        if not torch.equal(out[lo:hi], want):
            bad = lo + int(torch.nonzero(out[lo:hi] != want)[0])
            raise AssertionError(f"first mismatch at {bad}: got {float(out[bad])} want {float(want[bad - lo])}")
    # sampled outputs against the oracle (each sample walks its segment from the start)
    rng = np.random.default_rng(5)
    idx = np.concatenate([rng.integers(0, N, 6), [N - 1, (1 << 31) + 12345]]).astype(np.uint64)
    if seg == N:
        idx = idx[-2:]                                       # two long walks are enough
    ref = oracle.segmented_scan_at(x, seg, idx)
    got = out[torch.from_numpy(idx.astype(np.int64)).cuda()].cpu().numpy().astype(np.float64)
    assert np.array_equal(got, ref)
    tcr.check_device_flags()
    del out


def test_scan_variants_and_reduce_beyond_2_31_elements(tcr, oracle, data):
    x, xd = data
    seg = 1 << 20
    # small segments (one tile per wavefront kernels) and the binary16 / exclusive outputs
    out = tcr.segmented_scan(xd, 256)
    for lo in range(0, N, CHUNK):
        hi = min(lo + CHUNK, N)
        assert torch.equal(out[lo:hi], _expected_scan_chunk(lo, hi, 256, xd.device)), f"seg 256, chunk at {lo}"
    del out
    out16 = tcr.segmented_scan_ex(xd, seg, tcr.OUT_F16 | tcr.SCAN_EXCLUSIVE)
    for lo in range(0, N, CHUNK):
        hi = min(lo + CHUNK, N)
        want = _expected_scan_chunk(lo, hi, seg, xd.device) - xd[lo:hi].float()
        assert torch.equal(out16[lo:hi].float(), want), f"exclusive binary16, chunk at {lo}"
    del out16
    # reductions: a segment's total is the last entry of its scan
    last = torch.arange(seg - 1, N, seg, dtype=torch.int64, device=xd.device)
    want = torch.cat([_expected_scan_chunk(int(k), int(k) + 1, seg, xd.device) for k in last[:4]] +
                     [_expected_scan_chunk(int(k), int(k) + 1, seg, xd.device) for k in last[-4:]])
    red = tcr.segmented_reduce(xd, seg)
    assert torch.equal(torch.cat([red[:4], red[-4:]]), want)
    ref = oracle.segmented_scan_at(x, seg, (last.cpu().numpy()[[0, 1000, 2048]]).astype(np.uint64))
    assert np.array_equal(red[[0, 1000, 2048]].cpu().numpy().astype(np.float64), ref)
    total = float(tcr.reduce(xd).cpu()[0])
    assert total == float(np.sum(PATTERN[: N % 7].astype(np.float64)))
    red16 = tcr.segmented_reduce(xd, 16)
    k = torch.arange(0, N // 16, dtype=torch.int64, device=xd.device) * 16 + 15
    incl = torch.tensor(np.cumsum(PATTERN.astype(np.float64)), dtype=torch.float32, device=xd.device)
    start = k - 15
    before = torch.where(start % 7 == 0, torch.zeros((), device=xd.device), incl[(start - 1) % 7])
    assert torch.equal(red16, incl[k % 7] - before)
    tcr.check_device_flags()


def test_irregular_segments_beyond_2_31_elements(tcr, oracle, data):
    # 200 000 random cuts, a dense stretch of short segments across element 2^31 and a run of empty segments;
    # closed form as above with every element's own segment start
    x, xd = data
    rng = np.random.default_rng(17)
    cuts = np.concatenate([rng.integers(0, N, 200000, endpoint=True), (1 << 31) - 5000 + np.arange(0, 10000, 7),
                           np.full(300, (1 << 31) + 77), [5, N - 3]])
    off = np.concatenate([[5], np.sort(cuts[(cuts >= 5) & (cuts <= N - 3)]), [N - 3]]).astype(np.int64)   # x[:5], x[N-3:]: no segment
    od = torch.from_numpy(off).cuda()
    incl = torch.tensor(np.cumsum(PATTERN.astype(np.float64)), dtype=torch.float32, device=xd.device)

    def before(start):                                       # sum of x[0 .. start)
        return torch.where(start % 7 == 0, torch.zeros((), device=xd.device), incl[(start - 1) % 7])

    out = torch.full((N,), -5.0, dtype=torch.float32, device="cuda")
    tcr.irregular_scan(xd, od, out=out)
    assert torch.all(out[:5] == -5.0) and torch.all(out[N - 3:] == -5.0)
    for lo in range(0, N, CHUNK):
        hi = min(lo + CHUNK, N)
        k = torch.arange(max(lo, 5), min(hi, N - 3), dtype=torch.int64, device=xd.device)
        start = od[torch.searchsorted(od, k, right=True) - 1]
        want = incl[k % 7] - before(start)
        got = out[max(lo, 5):min(hi, N - 3)]
        if not torch.equal(got, want):
            bad = int(torch.nonzero(got != want)[0])
            raise AssertionError(f"first mismatch at {int(k[bad])}: got {float(got[bad])} want {float(want[bad])}")
    del out
    red = tcr.irregular_reduce(xd, od)
    want = torch.where(od[1:] > od[:-1], before(od[1:]) - before(od[:-1]), torch.zeros((), device=xd.device))
    if not torch.equal(red, want):
        bad = int(torch.nonzero(red != want)[0])
        raise AssertionError(f"segment {bad} [{off[bad]}, {off[bad + 1]}): got {float(red[bad])} want {float(want[bad])}")
    # sampled segments against the oracle: the short ones around 2^31 and a few of the long ones
    around = int(np.searchsorted(off, 1 << 31))
    for s in list(range(around - 3, around + 3)) + [0, 1000, off.size - 2]:
        piece = x[off[s]:off[s + 1]]
        assert float(red[s].cpu()) == oracle.reduce(piece) if piece.size else float(red[s].cpu()) == 0.0
    tcr.check_device_flags()


def test_beyond_2_32_elements(tcr):
    """Element indices that no longer fit 32 bits (the closed forms above, no host oracle: 8 GiB of input)."""
    if torch.cuda.get_device_properties(0).total_memory < 100 * (1 << 30):
        pytest.skip("needs 100 GiB of device memory")
    n = (1 << 32) + (1 << 20) + 24
    xd = torch.from_numpy(np.tile(PATTERN, n // 7 + 1)[:n].copy()).cuda()
    dev = xd.device
    incl = torch.tensor(np.cumsum(PATTERN.astype(np.float64)), dtype=torch.float32, device=dev)

    def before(start):                                       # sum of x[0 .. start)
        return torch.where(start % 7 == 0, torch.zeros((), device=dev), incl[(start - 1) % 7])

    for seg in (n, 1 << 20, 256, 3001):
        m = (n // seg) * seg
        print(f"  scan n={m} seg={seg} kernel={tcr.kernel_name(tcr.OP_SEGMENTED_SCAN, m, seg)}", flush=True)
        out = tcr.segmented_scan(xd[:m], seg)
        for lo in range(0, m, CHUNK):
            hi = min(lo + CHUNK, m)
            want = _expected_scan_chunk(lo, hi, seg, dev)
            if not torch.equal(out[lo:hi], want):
                raise AssertionError(f"scan seg {seg}: first mismatch at {lo + int(torch.nonzero(out[lo:hi] != want)[0])}")
        del out
    for seg in (16, 100, 4096, 1 << 20, 3001):
        m = (n // seg) * seg
        print(f"  reduce n={m} seg={seg} kernel={tcr.kernel_name(tcr.OP_SEGMENTED_REDUCE, m, seg)}", flush=True)
        k = torch.arange(0, m // seg, dtype=torch.int64, device=dev) * seg
        assert torch.equal(tcr.segmented_reduce(xd[:m], seg), before(k + seg) - before(k)), f"reduce seg {seg}"
    assert float(tcr.reduce(xd).cpu()[0]) == float(np.sum(PATTERN[: n % 7].astype(np.float64)))
    rng = np.random.default_rng(3)
    cuts = np.concatenate([rng.integers(0, n, 100000, endpoint=True), (1 << 32) - 3000 + np.arange(0, 6000, 5)])
    od = torch.from_numpy(np.concatenate([[0], np.sort(cuts), [n]]).astype(np.int64)).cuda()
    out = tcr.irregular_scan(xd, od)
    for lo in range(0, n, CHUNK):
        k = torch.arange(lo, min(lo + CHUNK, n), dtype=torch.int64, device=dev)
        want = incl[k % 7] - before(od[torch.searchsorted(od, k, right=True) - 1])
        assert torch.equal(out[lo:lo + CHUNK], want), f"irregular scan, chunk at {lo}"
    del out
    want = torch.where(od[1:] > od[:-1], before(od[1:]) - before(od[:-1]), torch.zeros((), device=dev))
    assert torch.equal(tcr.irregular_reduce(xd, od), want)
    tcr.check_device_flags()
