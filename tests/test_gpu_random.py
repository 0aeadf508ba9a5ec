"""Seeded random sweep over the dispatcher: operation, segment length (powers of two, multiples of 8, odd
lengths, one segment), segment count, flags and formulation are drawn at random and every output is compared
with the oracle bit for bit (integer-valued inputs).  It exists to catch a wrong turn between the many
kernels behind the five entry points; each case prints what it ran."""
import numpy as np
import pytest
import torch

from paper_1811_09736_amd import workloads

pytestmark = pytest.mark.gpu

MAX_N = 1 << 22


@pytest.fixture(scope="module")
def tcr():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1811_09736_amd import binding
    binding.set_variant("reset")
    binding.tuning_import("")
    yield binding
    binding.set_variant("reset")
    binding.check_device_flags()


def _draw_seg_len(rng) -> int:
    kind = rng.integers(0, 6)
    if kind == 0:
        return 1 << int(rng.integers(0, 22))                     # powers of two, 1 .. 2^21
    if kind == 1:
        return 8 * int(rng.integers(1, 40000))                   # multiples of 8 up to 320000
    if kind == 2:
        return int(rng.integers(1, 700))                         # short, any parity
    if kind == 3:
        return 2 * int(rng.integers(300, 100000)) + 1            # odd and long
    if kind == 4:
        return 32768 * int(rng.integers(1, 40)) + 8 * int(rng.integers(0, 2))   # around whole chain tiles
    return int(rng.integers(1, MAX_N))                           # anything


@pytest.mark.parametrize("block", range(8))
def test_random_dispatch(tcr, oracle, block):
    rng = np.random.default_rng(1000 + block)
    for case in range(25):
        seg = _draw_seg_len(rng)
        nseg = int(rng.integers(1, max(2, min(MAX_N // seg, 5000) + 1)))
        one_segment = rng.integers(0, 6) == 0
        if one_segment:
            seg, nseg = int(rng.integers(1, MAX_N)), 1
        n = seg * nseg
        op = ("reduce", "scan", "scan_ex", "moments")[int(rng.integers(0, 4))]
        flags = int(rng.integers(1, 4)) if op == "scan_ex" else 0
        dpp = rng.integers(0, 4) == 0 and op in ("reduce", "scan")
        # |x| <= 4 keeps every prefix below 2^24; the sums of squares of up to 2^22 values need |x| <= 1
        x = workloads.make_input(n, "int1" if op == "moments" else "int4", int(rng.integers(0, 1 << 30)))
        xd = torch.from_numpy(x).cuda()
        tcr.set_variant("formulation", "dpp" if dpp else "mfma")
        what = f"block {block} case {case}: {op} n={n} seg_len={seg} flags={flags} {'dpp' if dpp else 'mfma'}"
        print("  " + what, flush=True)
        try:
            if op == "reduce":
                got = tcr.segmented_reduce(xd, seg).cpu().numpy().astype(np.float64)
                ref = oracle.segmented_reduce(x, seg)
            elif op == "scan":
                got = tcr.segmented_scan(xd, seg).cpu().numpy().astype(np.float64)
                ref = oracle.segmented_scan(x, seg)
            elif op == "scan_ex":
                got = tcr.segmented_scan_ex(xd, seg, flags).cpu().numpy().astype(np.float64)
                ref = oracle.segmented_scan_exclusive(x, seg) if flags & 1 else oracle.segmented_scan(x, seg)
                if flags & 2:
                    ref = ref.astype(np.float16).astype(np.float64)
            else:
                a, q = tcr.segmented_moments(xd, seg)
                ra, rq = oracle.segmented_moments(x, seg)
                assert np.array_equal(a.cpu().numpy().astype(np.float64), ra), what + " (sum)"
                got, ref = q.cpu().numpy().astype(np.float64), rq
        finally:
            tcr.set_variant("reset")
        assert np.max(np.abs(ref)) < 2 ** 24 or flags & 2
        assert np.array_equal(got, ref), what
    tcr.check_device_flags()


def _draw_offsets(rng, n):
    """Random cover of part of [0, n): pieces drawn from several length scales, with empty segments and cuts placed
    on and around multiples of the 16384- and 32768-element tiles."""
    lo = int(rng.integers(0, max(1, min(n, 40000)))) if rng.integers(0, 3) == 0 else 0
    hi = n - int(rng.integers(0, max(1, min(n - lo, 40000)))) if rng.integers(0, 3) == 0 else n
    cuts = [np.array([lo, hi], dtype=np.int64)]
    for _ in range(int(rng.integers(0, 4))):
        scale = int((1, 8, 100, 5000, 200000)[int(rng.integers(0, 5))])
        start = int(rng.integers(lo, hi + 1))
        lens = rng.integers(0, 2 * scale + 1, int(rng.integers(1, 3000)))
        cuts.append(start + np.cumsum(lens))
    if rng.integers(0, 2):
        tiles = 16384 * rng.integers(0, n // 16384 + 1, int(rng.integers(1, 30)))
        cuts.append(tiles + rng.integers(-2, 3, tiles.size))
    if rng.integers(0, 2):
        cuts.append(np.full(int(rng.integers(1, 600)), int(rng.integers(lo, hi + 1))))      # a run of empty segments
    c = np.concatenate(cuts)
    return np.sort(c[(c >= lo) & (c <= hi)]).astype(np.int64)


@pytest.mark.parametrize("block", range(6))
def test_random_irregular_segments(tcr, oracle, block):
    # offsets, scan flags and the misalignment of both arrays drawn at random
    rng = np.random.default_rng(5000 + block)
    for case in range(20):
        n = int(rng.integers(1, MAX_N)) if rng.integers(0, 4) else int(rng.integers(1, 70000))
        off = _draw_offsets(rng, n)
        in_shift, out_shift = (int(rng.integers(0, 8)), int(rng.integers(0, 4))) if rng.integers(0, 2) else (0, 0)
        flags = int(rng.integers(0, 4))
        base = workloads.make_input(n + 8, "int4", int(rng.integers(0, 1 << 30)))
        x = base[in_shift:in_shift + n].copy()
        what = (f"block {block} case {case}: n={n} nseg={off.size - 1} cover=[{off[0]}, {off[-1]}) "
                f"shifts=({in_shift}, {out_shift}) flags={flags}")
        print("  " + what, flush=True)
        xd, od = torch.from_numpy(base).cuda()[in_shift:in_shift + n], torch.from_numpy(off).cuda()
        buf = torch.full((n + 8,), -7.0, dtype=torch.float16 if flags & 2 else torch.float32, device="cuda")
        tcr.irregular_scan_ex(xd, od, flags, out=buf[out_shift:out_shift + n])
        red = tcr.irregular_reduce(xd, od).cpu().numpy().astype(np.float64)
        got = buf.cpu().numpy().astype(np.float64)
        scan = got[out_shift:out_shift + n]
        ref = oracle.irregular_scan_exclusive(x, off) if flags & 1 else oracle.irregular_scan(x, off)
        assert np.max(np.abs(ref)) < 2 ** 24
        if flags & 2:
            ref = ref.astype(np.float16).astype(np.float64)
        lo, hi = int(off[0]), int(off[-1])
        assert np.array_equal(scan[lo:hi], ref[lo:hi]), what + " (scan)"
        assert np.all(scan[:lo] == -7.0) and np.all(scan[hi:] == -7.0), what + " (outside the segments)"
        assert np.all(got[:out_shift] == -7.0) and np.all(got[out_shift + n:] == -7.0), what + " (outside the array)"
        assert np.array_equal(red, oracle.irregular_reduce(x, off)), what + " (reduce)"
    tcr.check_device_flags()
