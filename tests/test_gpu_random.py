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
