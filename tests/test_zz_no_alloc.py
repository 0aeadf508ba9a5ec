"""tcr_segmented_scan_noalloc -- the scan on the library's fixed device scratch, for callers that cannot
allocate -- against tcr_segmented_scan, through the C ABI.

Same kernels, so integer-valued inputs must give identical outputs; for real-valued inputs the chained kernels
add the carries of earlier tiles in an order that may differ from launch to launch, so the bar is the one of
every other parity test: |y - ref| <= 1e-3 * max(|ref|, rho), rho = the root of the sum of squares of the inputs
the output adds up.  Every case runs two calls in a row on the shared scratch, the second on a smaller input.
"""
import ctypes

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


def _call(tcr, xd, seg, out):
    """Straight through the C ABI: pointers, sizes, the stream handle."""
    st = tcr.raw().tcr_segmented_scan_noalloc(xd.data_ptr(), out.data_ptr(), xd.numel(), seg,
                                              int(torch.cuda.current_stream().cuda_stream))
    assert st == tcr.OK, tcr.raw().tcr_status_string(st).decode()


def _compare(tcr, n, seg, dist, seed):
    x = workloads.make_input(n, dist, seed)
    xd = torch.from_numpy(x).cuda()
    want = tcr.segmented_scan(xd, seg)
    got = torch.full((n,), -7.0, dtype=torch.float32, device="cuda")
    _call(tcr, xd, seg, got)
    torch.cuda.synchronize()
    if dist.startswith("int"):
        assert torch.equal(got, want), f"n={n} seg={seg}: differs first at {int((got != want).nonzero()[0])}"
    else:
        ref = want.cpu().numpy().astype(np.float64)
        rho = np.sqrt(np.cumsum((x.astype(np.float64) ** 2).reshape(-1, seg), axis=1)).reshape(-1)
        err = np.abs(got.cpu().numpy().astype(np.float64) - ref)
        assert np.all(err <= 1e-3 * np.maximum(np.abs(ref), rho)), f"n={n} seg={seg} {dist}"


# (first call, second call on a smaller input); every pair shares the scratch of the GPU.
# 2^22 + 8 / 3 * 2^20 as one segment and seg_len 2^16: the pipelined chain; 16384: tiles by ticket;
# 2^21 + 3 as one segment: decoupled look-back; 100: fixed tiles with the segment starts marked; 256: no scratch at all.
PAIRS = [
    (((1 << 22) + 8, (1 << 22) + 8), (3 << 20, 1 << 16)),
    ((1 << 22, 16384), (1 << 20, 16384)),
    (((1 << 21) + 3, (1 << 21) + 3), (100 * 4001, 100)),
    ((1 << 22, 1 << 20), (1 << 18, 256)),
]


@pytest.mark.parametrize("dist", ["int4", "uniform_pm1"])
@pytest.mark.parametrize("first,second", PAIRS)
def test_two_calls_in_a_row_match_the_allocating_entry_point(tcr, first, second, dist):
    _compare(tcr, first[0], first[1], dist, 31)
    _compare(tcr, second[0], second[1], dist, 32)
    tcr.check_device_flags()


def test_back_to_back_without_a_host_wait_in_between(tcr):
    # the second launch starts from the counters the first one leaves behind, ordered by the stream only
    big = torch.from_numpy(workloads.make_input(1 << 23, "int4", 5)).cuda()
    small = torch.from_numpy(workloads.make_input((1 << 19) + 16, "int4", 6)).cuda()
    out_big = torch.empty(big.numel(), dtype=torch.float32, device="cuda")
    out_small = torch.empty(small.numel(), dtype=torch.float32, device="cuda")
    for _ in range(3):
        _call(tcr, big, big.numel(), out_big)
        _call(tcr, small, small.numel(), out_small)
    torch.cuda.synchronize()
    assert torch.equal(out_big, tcr.scan(big))
    assert torch.equal(out_small, tcr.scan(small))
    tcr.check_device_flags()


def test_sizes_beyond_the_scratch_are_rejected(tcr):
    # validated before anything is enqueued or touched: the pointers are never followed
    x = torch.zeros(64, dtype=torch.float16, device="cuda")
    out = torch.zeros(64, dtype=torch.float32, device="cuda")
    lib = tcr.raw()
    n = (1 << 30) + 16
    assert lib.tcr_segmented_scan_noalloc(x.data_ptr(), out.data_ptr(), n, 16, None) == tcr.ERR_UNSUPPORTED
    assert lib.tcr_segmented_scan_noalloc(x.data_ptr(), out.data_ptr(), 64, 0, None) == tcr.ERR_INVALID_ARG
    assert lib.tcr_segmented_scan_noalloc(x.data_ptr(), out.data_ptr(), 64, 7, None) == tcr.ERR_INVALID_ARG
    assert lib.tcr_segmented_scan_noalloc(None, out.data_ptr(), 64, 16, None) == tcr.ERR_INVALID_ARG
    assert lib.tcr_segmented_scan_noalloc(x.data_ptr(), out.data_ptr(), 0, 16, None) == tcr.OK
    torch.cuda.synchronize()
    assert not out.any()
