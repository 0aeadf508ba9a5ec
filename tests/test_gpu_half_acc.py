"""TCR_ACC_F16: the scan with a binary16 accumulator (tcr_segmented_scan_ex / tcr_scan_ex with
TCR_OUT_F16 | TCR_ACC_F16), against the oracle.

The library adds in a tree, the oracle (oracle_segmented_scan_half_acc) left to right, and a binary16 addition
rounds, so the two agree bit for bit exactly when no addition rounds: inputs whose sums over ANY run of
consecutive elements of a segment are binary16 values (integers within +-2048).  Those cases are compared bit
for bit with the binary16 oracle, which then also equals the exact scan.  For real-valued inputs the paper gives
no error bound; the bar is the one the arithmetic gives: at most 40 roundings of relative size 2^-11 on the way to
any output, |out - exact| <= 40 * 2^-11 * (sum of |x| over the elements the output adds up), against the
binary64 oracle -- beyond that bound parity is unpinned.
"""
import numpy as np
import pytest
import torch

from paper_1811_09736_amd import workloads

pytestmark = pytest.mark.gpu

EXCL, F16, ACC = 1, 2, 4
ROUNDINGS = 40


@pytest.fixture(scope="module")
def tcr():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1811_09736_amd import binding
    binding.set_variant("reset")
    yield binding
    binding.set_variant("reset")
    binding.check_device_flags()


def bounded_walk(n, seed, bound=1000):
    """Steps of +-1 whose running sum stays within +-bound from any starting point of a segment: a random walk
    folded back at +-bound (input generation only)."""
    rng = np.random.default_rng(seed)
    w = np.cumsum(rng.choice(np.array([-1, 1]), size=n))
    half = bound // 2                       # any run of consecutive steps then sums to within +-bound
    folded = np.abs((w + half) % (4 * half) - 2 * half) - half
    x = np.diff(np.concatenate([[0], folded]))
    assert np.all(np.abs(x) <= 1)
    return x.astype(np.float16)


SEGS = [1, 2, 4, 8, 16, 64, 512, 1024, 4096, 16384, 1 << 16, 1 << 17, 1 << 19]


@pytest.mark.parametrize("excl", [0, EXCL])
@pytest.mark.parametrize("seg", SEGS)
def test_bit_exact_while_no_addition_rounds(tcr, oracle, seg, excl):
    nseg = 3 if seg >= 8192 else (3 * 8192 // seg + 3)
    n = seg * nseg
    x = bounded_walk(n, seg + excl)
    xd = torch.from_numpy(x).cuda()
    got = tcr.segmented_scan_ex(xd, seg, F16 | ACC | excl).cpu().numpy()
    want = oracle.segmented_scan_half_acc(x, seg, bool(excl))
    exact = oracle.segmented_scan_exclusive(x, seg) if excl else oracle.segmented_scan(x, seg)
    assert np.array_equal(want.astype(np.float64), exact)                    # nothing rounded on the oracle's side either
    bad = np.flatnonzero(got.astype(np.float64) != want.astype(np.float64))
    assert bad.size == 0, f"L={seg}: first mismatch at {bad[0]}: {got[bad[0]]} != {want[bad[0]]}"


@pytest.mark.parametrize("excl", [0, EXCL])
@pytest.mark.parametrize("n", [1, 7, 513, 8193, 65536, 100003, (1 << 18) + 24, (1 << 21) + 9])
def test_full_scan_bit_exact(tcr, oracle, n, excl):
    x = bounded_walk(n, n % 997)
    got = tcr.scan_ex(torch.from_numpy(x).cuda(), F16 | ACC | excl).cpu().numpy()
    want = oracle.segmented_scan_half_acc(x, n, bool(excl))
    assert np.array_equal(got.astype(np.float64), want.astype(np.float64))


@pytest.mark.parametrize("dist", ["uniform_01", "uniform_pm1", "normal"])
@pytest.mark.parametrize("excl", [0, EXCL])
@pytest.mark.parametrize("seg", [4, 16, 256, 4096, 1 << 16, 1 << 18])
def test_real_valued_inputs_within_the_rounding_bound(tcr, oracle, seg, excl, dist):
    nseg = 3 if seg >= 8192 else (3 * 8192 // seg + 3)
    x = workloads.make_input(seg * nseg, dist, 4)
    got = tcr.segmented_scan_ex(torch.from_numpy(x).cuda(), seg, F16 | ACC | excl).cpu().numpy().astype(np.float64)
    exact = oracle.segmented_scan_exclusive(x, seg) if excl else oracle.segmented_scan(x, seg)
    mass = np.cumsum(np.abs(x.astype(np.float64)).reshape(-1, seg), axis=1)
    if excl:
        mass = np.concatenate([np.zeros((mass.shape[0], 1)), mass[:, :-1]], axis=1)
    mass = mass.reshape(-1)
    fin = mass < 60000.0                                       # (sums near the top of the format may overflow to infinity)
    bound = ROUNDINGS * 2.0 ** -11 * mass + ROUNDINGS * 2.0 ** -25
    assert np.all(np.abs(got - exact)[fin] <= bound[fin]), f"L={seg} {dist}"
    if excl:
        assert not got[::seg].any()


def test_a_tree_of_additions_does_not_stall_where_the_left_to_right_sum_does(tcr, oracle):
    # ones: left to right the count stops at 2048 (2048 + 1 rounds back); the tree adds 2048 + 2048.  Both are
    # binary16 accumulations; the library's stays within its bound of the exact count.
    x = np.ones(4096 * 4, dtype=np.float16)
    got = tcr.segmented_scan_ex(torch.from_numpy(x).cuda(), 4096, F16 | ACC).cpu().numpy().astype(np.float64)
    seq = oracle.segmented_scan_half_acc(x, 4096).astype(np.float64)
    exact = oracle.segmented_scan(x, 4096)
    assert seq.max() == 2048.0
    assert np.all(np.abs(got - exact) <= ROUNDINGS * 2.0 ** -11 * exact)
    assert got.reshape(4, 4096)[:, -1].tolist() == [4096.0] * 4


def test_flag_rules(tcr):
    x = torch.from_numpy(workloads.make_input(3000, "int4", 1)).cuda()
    out = torch.empty(3000, dtype=torch.float16, device="cuda")
    raw = tcr.raw()
    assert raw.tcr_segmented_scan_ex(x.data_ptr(), out.data_ptr(), 3000, 3000, ACC, None) == tcr.ERR_INVALID_ARG
    assert raw.tcr_segmented_scan_ex(x.data_ptr(), out.data_ptr(), 3000, 3000, 8, None) == tcr.ERR_INVALID_ARG
    assert raw.tcr_segmented_scan_ex(x.data_ptr(), out.data_ptr(), 3000, 100, F16 | ACC, None) == tcr.ERR_UNSUPPORTED
    assert raw.tcr_segmented_scan_ex(x[8:].data_ptr(), out.data_ptr(), 2048, 64, F16 | ACC, None) == tcr.OK
    assert raw.tcr_segmented_scan_ex(x[1:].data_ptr(), out.data_ptr(), 2048, 64, F16 | ACC, None) == tcr.ERR_UNSUPPORTED
    assert raw.tcr_scan_ex(None, None, 0, F16 | ACC, None) == tcr.OK
    assert raw.tcr_scan_ex(None, None, 0, ACC, None) == tcr.ERR_INVALID_ARG
    torch.cuda.synchronize()
