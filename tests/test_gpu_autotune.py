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


def test_autotune_picks_valid_shapes_and_results_stay_exact(tcr, oracle, data):
    x, xd = data
    out = torch.empty(N, dtype=torch.float32, device="cuda")
    try:
        tcr.autotune(tcr.OP_SEGMENTED_SCAN, xd[:N], out, 1 << 14)
        tcr.autotune(tcr.OP_SEGMENTED_REDUCE, xd[:N], out, 1 << 14)
        tcr.autotune(tcr.OP_SCAN, xd[:N], out, 0)
        tcr.autotune(tcr.OP_REDUCE, xd[:N], out, 0)
        tcr.autotune(tcr.OP_SEGMENTED_SCAN, xd[:N], out, 64)             # single shape: no entry
        table = dict(item.split("=") for item in tcr.tuning_export().split(";") if item)
        assert set(table) == {"scan:14", "reduce:14", "scan:41", "reduce:41"}
        assert int(table["scan:14"]) in range(4, 10)                     # shares that hold a 16384-element segment
        assert int(table["scan:41"]) in (7, 8, 9, 10, 11)
        assert np.array_equal(tcr.segmented_scan(xd[:N], 1 << 14).cpu().numpy().astype(np.float64),
                              oracle.segmented_scan(x[:N], 1 << 14))
        assert np.array_equal(tcr.segmented_reduce(xd[:N], 1 << 14).cpu().numpy().astype(np.float64),
                              oracle.segmented_reduce(x[:N], 1 << 14))
        assert np.array_equal(tcr.scan(xd[:N]).cpu().numpy().astype(np.float64), oracle.scan(x[:N]))
        assert float(tcr.reduce(xd[:N]).cpu()) == oracle.reduce(x[:N])
        tcr.check_device_flags()
    finally:
        tcr.tuning_import("")
