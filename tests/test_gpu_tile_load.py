"""The measured alternatives to loading matrix-core operands directly (tcr_set_variant("tile_load", ...)): tiles
staged through LDS from lane-ordered loads, and gfx950's load from memory into LDS.  Same arithmetic, so every
variant must give the oracle's result bit for bit on integer-valued inputs."""
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


@pytest.mark.parametrize("how", ["direct", "lds", "lds_dma"])
@pytest.mark.parametrize("seg", [16, 32, 64, 128, 256, 512])
def test_every_tile_load_matches_oracle(tcr, oracle, seg, how):
    n = (1 << 20) + 512 * 5 + seg * 3                    # full tiles, then a ragged tail
    x = workloads.make_input(n, "int8", seg)
    xd = torch.from_numpy(x).cuda()
    tcr.set_variant("tile_load", how)
    try:
        scan = tcr.segmented_scan(xd, seg).cpu().numpy().astype(np.float64)
        red = tcr.segmented_reduce(xd, seg).cpu().numpy().astype(np.float64)
    finally:
        tcr.set_variant("reset")
    assert np.array_equal(scan, oracle.segmented_scan(x, seg))
    assert np.array_equal(red, oracle.segmented_reduce(x, seg))


def test_unknown_value_is_rejected(tcr):
    with pytest.raises(tcr.TcrError):
        tcr.set_variant("tile_load", "texture")
