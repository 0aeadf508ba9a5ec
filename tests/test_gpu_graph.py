"""HIP graph capture: calls that need no library workspace can be recorded and replayed; calls that need it
refuse while the stream is capturing (their epoch and ticket arguments would be frozen into the graph)."""
import numpy as np
import pytest
import torch

from paper_1811_09736_amd import workloads

pytestmark = pytest.mark.gpu

N = 1 << 20


@pytest.fixture(scope="module")
def tcr():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_1811_09736_amd import binding
    binding.set_variant("reset")
    binding.tuning_import("")
    yield binding
    binding.check_device_flags()


def test_capture_and_replay_of_workspace_free_calls(tcr, oracle):
    inputs = [workloads.make_input(N, "int8", (21, k)) for k in range(3)]
    x = torch.from_numpy(inputs[0]).cuda()
    scan256 = torch.empty(N, dtype=torch.float32, device="cuda")
    scan4096 = torch.empty(N, dtype=torch.float32, device="cuda")
    red16 = torch.empty(N // 16, dtype=torch.float32, device="cuda")
    red64k = torch.empty(N // 65536, dtype=torch.float32, device="cuda")

    def calls():
        tcr.segmented_scan(x, 256, out=scan256)
        tcr.segmented_scan(x, 4096, out=scan4096)
        tcr.segmented_reduce(x, 16, out=red16)
        tcr.segmented_reduce(x, 65536, out=red64k)

    calls()                                              # eager once: nothing below is a first call
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        calls()
        with pytest.raises(tcr.TcrError) as err:         # needs the look-back workspace: refused, nothing recorded
            tcr.segmented_scan(x, 1 << 16, out=scan4096)
        assert err.value.status == tcr.ERR_UNSUPPORTED
        with pytest.raises(tcr.TcrError):
            tcr.scan(x, out=scan4096)
    for k in (1, 2, 0, 1):                               # several replays, eager work and synchronisation in between
        x.copy_(torch.from_numpy(inputs[k]).cuda())
        for t in (scan256, scan4096, red16, red64k):
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        h = inputs[k]
        assert np.array_equal(scan256.cpu().numpy().astype(np.float64), oracle.segmented_scan(h, 256))
        assert np.array_equal(scan4096.cpu().numpy().astype(np.float64), oracle.segmented_scan(h, 4096))
        assert np.array_equal(red16.cpu().numpy().astype(np.float64), oracle.segmented_reduce(h, 16))
        assert np.array_equal(red64k.cpu().numpy().astype(np.float64), oracle.segmented_reduce(h, 65536))
        # the eager long scan still works between replays
        got = tcr.scan(x).cpu().numpy().astype(np.float64)
        assert np.array_equal(got, oracle.scan(h))
