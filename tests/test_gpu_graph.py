"""HIP graph capture: calls that need no workspace can always be recorded and replayed; calls that need one can
once it exists (a recorded launch takes its epoch and ticket base from the device, not from frozen kernel
arguments), and refuse while it would have to be created during the capture."""
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


def test_chained_scans_in_a_graph(tcr, oracle):
    n = (1 << 22) + 4096
    inputs = [workloads.make_input(n, "int8", (23, k)) for k in range(3)]
    x = torch.from_numpy(inputs[0]).cuda()
    full = torch.empty(n, dtype=torch.float32, device="cuda")
    seg = torch.empty(1 << 22, dtype=torch.float32, device="cuda")
    look = torch.empty(n - 8, dtype=torch.float32, device="cuda")
    total = torch.empty(1, dtype=torch.float32, device="cuda")
    side = torch.cuda.Stream()

    def calls():
        tcr.scan(x, out=full)                                  # the pipelined chain
        tcr.segmented_scan(x[: 1 << 22], 1 << 17, out=seg)     # chained segments
        tcr.tuning_import("scan:41=9;")
        tcr.scan(x[: n - 8], out=look)                         # decoupled look-back on the same table
        tcr.tuning_import("")
        tcr.reduce(x, out=total)                               # partials + second kernel

    # a workspace that does not exist yet cannot be created while capturing
    tcr.release()
    torch.cuda.synchronize()
    fresh = torch.cuda.CUDAGraph()
    with torch.cuda.graph(fresh, stream=side):
        with pytest.raises(tcr.TcrError) as err:
            tcr.scan(x, out=full)
        assert err.value.status == tcr.ERR_UNSUPPORTED
        tcr.segmented_scan(x, 256, out=full)                   # something to record, so the capture is not empty
    with torch.cuda.stream(side):
        calls()                                                # eager once on the capture stream: its workspace exists now
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        calls()
    for k in (1, 2, 0, 1, 2):
        x.copy_(torch.from_numpy(inputs[k]).cuda())
        for t in (full, seg, look, total):
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        h = inputs[k]
        ref = oracle.scan(h)
        assert np.array_equal(full.cpu().numpy().astype(np.float64), ref)
        assert np.array_equal(look.cpu().numpy().astype(np.float64), ref[: n - 8])
        assert np.array_equal(seg.cpu().numpy().astype(np.float64), oracle.segmented_scan(h[: 1 << 22], 1 << 17))
        assert float(total.cpu()[0]) == oracle.reduce(h)
        # eager calls on the same stream share the device-managed counters with the graph
        with torch.cuda.stream(side):
            got = tcr.scan(x)
        side.synchronize()
        assert np.array_equal(got.cpu().numpy().astype(np.float64), ref)
    tcr.check_device_flags(side)
