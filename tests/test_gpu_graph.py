"""The schedules enqueue kernels, copies and event waits only (no allocation, no memset node, no
host wait), so a caller can capture them in a HIP graph; with offload the library's side streams
fork from and join back into the captured stream through events.  The graph is replayed
several times with eager work and synchronisations in between, and every replay is compared bit
for bit with the eager result."""
import pytest
import torch

from paper_2408_16978_amd import binding as B
from paper_2408_16978_amd import inputs, runner

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("flags", [0, B.FPDT_PAIRWISE | B.FPDT_BWD_KV_OUTER, B.FPDT_KV_ON_HOST,
                                   B.FPDT_KV_ON_HOST | B.FPDT_BWD_Q_OUTER,
                                   B.FPDT_KV_ON_HOST | B.FPDT_ACT_ON_HOST,
                                   B.FPDT_KV_ON_HOST | B.FPDT_BWD_STORE_DS])
def test_forward_and_backward_replay_from_a_graph(flags):
    S, chunk, Hq, Hkv, D = 2304, 256, 8, 2, 128  # nine chunks: every staging buffer is reused
    print("[case] graph capture", S, chunk, Hq, Hkv, D, flags, flush=True)
    Q, K, V, dO = inputs.make_qkvdo(S, Hq, Hkv, D, "bf16", seed=12)
    b = runner.make_buffers(Q, K, V, dO, chunk, D ** -0.5, flags)
    outs = ("O", "LSE", "dQ", "dK", "dV")
    runner.forward(b)
    runner.backward(b)
    torch.cuda.synchronize()
    want = {n: getattr(b, n).clone() for n in outs}

    side = torch.cuda.Stream()  # default priority
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        runner.forward(b)
        runner.backward(b)
    for rep in range(3):
        for n in outs:  # eager work between the replays: poison what the graph must rewrite
            getattr(b, n).fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for n in outs:
            assert torch.equal(getattr(b, n).view(torch.uint8), want[n].view(torch.uint8)), (n, rep)
    # and eagerly again after the capture, on the default stream
    for n in outs:
        getattr(b, n).fill_(float("nan"))
    runner.forward(b)
    runner.backward(b)
    torch.cuda.synchronize()
    for n in outs:
        assert torch.equal(getattr(b, n).view(torch.uint8), want[n].view(torch.uint8)), (n, "eager after")
