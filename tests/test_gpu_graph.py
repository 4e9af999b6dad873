"""The resident schedules enqueue kernels only (no allocation, no memset, no host wait), so a
caller can capture them in a HIP graph.  The graph is replayed several times with eager work and
synchronisations in between, and every replay is compared bit for bit with the eager result."""
import pytest
import torch

from paper_2408_16978_amd import binding as B
from paper_2408_16978_amd import inputs, runner

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("flags", [0, B.FPDT_PAIRWISE | B.FPDT_BWD_KV_OUTER])
def test_forward_and_backward_replay_from_a_graph(flags):
    S, chunk, Hq, Hkv, D = 2048, 512, 8, 2, 128
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


def test_offload_schedules_refuse_capture():
    """They fork onto the library's side streams, which a capture cannot follow: refused with a
    clear status before anything is enqueued, and the capture itself stays valid."""
    S, chunk, Hq, Hkv, D = 1024, 256, 4, 2, 128
    Q, K, V, dO = inputs.make_qkvdo(S, Hq, Hkv, D, "bf16", seed=13)
    b = runner.make_buffers(Q, K, V, dO, chunk, D ** -0.5, B.FPDT_KV_ON_HOST)
    runner.forward(b)  # eager: fine
    torch.cuda.synchronize()
    x = torch.zeros(8, device="cuda")
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=torch.cuda.Stream()):
        x.add_(1.0)
        with pytest.raises(B.FpdtError) as e:
            runner.forward(b)
        assert e.value.status == B.FPDT_ERR_UNSUPPORTED and "captured" in str(e.value)
    g.replay()
    torch.cuda.synchronize()
    assert float(x[0]) == 1.0
    runner.forward(b)  # and the library still works afterwards
    torch.cuda.synchronize()
