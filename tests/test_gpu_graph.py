"""GPU: the forward and backward calls recorded into a HIP graph (through torch's graph capture) and
replayed on new input data give the bits of the eager calls, replay after replay, with eager work and
synchronisations in between.  The library allocates nothing, never synchronises, and clears its queue
counters with kernels, which is what makes a call capturable; the first call of each kernel variant is
made outside the capture (it raises the kernel's dynamic-LDS limit)."""
import pytest
import torch

import workloads
from gpu_util import to_device

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("kind,N,d", [("causal_document", 1536, 128), ("shared_question", 1000, 64)])
def test_graph_replays_match_eager_calls(kind, N, d):
    import paper_2410_01359_amd as fm
    w = workloads.small_workload(kind, N, seed=900 + N, B=2, H=4, d=d)
    _, dev, vecs = to_device(w)
    q, k, v, dout = (dev[n].clone() for n in ("q", "k", "v", "dout"))
    ws_f = torch.empty(fm.flashmask_workspace_bytes(fm.FM_PASS_FWD, w.B, w.H, w.N, w.d), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(fm.flashmask_workspace_bytes(fm.FM_PASS_BWD, w.B, w.H, w.N, w.d), dtype=torch.uint8, device="cuda")

    def step():
        out, lse = fm.flashmask_fwd(q, k, v, *vecs, w.scale, workspace=ws_f)
        return (out, lse, *fm.flashmask_bwd(q, k, v, out, lse, dout, *vecs, w.scale, workspace=ws_b))

    step()                                   # outside the capture: LDS limits, lazy module loading
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        captured = step()
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5)
    for trial in range(4):
        for t in (q, k, v, dout):            # new data in the captured input buffers
            t.copy_(torch.randn(t.shape, device="cuda", generator=gen).bfloat16())
        eager = [x.clone() for x in step()]  # eager work between the replays, on the same workspaces
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name, a, b in zip(("out", "lse", "dq", "dk", "dv"), eager, captured):
            assert torch.equal(a, b), f"replay {trial}: {name} differs from the eager call"
