"""GPU: flashmask_fwd_noalloc (the forward with the library's static scratch, for callers that cannot
allocate) against flashmask_fwd, through the C ABI: two calls in a row, the second on a smaller input,
so that what the first call left in the shared scratch is shown to be harmless."""
import ctypes

import pytest
import torch

import workloads
from gpu_util import to_device

pytestmark = pytest.mark.gpu


def _both(w):
    import paper_2410_01359_amd as fm
    _, dev, vecs = to_device(w, ("q", "k", "v"))
    ref_out, ref_lse = fm.flashmask_fwd(dev["q"], dev["k"], dev["v"], *vecs, w.scale)
    out = torch.full_like(ref_out, float("nan"))
    lse = torch.full((w.B, w.H, w.N), float("nan"), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    fm.flashmask_fwd_noalloc(dev["q"], dev["k"], dev["v"], *vecs, w.scale, out, lse)
    after = torch.cuda.memory_stats()["allocation.all.allocated"]
    torch.cuda.synchronize()
    assert after == before, "the call went through torch's allocator"
    return ref_out, ref_lse, out, lse


def test_noalloc_forward_matches_forward_on_two_calls_in_a_row():
    # first a problem with many units and a ragged length (padded bound vectors in the scratch too),
    # then a smaller one whose tables and queues cover only the front of what the first call wrote
    big = workloads.small_workload("causal_document", 3000, seed=11, B=2, H=5, d=128)
    small = workloads.small_workload("shared_question", 640, seed=12, B=1, H=3, d=64)
    for w in (big, small, big):
        ref_out, ref_lse, out, lse = _both(w)
        assert torch.equal(ref_out.view(torch.int16), out.view(torch.int16)), w.name
        assert torch.equal(ref_lse.view(torch.int32), lse.view(torch.int32)), w.name


def test_noalloc_forward_rejects_what_does_not_fit():
    import paper_2410_01359_amd as fm
    lib = fm.load_library()
    B, H, N, d = 64, 64, 16384, 128          # 524288 row blocks: 8 MiB of queue records
    assert fm.flashmask_workspace_bytes(fm.FM_PASS_FWD, B, H, N, d) > (4 << 20)
    x = torch.zeros(16, dtype=torch.int32, device="cuda")       # never touched: the size check comes first
    p = x.data_ptr()
    rc = lib.flashmask_fwd_noalloc(p, p, p, p, p, p, p, ctypes.c_float(1.0), p, p, B, H, N, d, None)
    assert rc == -7 and b"static" in lib.flashmask_strerror(rc)
