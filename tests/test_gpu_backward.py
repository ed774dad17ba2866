"""GPU: backward parity (dq, dk, dv) vs the fp64 oracle through the C ABI.

The GPU backward consumes the GPU forward's own out (bf16) and lse (fp32), as a
training step would; the oracle backward uses its own fp64 forward."""
import numpy as np
import pytest
import torch

import workloads
from gpu_util import bf16_to_np, check_bwd, check_fwd, f64, to_device
from oracle import flashmask_oracle as orc

pytestmark = pytest.mark.gpu

KINDS = ["full", "causal", "sliding_window", "document", "causal_document", "shared_question", "prefix_lm",
         "prefix_document", "global_sliding_window", "causal_blockwise", "random_eviction", "qk_sparse", "random_intervals"]


def run_fwd_bwd(w):
    import paper_2410_01359_amd as fm
    bits, dev, vecs = to_device(w)
    out, lse = fm.flashmask_fwd(dev["q"], dev["k"], dev["v"], *vecs, w.scale)
    dq, dk, dv = fm.flashmask_bwd(dev["q"], dev["k"], dev["v"], out, lse, dev["dout"], *vecs, w.scale)
    torch.cuda.synchronize()
    return bits, out, lse, dq, dk, dv


def compare_all(w, bits, out, lse, dq, dk, dv, tag):
    for b in range(w.B):
        for h in range(w.H):
            args = [f64(bits[n][b, h]) for n in ("q", "k", "v", "dout")]
            rdq, rdk, rdv, ro, rl = orc.backward(*args, *w.vectors[b], w.scale)
            what = f"{tag} b={b} h={h}"
            check_fwd(bf16_to_np(out[b, h]), lse[b, h].cpu().numpy(), ro, rl, what)
            check_bwd(bf16_to_np(dq[b, h]), rdq, "dq", what)
            check_bwd(bf16_to_np(dk[b, h]), rdk, "dk", what)
            check_bwd(bf16_to_np(dv[b, h]), rdv, "dv", what)


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("N,d", [(128, 64), (384, 128), (640, 64), (1024, 128)])
def test_backward_small(kind, N, d):
    w = workloads.small_workload(kind, N, seed=29 + N + d, B=2, H=2, d=d)
    compare_all(w, *run_fwd_bwd(w), f"{kind} N={N} d={d}")


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("N,d", [(1, 64), (77, 128), (129, 64), (200, 128), (333, 64), (1000, 128)])
def test_backward_ragged_lengths(kind, N, d):
    """Sequence lengths that are not a multiple of the tile sizes (or of anything)."""
    if N < 8 and kind not in ("full", "causal", "random_intervals"):
        pytest.skip("family needs a few rows")
    w = workloads.small_workload(kind, N, seed=57 + N + d, B=2, H=2, d=d)
    compare_all(w, *run_fwd_bwd(w), f"{kind} N={N} d={d}")


@pytest.mark.parametrize("kind", ["causal_document", "random_intervals"])
def test_backward_many_slices(kind):
    """40 (batch row, head) slices: five per unit queue, i.e. three groups of slices per queue, the
    last one partial, each batch row with its own mask."""
    w = workloads.small_workload(kind, 384, seed=83, B=5, H=8, d=64)
    compare_all(w, *run_fwd_bwd(w), f"{kind} B=5 H=8")


def test_backward_config1_all_heads():
    w = workloads.config("1")
    compare_all(w, *run_fwd_bwd(w), "config 1")


def test_backward_is_bit_reproducible():
    import paper_2410_01359_amd as fm
    w = workloads.small_workload("shared_question", 1024, seed=5, B=1, H=4, d=128)
    bits, dev, vecs = to_device(w)
    out, lse = fm.flashmask_fwd(dev["q"], dev["k"], dev["v"], *vecs, w.scale)
    first = fm.flashmask_bwd(dev["q"], dev["k"], dev["v"], out, lse, dev["dout"], *vecs, w.scale)
    second = fm.flashmask_bwd(dev["q"], dev["k"], dev["v"], out, lse, dev["dout"], *vecs, w.scale)
    torch.cuda.synchronize()
    for x, y in zip(first, second):
        assert torch.equal(x.view(torch.int16), y.view(torch.int16))


def test_backward_rows_with_no_visible_key():
    N, d = 256, 64
    w = workloads.small_workload("causal", N, seed=3, B=1, H=1, d=d)
    lts, lte, uts, ute = (v.copy() for v in w.vectors[0])
    lts[:] = 100; lte[:] = 140
    w.vectors = [(lts, lte, uts, ute)]
    bits, out, lse, dq, dk, dv = run_fwd_bwd(w)
    compare_all(w, bits, out, lse, dq, dk, dv, "dead rows")
    assert np.all(bf16_to_np(dq[0, 0])[100:140] == 0.0)
