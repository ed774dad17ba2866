"""GPU: forward parity (out, lse) vs the fp64 oracle through the C ABI."""
import math

import numpy as np
import pytest
import torch

import workloads
from gpu_util import bf16_to_np, check_fwd, f64, to_device
from oracle import flashmask_oracle as orc

pytestmark = pytest.mark.gpu

KINDS = ["full", "causal", "sliding_window", "document", "causal_document", "shared_question", "prefix_lm",
         "prefix_document", "global_sliding_window", "causal_blockwise", "random_eviction", "qk_sparse", "random_intervals"]


def run_small(kind, N, d, seed, B=2, H=2):
    import paper_2410_01359_amd as fm
    w = workloads.small_workload(kind, N, seed=seed, B=B, H=H, d=d)
    bits, dev, vecs = to_device(w, ("q", "k", "v"))
    out, lse = fm.flashmask_fwd(dev["q"], dev["k"], dev["v"], *vecs, w.scale)
    torch.cuda.synchronize()
    out, lse = bf16_to_np(out), lse.cpu().numpy()
    for b in range(B):
        for h in range(H):
            ro, rl = orc.forward(f64(bits["q"][b, h]), f64(bits["k"][b, h]), f64(bits["v"][b, h]), *w.vectors[b], w.scale)
            check_fwd(out[b, h], lse[b, h], ro, rl, f"{kind} N={N} d={d} b={b} h={h}")


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("N,d", [(128, 64), (384, 128), (640, 64), (1024, 128)])
def test_forward_small(kind, N, d):
    run_small(kind, N, d, seed=17 + N + d)


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("N,d", [(1, 64), (77, 128), (129, 64), (200, 128), (333, 64), (1000, 128)])
def test_forward_ragged_lengths(kind, N, d):
    """Sequence lengths that are not a multiple of the tile sizes (or of anything)."""
    if N < 8 and kind not in ("full", "causal", "random_intervals"):
        pytest.skip("family needs a few rows")
    run_small(kind, N, d, seed=91 + N + d)


def test_forward_config1_all_heads():
    import paper_2410_01359_amd as fm
    w = workloads.config("1")
    bits, dev, vecs = to_device(w, ("q", "k", "v"))
    out, lse = fm.flashmask_fwd(dev["q"], dev["k"], dev["v"], *vecs, w.scale)
    torch.cuda.synchronize()
    for h in range(w.H):
        ro, rl = orc.forward(f64(bits["q"][0, h]), f64(bits["k"][0, h]), f64(bits["v"][0, h]), *w.vectors[0], w.scale)
        check_fwd(bf16_to_np(out[0, h]), lse[0, h].cpu().numpy(), ro, rl, f"config 1 head {h}")


def test_forward_rows_with_no_visible_key():
    """A column interval covering everything: rows lose every key -> out = 0, lse = -inf."""
    import paper_2410_01359_amd as fm
    N, d = 256, 64
    w = workloads.small_workload("causal", N, seed=3, B=1, H=1, d=d)
    lts, lte, uts, ute = (v.copy() for v in w.vectors[0])
    lts[:] = 100; lte[:] = 140          # rows 100..139 see nothing below/at the diagonal either
    uts[:] = 0; ute[:] = np.arange(N)
    w.vectors = [(lts, lte, uts, ute)]
    bits, dev, vecs = to_device(w, ("q", "k", "v"))
    out, lse = fm.flashmask_fwd(dev["q"], dev["k"], dev["v"], *vecs, w.scale)
    torch.cuda.synchronize()
    ro, rl = orc.forward(f64(bits["q"][0, 0]), f64(bits["k"][0, 0]), f64(bits["v"][0, 0]), *w.vectors[0], w.scale)
    assert np.isneginf(rl[100:140]).all()
    check_fwd(bf16_to_np(out[0, 0]), lse[0, 0].cpu().numpy(), ro, rl, "dead rows")
    assert np.all(bf16_to_np(out[0, 0])[100:140] == 0.0)


def test_forward_rejects_bad_arguments():
    import paper_2410_01359_amd as fm
    q = torch.zeros((1, 1, 256, 96), dtype=torch.bfloat16, device="cuda")
    vec = torch.zeros((1, 256), dtype=torch.int32, device="cuda")
    with pytest.raises(fm.FlashMaskError):
        fm.flashmask_fwd(q, q, q, vec, vec, vec, vec, 1.0)             # d not supported
    q = torch.zeros((1, 1, 256, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(fm.FlashMaskError):
        fm.flashmask_fwd(q, q, q, vec, vec, vec, vec, 1.0, workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
