"""GPU: sizes beyond the five configurations, checked through closed forms that need no N x N work.

With Q = 0 every score is 0, so P is uniform over the allowed keys of a row (Equations 1-2):
    lse_i = log c_i,  out_i = mean of the visible V rows,  c_i = number of allowed keys,
and the gradients of Algorithm 2 reduce to sums over the allowed sets:
    dV_j = sum_{i sees j} dO_i / c_i,      dK = scale * dS^T Q = 0 exactly,
    dQ_i = scale / c_i * ( sum_{j visible} (dO_i . V_j) K_j  -  D_i * sum_{j visible} K_j ),
    D_i = dO_i . out_i.
For a causal mask the allowed set of row i is the prefix [0, i], so everything is a prefix or
suffix sum.  N = 262144 makes every tile loop rebuild its live list several times (more key / row
blocks than one list holds) and is the largest sequence the tests run.
"""
import numpy as np
import pytest
import torch

import workloads
from gpu_util import ABS_BWD, ABS_FWD, REL_FWD, bf16_to_np

pytestmark = pytest.mark.gpu


def _bf16_dev(x_f32: np.ndarray) -> torch.Tensor:
    bits = workloads.to_bf16_bits(x_f32)
    return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()


def _rounded(x_f32: np.ndarray) -> np.ndarray:
    return workloads.bf16_bits_to_f32(workloads.to_bf16_bits(x_f32)).astype(np.float64)


@pytest.mark.parametrize("N,d", [(262144, 64), (131072, 128), (10001, 128), (4099, 64)])
def test_causal_zero_query_closed_forms(N, d):
    import paper_2410_01359_amd as fm
    rng = np.random.Generator(np.random.PCG64(991 + N + d))
    k32, v32, do32 = (rng.standard_normal((N, d), dtype=np.float32) for _ in range(3))
    k, v, do = _rounded(k32), _rounded(v32), _rounded(do32)
    scale = 1.0 / np.sqrt(d)
    vec = tuple(torch.from_numpy(x[None].astype(np.int32)).cuda() for x in workloads.causal_mask(N))
    q_dev = torch.zeros((1, 1, N, d), dtype=torch.bfloat16, device="cuda")
    k_dev, v_dev, do_dev = (_bf16_dev(x)[None, None] for x in (k32, v32, do32))

    out, lse = fm.flashmask_fwd(q_dev, k_dev, v_dev, *vec, scale)
    dq, dk, dv = fm.flashmask_bwd(q_dev, k_dev, v_dev, out, lse, do_dev, *vec, scale)
    torch.cuda.synchronize()
    out_g, lse_g = bf16_to_np(out[0, 0]).astype(np.float64), lse[0, 0].cpu().numpy().astype(np.float64)
    dq_g, dk_g, dv_g = (bf16_to_np(t[0, 0]).astype(np.float64) for t in (dq, dk, dv))

    c = np.arange(1, N + 1, dtype=np.float64)                  # allowed keys of row i: 0..i
    # forward
    ref_lse = np.log(c)
    ref_out = np.cumsum(v, axis=0) / c[:, None]
    assert np.abs(lse_g - ref_lse).max() <= ABS_FWD
    big = ref_lse >= 1.0
    assert (np.abs(lse_g - ref_lse)[big] / ref_lse[big]).max() <= REL_FWD
    assert np.abs(out_g - ref_out).max() <= ABS_FWD
    # dK is exactly zero (Q = 0), dV is a suffix sum
    assert np.all(dk_g == 0.0)
    ref_dv = np.cumsum((do / c[:, None])[::-1], axis=0)[::-1]
    assert np.abs(dv_g - ref_dv).max() <= ABS_BWD
    # dQ on sampled rows (each costs O(i d)); the GPU backward was fed its own bf16 out
    out_used = out_g
    rows = np.unique(np.concatenate([rng.integers(0, N, size=24), [0, 1, 63, 64, 127, 128, N // 2, N - 129, N - 1]]))
    for i in rows:
        w_j = v[: i + 1] @ do[i]                                # dO_i . V_j for visible j
        d_i = do[i] @ out_used[i]
        ref = scale / c[i] * (w_j @ k[: i + 1] - d_i * k[: i + 1].sum(axis=0))
        assert np.abs(dq_g[i] - ref).max() <= ABS_BWD, f"dq row {i}"


def test_calls_on_a_side_stream_match_the_default_stream():
    """The library enqueues on the caller's stream: the same call issued on a non-default stream
    (default priority), with its own workspace, gives bit-identical results."""
    import paper_2410_01359_amd as fm
    from gpu_util import to_device
    w = workloads.small_workload("causal_document", 1024, seed=77, B=2, H=3, d=128)
    _, dev, vecs = to_device(w)
    out0, lse0 = fm.flashmask_fwd(dev["q"], dev["k"], dev["v"], *vecs, w.scale)
    g0 = fm.flashmask_bwd(dev["q"], dev["k"], dev["v"], out0, lse0, dev["dout"], *vecs, w.scale)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        out1, lse1 = fm.flashmask_fwd(dev["q"], dev["k"], dev["v"], *vecs, w.scale)
        g1 = fm.flashmask_bwd(dev["q"], dev["k"], dev["v"], out1, lse1, dev["dout"], *vecs, w.scale)
    side.synchronize()
    assert torch.equal(out0, out1) and torch.equal(lse0, lse1)
    for a, b in zip(g0, g1):
        assert torch.equal(a, b)


def test_backward_and_table_entry_points_reject_bad_arguments():
    import paper_2410_01359_amd as fm
    q = torch.zeros((1, 1, 256, 64), dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros((1, 1, 256), dtype=torch.float32, device="cuda")
    vec = torch.zeros((1, 256), dtype=torch.int32, device="cuda")
    with pytest.raises(fm.FlashMaskError):
        fm.flashmask_bwd(q, q, q, q, lse, q, vec, vec, vec, vec, 0.0)      # scale must be positive
    with pytest.raises(fm.FlashMaskError):
        fm.flashmask_bwd(q, q, q, q, lse, q, vec, vec, vec, vec, float("nan"))
    with pytest.raises(fm.FlashMaskError):
        fm.flashmask_bwd(q, q, q, q, lse, q, vec, vec, vec, vec, 1.0,
                         workspace=torch.empty(512, dtype=torch.uint8, device="cuda"))   # workspace too small
    with pytest.raises(fm.FlashMaskError):
        fm.flashmask_fwd(q, q, q, vec, vec, vec, vec, -1.0)
    with pytest.raises(fm.FlashMaskError):
        fm.flashmask_preprocess(vec, vec, vec, vec, 48)                    # block size not a multiple of 32


def test_two_host_threads_on_two_streams_match_serial_calls():
    """Distinct streams with distinct workspaces may be driven from different host threads at the same
    time: forward + backward issued concurrently from two threads (different shapes, so different kernel
    instantiations raise their LDS limits for the first time in parallel too) give the bits of serial calls."""
    import threading
    import paper_2410_01359_amd as fm
    from gpu_util import to_device
    cases = [workloads.small_workload("causal_document", 2048, seed=301, B=1, H=6, d=128),
             workloads.small_workload("shared_question", 1500, seed=302, B=2, H=3, d=64)]
    inputs = [to_device(w)[1:] for w in cases]

    def run(idx, stream, rounds, sink):
        w, (dev, vecs) = cases[idx], inputs[idx]
        ws_f = torch.empty(fm.flashmask_workspace_bytes(fm.FM_PASS_FWD, w.B, w.H, w.N, w.d), dtype=torch.uint8, device="cuda")
        ws_b = torch.empty(fm.flashmask_workspace_bytes(fm.FM_PASS_BWD, w.B, w.H, w.N, w.d), dtype=torch.uint8, device="cuda")
        with torch.cuda.stream(stream):
            for _ in range(rounds):
                out, lse = fm.flashmask_fwd(dev["q"], dev["k"], dev["v"], *vecs, w.scale, workspace=ws_f)
                grads = fm.flashmask_bwd(dev["q"], dev["k"], dev["v"], out, lse, dev["dout"], *vecs, w.scale, workspace=ws_b)
            stream.synchronize()
        sink[idx] = (out, lse, *grads)

    serial, threaded = {}, {}
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    threads = [threading.Thread(target=run, args=(i, streams[i], 8, threaded)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    for i in range(2):
        run(i, torch.cuda.current_stream(), 1, serial)
    torch.cuda.synchronize()
    for i in range(2):
        assert len(threaded[i]) == 5
        for a, b in zip(serial[i], threaded[i]):
            assert torch.equal(a, b), f"case {i}"
