"""GPU: the strided / grouped-K/V-head entry points (flashmask_fwd_ex, flashmask_bwd_ex)
against the fp64 oracle, through the C ABI.

Layouts: [B,N,H,d] storage viewed as [B,H,N,d], and q/k/v taken as slices of one packed
[B,N,3,H,d] projection.  Grouped heads: query head h reads K/V head h // (H // H_kv); the
oracle is run per query head on that K/V head and its dk, dv are summed over the group."""
import numpy as np
import pytest
import torch

import workloads
from gpu_util import bf16_to_np, check_bwd, check_fwd, f64
from oracle import flashmask_oracle as orc

pytestmark = pytest.mark.gpu


def _dev(bits):
    return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()


def _inputs(kind, B, H, Hk, N, d, seed):
    w = workloads.small_workload(kind, N, seed=seed, B=B, H=H, d=d)
    bits = workloads.make_tensors(w.seed, B, H, N, d, ("q", "dout"))
    bits.update(workloads.make_tensors(w.seed + 1, B, Hk, N, d, ("k", "v")))
    vecs = tuple(torch.from_numpy(v).cuda() for v in w.stacked_vectors())
    return w, bits, vecs


def _oracle_check(w, bits, H, Hk, out, lse, dq, dk, dv, tag):
    for b in range(w.B):
        args = [np.stack([f64(bits[n][b, h]) for h in range(bits[n].shape[1])]) for n in ("q", "k", "v", "dout")]
        rdq, rdk, rdv, ro, rl = orc.backward_grouped(*args, *w.vectors[b], w.scale)
        for h in range(H):
            what = f"{tag} b={b} h={h}"
            check_fwd(bf16_to_np(out[b, h]), lse[b, h].cpu().numpy(), ro[h], rl[h], what)
            check_bwd(bf16_to_np(dq[b, h]), rdq[h], "dq", what)
        for hk in range(Hk):
            check_bwd(bf16_to_np(dk[b, hk]), rdk[hk], "dk", f"{tag} b={b} hk={hk}")
            check_bwd(bf16_to_np(dv[b, hk]), rdv[hk], "dv", f"{tag} b={b} hk={hk}")


def _bnhd(t):
    """The same values stored [B,N,H,d], viewed [B,H,N,d]."""
    return t.transpose(1, 2).contiguous().transpose(1, 2)


@pytest.mark.parametrize("kind", ["causal_document", "shared_question", "sliding_window", "random_intervals"])
@pytest.mark.parametrize("N,d", [(384, 128), (640, 64), (333, 128), (77, 64)])
def test_bnhd_layout_matches_oracle_and_contiguous_call(kind, N, d):
    import paper_2410_01359_amd as fm
    B, H = 2, 3
    w, bits, vecs = _inputs(kind, B, H, H, N, d, seed=101 + N + d)
    t = {n: _dev(bits[n]) for n in bits}
    s = {n: _bnhd(x) for n, x in t.items()}
    assert not s["q"].is_contiguous()
    out, lse = fm.flashmask_fwd_ex(s["q"], s["k"], s["v"], *vecs, w.scale)
    assert out.stride() == s["q"].stride()
    dq, dk, dv = fm.flashmask_bwd_ex(s["q"], s["k"], s["v"], out, lse, s["dout"], *vecs, w.scale)
    torch.cuda.synchronize()
    _oracle_check(w, bits, H, H, out, lse, dq, dk, dv, f"bnhd {kind} N={N} d={d}")
    # same arithmetic in the same order as the contiguous entry points: identical bits
    out_c, lse_c = fm.flashmask_fwd(t["q"], t["k"], t["v"], *vecs, w.scale)
    dq_c, dk_c, dv_c = fm.flashmask_bwd(t["q"], t["k"], t["v"], out_c, lse_c, t["dout"], *vecs, w.scale)
    torch.cuda.synchronize()
    assert torch.equal(out.contiguous().view(torch.int16), out_c.view(torch.int16))
    assert torch.equal(lse, lse_c)
    for x, y in ((dq, dq_c), (dk, dk_c), (dv, dv_c)):
        assert torch.equal(x.contiguous().view(torch.int16), y.view(torch.int16))


@pytest.mark.parametrize("N,d", [(512, 128), (200, 64)])
def test_packed_qkv_projection(N, d):
    """q, k, v are slices of one [B,N,3,H,d] tensor (row stride 3*H*d)."""
    import paper_2410_01359_amd as fm
    B, H = 1, 2
    w, bits, vecs = _inputs("causal_document", B, H, H, N, d, seed=211 + N)
    packed = torch.empty((B, N, 3, H, d), dtype=torch.bfloat16, device="cuda")
    for idx, n in enumerate(("q", "k", "v")):
        packed[:, :, idx] = _dev(bits[n]).transpose(1, 2)
    q, k, v = (packed[:, :, idx].transpose(1, 2) for idx in range(3))
    dout = _dev(bits["dout"])
    out, lse = fm.flashmask_fwd_ex(q, k, v, *vecs, w.scale)
    dq, dk, dv = fm.flashmask_bwd_ex(q, k, v, out, lse, dout, *vecs, w.scale)
    torch.cuda.synchronize()
    _oracle_check(w, bits, H, H, out, lse, dq, dk, dv, f"packed N={N} d={d}")


@pytest.mark.parametrize("kind", ["causal_document", "shared_question", "prefix_lm", "document"])
@pytest.mark.parametrize("H,Hk,N,d", [(4, 2, 384, 128), (4, 1, 300, 64), (8, 2, 1024, 128), (6, 3, 129, 64)])
def test_grouped_kv_heads(kind, H, Hk, N, d):
    import paper_2410_01359_amd as fm
    B = 2
    w, bits, vecs = _inputs(kind, B, H, Hk, N, d, seed=307 + N + H)
    t = {n: _dev(bits[n]) for n in bits}
    out, lse = fm.flashmask_fwd_ex(t["q"], t["k"], t["v"], *vecs, w.scale)
    dq, dk, dv = fm.flashmask_bwd_ex(t["q"], t["k"], t["v"], out, lse, t["dout"], *vecs, w.scale)
    torch.cuda.synchronize()
    assert tuple(dk.shape) == (B, Hk, N, d) and tuple(dv.shape) == (B, Hk, N, d)
    _oracle_check(w, bits, H, Hk, out, lse, dq, dk, dv, f"gqa {kind} H={H}/{Hk} N={N} d={d}")


def test_grouped_heads_in_bnhd_layout_inference_shape():
    """The head configuration of the paper's inference appendix (32 query heads on 8 K/V heads,
    d = 128) at a length the oracle still finishes quickly, stored [B,N,H,d]; two heads checked."""
    import paper_2410_01359_amd as fm
    B, H, Hk, N, d = 1, 32, 8, 2048, 128
    w, bits, vecs = _inputs("causal_document", B, H, Hk, N, d, seed=409)
    s = {n: _bnhd(_dev(bits[n])) for n in bits}
    out, lse = fm.flashmask_fwd_ex(s["q"], s["k"], s["v"], *vecs, w.scale)
    dq, dk, dv = fm.flashmask_bwd_ex(s["q"], s["k"], s["v"], out, lse, s["dout"], *vecs, w.scale)
    torch.cuda.synchronize()
    G = H // Hk
    for hk in (0, Hk - 1):
        ref_dk, ref_dv = 0.0, 0.0
        for h in range(hk * G, (hk + 1) * G):
            rdq, rdk, rdv, ro, rl = orc.backward(f64(bits["q"][0, h]), f64(bits["k"][0, hk]), f64(bits["v"][0, hk]),
                                                 f64(bits["dout"][0, h]), *w.vectors[0], w.scale)
            check_fwd(bf16_to_np(out[0, h]), lse[0, h].cpu().numpy(), ro, rl, f"h={h}")
            check_bwd(bf16_to_np(dq[0, h]), rdq, "dq", f"h={h}")
            ref_dk, ref_dv = ref_dk + rdk, ref_dv + rdv
        check_bwd(bf16_to_np(dk[0, hk]), ref_dk, "dk", f"hk={hk}")
        check_bwd(bf16_to_np(dv[0, hk]), ref_dv, "dv", f"hk={hk}")


def test_grouped_heads_bnhd_long_sequence_closed_form():
    """Q = 0 under a causal mask: lse_i = log(i + 1), out_i = prefix mean of V, dK = 0 and dV a
    suffix sum (summed over the query heads of a group) -- checked on every row at a ragged length
    whose live lists are rebuilt (more key blocks than one list holds), stored [B,N,H,d]."""
    import paper_2410_01359_amd as fm
    from gpu_util import ABS_BWD, ABS_FWD
    B, H, Hk, N, d = 1, 4, 2, 70001, 128
    G = H // Hk
    rng = np.random.Generator(np.random.PCG64(5150))
    kv = rng.standard_normal((2, B, Hk, N, d), dtype=np.float32)
    do32 = rng.standard_normal((B, H, N, d), dtype=np.float32)
    to_dev = lambda x: _bnhd(_dev(workloads.to_bf16_bits(x)))
    rounded = lambda x: workloads.bf16_bits_to_f32(workloads.to_bf16_bits(x)).astype(np.float64)
    q = _bnhd(torch.zeros((B, H, N, d), dtype=torch.bfloat16, device="cuda"))
    k, v, do = to_dev(kv[0]), to_dev(kv[1]), to_dev(do32)
    vecs = tuple(torch.from_numpy(x[None].astype(np.int32)).cuda() for x in workloads.causal_mask(N))
    scale = 1.0 / np.sqrt(d)
    out, lse = fm.flashmask_fwd_ex(q, k, v, *vecs, scale)
    dq, dk, dv = fm.flashmask_bwd_ex(q, k, v, out, lse, do, *vecs, scale)
    torch.cuda.synchronize()
    c = np.arange(1, N + 1, dtype=np.float64)
    vr, dor = rounded(kv[1]), rounded(do32)
    for h in range(H):
        assert np.abs(lse[0, h].cpu().numpy() - np.log(c)).max() <= ABS_FWD
        assert np.abs(bf16_to_np(out[0, h]) - np.cumsum(vr[0, h // G], axis=0) / c[:, None]).max() <= ABS_FWD
    assert torch.count_nonzero(dk.float()) == 0
    for hk in range(Hk):
        ref = sum(np.cumsum((dor[0, h] / c[:, None])[::-1], axis=0)[::-1] for h in range(hk * G, (hk + 1) * G))
        assert np.abs(bf16_to_np(dv[0, hk]) - ref).max() <= ABS_BWD


def test_forward_backward_inside_a_hip_graph():
    """The whole path (preprocessing, unit queues, tile loops) captured into a HIP graph and
    replayed with new inputs: every replay is bit-identical to the eager call on the same
    inputs (the library allocates nothing and its only global-memory clears are kernels)."""
    import paper_2410_01359_amd as fm
    B, H, Hk, N, d = 2, 4, 2, 1000, 128
    w, bits, vecs = _inputs("shared_question", B, H, Hk, N, d, seed=613)
    t = {n: _dev(bits[n]) for n in bits}
    ws_f = torch.empty(fm.flashmask_workspace_bytes(fm.FM_PASS_FWD, B, H, N, d), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(fm.flashmask_workspace_bytes(fm.FM_PASS_BWD, B, H, N, d), dtype=torch.uint8, device="cuda")

    def run():
        out, lse = fm.flashmask_fwd_ex(t["q"], t["k"], t["v"], *vecs, w.scale, workspace=ws_f)
        return (out, lse) + tuple(fm.flashmask_bwd_ex(t["q"], t["k"], t["v"], out, lse, t["dout"], *vecs, w.scale,
                                                      workspace=ws_b))

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()                                  # warm-up outside the capture (kernel attributes are set on first use)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        captured = run()
    gen = torch.Generator(device="cuda")
    gen.manual_seed(7)
    for replay in range(3):
        for n in ("q", "dout"):                # new values in the captured buffers
            t[n].copy_(torch.randn(t[n].shape, device="cuda", generator=gen).bfloat16())
        graph.replay()
        torch.cuda.synchronize()
        eager = run()
        torch.cuda.synchronize()
        for name, a, b in zip(("out", "lse", "dq", "dk", "dv"), captured, eager):
            assert torch.equal(a, b), f"replay {replay}: {name} differs from the eager call"
