"""Helpers shared by the GPU parity tests: move a Workload to the device and
run the oracle on exactly the bf16-rounded values the kernels see."""
import numpy as np
import torch

import workloads
from oracle import flashmask_oracle as orc

# Parity bars (spec tolerances): out and lse max-abs 2e-2 and relative 1e-2; gradients
# max-abs 5e-2.  The relative bar is applied in two forms.  Where the reference magnitude is >= 1 it
# is the plain elementwise bound.  Everywhere, it is applied with a floor of two bf16 rounding steps
# (2 x 2^-8: P is rounded to bf16 as a matrix-core operand, out is stored in bf16) of the scale the
# element lives at: for `out`, the largest magnitude in the element's row (a row of out is one convex
# combination of V rows, so its entries share that scale); for lse, which is O(1) by construction,
# 2^-7 itself.  At the benchmark sizes out is an average over many keys (|out| ~ 0.05), so without the
# floored form only the absolute bar would ever act there.
ABS_FWD, REL_FWD, ABS_BWD = 2e-2, 1e-2, 5e-2
REL_FLOOR = 2.0 ** -7


def to_device(w: workloads.Workload, names=("q", "k", "v", "dout")):
    bits = w.tensors(names)
    dev = {n: torch.from_numpy(b.view(np.int16)).view(torch.bfloat16).cuda() for n, b in bits.items()}
    vecs = tuple(torch.from_numpy(v).cuda() for v in w.stacked_vectors())
    return bits, dev, vecs


def f64(bits_bh):
    return workloads.bf16_bits_to_f32(bits_bh).astype(np.float64)


def check_fwd(got_out, got_lse, ref_out, ref_lse, what=""):
    got_out = np.asarray(got_out, dtype=np.float64)
    got_lse = np.asarray(got_lse, dtype=np.float64)
    inf = np.isinf(ref_lse)
    assert np.array_equal(np.isneginf(got_lse), np.isneginf(ref_lse)), f"{what}: -inf pattern of lse differs"
    for name, g, r in (("out", got_out, ref_out), ("lse", got_lse[~inf], ref_lse[~inf])):
        err = np.abs(g - r)
        assert np.all(np.isfinite(g)), f"{what}: {name} has non-finite values"
        assert err.max(initial=0.0) <= ABS_FWD, f"{what}: {name} max-abs {err.max():.4g} > {ABS_FWD}"
        big = np.abs(r) >= 1.0
        if big.any():
            rel = (err[big] / np.abs(r[big])).max()
            assert rel <= REL_FWD, f"{what}: {name} max-rel {rel:.4g} > {REL_FWD}"
        if err.size:
            scale_of = np.abs(r).max(axis=-1, keepdims=True) if name == "out" else 1.0
            excess = err - (REL_FWD * np.abs(r) + REL_FLOOR * scale_of)
            assert excess.max() <= 0.0, (f"{what}: {name} error exceeds {REL_FWD} * |ref| + 2^-7 * row scale by "
                                         f"{excess.max():.4g}")


def check_bwd(got, ref, name, what=""):
    got = np.asarray(got, dtype=np.float64)
    assert np.all(np.isfinite(got)), f"{what}: {name} has non-finite values"
    err = np.abs(got - ref).max(initial=0.0)
    assert err <= ABS_BWD, f"{what}: {name} max-abs {err:.4g} > {ABS_BWD}"


def bf16_to_np(t: torch.Tensor):
    return t.detach().float().cpu().numpy()
