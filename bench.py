#!/usr/bin/env python3
"""Benchmark of the FlashMask hot path on one MI355X.

One "step" = one forward + one backward pass of the whole C-ABI path
(preprocessing, launch order, tile loops, D pre-pass) over one batch of
synthetic bf16 input already resident in HBM.  Throughput counts only unmasked
FLOPs: 4*d per unmasked score element forward, 2.5x that backward.

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak (published)
DEFAULT_WORKLOAD = "5"


def hip_runtime():
    lib = ctypes.CDLL("libamdhip64.so")
    lib.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
    lib.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
    lib.hipEventSynchronize.argtypes = [ctypes.c_void_p]
    lib.hipEventDestroy.argtypes = [ctypes.c_void_p]
    return lib


def make_events(hip, n):
    arr = (ctypes.c_void_p * n)()
    for i in range(n):
        ev = ctypes.c_void_p()
        rc = hip.hipEventCreate(ctypes.byref(ev))
        if rc != 0:
            raise RuntimeError(f"hipEventCreate failed: {rc}")
        arr[i] = ev
    return arr


def elapsed(hip, a, b):
    ms = ctypes.c_float()
    rc = hip.hipEventElapsedTime(ctypes.byref(ms), a, b)
    if rc != 0:
        raise RuntimeError(f"hipEventElapsedTime failed: {rc}")
    return float(ms.value)


def device_inputs(w, torch):
    """bf16 ~N(0,1) tensors drawn on the device from a seeded generator (same
    distribution as the parity inputs; the bench needs no host copy)."""
    g = torch.Generator(device="cuda")
    g.manual_seed(w.seed)
    shape = (w.B, w.H, w.N, w.d)
    t = {n: torch.randn(shape, device="cuda", dtype=torch.float32, generator=g).bfloat16() for n in ("q", "k", "v", "dout")}
    vecs = tuple(torch.from_numpy(x).cuda() for x in w.stacked_vectors())
    return t, vecs


def run_workload(name, steps, warmup, torch, fm, orc, workloads, hip, with_events):
    w = name if isinstance(name, workloads.Workload) else workloads.config(name)
    name = w.name
    t, vecs = device_inputs(w, torch)
    ws = torch.empty(max(fm.flashmask_workspace_bytes(fm.FM_PASS_BWD, w.B, w.H, w.N, w.d),
                         fm.flashmask_workspace_bytes(fm.FM_PASS_FWD, w.B, w.H, w.N, w.d)),
                     dtype=torch.uint8, device="cuda")
    n_unmasked = sum(orc.count_unmasked_elements(*v) for v in w.vectors) * w.H
    f_fwd = 4.0 * w.d * n_unmasked
    f_total = 3.5 * f_fwd
    cls128 = [orc.classify_tiles_fast(orc.minmax_tables(*v, 128), w.N, 128, 128) for v in w.vectors]
    rho = float(np.mean([orc.block_sparsity(c) for c in cls128]))
    f_tile = 3.5 * sum(orc.flops_tile(c, w.H, w.d)[0] for c in cls128)

    lib = fm.load_library()

    def step(ev_f=None, ev_b=None):
        if ev_f is not None:
            lib.flashmask_profile_events(ev_f, 3)
        out, lse = fm.flashmask_fwd(t["q"], t["k"], t["v"], *vecs, w.scale, workspace=ws)
        if ev_b is not None:
            lib.flashmask_profile_events(ev_b, 4)
        fm.flashmask_bwd(t["q"], t["k"], t["v"], out, lse, t["dout"], *vecs, w.scale, workspace=ws)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    evs = [(make_events(hip, 3), make_events(hip, 4)) for _ in range(steps)] if with_events else [(None, None)] * steps
    t0 = time.perf_counter()
    for ev_f, ev_b in evs:
        step(ev_f, ev_b)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    lib.flashmask_profile_events(None, 0)

    res = {"workload": name, "ms_per_step": wall_ms, "tflops": f_total / wall_ms / 1e9, "block_sparsity": rho,
           "unmasked_tflop": f_total / 1e12, "tile_tflop": f_tile / 1e12, "workload_obj": w}
    if with_events:
        stage = {"fwd_setup": [], "fwd_tiles": [], "bwd_setup": [], "bwd_dq": [], "bwd_dkdv": []}
        fwd_ms, bwd_ms = [], []
        for ev_f, ev_b in evs:
            stage["fwd_setup"].append(elapsed(hip, ev_f[0], ev_f[1]))
            stage["fwd_tiles"].append(elapsed(hip, ev_f[1], ev_f[2]))
            stage["bwd_setup"].append(elapsed(hip, ev_b[0], ev_b[1]))
            stage["bwd_dq"].append(elapsed(hip, ev_b[1], ev_b[2]))       # includes the D pre-pass (its prologue)
            stage["bwd_dkdv"].append(elapsed(hip, ev_b[2], ev_b[3]))
            fwd_ms.append(elapsed(hip, ev_f[0], ev_f[2]))
            bwd_ms.append(elapsed(hip, ev_b[0], ev_b[3]))
        res["stage_ms"] = {k: float(np.mean(v)) for k, v in stage.items()}
        res["fwd_ms"], res["bwd_ms"] = float(np.mean(fwd_ms)), float(np.mean(bwd_ms))
        # algorithmic FLOPs of each tile loop per launch: matrix products per tile x 2*d per unmasked element
        res["kernel_flop"] = {"fwd_tiles": 4.0 * w.d * n_unmasked, "bwd_dkdv": 8.0 * w.d * n_unmasked,
                              "bwd_dq": 6.0 * w.d * n_unmasked}
        for ev_f, ev_b in evs:
            for e in list(ev_f) + list(ev_b):
                hip.hipEventDestroy(e)
    return res


def kernels_digest():
    """Digest of the HIP sources: recorded with the counter-derived traffic figures, which are only
    reported while the kernels they were measured on are the ones being timed."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2410_01359_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".h")) and name != "fm_probe.hip":      # the measurement kernels are not timed code
            h.update(name.encode())
            h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


def load_traffic():
    """profiles/hbm_traffic.json: {"kernels_digest": ..., "entries": {"<workload>:<kernel>": bytes per launch}}
    written from rocprofv3 FETCH_SIZE / WRITE_SIZE runs.  Entries measured on other kernels are not used."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        rec = json.load(open(path))
    except Exception:
        return {}, "no profiles/hbm_traffic.json"
    if rec.get("kernels_digest") != kernels_digest():
        return {}, "profiles/hbm_traffic.json was measured on other kernel sources; traffic not reported"
    return rec.get("entries", {}), None


def roofline_of(res, traffic_entries, onbox):
    """The tile loop with the largest event-timed duration of one workload against the bf16 MFMA peak."""
    st = res["stage_ms"]
    dominant = max(("fwd_tiles", "bwd_dkdv", "bwd_dq"), key=lambda k: st[k])
    achieved = res["kernel_flop"][dominant] / st[dominant] / 1e9
    roof = {"bound": "mfma", "kernel": dominant, "achieved": round(achieved, 2), "peak": PEAK_BF16_TFLOPS,
            "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
            "traffic": traffic_entries.get(f"{res['workload']}:{dominant}"),
            "kernel_ms": round(st[dominant], 4),
            "all_loops_tflops": {k: round(res["kernel_flop"][k] / st[k] / 1e9, 1) for k in ("fwd_tiles", "bwd_dkdv", "bwd_dq")}}
    if onbox:
        roof["onbox_peak"] = onbox["tflops"]
        roof["frac_of_onbox_peak"] = round(achieved / onbox["tflops"], 4)
    return roof


def backward_rates(res):
    """The backward's rate on the five matrix products Algorithm 2 has (10 d FLOP per unmasked element:
    what the metric counts) beside its rate on the seven it executes (the row-parallel dQ pass forms S and
    dP a second time: 14 d)."""
    counted = 2.5 * res["kernel_flop"]["fwd_tiles"]
    executed = res["kernel_flop"]["bwd_dkdv"] + res["kernel_flop"]["bwd_dq"]
    return {"alg2_products_tflops": round(counted / res["bwd_ms"] / 1e9, 1),
            "executed_products_tflops": round(executed / res["bwd_ms"] / 1e9, 1),
            "alg2_frac_of_peak": round(counted / res["bwd_ms"] / 1e9 / PEAK_BF16_TFLOPS, 4)}


def mfma_ceiling(torch, fm, hip, iters=4000, reps=5, shape=0, zeros=False):
    """On-box matrix-core ceiling: a kernel of nothing but bf16 MFMAs (shape 0: the 32x32x16 instruction of the
    tile loops; 1: 16x16x32) on random operands (or zeros), the whole chip filled as the tile loops fill it
    (2 workgroups of 4 waves per CU), timed with events on the launch stream; the LAST of `reps` back-to-back
    launches of ~20 ms is reported (the sustained rate: the first launches still run at a higher clock).
    `implied_clock_ghz` = rate / (256 CUs x 4096 FLOP per clock): the clock the chip held if every SIMD issued
    back to back."""
    g = torch.Generator(device="cuda")
    g.manual_seed(7)
    operands = torch.randn(8192, device="cuda", generator=g).bfloat16()
    if zeros:
        operands.zero_()
    wgs = 256 * 2 * 4                      # four rounds of full occupancy
    sink = torch.empty(wgs * 256, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    fm.flashmask_mfma_ceiling(operands, sink, wgs, iters // 10, shape)
    torch.cuda.synchronize()
    ev = make_events(hip, 2)
    hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    times = []
    for _ in range(reps):
        hip.hipEventRecord(ev[0], ctypes.c_void_p(stream))
        flop = fm.flashmask_mfma_ceiling(operands, sink, wgs, iters, shape)
        hip.hipEventRecord(ev[1], ctypes.c_void_p(stream))
        hip.hipEventSynchronize(ev[1])
        times.append(elapsed(hip, ev[0], ev[1]))
    for e in ev:
        hip.hipEventDestroy(e)
    tflops = flop / times[-1] / 1e9
    return {"tflops": round(tflops, 1), "ms": round(times[-1], 4), "first_launch_tflops": round(flop / times[0] / 1e9, 1),
            "implied_clock_ghz": round(tflops * 1e12 / (256 * 4096) / 1e9, 3),
            "kernel": ("v_mfma_f32_16x16x32_bf16 only" if shape == 1 else "v_mfma_f32_32x32x16_bf16 only" if shape == 0 else
                       "v_mfma_f32_32x32x16_bf16 + per MFMA one ds_read_b128, four fma, one exp (the forward's mix)") + ", " +
                      ("zero" if zeros else "random N(0,1)") + " operands, 2048 workgroups x 4 waves, 4 chains per wave"}


def atomic_ceiling(torch, fm, hip, reps=4):
    """Rate of the dQ update as Algorithm 2's column-parallel loop would issue it (a 64 x 128 fp32 block per
    tile, no-return atomic adds into HBM), and the cap it would put on a backward that fuses dQ into the
    dK/dV loop: one such block per 64 x 128-key tile, whose five matrix products are 10 d FLOP per score
    element."""
    heads, n_tiles, tiles, wgs = 8, 512, 64, 2048
    acc = torch.zeros((heads, n_tiles, 64, 128), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    fm.flashmask_atomic_ceiling(acc, 4, wgs)
    torch.cuda.synchronize()
    ev = make_events(hip, 2)
    best = None
    for _ in range(reps):
        hip.hipEventRecord(ev[0], ctypes.c_void_p(stream))
        nbytes = fm.flashmask_atomic_ceiling(acc, tiles, wgs)
        hip.hipEventRecord(ev[1], ctypes.c_void_p(stream))
        hip.hipEventSynchronize(ev[1])
        ms = elapsed(hip, ev[0], ev[1])
        best = ms if best is None else min(best, ms)
    for e in ev:
        hip.hipEventDestroy(e)
    tbs = nbytes / best / 1e9
    d = 128
    cap = tbs * 1e12 / (64 * 128 * 4) * (10.0 * d * 64 * 128) / 1e12
    return {"fp32_atomic_add_TBps": round(tbs, 3), "ms": round(best, 4),
            "pattern": "2048 workgroups x 64 tiles of 64 x 128 fp32, 8 heads x 32768 rows, a head's adds from one XCD",
            "fused_dq_backward_cap_tflops": round(cap, 1),
            "note": "cap on a backward that adds dQ per 64 x 128-key tile from the column-parallel loop (10 d FLOP per element, d = 128)"}


def forward_only_grouped(torch, fm, orc, workloads, steps):
    """Forward pass alone at the head configuration of the paper's inference appendix (32 query
    heads on 8 K/V heads, d = 128, batch 1) under a causal-document mask of 16 equal documents at
    N = 32768, tensors stored [B,N,H,d]: the strided / grouped-head entry point."""
    B, H, Hk, N, d = 1, 32, 8, 32768, 128
    spans = workloads.spans_from_lengths([N // 16] * 16)
    vec = workloads.causal_document_mask(N, spans)
    vecs = tuple(torch.from_numpy(np.asarray(x, dtype=np.int32)[None]).cuda() for x in vec)
    g = torch.Generator(device="cuda")
    g.manual_seed(20241002)
    q = torch.randn((B, N, H, d), device="cuda", generator=g).bfloat16().transpose(1, 2)
    k, v = (torch.randn((B, N, Hk, d), device="cuda", generator=g).bfloat16().transpose(1, 2) for _ in range(2))
    ws = torch.empty(fm.flashmask_workspace_bytes(fm.FM_PASS_FWD, B, H, N, d), dtype=torch.uint8, device="cuda")
    scale = 1.0 / math.sqrt(d)
    for _ in range(2):
        fm.flashmask_fwd_ex(q, k, v, *vecs, scale, workspace=ws)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fm.flashmask_fwd_ex(q, k, v, *vecs, scale, workspace=ws)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    flop = 4.0 * d * orc.count_unmasked_elements(*vec) * H
    return {"workload": "forward only, 32 query heads on 8 K/V heads, d=128, N=32768, causal document (16 x 2048), "
                        "[B,N,H,d] storage", "ms": round(ms, 4), "tflops": round(flop / ms / 1e9, 1)}


def cpu_baseline(w, orc, workloads, budget_rows):
    """The fp64 oracle, as it stands, timed on the host on a bounded sample of
    the same workload: the full forward+backward work of `budget_rows` query
    rows of head 0 (every key column), in the metric's unit."""
    import threadpoolctl
    bits = workloads.make_tensors(w.seed, 1, 1, w.N, w.d)     # one head's worth of the same recipe
    arrs = [workloads.bf16_bits_to_f32(bits[n][0, 0]).astype(np.float64) for n in ("q", "k", "v", "dout")]
    vec = w.vectors[0]
    rows_total = min(budget_rows, w.N)
    r_start = (w.N - rows_total) // 2
    allowed = orc.allowed_keys_per_row(*vec)
    t0 = time.perf_counter()
    for r0 in range(r_start, r_start + rows_total, orc.ROW_CHUNK):
        rows = np.arange(r0, min(r0 + orc.ROW_CHUNK, r_start + rows_total))
        orc.backward_row_block(*arrs, *vec, w.scale, rows)
    secs = time.perf_counter() - t0
    unmasked = int(allowed[r_start:r_start + rows_total].sum())
    flop = 14.0 * w.d * unmasked
    threads = max([p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()] or [1])
    return {"value": flop / secs / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
            "sample": f"fp64 oracle forward+backward of {rows_total} query rows x all {w.N} keys of one head of "
                      f"workload {w.name} ({secs:.1f} s; dense work, unmasked FLOPs counted)"}


def sparsity_sweep(torch, fm, orc, workloads, hip, steps, warmup):
    """Wall time of forward+backward against the fraction of tiles that are not skipped, at the
    shape of config 4 with the three masks of the paper's sparsity experiment (causal document,
    document, shared question); least-squares lines per mask and over all points."""
    pts = []
    for w in workloads.sweep_workloads():
        # two measurements per point, the faster one kept: a single disturbed run (another tenant of the box,
        # a clock ramp) otherwise shows up as an outlier of the fit
        r = min((run_workload(w, steps, warmup, torch, fm, orc, workloads, hip, False) for _ in range(2)),
                key=lambda x: x["ms_per_step"])
        pts.append({"workload": w.name, "mask": w.mask_kind, "parts": len(w.structure[0]),
                    "block_sparsity": round(r["block_sparsity"], 4),
                    "ms": round(r["ms_per_step"], 4), "tflops": round(r["tflops"], 1)})
        torch.cuda.empty_cache()

    def fit(sel):
        x = np.array([1.0 - p["block_sparsity"] for p in sel])
        y = np.array([p["ms"] for p in sel])
        slope, intercept = np.polyfit(x, y, 1)
        resid = y - (slope * x + intercept)
        r2 = 1.0 - float(resid @ resid) / float(((y - y.mean()) @ (y - y.mean())))
        return {"points": len(sel), "slope_ms": round(float(slope), 4), "intercept_ms": round(float(intercept), 4),
                "r2": round(r2, 5)}

    fits = {"all": fit(pts)}
    for kind in sorted({p["mask"] for p in pts}):
        fits[kind] = fit([p for p in pts if p["mask"] == kind])
    return {"metric": "fwd+bwd ms vs fraction of 128x128 tiles not skipped (1 - block sparsity)",
            "shape": "B=1, H=16, N=32768, d=128; causal-document, document and shared-question masks",
            "steps": steps, "warmup": warmup, "fit": fits["all"], "fits": fits, "points": pts}


def paper_table(torch, fm, orc, workloads, hip, steps, warmup):
    """Forward and backward time at the shapes of the paper's kernel-speed tables (d = 128, 128K tokens,
    32 heads, N = 8K / 32K / 128K; the rows whose masks have no random structure), with the paper's own
    FLOP accounting (128 x 128 tiles not skipped) next to the strict one (unmasked elements)."""
    rows = []
    for w in workloads.paper_table_workloads():
        r = run_workload(w, steps, warmup, torch, fm, orc, workloads, hip, True)
        fw_tile = r["tile_tflop"] / 3.5
        rows.append({"workload": w.name, "B": w.B, "H": w.H, "N": w.N, "block_sparsity": round(r["block_sparsity"], 4),
                     "fwd_ms": round(r["fwd_ms"], 3), "bwd_ms": round(r["bwd_ms"], 3), "total_ms": round(r["ms_per_step"], 3),
                     "tile_tflop_fwd": round(fw_tile, 2), "tile_tflop_bwd": round(2.5 * fw_tile, 2),
                     "fwd_tile_tflops": round(fw_tile * 1e3 / r["fwd_ms"], 1),
                     "bwd_tile_tflops": round(2.5 * fw_tile * 1e3 / r["bwd_ms"], 1),
                     "total_tile_tflops": round(r["tile_tflop"] * 1e3 / r["ms_per_step"], 1),
                     "total_unmasked_tflops": round(r["tflops"], 1),
                     "pct_of_bf16_mfma_peak": round(100.0 * r["tflops"] / PEAK_BF16_TFLOPS, 2)})
        print(f"# {rows[-1]}", file=sys.stderr, flush=True)
        del r
        torch.cuda.empty_cache()
    return {"metric": "fwd / bwd / total TFLOP/s at the shapes of the paper's d=128 kernel-speed tables, 1 MI355X",
            "steps": steps, "warmup": warmup, "dtype": "bf16", "data": "synthetic", "rows": rows}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD, help="1, 2, 3, 4a, 4b, 5 or 4b-d64")
    ap.add_argument("--others", default="2,3,4a,4b,4b-d64",
                    help="extra workloads reported in `other_workloads` ('' = none); 4b-d64 = run 4b at d = 64, 32 heads")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-rows", type=int, default=12288)
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the benchmark line, print the block-sparsity sweep (time vs 1 - sparsity)")
    ap.add_argument("--paper-table", action="store_true",
                    help="instead of the benchmark line, time the deterministic rows of the paper's d=128 "
                         "kernel-speed tables (128K tokens, 32 heads, N = 8K / 32K / 128K)")
    ap.add_argument("--mfma-ceiling", action="store_true",
                    help="only measure the on-box matrix-core ceiling (an MFMA-only kernel) and print it")
    ap.add_argument("--atomic-ceiling", action="store_true",
                    help="only measure the fp32 atomic-add rate of a dQ update fused into the dK/dV loop and print it")
    ap.add_argument("--copy-calibration-mib", type=int, default=0,
                    help="also run plain device copies of this many MiB (read once, written once): a kernel of known "
                         "HBM traffic against which rocprofv3's FETCH_SIZE / WRITE_SIZE counters are scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (batch x heads is the sharding axis); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2410_01359_amd as fm
    import workloads
    from oracle import flashmask_oracle as orc      # FLOP counters and the cpu_baseline leg only

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    fm.load_library()
    hip = hip_runtime()

    if args.mfma_ceiling:
        print(json.dumps({"metric": "sustained bf16 MFMA-only rate on this box (TFLOP/s), nominal peak 2500",
                          "runs": [mfma_ceiling(torch, fm, hip, shape=sh, zeros=z) for z in (False, True) for sh in (0, 1, 2)]}),
              flush=True)
        return

    if args.atomic_ceiling:
        print(json.dumps(atomic_ceiling(torch, fm, hip)), flush=True)
        return

    if args.sweep:
        print(json.dumps(sparsity_sweep(torch, fm, orc, workloads, hip, max(3, args.steps // 4), 2)), flush=True)
        return

    if args.paper_table:
        print(json.dumps(paper_table(torch, fm, orc, workloads, hip, max(2, args.steps // 5), 1)), flush=True)
        return

    onbox = mfma_ceiling(torch, fm, hip)
    onbox_mix = mfma_ceiling(torch, fm, hip, shape=2)
    traffic_entries, traffic_note = load_traffic()
    main_res = run_workload(args.workload, args.steps, args.warmup, torch, fm, orc, workloads, hip, True)
    w = main_res.pop("workload_obj")
    others = []
    for name in [x for x in args.others.split(",") if x and x != args.workload]:
        r = run_workload(name, max(3, args.steps // 2), 2, torch, fm, orc, workloads, hip, True)
        r.pop("workload_obj")
        r["pct_of_bf16_mfma_peak"] = 100.0 * r["tflops"] / PEAK_BF16_TFLOPS
        r["tile_tflops"] = r["tile_tflop"] * 1e3 / r["ms_per_step"]      # the paper's accounting: 128x128 tiles not skipped
        entry = {k: (round(v, 4) if isinstance(v, float) else v) for k, v in r.items()
                 if k in ("workload", "ms_per_step", "tflops", "pct_of_bf16_mfma_peak", "tile_tflops",
                          "block_sparsity", "unmasked_tflop", "tile_tflop", "fwd_ms", "bwd_ms")}
        entry["stage_ms"] = {k: round(v, 4) for k, v in r["stage_ms"].items()}
        entry["roofline"] = roofline_of(r, traffic_entries, onbox)
        entry["backward"] = backward_rates(r)
        others.append(entry)
        torch.cuda.empty_cache()

    if args.copy_calibration_mib > 0:
        n = args.copy_calibration_mib * (1 << 20) // 4
        src = torch.arange(n, dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    st = main_res["stage_ms"]
    roof = roofline_of(main_res, traffic_entries, onbox)
    if traffic_note:
        roof["traffic_note"] = traffic_note
    line = {
        "metric": "fwd+bwd TFLOPs/s (unmasked FLOPs) on 1 MI355X",
        "value": round(main_res["tflops"], 2),
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(main_res["ms_per_step"], 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "pct_of_bf16_mfma_peak": round(100.0 * main_res["tflops"] / PEAK_BF16_TFLOPS, 2),
        "config": {"workload": f"config {w.name}: {w.mask_kind} mask, B={w.B}, H={w.H}, N={w.N}, d={w.d}, bf16, "
                               f"forward+backward, scale=1/sqrt(d)",
                   "block_sparsity_128": round(main_res["block_sparsity"], 4),
                   "unmasked_tflop_per_step": round(main_res["unmasked_tflop"], 4),
                   "tile_tflop_per_step": round(main_res["tile_tflop"], 4),
                   "fwd_ms": round(main_res["fwd_ms"], 4), "bwd_ms": round(main_res["bwd_ms"], 4),
                   "stage_ms": {k: round(v, 4) for k, v in st.items()}},
        "roofline": roof,
        "backward": backward_rates(main_res),
        "onbox_mfma_ceiling": onbox,
        "onbox_forward_mix_ceiling": onbox_mix,
        "other_workloads": others,
    }
    if args.others:   # the extra measurements are left out of single-workload (profiling) runs
        line["forward_only_grouped_heads"] = forward_only_grouped(torch, fm, orc, workloads, max(5, args.steps))
        line["dq_atomic_ceiling"] = atomic_ceiling(torch, fm, hip)
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(w, orc, workloads, args.cpu_rows)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
