"""Host-side check of the wait states around the dK/dV loop's inline-assembly MFMAs.

The two accumulating products of the dK/dV kernel are issued from inline assembly so that their
accumulators live in AGPRs; the compiler does not look into the asm, so the wait states it would
insert for an ordinary MFMA are the source's responsibility (see mfma32_acc in fm_common.h).  This
test compiles the backward source to gfx950 assembly (no GPU needed, ~15 s) and checks, in every
instantiation of the kernel, what the source relies on:
  * no vector instruction writes an A/B source of such an MFMA within the two instructions before
    it, unless the MFMA carries its own idle instruction (`s_nop 1`);
  * every path from such an MFMA to any other instruction that touches an accumulator register (the
    stores' reads, the zero-initialisation, copies the compiler inserts between the tile loops) passes
    the drain (`s_nop 15` x 3): checked by data flow over the kernel's basic blocks.
"""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _assembly(tmp_path, source="fm_bwd.hip"):
    import importlib
    build = importlib.import_module("paper_2410_01359_amd.build")
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("hipcc not available")
    out = os.path.join(tmp_path, source.replace(".hip", ".s"))
    flags = [f for f in build.FLAGS if f != "-shared"]
    cmd = [hipcc, *flags, "--cuda-device-only", "-S", os.path.join(build.CSRC, source), "-o", out]
    subprocess.run(cmd, check=True, stdout=subprocess.PIPE, stderr=subprocess.PIPE, timeout=600)
    return open(out).read()


def _regs(text, prefix):
    """Register numbers named in an operand string, for v (prefix 'v') or a (prefix 'a') registers."""
    regs = set()
    for lo, hi in re.findall(r"\b%s\[(\d+):(\d+)\]" % prefix, text):
        regs.update(range(int(lo), int(hi) + 1))
    regs.update(int(x) for x in re.findall(r"\b%s(\d+)\b" % prefix, text))
    return regs


def _blocks(lines):
    """Basic blocks of one function's assembly: [{"label", "ins": [...], "succ": [labels...]}], split at labels,
    at the compiler's own block comments (; %bb.N) and behind every branch."""
    blocks, cur = [], {"label": "entry", "ins": []}
    for raw in lines:
        l = raw.strip()
        m = re.match(r"^(\.LBB\d+_\d+):", l)
        if m or l.startswith("; %bb."):
            blocks.append(cur)
            cur = {"label": m.group(1) if m else l.split(":")[0][2:], "ins": []}
            continue
        if not l or l.startswith(";") or l.startswith(".") or l.endswith(":"):
            continue
        cur["ins"].append(l)
        if l.startswith("s_cbranch") or l.startswith("s_branch") or l.startswith("s_endpgm"):
            blocks.append(cur)
            cur = {"label": None, "ins": []}
    blocks.append(cur)
    blocks = [b for b in blocks if b["ins"] or b["label"]]
    index = {b["label"]: k for k, b in enumerate(blocks) if b["label"]}
    for k, b in enumerate(blocks):
        last = b["ins"][-1] if b["ins"] else ""
        succ = []
        if last.startswith("s_branch") or last.startswith("s_cbranch"):
            succ.append(index[last.split()[-1]])
        if not last.startswith("s_branch") and not last.startswith("s_endpgm") and k + 1 < len(blocks):
            succ.append(k + 1)
        b["succ"] = succ
    return blocks


def test_dkdv_inline_asm_mfma_wait_states(tmp_path):
    asm = _assembly(str(tmp_path))
    kernels = list(re.finditer(r"^(_ZN2fm11dkdv_kernel\w+):.*?^\.Lfunc_end\d+:", asm, re.S | re.M))
    assert len(kernels) == 8, "two head dims x ragged x general"
    for m in kernels:
        name = m.group(1)
        blocks = _blocks(m.group(0).split("\n")[1:])
        real = [l for b in blocks for l in b["ins"]]
        is_acc_mfma = lambda l: l.startswith("v_mfma_f32_32x32x16_bf16 a")
        accs = set()
        n_mfma = 0
        for k, l in enumerate(real):
            if not is_acc_mfma(l):
                continue
            n_mfma += 1
            dst, rest = l.split(",", 1)
            accs |= _regs(dst, "a")
            srcs = _regs(rest, "v")
            if real[k - 1] == "s_nop 1":
                continue
            for prev in real[max(0, k - 2):k]:
                w = re.match(r"v_(?!mfma)\w+ (v\d+|v\[\d+:\d+\])", prev)
                assert not (w and _regs(w.group(1), "v") & srcs), f"{name}: '{prev}' right before '{l}'"
        d = 128 if "ILi128E" in name else 64
        if d == 64:
            # d = 64 keeps its accumulators in compiler-managed registers (ordinary MFMA builtins, whose wait
            # states the compiler handles): no inline-assembly MFMA may be left in these instantiations
            assert n_mfma == 0, f"{name}: {n_mfma} inline-assembly MFMAs"
            continue
        # (dK + dV) x d/32 blocks x 8 steps per tile body: one body per tile loop, plus the copies the compiler
        # makes of a body (a loop's last iteration, which ends with the drain, may be peeled off)
        assert n_mfma % ((d // 32) * 8) == 0 and 2 <= n_mfma // ((d // 32) * 8) <= 6, f"{name}: {n_mfma} accumulating MFMAs"
        assert len(accs) >= 4 * d // 32 * 16 // 2, f"{name}: {len(accs)} accumulator registers"
        # Every path from an accumulating MFMA to any other instruction that touches an accumulator register
        # (the stores' reads, the zero-initialisation, and the copies the compiler makes where it keeps the
        # accumulators in different registers in the two tile loops) must pass the drain: 3 x `s_nop 15`.
        # Forward data flow over the basic blocks; state = the registers an MFMA may still be writing.
        busy_in = [frozenset()] * len(blocks)
        changed = True
        while changed:
            changed = False
            for k, b in enumerate(blocks):
                busy, nops = set(busy_in[k]), 0
                for l in b["ins"]:
                    if is_acc_mfma(l):
                        busy |= _regs(l.split(",", 1)[0], "a")
                        nops = 0
                    elif l == "s_nop 15":
                        nops += 1
                        if nops >= 3:
                            busy.clear()
                    else:
                        nops = 0
                        hit = _regs(l, "a") & busy
                        assert not hit, f"{name}: '{l}' touches a{sorted(hit)[0]} before the drain"
                for t in b["succ"]:
                    if not busy <= busy_in[t]:
                        busy_in[t] = frozenset(busy_in[t] | busy)
                        changed = True
        # and inside the tile loops (blocks with accumulating MFMAs) nothing but those MFMAs touches them
        for b in blocks:
            if any(is_acc_mfma(l) for l in b["ins"]):
                for l in b["ins"]:
                    assert is_acc_mfma(l) or not (_regs(l, "a") & accs) or l.startswith("v_accvgpr"), f"{name}: '{l}'"
                assert sum(1 for l in b["ins"] if l.startswith("v_accvgpr") and _regs(l, "a") & accs) == 0 or \
                    not any(is_acc_mfma(l) for l in b["ins"][-1:]), name


@pytest.mark.parametrize("source", ["fm_fwd.hip", "fm_bwd.hip"])
def test_lds_window_register_is_written_only_by_the_copy_helpers(tmp_path, source):
    """The tile copies (global_load_lds) take their LDS destination from M0, which the copy helpers set
    in one inline-assembly statement (async_window) and use in later ones (async_copy16_window) without
    the compiler knowing of the dependency.  That is sound as long as nothing the COMPILER emits writes
    M0 in a tile-loop kernel: every write of M0, and every global_load_lds, must sit inside an
    inline-assembly block of the generated code."""
    asm = _assembly(str(tmp_path), source)
    kernels = list(re.finditer(r"^(_ZN2fm\d+(?:fwd|dq|dkdv)_kernel\w+):.*?^\.Lfunc_end\d+:", asm, re.S | re.M))
    assert len(kernels) == (8 if source == "fm_fwd.hip" else 16)
    for m in kernels:
        inside, copies, windows = False, 0, 0
        for raw in m.group(0).split("\n"):
            l = raw.strip()
            if l.startswith(";;#ASMSTART"):
                inside = True
            elif l.startswith(";;#ASMEND"):
                inside = False
            elif l and not l.startswith(";") and not l.startswith("."):
                writes_m0 = re.match(r"s_\w+\s+m0\b", l) is not None
                if writes_m0:
                    windows += 1
                if l.startswith("global_load_lds"):
                    copies += 1
                assert inside or not (writes_m0 or l.startswith("global_load_lds")), f"{m.group(1)}: '{l}' outside inline assembly"
        assert copies > 0 and windows > 0, m.group(1)
