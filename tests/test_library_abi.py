"""No GPU: the C-ABI library loads and exports every symbol the header declares,
and the host-only entry points behave."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "flashmask.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(flashmask_\w+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    import paper_2410_01359_amd as fm
    if not os.path.exists(fm.library_path()):
        from paper_2410_01359_amd import build
        build.build()
    lib = fm.load_library()
    names = _declared_symbols()
    assert {"flashmask_fwd", "flashmask_bwd", "flashmask_preprocess", "flashmask_classify",
            "flashmask_workspace_bytes", "flashmask_tile_shape", "flashmask_strerror"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in flashmask.h but not exported"


def test_host_only_entry_points():
    import paper_2410_01359_amd as fm
    fm.load_library()
    for p in (fm.FM_PASS_FWD, fm.FM_PASS_BWD_DKDV, fm.FM_PASS_BWD_DQ):
        for d in (64, 128):
            br, bc = fm.flashmask_tile_shape(p, d)
            assert br > 0 and bc > 0 and br % 32 == 0 and bc % 32 == 0
    with pytest.raises(fm.FlashMaskError):
        fm.flashmask_tile_shape(99, 128)
    assert fm.flashmask_workspace_bytes(fm.FM_PASS_FWD, 1, 16, 32768, 128) > 0
    assert fm.flashmask_workspace_bytes(fm.FM_PASS_BWD, 1, 16, 32768, 128) > 0
    assert fm.flashmask_workspace_bytes(fm.FM_PASS_FWD, 1, 16, 100, 128) > 0      # any N >= 1 is supported
    assert fm.flashmask_workspace_bytes(fm.FM_PASS_FWD, 1, 16, 0, 128) == 0       # bad N
    assert fm.flashmask_workspace_bytes(fm.FM_PASS_FWD, 1, 16, 256, 96) == 0      # bad d
    lib = fm.load_library()
    assert lib.flashmask_strerror(0) == b"ok"
    assert b"NULL" in lib.flashmask_strerror(-1)
    # NULL pointers are rejected on the host before anything touches a device
    assert lib.flashmask_fwd(None, None, None, None, None, None, None, ctypes.c_float(1.0), None, None,
                             1, 1, 128, 64, None, 0, None) == -1


def test_strided_entry_points_check_their_arguments_on_the_host():
    """flashmask_fwd_ex / flashmask_bwd_ex reject unusable head counts and strides before any
    device pointer is looked at (all tensor pointers are NULL here)."""
    import paper_2410_01359_amd as fm
    lib = fm.load_library()
    S = fm.Strides
    ok = S(4 * 256 * 64, 256 * 64, 64)

    def fwd(H, Hk, sq, sk=ok, sv=ok, so=ok, N=256, d=64):
        return lib.flashmask_fwd_ex(None, None, None, None, None, None, None, ctypes.c_float(1.0), None, None,
                                    1, H, Hk, N, d, ctypes.byref(sq), ctypes.byref(sk), ctypes.byref(sv),
                                    ctypes.byref(so), None, 0, None)

    assert fwd(4, 4, ok) == -1                         # strides fine: falls through to the NULL-pointer check
    assert fwd(4, 3, ok) == -2                         # H not a multiple of H_kv
    assert fwd(4, 0, ok) == -2
    assert fwd(4, 4, S(4 * 256 * 64, 256 * 64, 60)) == -3     # row stride not a multiple of 8 elements
    assert fwd(4, 4, S(4 * 256 * 64 + 4, 256 * 64, 64)) == -3
    assert fwd(4, 4, S(4 * 256 * 64, 256 * 64, 32)) == -2     # rows would overlap (row < d)
    assert fwd(4, 4, S(4 * 256 * 64, 256 * 64, 1 << 24)) == -2
    assert fwd(4, 4, ok, sk=S(0, 0, 64)) == -2         # several K/V heads on one address
    assert fwd(4, 1, ok, sk=S(0, 0, 64), sv=S(0, 0, 64)) == -1   # one K/V head, batch 1: any stride will do
    arr = (S * 8)(*([ok] * 8))
    assert lib.flashmask_bwd_ex(None, None, None, None, None, None, None, None, None, None, ctypes.c_float(1.0),
                                None, None, None, 1, 4, 4, 256, 64, arr, None, 0, None) == -1
    arr[6] = S(4 * 256 * 64, 256 * 64, 68)
    assert lib.flashmask_bwd_ex(None, None, None, None, None, None, None, None, None, None, ctypes.c_float(1.0),
                                None, None, None, 1, 4, 4, 256, 64, arr, None, 0, None) == -3
    assert lib.flashmask_bwd_ex(None, None, None, None, None, None, None, None, None, None, ctypes.c_float(1.0),
                                None, None, None, 1, 4, 4, 256, 64, None, None, 0, None) == -1
