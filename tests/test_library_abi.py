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
