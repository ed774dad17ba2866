"""ctypes binding of libflashmask.so (see include/flashmask.h for the contract).

Argument marshalling only.  There is no fallback: if the HIP library is not
built, or a tensor is not on the GPU, the call raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

FM_PASS_FWD, FM_PASS_BWD_DKDV, FM_PASS_BWD_DQ, FM_PASS_BWD = 0, 1, 2, 3

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class FlashMaskError(RuntimeError):
    pass


class Strides(ctypes.Structure):
    """flashmask_strides: element strides of a tensor indexed [batch][head][row][d]."""
    _fields_ = [("batch", ctypes.c_int64), ("head", ctypes.c_int64), ("row", ctypes.c_int64)]


def library_path() -> str:
    return os.path.join(_HERE, "libflashmask.so")


def load_library() -> ctypes.CDLL:
    """Load the in-tree shared library; raise if it has not been built."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise FlashMaskError(f"{path} is missing: build it with `python -m paper_2410_01359_amd.build` "
                             "(or __graft_entry__.build()); there is no fallback path")
    lib = ctypes.CDLL(path)
    vp, ip, fp = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p
    i, f, sz = ctypes.c_int, ctypes.c_float, ctypes.c_size_t
    lib.flashmask_fwd.restype = i
    lib.flashmask_fwd.argtypes = [vp, vp, vp, ip, ip, ip, ip, f, vp, fp, i, i, i, i, vp, sz, vp]
    lib.flashmask_fwd_noalloc.restype = i
    lib.flashmask_fwd_noalloc.argtypes = [vp, vp, vp, ip, ip, ip, ip, f, vp, fp, i, i, i, i, vp]
    lib.flashmask_bwd.restype = i
    lib.flashmask_bwd.argtypes = [vp, vp, vp, vp, fp, vp, ip, ip, ip, ip, f, vp, vp, vp, i, i, i, i, vp, sz, vp]
    sp = ctypes.POINTER(Strides)
    lib.flashmask_fwd_ex.restype = i
    lib.flashmask_fwd_ex.argtypes = [vp, vp, vp, ip, ip, ip, ip, f, vp, fp, i, i, i, i, i, sp, sp, sp, sp, vp, sz, vp]
    lib.flashmask_bwd_ex.restype = i
    lib.flashmask_bwd_ex.argtypes = [vp, vp, vp, vp, fp, vp, ip, ip, ip, ip, f, vp, vp, vp, i, i, i, i, i, sp, vp, sz, vp]
    lib.flashmask_unit_queues.restype = i
    lib.flashmask_unit_queues.argtypes = [i, ip, ip, ip, ip, i, i, i, i, ip, ctypes.POINTER(i), vp, sz, vp]
    lib.flashmask_workspace_bytes.restype = sz
    lib.flashmask_workspace_bytes.argtypes = [i, i, i, i, i]
    lib.flashmask_preprocess.restype = i
    lib.flashmask_preprocess.argtypes = [ip, ip, ip, ip, i, i, i, ip, vp]
    lib.flashmask_classify.restype = i
    lib.flashmask_classify.argtypes = [ip, i, i, i, i, vp, vp]
    lib.flashmask_tile_shape.restype = i
    lib.flashmask_tile_shape.argtypes = [i, i, ctypes.POINTER(i), ctypes.POINTER(i)]
    lib.flashmask_strerror.restype = ctypes.c_char_p
    lib.flashmask_strerror.argtypes = [i]
    lib.flashmask_last_hip_error.restype = ctypes.c_char_p
    lib.flashmask_last_hip_error.argtypes = []
    lib.flashmask_mfma_ceiling.restype = i
    lib.flashmask_mfma_ceiling.argtypes = [vp, fp, i, i, i, ctypes.POINTER(ctypes.c_double), vp]
    lib.flashmask_atomic_ceiling.restype = i
    lib.flashmask_atomic_ceiling.argtypes = [fp, i, i, i, i, ctypes.POINTER(ctypes.c_double), vp]
    lib.flashmask_profile_events.restype = i
    lib.flashmask_profile_events.argtypes = [ctypes.POINTER(ctypes.c_void_p), i]
    _LIB = lib
    return lib


def _check(rc: int, what: str):
    if rc != 0:
        lib = load_library()
        msg = lib.flashmask_strerror(rc).decode()
        hip = lib.flashmask_last_hip_error().decode()
        raise FlashMaskError(f"{what} failed: {msg} (code {rc}){' [' + hip + ']' if hip and rc == -5 else ''}")


def _dev(t: torch.Tensor, dtype, name: str) -> torch.Tensor:
    if not t.is_cuda:
        raise FlashMaskError(f"{name} must live on the GPU")
    if t.dtype != dtype:
        raise FlashMaskError(f"{name} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise FlashMaskError(f"{name} must be contiguous")
    return t


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def flashmask_tile_shape(pass_id: int, d: int):
    br, bc = ctypes.c_int(0), ctypes.c_int(0)
    _check(load_library().flashmask_tile_shape(pass_id, d, ctypes.byref(br), ctypes.byref(bc)), "flashmask_tile_shape")
    return br.value, bc.value


def flashmask_workspace_bytes(pass_id: int, B: int, H: int, N: int, d: int) -> int:
    return int(load_library().flashmask_workspace_bytes(pass_id, B, H, N, d))


def _workspace(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def flashmask_preprocess(lts, lte, uts, ute, block_c: int) -> torch.Tensor:
    """int32 [B, 8, T_c] min/max table."""
    vecs = [_dev(x, torch.int32, n) for x, n in zip((lts, lte, uts, ute), ("lts", "lte", "uts", "ute"))]
    B, N = vecs[0].shape
    t_c = (N + block_c - 1) // block_c
    out = torch.empty((B, 8, t_c), dtype=torch.int32, device=vecs[0].device)
    _check(load_library().flashmask_preprocess(*(v.data_ptr() for v in vecs), B, N, block_c, out.data_ptr(), _stream()),
           "flashmask_preprocess")
    return out


def flashmask_classify(minmax: torch.Tensor, N: int, block_r: int, block_c: int) -> torch.Tensor:
    """uint8 [B, T_r, T_c] tile classes."""
    _dev(minmax, torch.int32, "minmax")
    B = minmax.shape[0]
    t_r, t_c = (N + block_r - 1) // block_r, (N + block_c - 1) // block_c
    if tuple(minmax.shape) != (B, 8, t_c):
        raise FlashMaskError("minmax must be [B, 8, ceil(N / block_c)]")
    cls = torch.empty((B, t_r, t_c), dtype=torch.uint8, device=minmax.device)
    _check(load_library().flashmask_classify(minmax.data_ptr(), B, N, block_r, block_c, cls.data_ptr(), _stream()),
           "flashmask_classify")
    return cls


def flashmask_fwd(q, k, v, lts, lte, uts, ute, scale: float, workspace: torch.Tensor | None = None):
    """out (bf16 [B,H,N,d]) and lse (fp32 [B,H,N])."""
    for t, n in zip((q, k, v), "qkv"):
        _dev(t, torch.bfloat16, n)
    for t, n in zip((lts, lte, uts, ute), ("lts", "lte", "uts", "ute")):
        _dev(t, torch.int32, n)
    B, H, N, d = q.shape
    if k.shape != q.shape or v.shape != q.shape or any(tuple(x.shape) != (B, N) for x in (lts, lte, uts, ute)):
        raise FlashMaskError("shape mismatch: q,k,v [B,H,N,d]; lts,lte,uts,ute [B,N]")
    need = flashmask_workspace_bytes(FM_PASS_FWD, B, H, N, d)
    ws = workspace if workspace is not None else _workspace(need, q.device)
    out = torch.empty_like(q)
    lse = torch.empty((B, H, N), dtype=torch.float32, device=q.device)
    _check(load_library().flashmask_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), lts.data_ptr(), lte.data_ptr(),
                                        uts.data_ptr(), ute.data_ptr(), float(scale), out.data_ptr(), lse.data_ptr(),
                                        B, H, N, d, ws.data_ptr(), ws.numel(), _stream()), "flashmask_fwd")
    return out, lse


def flashmask_fwd_noalloc(q, k, v, lts, lte, uts, ute, scale: float, out: torch.Tensor, lse: torch.Tensor):
    """flashmask_fwd into caller-provided out / lse, with the library's static scratch: this call
    itself allocates nothing (not even through torch)."""
    for t, n in zip((q, k, v, out), ("q", "k", "v", "out")):
        _dev(t, torch.bfloat16, n)
    _dev(lse, torch.float32, "lse")
    for t, n in zip((lts, lte, uts, ute), ("lts", "lte", "uts", "ute")):
        _dev(t, torch.int32, n)
    B, H, N, d = q.shape
    if any(x.shape != q.shape for x in (k, v, out)) or tuple(lse.shape) != (B, H, N) or \
            any(tuple(x.shape) != (B, N) for x in (lts, lte, uts, ute)):
        raise FlashMaskError("shape mismatch: q,k,v,out [B,H,N,d]; lse [B,H,N]; lts,lte,uts,ute [B,N]")
    _check(load_library().flashmask_fwd_noalloc(q.data_ptr(), k.data_ptr(), v.data_ptr(), lts.data_ptr(),
                                                lte.data_ptr(), uts.data_ptr(), ute.data_ptr(), float(scale),
                                                out.data_ptr(), lse.data_ptr(), B, H, N, d, _stream()),
           "flashmask_fwd_noalloc")
    return out, lse


def flashmask_bwd(q, k, v, out, lse, dout, lts, lte, uts, ute, scale: float, workspace: torch.Tensor | None = None):
    """dq, dk, dv (bf16 [B,H,N,d])."""
    for t, n in zip((q, k, v, out, dout), ("q", "k", "v", "out", "dout")):
        _dev(t, torch.bfloat16, n)
    _dev(lse, torch.float32, "lse")
    for t, n in zip((lts, lte, uts, ute), ("lts", "lte", "uts", "ute")):
        _dev(t, torch.int32, n)
    B, H, N, d = q.shape
    if any(x.shape != q.shape for x in (k, v, out, dout)) or tuple(lse.shape) != (B, H, N) or \
            any(tuple(x.shape) != (B, N) for x in (lts, lte, uts, ute)):
        raise FlashMaskError("shape mismatch")
    need = flashmask_workspace_bytes(FM_PASS_BWD, B, H, N, d)
    ws = workspace if workspace is not None else _workspace(need, q.device)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)
    _check(load_library().flashmask_bwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), lse.data_ptr(),
                                        dout.data_ptr(), lts.data_ptr(), lte.data_ptr(), uts.data_ptr(),
                                        ute.data_ptr(), float(scale), dq.data_ptr(), dk.data_ptr(), dv.data_ptr(),
                                        B, H, N, d, ws.data_ptr(), ws.numel(), _stream()), "flashmask_bwd")
    return dq, dk, dv


def _view(t: torch.Tensor, name: str) -> Strides:
    """Strides of a bf16 tensor indexed [B, heads, N, d]; d must be contiguous."""
    if not t.is_cuda:
        raise FlashMaskError(f"{name} must live on the GPU")
    if t.dtype != torch.bfloat16:
        raise FlashMaskError(f"{name} must be bfloat16, got {t.dtype}")
    if t.dim() != 4 or t.stride(3) != 1:
        raise FlashMaskError(f"{name} must be indexed [B, heads, N, d] with d contiguous")
    return Strides(t.stride(0), t.stride(1), t.stride(2))


def flashmask_fwd_ex(q, k, v, lts, lte, uts, ute, scale: float, workspace: torch.Tensor | None = None):
    """Forward for tensors of any strides (indexed [B,heads,N,d], d contiguous: pass `x.transpose(1, 2)` of
    a [B,N,H,d] tensor) and for k, v with fewer heads than q (H % H_kv == 0).  Returns out (bf16, laid
    out like q) and lse (fp32 [B,H,N])."""
    sq, sk, sv = _view(q, "q"), _view(k, "k"), _view(v, "v")
    for t, n in zip((lts, lte, uts, ute), ("lts", "lte", "uts", "ute")):
        _dev(t, torch.int32, n)
    B, H, N, d = q.shape
    Hk = k.shape[1]
    if tuple(k.shape) != (B, Hk, N, d) or v.shape != k.shape or any(tuple(x.shape) != (B, N) for x in (lts, lte, uts, ute)):
        raise FlashMaskError("shape mismatch: q [B,H,N,d]; k,v [B,H_kv,N,d]; lts,lte,uts,ute [B,N]")
    need = flashmask_workspace_bytes(FM_PASS_FWD, B, H, N, d)
    ws = workspace if workspace is not None else _workspace(need, q.device)
    out = torch.empty_like(q)
    so = _view(out, "out")
    lse = torch.empty((B, H, N), dtype=torch.float32, device=q.device)
    _check(load_library().flashmask_fwd_ex(q.data_ptr(), k.data_ptr(), v.data_ptr(), lts.data_ptr(), lte.data_ptr(),
                                           uts.data_ptr(), ute.data_ptr(), float(scale), out.data_ptr(),
                                           lse.data_ptr(), B, H, Hk, N, d, ctypes.byref(sq), ctypes.byref(sk),
                                           ctypes.byref(sv), ctypes.byref(so), ws.data_ptr(), ws.numel(), _stream()),
           "flashmask_fwd_ex")
    return out, lse


def flashmask_bwd_ex(q, k, v, out, lse, dout, lts, lte, uts, ute, scale: float,
                     workspace: torch.Tensor | None = None):
    """Backward for tensors of any strides and grouped K/V heads (see flashmask_fwd_ex).  Returns dq (laid
    out like q), dk and dv (laid out like k and v, summed over the query heads of each group)."""
    tensors = (q, k, v, out, dout)
    names = ("q", "k", "v", "out", "dout")
    st = [_view(t, n) for t, n in zip(tensors, names)]
    _dev(lse, torch.float32, "lse")
    for t, n in zip((lts, lte, uts, ute), ("lts", "lte", "uts", "ute")):
        _dev(t, torch.int32, n)
    B, H, N, d = q.shape
    Hk = k.shape[1]
    if tuple(k.shape) != (B, Hk, N, d) or v.shape != k.shape or out.shape != q.shape or dout.shape != q.shape or \
            tuple(lse.shape) != (B, H, N) or any(tuple(x.shape) != (B, N) for x in (lts, lte, uts, ute)):
        raise FlashMaskError("shape mismatch")
    need = flashmask_workspace_bytes(FM_PASS_BWD, B, H, N, d)
    ws = workspace if workspace is not None else _workspace(need, q.device)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
    st += [_view(dq, "dq"), _view(dk, "dk"), _view(dv, "dv")]
    arr = (Strides * 8)(*st)
    _check(load_library().flashmask_bwd_ex(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), lse.data_ptr(),
                                           dout.data_ptr(), lts.data_ptr(), lte.data_ptr(), uts.data_ptr(),
                                           ute.data_ptr(), float(scale), dq.data_ptr(), dk.data_ptr(), dv.data_ptr(),
                                           B, H, Hk, N, d, arr, ws.data_ptr(), ws.numel(), _stream()),
           "flashmask_bwd_ex")
    return dq, dk, dv


def flashmask_mfma_ceiling(operands: torch.Tensor, sink: torch.Tensor, workgroups: int, iters: int,
                           shape: int = 0) -> float:
    """Enqueue the matrix-core-only measurement kernel; returns the floating-point operations it performs."""
    _dev(operands, torch.bfloat16, "operands")
    _dev(sink, torch.float32, "sink")
    if operands.numel() < 8192 or sink.numel() < workgroups * 256:
        raise FlashMaskError("operands needs 8192 bf16 values, sink workgroups * 256 floats")
    flop = ctypes.c_double(0.0)
    _check(load_library().flashmask_mfma_ceiling(operands.data_ptr(), sink.data_ptr(), workgroups, iters, shape,
                                                 ctypes.byref(flop), _stream()), "flashmask_mfma_ceiling")
    return float(flop.value)


def flashmask_atomic_ceiling(acc: torch.Tensor, tiles: int, workgroups: int) -> float:
    """Enqueue the atomic-add measurement kernel on acc (fp32 [heads, n_tiles, 64, 128]); returns the bytes of
    fp32 updates it issues."""
    _dev(acc, torch.float32, "acc")
    if acc.dim() != 4 or tuple(acc.shape[2:]) != (64, 128):
        raise FlashMaskError("acc must be [heads, n_tiles, 64, 128]")
    nbytes = ctypes.c_double(0.0)
    _check(load_library().flashmask_atomic_ceiling(acc.data_ptr(), acc.shape[0], acc.shape[1], tiles, workgroups,
                                                   ctypes.byref(nbytes), _stream()), "flashmask_atomic_ceiling")
    return float(nbytes.value)


def flashmask_unit_queues(pass_id: int, lts, lte, uts, ute, H: int, d: int) -> torch.Tensor:
    """int32 [slots, 4] slot records of the pass's unit queues (see flashmask.h)."""
    vecs = [_dev(x, torch.int32, n) for x, n in zip((lts, lte, uts, ute), ("lts", "lte", "uts", "ute"))]
    B, N = vecs[0].shape
    lib = load_library()
    slots = ctypes.c_int(0)
    ptrs = [v.data_ptr() for v in vecs]
    _check(lib.flashmask_unit_queues(pass_id, *ptrs, B, H, N, d, None, ctypes.byref(slots), None, 0, None),
           "flashmask_unit_queues")
    rec = torch.empty((slots.value, 4), dtype=torch.int32, device=vecs[0].device)
    ws = _workspace(flashmask_workspace_bytes(FM_PASS_FWD if pass_id == FM_PASS_FWD else FM_PASS_BWD, B, H, N, d),
                    vecs[0].device)
    _check(lib.flashmask_unit_queues(pass_id, *ptrs, B, H, N, d, rec.data_ptr(), ctypes.byref(slots), ws.data_ptr(),
                                     ws.numel(), _stream()), "flashmask_unit_queues")
    return rec
