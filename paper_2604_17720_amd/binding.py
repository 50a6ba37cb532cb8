"""Thin Python binding of libflashfps.so: same names as the C ABI
(include/flashfps.h), argument marshalling only.  Every step of the sampling
path runs in the library's HIP kernels; PyTorch supplies device memory and the
stream and nothing else.  There is no CPU fallback: without the built library
or without a GPU the calls raise."""
from __future__ import annotations

import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libflashfps.so")

FFPS_OK = 0
FFPS_ERR_INVALID_ARG = -1
FFPS_ERR_WORKSPACE_TOO_SMALL = -2
FFPS_ERR_UNSUPPORTED_DEVICE = -3
FFPS_ERR_LAUNCH_FAILED = -4
FFPS_ERR_TIMEOUT = -5
FFPS_ERR_UNSUPPORTED_SIZE = -6
FFPS_ERR_INTERNAL = -7
FFPS_FLAG_CP = 1
FFPS_FLAG_IP = 2
FFPS_FLAG_PERM = 4
FFPS_MODE_CACHED = 0
FFPS_MODE_CHAIN = 1
FFPS_VARIANT_AUTO = 0
FFPS_VARIANT_WG = 1
FFPS_VARIANT_GRID = 2
FFPS_VARIANT_STREAM = 3



FFPS_VARIANT_TEST_NO_WAIT = 1 << 16


def variant_with_picks(variant: int, picks: int) -> int:
    """FFPS_VARIANT_WITH_PICKS of the header."""
    return variant | (picks << 8)


EXPORTS = ["ffps_version", "ffps_strerror", "ffps_prune_sizes", "ffps_workspace_bytes",
           "ffps_exact", "ffps_prune", "ffps_cached_stages", "ffps_last_status",
           "ffps_last_rounds", "ffps_barrier_probe", "ffps_alu_probe", "ffps_gather_rows", "ffps_describe_plan",
           "ffps_exact_noalloc"]


class FlashFPSError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {ffps_strerror(code)} ({code})")


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library (built in-tree by build.py if absent)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            from . import build as _build
            _build.build(force=True)
        L = ctypes.CDLL(LIB_PATH)
        c_int, c_vp, c_sz = ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
        ip = ctypes.POINTER(c_int)
        L.ffps_version.restype = c_int
        L.ffps_strerror.argtypes = [c_int]
        L.ffps_strerror.restype = ctypes.c_char_p
        L.ffps_prune_sizes.argtypes = [c_int, c_int, c_int, c_int, ctypes.c_uint, ip, ip, ip]
        L.ffps_workspace_bytes.argtypes = [c_int, c_int, c_int, ctypes.POINTER(c_sz)]
        L.ffps_exact.argtypes = [c_vp, c_int, c_int, c_int, c_int, c_int, c_vp, c_vp, c_vp, c_sz, c_vp]
        L.ffps_exact_noalloc.argtypes = [c_vp, c_int, c_int, c_int, c_int, c_int, c_vp, c_vp, c_vp, c_vp]
        L.ffps_prune.argtypes = [c_vp, c_int, c_int, c_int, c_int, c_int, c_int, ctypes.c_uint,
                                 ctypes.c_uint64, c_int, c_vp, ip, c_vp, c_sz, c_vp]
        L.ffps_cached_stages.argtypes = [c_vp, c_int, c_int, c_int, ip, c_int, c_int, c_int,
                                         ctypes.c_uint, ctypes.c_uint64, c_int, c_int, c_vp, c_vp,
                                         c_sz, c_vp]
        L.ffps_last_status.argtypes = [c_vp, c_vp]
        L.ffps_last_rounds.argtypes = [c_vp, c_vp]
        L.ffps_gather_rows.argtypes = [c_vp, c_int, c_int, c_int, c_vp, ctypes.c_long, c_int, c_vp, c_vp]
        L.ffps_barrier_probe.argtypes = [c_int, c_vp, c_sz, c_vp, ctypes.POINTER(ctypes.c_float)]
        L.ffps_alu_probe.argtypes = [c_int, c_int, c_vp, c_sz, c_vp, ctypes.POINTER(ctypes.c_double)]
        L.ffps_describe_plan.argtypes = [c_int, c_int, c_int, c_int, ip, ip, ip, ip]
        for n in EXPORTS:
            if n not in ("ffps_strerror",):
                getattr(L, n).restype = c_int
        _lib = L
    return _lib


# ---- host-only calls ---------------------------------------------------------
def ffps_version() -> int:
    return lib().ffps_version()


def ffps_strerror(code: int) -> str:
    return lib().ffps_strerror(code).decode()


def ffps_prune_sizes(N, M, keep_num, keep_den, flags):
    nc, k, r = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    rc = lib().ffps_prune_sizes(N, M, keep_num, keep_den, flags, ctypes.byref(nc),
                                ctypes.byref(k), ctypes.byref(r))
    if rc:
        raise FlashFPSError(rc, "ffps_prune_sizes")
    return nc.value, k.value, r.value


def ffps_describe_plan(B, N, variant=FFPS_VARIANT_AUTO, num_cu=256):
    """(kernel, workgroups per cloud, reporting units per cloud, clouds per launch)
    a call on B clouds of N points would use on a device with num_cu CUs."""
    k, g, u, c = ctypes.c_int(), ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    rc = lib().ffps_describe_plan(B, N, variant, num_cu, ctypes.byref(k), ctypes.byref(g),
                                  ctypes.byref(u), ctypes.byref(c))
    if rc:
        raise FlashFPSError(rc, "ffps_describe_plan")
    return k.value, g.value, u.value, c.value


def ffps_workspace_bytes(B, N, M) -> int:
    out = ctypes.c_size_t()
    rc = lib().ffps_workspace_bytes(B, N, M, ctypes.byref(out))
    if rc:
        raise FlashFPSError(rc, "ffps_workspace_bytes")
    return out.value


# ---- device calls --------------------------------------------------------------
def _torch():
    import torch
    if not torch.cuda.is_available():
        raise RuntimeError("flashfps needs a GPU: there is no CPU path")
    return torch


def _prep(xyz):
    torch = _torch()
    if not (xyz.is_cuda and xyz.dtype == torch.float32 and xyz.is_contiguous()):
        raise ValueError("xyz must be a contiguous float32 CUDA tensor")
    if xyz.dim() == 2:
        xyz = xyz.unsqueeze(0)
    if xyz.dim() != 3 or xyz.shape[2] != 3:
        raise ValueError("xyz must be [B,N,3] or [N,3]")
    return torch, xyz, int(xyz.shape[0]), int(xyz.shape[1])


def make_workspace(B, N, M, device="cuda", stream=None):
    """Device workspace (uint8 tensor) large enough for any call with these sizes.
    With `stream` it is allocated as that stream's memory, so the caching
    allocator does not hand it to other work before the stream has finished."""
    torch = _torch()
    n = ffps_workspace_bytes(B, N, M)
    if stream is None:
        return torch.empty(n, dtype=torch.uint8, device=device)
    with torch.cuda.stream(stream):
        return torch.empty(n, dtype=torch.uint8, device=device)


def _empty(torch, shape, dtype, device, stream):
    if stream is None:
        return torch.empty(shape, dtype=dtype, device=device)
    with torch.cuda.stream(stream):
        return torch.empty(shape, dtype=dtype, device=device)


def _stream(torch, stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def ffps_exact(xyz, M, start_idx=0, variant=FFPS_VARIANT_AUTO, return_maxdist=False,
               workspace=None, stream=None, out=None):
    """Exact FPS.  xyz: CUDA float32 [B,N,3] (or [N,3]).  Returns int32 [B,M]
    (and fp32 [B,M] squared pick distances when return_maxdist)."""
    torch, x, B, N = _prep(xyz)
    if not (1 <= M <= N):
        raise FlashFPSError(FFPS_ERR_INVALID_ARG, "ffps_exact")
    ws = make_workspace(B, N, M, x.device, stream) if workspace is None else workspace
    idx = _empty(torch, (B, M), torch.int32, x.device, stream) if out is None else out
    md = _empty(torch, (B, M), torch.float32, x.device, stream) if return_maxdist else None
    rc = lib().ffps_exact(x.data_ptr(), B, N, M, start_idx, variant, idx.data_ptr(),
                          md.data_ptr() if md is not None else None, ws.data_ptr(), ws.numel(),
                          _stream(torch, stream))
    if rc:
        raise FlashFPSError(rc, "ffps_exact")
    return (idx, md) if return_maxdist else idx


def ffps_exact_noalloc(xyz, M, out, start_idx=0, variant=FFPS_VARIANT_AUTO, out_maxdist=None,
                       out_status=None, stream=None):
    """ffps_exact without a workspace and without any allocation: the caller
    passes every output (out int32 [B,M]; optionally out_maxdist fp32 [B,M] and
    out_status int32 [2]).  Returns out."""
    torch, x, B, N = _prep(xyz)
    if not (1 <= M <= N):
        raise FlashFPSError(FFPS_ERR_INVALID_ARG, "ffps_exact_noalloc")
    rc = lib().ffps_exact_noalloc(x.data_ptr(), B, N, M, start_idx, variant, out.data_ptr(),
                                  out_maxdist.data_ptr() if out_maxdist is not None else None,
                                  out_status.data_ptr() if out_status is not None else None,
                                  _stream(torch, stream))
    if rc:
        raise FlashFPSError(rc, "ffps_exact_noalloc")
    return out


def ffps_prune(xyz, M, keep_num, keep_den, flags=FFPS_FLAG_CP | FFPS_FLAG_IP, start_idx=0,
               variant=FFPS_VARIANT_AUTO, workspace=None, stream=None, out=None, seed=0):
    """FPS-Prune.  Returns (idx int32 [B,M], k): idx[:, :k] is FPS order, idx[:, k:] the fill."""
    torch, x, B, N = _prep(xyz)
    if not (1 <= M <= N):
        raise FlashFPSError(FFPS_ERR_INVALID_ARG, "ffps_prune")
    ws = make_workspace(B, N, M, x.device, stream) if workspace is None else workspace
    idx = _empty(torch, (B, M), torch.int32, x.device, stream) if out is None else out
    k = ctypes.c_int()
    rc = lib().ffps_prune(x.data_ptr(), B, N, M, start_idx, keep_num, keep_den, flags, seed, variant,
                          idx.data_ptr(), ctypes.byref(k), ws.data_ptr(), ws.numel(),
                          _stream(torch, stream))
    if rc:
        raise FlashFPSError(rc, "ffps_prune")
    return idx, k.value


def ffps_cached_stages(xyz, M_stages, mode=FFPS_MODE_CACHED, keep_num=1, keep_den=1, flags=0,
                       start_idx=0, variant=FFPS_VARIANT_AUTO, workspace=None, stream=None,
                       out=None, seed=0):
    """Stage chain.  Returns a list of int32 [B,M_l] views, one per layer, of one
    [B, sum(M_stages)] tensor."""
    torch, x, B, N = _prep(xyz)
    ms = [int(m) for m in M_stages]
    if not ms or not (1 <= ms[0] <= N):
        raise FlashFPSError(FFPS_ERR_INVALID_ARG, "ffps_cached_stages")
    ws = make_workspace(B, N, ms[0], x.device, stream) if workspace is None else workspace
    S = sum(ms)
    idx = _empty(torch, (B, S), torch.int32, x.device, stream) if out is None else out
    arr = (ctypes.c_int * len(ms))(*ms)
    rc = lib().ffps_cached_stages(x.data_ptr(), B, N, len(ms), arr, start_idx, keep_num, keep_den,
                                  flags, seed, mode, variant, idx.data_ptr(), ws.data_ptr(), ws.numel(),
                                  _stream(torch, stream))
    if rc:
        raise FlashFPSError(rc, "ffps_cached_stages")
    outs, off = [], 0
    for m in ms:
        outs.append(idx[:, off:off + m])
        off += m
    return outs


def ffps_last_status(workspace, stream=None) -> int:
    torch = _torch()
    return lib().ffps_last_status(workspace.data_ptr(), _stream(torch, stream))


def ffps_last_rounds(workspace, stream=None) -> int:
    torch = _torch()
    return lib().ffps_last_rounds(workspace.data_ptr(), _stream(torch, stream))


def ffps_alu_probe(waves_per_cu, iters, workspace=None, stream=None) -> float:
    """Sustained individually rounded fp32 vector operations per second (diagnostic)."""
    torch = _torch()
    ws = workspace if workspace is not None else make_workspace(1, 1, 1, stream=stream)
    out = ctypes.c_double(0.0)
    rc = lib().ffps_alu_probe(int(waves_per_cu), int(iters), ws.data_ptr(), ws.numel(), _stream(torch, stream),
                              ctypes.byref(out))
    if rc != 0:
        raise FlashFPSError(rc, "ffps_alu_probe")
    return out.value


def ffps_barrier_probe(iters, workspace=None, stream=None) -> float:
    """Mean time of one plain grid barrier (microseconds) in the GRID launch shape."""
    torch = _torch()
    ws = make_workspace(1, 1, 1, stream=stream) if workspace is None else workspace
    out = ctypes.c_float()
    rc = lib().ffps_barrier_probe(iters, ws.data_ptr(), ws.numel(), _stream(torch, stream),
                                  ctypes.byref(out))
    if rc:
        raise FlashFPSError(rc, "ffps_barrier_probe")
    return out.value


def ffps_gather_rows(rows, idx, stream=None):
    """rows: CUDA float32 [B,N,C]; idx: CUDA int32 [B,S] (may be a column slice of a
    wider tensor, e.g. one stage of ffps_cached_stages).  Returns float32 [B,S,C]."""
    torch = _torch()
    if not (rows.is_cuda and rows.dtype == torch.float32 and rows.is_contiguous() and rows.dim() == 3):
        raise ValueError("rows must be a contiguous float32 CUDA tensor [B,N,C]")
    if not (idx.is_cuda and idx.dtype == torch.int32 and idx.dim() == 2 and idx.stride(1) == 1):
        raise ValueError("idx must be an int32 CUDA tensor [B,S] with unit inner stride")
    B, N, C = (int(v) for v in rows.shape)
    S = int(idx.shape[1])
    if int(idx.shape[0]) != B:
        raise ValueError("batch sizes differ")
    stride = int(idx.stride(0)) if B > 1 else max(int(idx.stride(0)), S)
    out = _empty(torch, (B, S, C), torch.float32, rows.device, stream)
    rc = lib().ffps_gather_rows(rows.data_ptr(), B, N, C, idx.data_ptr(), stride, S, out.data_ptr(),
                                _stream(torch, stream))
    if rc:
        raise FlashFPSError(rc, "ffps_gather_rows")
    return out
