"""ctypes front end of the CPU oracle (oracle/fps_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and
by bench.py's cpu_baseline leg.  The product package never imports it and it
never imports the product package.  All arithmetic lives in the C file; this
module only marshals NumPy arrays and loops over the batch dimension.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fps_oracle.c")
_LIB = os.path.join(_HERE, "libfps_oracle.so")

FLAG_CP = 1
FLAG_IP = 2
FLAG_PERM = 4
MODE_CACHED = 0
MODE_CHAIN = 1

CFLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC", "-std=gnu11", "-pthread"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (contraction off).  Returns the .so path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", *CFLAGS, "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        fp = ctypes.POINTER(ctypes.c_float)
        ip = ctypes.POINTER(ctypes.c_int32)
        ci = ctypes.c_int
        lib.oracle_fps_exact.argtypes = [fp, ci, ci, ci, ip, fp]
        lib.oracle_fps_exact.restype = ci
        lib.oracle_fps_exact_mt.argtypes = [fp, ci, ci, ci, ip, fp, ci]
        lib.oracle_fps_exact_mt.restype = ci
        lib.oracle_prune_sizes.argtypes = [ci, ci, ci, ci, ctypes.c_uint,
                                           ctypes.POINTER(ci), ctypes.POINTER(ci), ctypes.POINTER(ci)]
        lib.oracle_prune_sizes.restype = ci
        lib.oracle_candidates.argtypes = [ci, ci, ci, ip, ctypes.POINTER(ci)]
        lib.oracle_candidates.restype = ci
        lib.oracle_fps_prune.argtypes = [fp, ci, ci, ci, ci, ci, ctypes.c_uint, ctypes.c_uint64, ip,
                                         ctypes.POINTER(ci)]
        lib.oracle_perm.argtypes = [ctypes.c_int64, ctypes.c_uint64, ctypes.c_int64]
        lib.oracle_perm.restype = ctypes.c_int64
        lib.oracle_candidates_perm.argtypes = [ci, ci, ci, ctypes.c_uint64, ip, ctypes.POINTER(ci)]
        lib.oracle_candidates_perm.restype = ci
        lib.oracle_fps_prune.restype = ci
        lib.oracle_fps_stages.argtypes = [fp, ci, ci, ctypes.POINTER(ci), ci, ci, ci,
                                          ctypes.c_uint, ctypes.c_uint64, ci, ip]
        lib.oracle_fps_stages.restype = ci
        lib.oracle_coverage_radius.argtypes = [fp, ci, ip, ci]
        lib.oracle_coverage_radius.restype = ctypes.c_double
        _lib = lib
    return _lib


def _fptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _iptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _cloud(xyz):
    a = np.ascontiguousarray(xyz, dtype=np.float32)
    if a.ndim != 2 or a.shape[1] != 3:
        raise ValueError("expected a [N,3] cloud")
    return a


def _batched(fn, xyz, *args, **kw):
    a = np.asarray(xyz)
    if a.ndim == 3:
        outs = [fn(a[b], *args, **kw) for b in range(a.shape[0])]
        if isinstance(outs[0], tuple):
            return tuple(np.stack([o[i] for o in outs]) for i in range(len(outs[0])))
        return np.stack(outs)
    return fn(a, *args, **kw)


def _fps_exact1(xyz, M, start=0, return_maxdist=False):
    a = _cloud(xyz)
    idx = np.empty(M, dtype=np.int32)
    md = np.empty(M, dtype=np.float32)
    rc = _load().oracle_fps_exact(_fptr(a), a.shape[0], M, start, _iptr(idx), _fptr(md))
    if rc:
        raise ValueError(f"oracle_fps_exact: invalid arguments (rc={rc})")
    return (idx, md) if return_maxdist else idx


def fps_exact(xyz, M, start=0, return_maxdist=False):
    """Exact FPS (Eq. 1).  xyz [N,3] or [B,N,3]; returns int32 idx [M] or [B,M]
    (and the squared pick distances when return_maxdist)."""
    return _batched(_fps_exact1, xyz, M, start, return_maxdist)


def host_threads() -> int:
    """Threads the all-cores run may use: the cores this process may run on,
    capped by OMP_NUM_THREADS when that is set."""
    n = len(os.sched_getaffinity(0))
    env = os.environ.get("OMP_NUM_THREADS", "")
    if env.isdigit() and int(env) >= 1:
        n = min(n, int(env))
    return max(1, n)


def fps_exact_mt(xyz, M, start=0, threads=None, return_maxdist=False):
    """Exact FPS of ONE cloud on `threads` host threads (default host_threads());
    identical to fps_exact for any thread count."""
    a = _cloud(xyz)
    idx = np.empty(M, dtype=np.int32)
    md = np.empty(M, dtype=np.float32)
    t = host_threads() if threads is None else int(threads)
    rc = _load().oracle_fps_exact_mt(_fptr(a), a.shape[0], M, start, _iptr(idx), _fptr(md), t)
    if rc:
        raise ValueError(f"oracle_fps_exact_mt: invalid arguments (rc={rc})")
    return (idx, md) if return_maxdist else idx


def prune_sizes(N, M, keep_num, keep_den, flags):
    """(N', k, R) of FPS-Prune (Alg. 1, layer 1)."""
    nc, k, r = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    rc = _load().oracle_prune_sizes(N, M, keep_num, keep_den, flags,
                                    ctypes.byref(nc), ctypes.byref(k), ctypes.byref(r))
    if rc:
        raise ValueError("oracle_prune_sizes: invalid arguments")
    return nc.value, k.value, r.value


def candidates(N, Nc, start=0):
    """(cand[N'], position of start in cand) of candidate pruning."""
    cand = np.empty(Nc, dtype=np.int32)
    pos = ctypes.c_int()
    rc = _load().oracle_candidates(N, Nc, start, _iptr(cand), ctypes.byref(pos))
    if rc:
        raise ValueError("oracle_candidates: invalid arguments")
    return cand, pos.value


def perm(N, seed, j):
    """Image of j under the seeded bijection of [0, N) (random select / fill)."""
    return int(_load().oracle_perm(N, seed, j))


def candidates_perm(N, Nc, start, seed):
    cand = np.empty(Nc, dtype=np.int32)
    pos = ctypes.c_int()
    rc = _load().oracle_candidates_perm(N, Nc, start, seed, _iptr(cand), ctypes.byref(pos))
    if rc:
        raise ValueError("oracle_candidates_perm: invalid arguments")
    return cand, pos.value


def _fps_prune1(xyz, M, keep_num, keep_den, flags=FLAG_CP | FLAG_IP, start=0, seed=0):
    a = _cloud(xyz)
    idx = np.empty(M, dtype=np.int32)
    k = ctypes.c_int()
    rc = _load().oracle_fps_prune(_fptr(a), a.shape[0], M, start, keep_num, keep_den, flags, seed,
                                  _iptr(idx), ctypes.byref(k))
    if rc:
        raise ValueError(f"oracle_fps_prune: invalid arguments (rc={rc})")
    return idx


def fps_prune(xyz, M, keep_num, keep_den, flags=FLAG_CP | FLAG_IP, start=0, seed=0):
    """FPS-Prune (Alg. 1, layer 1).  First k entries are FPS order, then the fill.
    With FLAG_PERM cloud b of a batch uses seed + b."""
    a = np.asarray(xyz)
    if a.ndim == 3:
        return np.stack([_fps_prune1(a[b], M, keep_num, keep_den, flags, start, seed + b)
                         for b in range(a.shape[0])])
    return _fps_prune1(a, M, keep_num, keep_den, flags, start, seed)


def _fps_stages1(xyz, Ms, mode, keep_num=1, keep_den=1, flags=0, start=0, seed=0):
    a = _cloud(xyz)
    ms = (ctypes.c_int * len(Ms))(*[int(m) for m in Ms])
    out = np.empty(int(sum(Ms)), dtype=np.int32)
    rc = _load().oracle_fps_stages(_fptr(a), a.shape[0], len(Ms), ms, start, keep_num, keep_den,
                                   flags, seed, mode, _iptr(out))
    if rc:
        raise ValueError(f"oracle_fps_stages: invalid arguments (rc={rc})")
    return out


def fps_stages(xyz, Ms, mode, keep_num=1, keep_den=1, flags=0, start=0, seed=0):
    """Stage chain (Alg. 1 / Sec. 3.3); returns the layers back to back."""
    a = np.asarray(xyz)
    if a.ndim == 3:
        return np.stack([_fps_stages1(a[b], Ms, mode, keep_num, keep_den, flags, start, seed + b)
                         for b in range(a.shape[0])])
    return _fps_stages1(a, Ms, mode, keep_num, keep_den, flags, start, seed)


def coverage_radius(xyz, sel):
    """R_P(S): largest distance from any point of the cloud to its nearest sample."""
    a = _cloud(xyz)
    s = np.ascontiguousarray(sel, dtype=np.int32)
    return float(_load().oracle_coverage_radius(_fptr(a), a.shape[0], _iptr(s), s.shape[0]))
