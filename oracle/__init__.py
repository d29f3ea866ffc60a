"""CPU fp64 oracle for the window-over-history attention (TEST INFRASTRUCTURE ONLY).

Thin ctypes wrapper over ``tlin_oracle.c``; see that file's header for what is computed and
what pins it.  Only the tests, the smoke check and the benchmark's ``cpu_baseline`` leg may
import this package; the product path never does.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libtlin_oracle.so")
_lib = None

F32, BF16 = 0, 1
SUM, JOINT = 0, 1


def build(verbose: bool = False) -> str:
    """Compile tlin_oracle.c (gcc -O2, OpenMP, no fast-math)."""
    cmd = ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB_PATH,
           os.path.join(_HERE, "tlin_oracle.c"), "-lm"]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    global _lib
    _lib = None
    return _LIB_PATH


def use_library(path: str) -> None:
    """Load another build of tlin_oracle.c instead of the one next to this file.  Only the pin
    tests call this (through their --oracle-lib option, which the GPU tests refuse): the
    mutation test points them at deliberately broken builds to show that the pins notice."""
    global _lib, _LIB_PATH
    if not os.path.exists(path):
        raise FileNotFoundError(path)
    _LIB_PATH = path
    _lib = None


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            build()
        lib = ctypes.CDLL(_LIB_PATH)
        vp, ci, cd = ctypes.c_void_p, ctypes.c_int, ctypes.c_double
        lib.tlin_oracle_history.restype = ci
        lib.tlin_oracle_history.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, ci, cd, vp, ci, vp, vp]
        lib.tlin_oracle_window_causal.restype = ci
        lib.tlin_oracle_window_causal.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, cd, vp, ci, vp, vp]
        lib.tlin_oracle_layer.restype = ci
        lib.tlin_oracle_layer.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, cd, ci, vp, ci, vp]
        lib.tlin_oracle_slide.restype = ci
        lib.tlin_oracle_slide.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, cd, ci, vp, ci, vp]
        lib.tlin_oracle_threads.restype = ci
        _lib = lib
    return _lib


def _prep(a, dtype):
    want = np.float32 if dtype == F32 else np.uint16
    a = np.ascontiguousarray(a)
    if a.dtype != want:
        raise TypeError(f"expected {want} storage for dtype {dtype}, got {a.dtype}")
    if a.ndim != 4:
        raise ValueError("expected [B,H,rows,D]")
    return a


def _rows(rows, W):
    if rows is None:
        return None, 0, W
    r = np.ascontiguousarray(rows, dtype=np.int32)
    return r, int(r.size), int(r.size)


def _ptr(a):
    return None if a is None else a.ctypes.data


def history(Q, Kh, Vh, dtype, scale, rows=None):
    """Unmasked attention of the window rows over the history.  Returns (O, lse) in fp64:
    O [B,H,R,D], lse [B,H,R], R = len(rows) or W."""
    Q, Kh, Vh = _prep(Q, dtype), _prep(Kh, dtype), _prep(Vh, dtype)
    B, H, W, D = Q.shape
    N = Kh.shape[2]
    assert Kh.shape == (B, H, N, D) and Vh.shape == (B, H, N, D)
    r, nr, R = _rows(rows, W)
    O = np.empty((B, H, R, D), dtype=np.float64)
    lse = np.empty((B, H, R), dtype=np.float64)
    rc = _load().tlin_oracle_history(_ptr(Q), _ptr(Kh), _ptr(Vh), dtype, B, H, W, N, D, float(scale),
                                     _ptr(r), nr, _ptr(O), _ptr(lse))
    if rc != 0:
        raise RuntimeError(f"tlin_oracle_history failed ({rc})")
    return O, lse


def window_causal(Q, Kw, Vw, dtype, scale, rows=None):
    """Causal attention inside the window (row i sees rows j <= i).  Returns (O, lse)."""
    Q, Kw, Vw = _prep(Q, dtype), _prep(Kw, dtype), _prep(Vw, dtype)
    B, H, W, D = Q.shape
    assert Kw.shape == (B, H, W, D) and Vw.shape == (B, H, W, D)
    r, nr, R = _rows(rows, W)
    O = np.empty((B, H, R, D), dtype=np.float64)
    lse = np.empty((B, H, R), dtype=np.float64)
    rc = _load().tlin_oracle_window_causal(_ptr(Q), _ptr(Kw), _ptr(Vw), dtype, B, H, W, D, float(scale),
                                           _ptr(r), nr, _ptr(O), _ptr(lse))
    if rc != 0:
        raise RuntimeError(f"tlin_oracle_window_causal failed ({rc})")
    return O, lse


def layer(Q, Kh, Vh, Kw, Vw, dtype, scale, combine, rows=None):
    """History attention and window causal attention combined (SUM or JOINT).  Kh/Vh may be
    None or have zero rows (empty history).  Returns O [B,H,R,D] in fp64."""
    Q, Kw, Vw = _prep(Q, dtype), _prep(Kw, dtype), _prep(Vw, dtype)
    B, H, W, D = Q.shape
    N = 0 if Kh is None else Kh.shape[2]
    if N > 0:
        Kh, Vh = _prep(Kh, dtype), _prep(Vh, dtype)
        assert Kh.shape == (B, H, N, D) and Vh.shape == (B, H, N, D)
    else:
        Kh = Vh = None
    r, nr, R = _rows(rows, W)
    O = np.empty((B, H, R, D), dtype=np.float64)
    rc = _load().tlin_oracle_layer(_ptr(Q), _ptr(Kh), _ptr(Vh), _ptr(Kw), _ptr(Vw), dtype, B, H, W, N, D,
                                   float(scale), int(combine), _ptr(r), nr, _ptr(O))
    if rc != 0:
        raise RuntimeError(f"tlin_oracle_layer failed ({rc})")
    return O


def slide(Q, Kh, Vh, Kw, Vw, dtype, scale, chunk, combine, rows=None):
    """Sliding schedule of Section 5.1 over a whole sequence: all tensors [B,H,L,D]; position
    p = c*chunk + i attends history rows [0, c*chunk) of Kh/Vh unmasked and window rows
    [c*chunk, p] of Kw/Vw, combined by SUM or JOINT.  Returns O [B,H,R,D] in fp64."""
    Q, Kh, Vh, Kw, Vw = (_prep(a, dtype) for a in (Q, Kh, Vh, Kw, Vw))
    B, H, L, D = Q.shape
    for a in (Kh, Vh, Kw, Vw):
        assert a.shape == (B, H, L, D)
    r, nr, R = _rows(rows, L)
    O = np.empty((B, H, R, D), dtype=np.float64)
    rc = _load().tlin_oracle_slide(_ptr(Q), _ptr(Kh), _ptr(Vh), _ptr(Kw), _ptr(Vw), dtype, B, H, L, int(chunk), D,
                                   float(scale), int(combine), _ptr(r), nr, _ptr(O))
    if rc != 0:
        raise RuntimeError(f"tlin_oracle_slide failed ({rc})")
    return O


def threads() -> int:
    """OpenMP threads the oracle runs on."""
    return int(_load().tlin_oracle_threads())
