"""ctypes binding of libtlinattn.so: argument marshalling only.

Every step of the attention path runs in the library's HIP kernels; PyTorch supplies device
memory and streams.  There is no fallback: if the library has not been built the import of
the entry points fails with an error that says so.
"""
from __future__ import annotations

import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libtlinattn.so")

TLIN_OK, TLIN_ERR_INVALID_ARG, TLIN_ERR_UNSUPPORTED, TLIN_ERR_WORKSPACE, TLIN_ERR_HIP = range(5)
TLIN_F32, TLIN_BF16 = 0, 1
TLIN_COMBINE_SUM, TLIN_COMBINE_JOINT = 0, 1

EXPORTS = ("tlin_workspace_bytes", "tlin_num_splits", "tlin_history_attn", "tlin_window_causal_attn",
           "tlin_layer_attn", "tlin_layer_attn_static_ws", "tlin_slide_workspace_bytes", "tlin_slide_layer_attn", "tlin_profile_enable", "tlin_profile_read", "tlin_profile_stream_read", "tlin_status_string", "tlin_version")


class TlinParams(ctypes.Structure):
    """Mirror of ``tlin_params`` in include/tlinattn.h."""
    _fields_ = [
        ("B", ctypes.c_int32), ("H", ctypes.c_int32), ("W", ctypes.c_int32), ("N", ctypes.c_int32),
        ("D", ctypes.c_int32), ("in_dtype", ctypes.c_int32), ("out_dtype", ctypes.c_int32),
        ("scale", ctypes.c_float), ("num_splits", ctypes.c_int32), ("combine", ctypes.c_int32),
        ("q_stride", ctypes.c_int64 * 3), ("kh_stride", ctypes.c_int64 * 3), ("vh_stride", ctypes.c_int64 * 3),
        ("kw_stride", ctypes.c_int64 * 3), ("vw_stride", ctypes.c_int64 * 3), ("o_stride", ctypes.c_int64 * 3),
    ]


class TlinError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library.  Raises if it has not been built (no CPU fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2508_20407_amd.build` "
                "(hipcc, gfx950).  There is no fallback implementation.")
        L = ctypes.CDLL(LIB_PATH)
        pp, vp, sz = ctypes.POINTER(TlinParams), ctypes.c_void_p, ctypes.c_size_t
        L.tlin_workspace_bytes.restype = sz
        L.tlin_workspace_bytes.argtypes = [pp]
        L.tlin_num_splits.restype = ctypes.c_int32
        L.tlin_num_splits.argtypes = [pp]
        L.tlin_history_attn.restype = ctypes.c_int
        L.tlin_history_attn.argtypes = [pp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.tlin_window_causal_attn.restype = ctypes.c_int
        L.tlin_window_causal_attn.argtypes = [pp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.tlin_layer_attn.restype = ctypes.c_int
        L.tlin_layer_attn.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.tlin_layer_attn_static_ws.restype = ctypes.c_int
        L.tlin_layer_attn_static_ws.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp]
        L.tlin_slide_workspace_bytes.restype = sz
        L.tlin_slide_workspace_bytes.argtypes = [pp]
        L.tlin_slide_layer_attn.restype = ctypes.c_int
        L.tlin_slide_layer_attn.argtypes = [pp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.tlin_profile_enable.restype = ctypes.c_int
        L.tlin_profile_enable.argtypes = [ctypes.c_int32]
        L.tlin_profile_read.restype = ctypes.c_int
        L.tlin_profile_read.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]
        L.tlin_profile_stream_read.restype = ctypes.c_int
        L.tlin_profile_stream_read.argtypes = [vp, sz, ctypes.c_int32, vp]
        L.tlin_status_string.restype = ctypes.c_char_p
        L.tlin_status_string.argtypes = [ctypes.c_int]
        L.tlin_version.restype = ctypes.c_int32
        L.tlin_version.argtypes = []
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().tlin_status_string(int(status)).decode()


def version() -> int:
    return int(lib().tlin_version())


def make_params(B, H, W, N, D, in_dtype, out_dtype, scale, num_splits=0, combine=TLIN_COMBINE_SUM,
                **strides) -> TlinParams:
    p = TlinParams()
    p.B, p.H, p.W, p.N, p.D = int(B), int(H), int(W), int(N), int(D)
    p.in_dtype, p.out_dtype = int(in_dtype), int(out_dtype)
    p.scale, p.num_splits, p.combine = float(scale), int(num_splits), int(combine)
    for name, val in strides.items():
        arr = getattr(p, name)
        for i in range(3):
            arr[i] = int(val[i])
    return p


def workspace_bytes(p: TlinParams) -> int:
    return int(lib().tlin_workspace_bytes(ctypes.byref(p)))


def num_splits(p: TlinParams) -> int:
    return int(lib().tlin_num_splits(ctypes.byref(p)))


def _check(status: int, where: str):
    if status != TLIN_OK:
        raise TlinError(status, where)


def history_attn_raw(p, q, kh, vh, o, lse, ws, ws_bytes, stream) -> int:
    """Raw call with integer device addresses; returns the status code."""
    return int(lib().tlin_history_attn(ctypes.byref(p), q, kh, vh, o, lse, ws, ws_bytes, stream))


def window_causal_attn_raw(p, q, kw, vw, o, lse, ws, ws_bytes, stream) -> int:
    return int(lib().tlin_window_causal_attn(ctypes.byref(p), q, kw, vw, o, lse, ws, ws_bytes, stream))


def layer_attn_raw(p, q, kh, vh, kw, vw, o, ws, ws_bytes, stream) -> int:
    return int(lib().tlin_layer_attn(ctypes.byref(p), q, kh, vh, kw, vw, o, ws, ws_bytes, stream))


STATIC_WS_BYTES = 64 << 20   # TLIN_STATIC_WS_BYTES


def layer_attn_static_ws_raw(p, q, kh, vh, kw, vw, o, stream) -> int:
    return int(lib().tlin_layer_attn_static_ws(ctypes.byref(p), q, kh, vh, kw, vw, o, stream))


def slide_workspace_bytes(p: TlinParams) -> int:
    return int(lib().tlin_slide_workspace_bytes(ctypes.byref(p)))


def slide_layer_attn_raw(p, q, kh, vh, kw, vw, o, ws, ws_bytes, stream) -> int:
    return int(lib().tlin_slide_layer_attn(ctypes.byref(p), q, kh, vh, kw, vw, o, ws, ws_bytes, stream))


def profile_enable(on: bool) -> None:
    _check(int(lib().tlin_profile_enable(1 if on else 0)), "tlin_profile_enable")


def profile_stream_read(addr: int, nbytes: int, nontemporal: bool, stream) -> None:
    """Enqueue the read-only streaming kernel over a device buffer (measurement aid)."""
    _check(int(lib().tlin_profile_stream_read(addr, nbytes, 1 if nontemporal else 0, stream)), "tlin_profile_stream_read")


def profile_read():
    """(ms, launches) per kernel class: history partition kernel, window causal kernel, merge."""
    ms = (ctypes.c_double * 3)()
    n = (ctypes.c_int64 * 3)()
    _check(int(lib().tlin_profile_read(ms, n)), "tlin_profile_read")
    return list(ms), list(n)
