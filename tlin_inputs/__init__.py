"""Seeded synthetic inputs for the window-over-history attention workloads.

Shared by the tests, the bench and the CPU oracle's callers.  It holds none of the method's
arithmetic: only the workload table (shapes, dtypes, value distributions) and a counter-based
Gaussian generator implemented in ``gen.c`` (built by :func:`build`).

The workloads stand in for the paper's long-sequence inference runs (Section 6.4: batch 1,
random content, history length swept to ~1e6, fixed windows of a few hundred rows): the
trained weights and the text corpus are not available, and the attention path takes already
projected Q/K/V, so Gaussian Q/K/V of the same shapes are used.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, replace

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libtlin_inputs.so")
_lib = None

F32, BF16 = 0, 1
TAG_Q, TAG_KH, TAG_VH, TAG_KW, TAG_VW = 1, 2, 3, 4, 5


def build(verbose: bool = False) -> str:
    """Compile gen.c into libtlin_inputs.so (gcc, OpenMP)."""
    cmd = ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB_PATH,
           os.path.join(_HERE, "gen.c"), "-lm"]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    global _lib
    _lib = None
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            build()
        lib = ctypes.CDLL(_LIB_PATH)
        lib.tlin_gen_normal.restype = ctypes.c_int
        lib.tlin_gen_normal.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64,
                                        ctypes.c_uint64, ctypes.c_size_t, ctypes.c_float,
                                        ctypes.c_size_t, ctypes.c_uint32, ctypes.c_float]
        _lib = lib
    return _lib


@dataclass(frozen=True)
class Workload:
    """One synthetic attention problem.  N = history rows, W = window rows, D = head dim."""
    name: str
    B: int
    H: int
    D: int
    N: int
    W: int
    dtype: int            # F32 or BF16 (storage type of Q/K/V)
    mul: float            # every tensor is N(0,1) * mul
    seed: int
    peaky_mod: int = 0    # >0: one history key row in peaky_mod is scaled by peaky_factor
    peaky_factor: float = 1.0

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.D))

    def flops_history(self) -> float:
        return 4.0 * self.B * self.H * self.W * self.N * self.D

    def flops_window(self) -> float:
        return 4.0 * self.B * self.H * self.D * self.W * (self.W + 1) / 2.0


_BASE_SEED = 204070


def config(idx: int) -> Workload:
    """The four fixed workloads (0-based index) of the benchmark definition."""
    if idx == 0:
        return Workload("cfg1_f32_N1024_W64", 1, 1, 64, 1024, 64, F32, 0.5, _BASE_SEED + 1)
    if idx == 1:
        return Workload("cfg2_bf16_N8192_W128", 2, 8, 64, 8192, 128, BF16, 1.0 / 8.0, _BASE_SEED + 2)
    if idx == 2:
        return Workload("cfg3_bf16_N32768_W256_peaky", 4, 16, 128, 32768, 256, BF16, 1.0,
                        _BASE_SEED + 3, peaky_mod=100, peaky_factor=8.0)
    if idx == 3:
        return Workload("cfg4_bf16_N131072_W512", 1, 32, 128, 131072, 512, BF16, 1.0, _BASE_SEED + 4)
    raise ValueError("config index must be 0..3")


def sweep_point(N: int, W: int) -> Workload:
    """A point of the latency-vs-N sweep (batch 1, 32 heads, head dim 128, bf16)."""
    return Workload(f"sweep_bf16_N{N}_W{W}", 1, 32, 128, N, W, BF16, 1.0,
                    _BASE_SEED + 5 + 7919 * N + 104729 * W)


def sweep_points():
    pts = [sweep_point(N, W) for W in (64, 512) for N in (4096, 16384, 65536, 262144)]
    return pts


def decode_point(N: int, W: int = 1) -> Workload:
    """Cache-hit step (Section 4.2): only the newest W rows (1 in the paper) query an N-row history."""
    return Workload(f"decode_bf16_N{N}_W{W}", 1, 32, 128, N, W, BF16, 1.0,
                    _BASE_SEED + 6 + 7919 * N + 104729 * W)


def restore_point(n_queries: int, w_oh: int = 256) -> Workload:
    """Last layer of the context path (Section 3, restoration of the sequence length): every
    history row queries the w_oh compressed rows.  In Workload terms W = n_queries query rows
    and N = w_oh key/value rows."""
    return Workload(f"restore_bf16_Q{n_queries}_K{w_oh}", 1, 32, 128, w_oh, n_queries, BF16, 1.0,
                    _BASE_SEED + 7 + 7919 * w_oh + 104729 * n_queries)


def paper_model_point(N: int, W: int = 256) -> Workload:
    """The attention shape of the paper's own model (Section 6.2: width 432 in 12 heads, so head
    dimension 36; windows of 256 rows, Section 5.1) over an N-row history."""
    return Workload(f"paper_bf16_H12_D36_N{N}_W{W}", 1, 12, 36, N, W, BF16, 1.0,
                    _BASE_SEED + 8 + 7919 * N + 104729 * W)


def f32_point(N: int, W: int = 512) -> Workload:
    """cfg4's shape with fp32 inputs (the precision of the paper's runs is not stated): what the
    fp32 kernel sustains on a workload large enough to fill the chip."""
    return Workload(f"f32_N{N}_W{W}", 1, 32, 128, N, W, F32, 1.0, _BASE_SEED + 9 + 7919 * N + 104729 * W)


def degenerate_causal() -> Workload:
    """Empty history, window of 4096 rows: the layer reduces to standard causal attention."""
    return sweep_point(0, 4096)


def shrink(w: Workload, **kw) -> Workload:
    """The workload with some fields changed; unless a name is given, the new one says which."""
    if kw and "name" not in kw:
        kw["name"] = w.name + "_changed_" + "_".join(f"{k}{v}" for k, v in sorted(kw.items()))
    return replace(w, **kw)


def normal(shape, dtype: int, seed: int, tag: int, mul: float = 1.0,
           peaky_mod: int = 0, peaky_factor: float = 1.0) -> np.ndarray:
    """Array of the given shape: float32 for F32, uint16 holding bf16 bit patterns for BF16.

    The last axis is the row length used by the peaky-row rule.
    """
    shape = tuple(int(s) for s in shape)
    n = int(np.prod(shape)) if shape else 1
    out = np.empty(shape, dtype=np.float32 if dtype == F32 else np.uint16)
    if n == 0:
        return out
    rc = _load().tlin_gen_normal(out.ctypes.data, dtype, seed, tag, n, mul,
                                 shape[-1], peaky_mod, peaky_factor)
    if rc != 0:
        raise RuntimeError("tlin_gen_normal failed")
    return out


def make(w: Workload, which=("Q", "Kh", "Vh", "Kw", "Vw")) -> dict:
    """Host arrays of workload ``w`` in dense [B,H,rows,D] layout."""
    out = {}
    for name, tag, rows in (("Q", TAG_Q, w.W), ("Kh", TAG_KH, w.N), ("Vh", TAG_VH, w.N),
                            ("Kw", TAG_KW, w.W), ("Vw", TAG_VW, w.W)):
        if name not in which:
            continue
        peaky = (w.peaky_mod, w.peaky_factor) if name == "Kh" else (0, 1.0)
        out[name] = normal((w.B, w.H, rows, w.D), w.dtype, w.seed, tag, w.mul, *peaky)
    return out


def bf16_bits_to_f32(a: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to float32."""
    return (a.astype(np.uint32) << 16).view(np.float32)


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even narrowing of float32 to bf16 bit patterns (finite inputs)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


def to_f64(a: np.ndarray, dtype: int) -> np.ndarray:
    return (a if dtype == F32 else bf16_bits_to_f32(a)).astype(np.float64)
