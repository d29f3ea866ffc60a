"""TLinFormer window-over-history attention for MI355X: Python face of libtlinattn.

``tlin_history_attn``, ``tlin_window_causal_attn`` and ``tlin_layer_attn`` take torch tensors
that live on the GPU ([B,H,rows,D], last axis contiguous), marshal their addresses and strides
into the C-ABI call of the same name and return the output tensor.  All arithmetic happens in
the library's HIP kernels.
"""
from __future__ import annotations

from . import binding
from .binding import (TLIN_BF16, TLIN_COMBINE_JOINT, TLIN_COMBINE_SUM, TLIN_F32, TlinError, TlinParams)

__all__ = ["tlin_history_attn", "tlin_window_causal_attn", "tlin_layer_attn", "tlin_layer_attn_static_ws", "tlin_slide_layer_attn", "Workspace", "params_for",
           "TLIN_F32", "TLIN_BF16", "TLIN_COMBINE_SUM", "TLIN_COMBINE_JOINT", "TlinError", "TlinParams",
           "binding"]


def _torch():
    import torch
    return torch


def _dtype_code(t):
    torch = _torch()
    if t.dtype == torch.float32:
        return TLIN_F32
    if t.dtype == torch.bfloat16:
        return TLIN_BF16
    raise TypeError(f"unsupported dtype {t.dtype}: float32 or bfloat16 expected")


def _strides(t):
    if t.dim() != 4 or t.stride(3) != 1:
        raise ValueError("expected a [B,H,rows,D] tensor whose last axis is contiguous")
    return (t.stride(0), t.stride(1), t.stride(2))


def _require_gpu(*ts):
    for t in ts:
        if t is not None and not t.is_cuda:
            raise ValueError("libtlinattn takes device tensors only")


def params_for(q, n_hist, out_dtype=None, scale=None, num_splits=0, combine=TLIN_COMBINE_SUM,
               kh=None, vh=None, kw=None, vw=None, o=None) -> TlinParams:
    B, H, W, D = q.shape
    code = _dtype_code(q)
    oc = code if out_dtype is None else (TLIN_F32 if out_dtype == _torch().float32 else TLIN_BF16)
    st = {"q_stride": _strides(q)}
    for name, t in (("kh_stride", kh), ("vh_stride", vh), ("kw_stride", kw), ("vw_stride", vw), ("o_stride", o)):
        if t is not None:
            st[name] = _strides(t)
    return binding.make_params(B, H, W, n_hist, D, code, oc, (D ** -0.5) if scale is None else scale,
                               num_splits, combine, **st)


class Workspace:
    """Caller-owned device scratch for split partials, grown on demand and reused."""

    def __init__(self):
        self.buf = None

    def get(self, nbytes: int, device):
        """(256-byte aligned address, bytes) of a region of at least nbytes inside the buffer."""
        torch = _torch()
        if nbytes == 0:
            return 0, 0
        if self.buf is not None and self.buf.device == device:
            addr = (self.buf.data_ptr() + 255) // 256 * 256
            if self.buf.data_ptr() + self.buf.numel() - addr >= nbytes:      # capacity behind the aligned address
                return addr, nbytes
        self.buf = torch.empty(nbytes + 256, dtype=torch.uint8, device=device)
        return (self.buf.data_ptr() + 255) // 256 * 256, nbytes


# Calls that share a workspace must be ordered on one stream, so the workspaces the wrappers
# fall back to are kept per (device, stream).
_default_ws = {}


def _workspace_for(t, workspace):
    if workspace is not None:
        return workspace
    key = (t.device, _stream(t))
    ws = _default_ws.get(key)
    if ws is None:
        ws = _default_ws[key] = Workspace()
    return ws


def _stream(t):
    return _torch().cuda.current_stream(t.device).cuda_stream


def _out(q, out_dtype):
    """Output tensor [B,H,rows,D]; its rows are padded to whole 16-byte pieces when D is not."""
    torch = _torch()
    dt = q.dtype if out_dtype is None else out_dtype
    per16 = 16 // torch.empty((), dtype=dt).element_size()
    B, H, R, D = q.shape
    row = (D + per16 - 1) // per16 * per16
    return torch.empty((B, H, R, row), dtype=dt, device=q.device)[..., :D]


def tlin_history_attn(q_win, k_hist, v_hist, *, scale=None, out_dtype=None, num_splits=0, return_lse=False,
                      workspace: Workspace | None = None):
    """softmax(scale * Q_win K_hist^T) V_hist, no mask.  Returns O, or (O, lse) with return_lse."""
    _require_gpu(q_win, k_hist, v_hist)
    torch = _torch()
    o = _out(q_win, out_dtype)
    p = params_for(q_win, k_hist.shape[2], o.dtype, scale, num_splits, kh=k_hist, vh=v_hist, o=o)
    lse = torch.empty(q_win.shape[:3], dtype=torch.float32, device=q_win.device) if return_lse else None
    ws, nb = _workspace_for(q_win, workspace).get(binding.workspace_bytes(p), q_win.device)
    st = binding.history_attn_raw(p, q_win.data_ptr(), k_hist.data_ptr(), v_hist.data_ptr(), o.data_ptr(),
                                  lse.data_ptr() if return_lse else None, ws or None, nb, _stream(q_win))
    binding._check(st, "tlin_history_attn")
    return (o, lse) if return_lse else o


def tlin_window_causal_attn(q_win, k_win, v_win, *, scale=None, out_dtype=None, return_lse=False):
    """Causal attention inside the window (query i sees keys j <= i)."""
    _require_gpu(q_win, k_win, v_win)
    torch = _torch()
    o = _out(q_win, out_dtype)
    p = params_for(q_win, 0, o.dtype, scale, kw=k_win, vw=v_win, o=o)
    lse = torch.empty(q_win.shape[:3], dtype=torch.float32, device=q_win.device) if return_lse else None
    st = binding.window_causal_attn_raw(p, q_win.data_ptr(), k_win.data_ptr(), v_win.data_ptr(), o.data_ptr(),
                                        lse.data_ptr() if return_lse else None, None, 0, _stream(q_win))
    binding._check(st, "tlin_window_causal_attn")
    return (o, lse) if return_lse else o


def tlin_layer_attn(q_win, k_hist, v_hist, k_win, v_win, *, combine=TLIN_COMBINE_SUM, scale=None, out_dtype=None,
                    num_splits=0, workspace: Workspace | None = None):
    """History attention and window causal attention of the same rows, combined."""
    _require_gpu(q_win, k_hist, v_hist, k_win, v_win)
    n = 0 if k_hist is None else k_hist.shape[2]
    o = _out(q_win, out_dtype)
    p = params_for(q_win, n, o.dtype, scale, num_splits, combine,
                   kh=k_hist if n else None, vh=v_hist if n else None, kw=k_win, vw=v_win, o=o)
    ws, nb = _workspace_for(q_win, workspace).get(binding.workspace_bytes(p), q_win.device)
    st = binding.layer_attn_raw(p, q_win.data_ptr(), k_hist.data_ptr() if n else None,
                                v_hist.data_ptr() if n else None, k_win.data_ptr(), v_win.data_ptr(),
                                o.data_ptr(), ws or None, nb, _stream(q_win))
    binding._check(st, "tlin_layer_attn")
    return o


def tlin_layer_attn_static_ws(q_win, k_hist, v_hist, k_win, v_win, *, combine=TLIN_COMBINE_SUM, scale=None, out=None,
                              num_splits=0):
    """tlin_layer_attn with the library's own static device array as workspace.  With `out` (a
    [B,H,W,D] tensor of the wanted output type) the call allocates nothing at all."""
    _require_gpu(q_win, k_hist, v_hist, k_win, v_win, out)
    n = 0 if k_hist is None else k_hist.shape[2]
    o = _out(q_win, None) if out is None else out
    if tuple(o.shape) != tuple(q_win.shape):
        raise ValueError("out must have the shape of q_win")
    p = params_for(q_win, n, o.dtype, scale, num_splits, combine,
                   kh=k_hist if n else None, vh=v_hist if n else None, kw=k_win, vw=v_win, o=o)
    st = binding.layer_attn_static_ws_raw(p, q_win.data_ptr(), k_hist.data_ptr() if n else None,
                                          v_hist.data_ptr() if n else None, k_win.data_ptr(), v_win.data_ptr(),
                                          o.data_ptr(), _stream(q_win))
    binding._check(st, "tlin_layer_attn_static_ws")
    return o


def tlin_slide_layer_attn(q, k_hist, v_hist, k_win, v_win, chunk, *, combine=TLIN_COMBINE_SUM, scale=None,
                          out_dtype=None, num_splits=0, workspace: Workspace | None = None):
    """tlin_layer_attn for every chunk of `chunk` rows of a whole sequence [B,H,L,D] at once;
    the history of a chunk is every earlier chunk (k_hist/v_hist rows before it)."""
    _require_gpu(q, k_hist, v_hist, k_win, v_win)
    B, H, L, D = q.shape
    for t in (k_hist, v_hist, k_win, v_win):
        if tuple(t.shape) != (B, H, L, D):
            raise ValueError("all tensors of the sliding schedule are [B,H,L,D]")
    o = _out(q, out_dtype)
    code = _dtype_code(q)
    oc = TLIN_F32 if o.dtype == _torch().float32 else TLIN_BF16
    p = binding.make_params(B, H, int(chunk), L, D, code, oc, (D ** -0.5) if scale is None else scale, num_splits,
                            combine, q_stride=_strides(q), kh_stride=_strides(k_hist), vh_stride=_strides(v_hist),
                            kw_stride=_strides(k_win), vw_stride=_strides(v_win), o_stride=_strides(o))
    ws, nb = _workspace_for(q, workspace).get(binding.slide_workspace_bytes(p), q.device)
    st = binding.slide_layer_attn_raw(p, q.data_ptr(), k_hist.data_ptr(), v_hist.data_ptr(), k_win.data_ptr(),
                                      v_win.data_ptr(), o.data_ptr(), ws or None, nb, _stream(q))
    binding._check(st, "tlin_slide_layer_attn")
    return o
