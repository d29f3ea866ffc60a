"""The layer call that takes its workspace from the library's static device array, through the
C-ABI, against the ordinary layer call (same kernels: bit for bit) and against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import tlin_inputs as ti
import paper_2508_20407_amd as tl
from paper_2508_20407_amd import binding
from helpers import assert_close, upload

pytestmark = pytest.mark.gpu
NAMES = ("Q", "Kh", "Vh", "Kw", "Vw")


def call_pair(w, mode):
    host = ti.make(w)
    dev = upload(host, w.dtype)
    want = tl.tlin_layer_attn(*(dev[k] for k in NAMES), combine=mode, scale=w.scale)
    out = torch.full_like(want, float("nan"))
    before = torch.cuda.memory_allocated()
    got = tl.tlin_layer_attn_static_ws(*(dev[k] for k in NAMES), combine=mode, scale=w.scale, out=out)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    assert got.data_ptr() == out.data_ptr()
    assert torch.equal(got, want), f"{w.name}: static-workspace call differs from tlin_layer_attn"
    omode = oracle.SUM if mode == tl.TLIN_COMBINE_SUM else oracle.JOINT
    ro = oracle.layer(*(host[k] for k in NAMES), w.dtype, w.scale, omode)
    assert_close(got, ro, w.dtype, w.name)


@pytest.mark.parametrize("dtype", [ti.BF16, ti.F32])
def test_two_calls_in_a_row_the_second_smaller(dtype):
    """The array keeps the first call's partials; the second, smaller call (fewer rows, fewer
    partitions) must not see them."""
    big = ti.Workload(f"static_ws_big_{dtype}", 2, 6, 128, 9000 + 41, 300, dtype, 1.0, 5501)
    small = ti.Workload(f"static_ws_small_{dtype}", 1, 3, 128, 700, 70, dtype, 1.0, 5502)
    assert binding.num_splits(binding.make_params(big.B, big.H, big.W, big.N, big.D, 1, 1, big.scale)) > 1
    for mode in (tl.TLIN_COMBINE_SUM, tl.TLIN_COMBINE_JOINT):
        call_pair(big, mode)
        call_pair(small, mode)


def test_empty_history_and_the_size_limit():
    w = ti.Workload("static_ws_empty", 1, 4, 64, 0, 200, ti.BF16, 1.0, 5503)
    host = ti.make(w, which=("Q", "Kw", "Vw"))
    dev = upload(host, w.dtype)
    got = tl.tlin_layer_attn_static_ws(dev["Q"], None, None, dev["Kw"], dev["Vw"], scale=w.scale)
    want = tl.tlin_window_causal_attn(dev["Q"], dev["Kw"], dev["Vw"], scale=w.scale)
    assert torch.equal(got, want)
    # beyond the array: refused with the workspace status, nothing launched
    B, H, W, N, D = 4, 32, 512, 131072, 128
    p = binding.make_params(B, H, W, N, D, binding.TLIN_BF16, binding.TLIN_BF16, D ** -0.5)
    assert binding.workspace_bytes(p) > binding.STATIC_WS_BYTES
    a = dev["Q"].data_ptr()
    assert binding.layer_attn_static_ws_raw(p, a, a, a, a, a, a, None) == binding.TLIN_ERR_WORKSPACE
