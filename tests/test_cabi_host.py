"""Host-only checks of the C-ABI library: it loads without a GPU, exports every symbol the
header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

from paper_2508_20407_amd import binding as b

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

pytestmark = pytest.mark.skipif(not os.path.exists(b.LIB_PATH), reason="libtlinattn.so not built")


def header_symbols():
    syms = set()
    for name in sorted(os.listdir(os.path.join(ROOT, "include"))):
        if not name.endswith(".h"):
            continue
        text = open(os.path.join(ROOT, "include", name)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        syms |= set(re.findall(r"\b(tlin_[a-z_]+)\s*\(", text))
    return sorted(syms)


def test_library_exports_every_declared_symbol():
    syms = header_symbols()
    assert set(syms) == set(b.EXPORTS)
    L = b.lib()
    for s in syms:
        assert getattr(L, s) is not None


def test_version_and_status_strings():
    assert b.version() >= 100
    seen = {b.status_string(i) for i in range(5)}
    assert len(seen) == 5 and b.status_string(0) == "ok"
    assert b.status_string(99) == "unknown status"


def test_params_struct_matches_header_layout():
    # 10 four-byte fields, then six int64[3] arrays aligned to 8
    assert ctypes.sizeof(b.TlinParams) == 40 + 6 * 24
    assert b.TlinParams.q_stride.offset == 40 and b.TlinParams.o_stride.offset == 40 + 5 * 24


def P(**kw):
    d = dict(B=1, H=2, W=64, N=1024, D=64, in_dtype=b.TLIN_BF16, out_dtype=b.TLIN_BF16, scale=0.125)
    d.update(kw)
    return b.make_params(**d)


def test_workspace_and_split_planning_is_pure_host_arithmetic():
    p = P(B=1, H=32, W=512, N=131072, D=128)
    s = b.num_splits(p)
    assert s >= 1
    need = b.workspace_bytes(p)
    rows = 32 * (s + 1) * 512
    assert need == rows * 128 * 4 + 2 * rows * 4
    assert b.num_splits(P(num_splits=4)) == 4
    assert b.num_splits(P(num_splits=5)) == 4      # 16 tiles: 4 per partition, none empty
    assert b.num_splits(P(num_splits=10 ** 6)) == 1024 // 64   # one 64-key tile per partition at most
    assert b.num_splits(P(N=1)) == 1
    assert b.workspace_bytes(P(W=0)) == 0 and b.num_splits(P(D=30)) == 0


A = 1 << 20   # a fake, suitably aligned device address: validation must fail before it is used


@pytest.mark.parametrize("kw,status", [
    (dict(B=0), b.TLIN_ERR_INVALID_ARG), (dict(H=-1), b.TLIN_ERR_INVALID_ARG), (dict(W=0), b.TLIN_ERR_INVALID_ARG),
    (dict(N=0), b.TLIN_ERR_INVALID_ARG), (dict(D=30), b.TLIN_ERR_UNSUPPORTED), (dict(D=256), b.TLIN_ERR_UNSUPPORTED), (dict(D=0), b.TLIN_ERR_UNSUPPORTED), (dict(D=4), b.TLIN_ERR_UNSUPPORTED),
    (dict(D=36), b.TLIN_ERR_INVALID_ARG),                                      # dense bf16 rows of 72 bytes
    (dict(in_dtype=7), b.TLIN_ERR_INVALID_ARG), (dict(out_dtype=-1), b.TLIN_ERR_INVALID_ARG),
    (dict(scale=0.0), b.TLIN_ERR_INVALID_ARG), (dict(scale=float("nan")), b.TLIN_ERR_INVALID_ARG),
    (dict(scale=float("inf")), b.TLIN_ERR_INVALID_ARG), (dict(num_splits=-2), b.TLIN_ERR_INVALID_ARG),
    (dict(N=(1 << 30) + 1), b.TLIN_ERR_INVALID_ARG), (dict(W=(1 << 30) + 64), b.TLIN_ERR_INVALID_ARG),   # beyond 32-bit tile arithmetic
    (dict(kh_stride=(0, 0, 1 << 24)), b.TLIN_ERR_INVALID_ARG),                 # row stride of 32 MiB
    (dict(q_stride=(64 * 64 * 2, 64 * 64, 60)), b.TLIN_ERR_INVALID_ARG),       # row stride < D
    (dict(kh_stride=(1024 * 68 * 2, 1024 * 68, 68)), b.TLIN_ERR_INVALID_ARG),  # rows not 16-byte aligned
])
def test_history_rejects_bad_params(kw, status):
    assert b.history_attn_raw(P(**kw), A, A, A, A, None, A, 1 << 30, None) == status


def test_other_head_dimensions_run_in_the_next_native_size():
    # rows padded to whole 16-byte pieces are accepted; the workspace is sized for the kernel's 64 / 128 columns
    st40 = lambda rows: (2 * rows * 40, rows * 40, 40)
    p36 = P(D=36, q_stride=st40(64), kh_stride=st40(1024), vh_stride=st40(1024), kw_stride=st40(64), vw_stride=st40(64),
            o_stride=st40(64))
    assert b.num_splits(p36) == b.num_splits(P()) and b.workspace_bytes(p36) == b.workspace_bytes(P())
    p96 = P(D=96)
    assert b.workspace_bytes(p96) == b.workspace_bytes(P(D=128))
    # fp32 rows of 36 floats are whole pieces already
    assert b.num_splits(P(D=36, in_dtype=b.TLIN_F32, out_dtype=b.TLIN_F32)) >= 1
    # a row stride that cannot hold the last piece
    bad = P(D=36, q_stride=(2 * 64 * 36, 64 * 36, 36))
    assert b.history_attn_raw(bad, A, A, A, A, None, A, 1 << 30, None) == b.TLIN_ERR_INVALID_ARG


def test_null_and_misaligned_pointers_and_workspace():
    p = P()
    assert b.num_splits(p) > 1
    big = 1 << 30
    assert b.history_attn_raw(p, None, A, A, A, None, A, big, None) == b.TLIN_ERR_INVALID_ARG
    assert b.history_attn_raw(p, A, A, None, A, None, A, big, None) == b.TLIN_ERR_INVALID_ARG
    assert b.history_attn_raw(p, A, A, A, None, None, A, big, None) == b.TLIN_ERR_INVALID_ARG
    assert b.history_attn_raw(p, A + 2, A, A, A, None, A, big, None) == b.TLIN_ERR_INVALID_ARG
    assert b.history_attn_raw(p, A, A, A, A, None, None, 0, None) == b.TLIN_ERR_WORKSPACE
    assert b.history_attn_raw(p, A, A, A, A, None, A, 16, None) == b.TLIN_ERR_WORKSPACE
    assert b.history_attn_raw(p, A, A, A, A, None, A + 16, big, None) == b.TLIN_ERR_WORKSPACE
    assert b.window_causal_attn_raw(p, A, None, A, A, None, None, 0, None) == b.TLIN_ERR_INVALID_ARG
    assert b.layer_attn_raw(p, A, A, A, A, A, A, None, 0, None) == b.TLIN_ERR_WORKSPACE
    assert b.layer_attn_raw(p, A, None, A, A, A, A, A, big, None) == b.TLIN_ERR_INVALID_ARG
    assert b.layer_attn_raw(P(combine=3), A, A, A, A, A, A, A, big, None) == b.TLIN_ERR_INVALID_ARG
    assert b.layer_attn_raw(P(N=-1), A, A, A, A, A, A, A, big, None) == b.TLIN_ERR_INVALID_ARG


def test_static_workspace_entry_point_checks_arguments_and_its_limit_on_the_host():
    p = P()
    assert b.layer_attn_static_ws_raw(p, None, A, A, A, A, A, None) == b.TLIN_ERR_INVALID_ARG
    assert b.layer_attn_static_ws_raw(P(combine=3), A, A, A, A, A, A, None) == b.TLIN_ERR_INVALID_ARG
    assert b.layer_attn_static_ws_raw(P(W=0), A, A, A, A, A, A, None) == b.TLIN_ERR_INVALID_ARG
    # a workspace need beyond the array's size is refused before any device call
    big = P(B=4, H=32, W=512, N=131072, D=128)
    assert b.workspace_bytes(big) > b.STATIC_WS_BYTES
    assert b.layer_attn_static_ws_raw(big, A, A, A, A, A, A, None) == b.TLIN_ERR_WORKSPACE
    # the largest fixed workload fits
    assert b.workspace_bytes(P(B=1, H=32, W=512, N=131072, D=128)) <= b.STATIC_WS_BYTES
    text = open(os.path.join(ROOT, "include", "tlinattn.h")).read()
    assert "#define TLIN_STATIC_WS_BYTES ((size_t)64 << 20)" in text and b.STATIC_WS_BYTES == 64 << 20


def test_slide_planning_and_argument_checks():
    # 256 chunks of 512 rows, 32 heads: plenty of work items, so one partition per chunk history
    # plus the window partial = 2 fp32 partial slots per output row
    p = P(B=1, H=32, W=512, N=131072, D=128)
    rows = 32 * 256 * 2 * 512
    assert b.slide_workspace_bytes(p) == rows * 128 * 4 + 2 * rows * 4
    # a short sequence is split further; the ragged last chunk still gets whole slots
    small = P(B=1, H=1, W=128, N=1000, D=64)
    need = b.slide_workspace_bytes(small)
    per_slot = 128 * 64 * 4 + 2 * 128 * 4
    assert need % (8 * per_slot) == 0 and need // (8 * per_slot) >= 2
    forced = P(B=1, H=1, W=128, N=1000, D=64, num_splits=3)
    assert b.slide_workspace_bytes(forced) == 8 * 4 * per_slot
    assert b.slide_workspace_bytes(P(N=0)) == 0 and b.slide_workspace_bytes(P(D=130)) == 0
    big = 1 << 40
    assert b.slide_layer_attn_raw(P(N=0), A, A, A, A, A, A, A, big, None) == b.TLIN_ERR_INVALID_ARG
    assert b.slide_layer_attn_raw(P(combine=2), A, A, A, A, A, A, A, big, None) == b.TLIN_ERR_INVALID_ARG
    assert b.slide_layer_attn_raw(p, A, A, None, A, A, A, A, big, None) == b.TLIN_ERR_INVALID_ARG
    assert b.slide_layer_attn_raw(p, A, A, A, A, A + 4, A, A, big, None) == b.TLIN_ERR_INVALID_ARG
    assert b.slide_layer_attn_raw(p, A, A, A, A, A, A, None, 0, None) == b.TLIN_ERR_WORKSPACE
    assert b.slide_layer_attn_raw(p, A, A, A, A, A, A, A, 1 << 20, None) == b.TLIN_ERR_WORKSPACE


def test_binding_fails_loudly_when_library_is_missing(monkeypatch):
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "LIB_PATH", "/nonexistent/libtlinattn.so")
    with pytest.raises(ImportError, match="no fallback"):
        b.lib()
