"""GPU parity: libtlinattn (through its C-ABI) against the CPU fp64 oracle, element by element,
on identical seeded inputs."""
import numpy as np
import pytest
import torch

import oracle
import tlin_inputs as ti
import paper_2508_20407_amd as tl
from helpers import assert_close, f32_rel_bound, sample_rows, stratified_rows, to_host64, upload

pytestmark = pytest.mark.gpu

TDT = {ti.F32: torch.float32, ti.BF16: torch.bfloat16}


def lse_atol(dtype, rl):
    """fp32 path: rounding of an fp32 log-sum-exp.  bf16 path: the row sum is accumulated from
    the bf16-rounded weights (the values the value product uses), each within 2^-8 relative of
    the exact weight (bf16 keeps 8 significant bits), so the sum is within 2^-8 relative and
    its log within 2^-8 = 3.9e-3 absolute."""
    return (2e-4 if dtype == ti.F32 else 4.5e-3) * max(1.0, float(np.abs(rl).max()) if dtype == ti.F32 else 1.0)


def run_all(w: ti.Workload, rows=None, num_splits=0, check_lse=True, tag=""):
    """History, window, and both layer modes of one workload against the oracle."""
    host = ti.make(w)
    dev = upload(host, w.dtype)
    Q, Kh, Vh, Kw, Vw = (dev[k] for k in ("Q", "Kh", "Vh", "Kw", "Vw"))
    sel = (lambda t: t) if rows is None else (lambda t: t[:, :, torch.from_numpy(rows).long().cuda()])
    name = f"{w.name}{tag}"
    if w.N > 0:
        o, lse = tl.tlin_history_attn(Q, Kh, Vh, scale=w.scale, num_splits=num_splits, return_lse=True)
        ro, rl = oracle.history(host["Q"], host["Kh"], host["Vh"], w.dtype, w.scale, rows)
        assert_close(sel(o), ro, w.dtype, f"{name} history")
        if check_lse:
            np.testing.assert_allclose(to_host64(sel(lse.unsqueeze(-1)))[..., 0], rl, rtol=1e-6, atol=lse_atol(w.dtype, rl))
    o, lse = tl.tlin_window_causal_attn(Q, Kw, Vw, scale=w.scale, return_lse=True)
    ro, rl = oracle.window_causal(host["Q"], host["Kw"], host["Vw"], w.dtype, w.scale, rows)
    assert_close(sel(o), ro, w.dtype, f"{name} window")
    if check_lse:
        np.testing.assert_allclose(to_host64(sel(lse.unsqueeze(-1)))[..., 0], rl, rtol=1e-6, atol=lse_atol(w.dtype, rl))
    for mode, omode in ((tl.TLIN_COMBINE_SUM, oracle.SUM), (tl.TLIN_COMBINE_JOINT, oracle.JOINT)):
        o = tl.tlin_layer_attn(Q, Kh if w.N else None, Vh if w.N else None, Kw, Vw, combine=mode, scale=w.scale,
                               num_splits=num_splits)
        ro = oracle.layer(host["Q"], host["Kh"] if w.N else None, host["Vh"] if w.N else None, host["Kw"],
                          host["Vw"], w.dtype, w.scale, omode, rows)
        assert_close(sel(o), ro, w.dtype, f"{name} layer mode {mode}")


# ---------------------------------------------------------------- the fixed workloads
def test_config1_f32_full():
    run_all(ti.config(0))


def test_config2_bf16_full():
    run_all(ti.config(1))


def test_config3_peaky_reduced_full_compare():
    # several key tiles and partitions, ragged tail in N, every row compared
    run_all(ti.shrink(ti.config(2), B=1, H=2, N=4096 + 37))


def test_config3_peaky_full_size_stratified_rows():
    """Full size, in the launch configuration the bench times; first and last row of every
    32-row wave block of every query block of every head."""
    w = ti.config(2)
    run_all(w, rows=stratified_rows(w.W))


def test_config4_full_size_stratified_rows():
    w = ti.config(3)
    run_all(w, rows=stratified_rows(w.W))


@pytest.mark.parametrize("W", [64, 512])
@pytest.mark.parametrize("N", [4096, 16384, 65536, 262144])
def test_sweep_points_full_size_stratified_rows(N, W):
    """Every point of the latency-vs-N sweep (Section 4.1, equations (1)-(4): cost linear in N at
    fixed window), full size, history / window / both layer modes."""
    w = ti.sweep_point(N, W)
    run_all(w, rows=stratified_rows(W))


def test_degenerate_empty_history_is_standard_causal_attention():
    """N_hist = 0, W = 4096: the layer, in both modes, is plain causal attention of length W."""
    w = ti.degenerate_causal()
    host = ti.make(w, which=("Q", "Kw", "Vw"))
    dev = upload(host, w.dtype)
    rows = sample_rows(w.W, 48, seed=5)
    ro, _ = oracle.window_causal(host["Q"], host["Kw"], host["Vw"], w.dtype, w.scale, rows)
    idx = torch.from_numpy(rows).long().cuda()
    o_win = tl.tlin_window_causal_attn(dev["Q"], dev["Kw"], dev["Vw"], scale=w.scale)
    assert_close(o_win[:, :, idx], ro, w.dtype, "window W=4096")
    for mode in (tl.TLIN_COMBINE_SUM, tl.TLIN_COMBINE_JOINT):
        o = tl.tlin_layer_attn(dev["Q"], None, None, dev["Kw"], dev["Vw"], combine=mode, scale=w.scale)
        assert torch.equal(o, o_win)


# ---------------------------------------------------------------- cache-hit and restoration shapes
@pytest.mark.parametrize("W", [1, 2, 4, 8])
def test_decode_shape_full_size_every_row(W):
    """Cache-hit step (Section 4.2): the newest rows against the whole history, in the launch
    configuration the bench times; also through the layer call with the W newest rows as window."""
    run_all(ti.decode_point(131072, W))


@pytest.mark.parametrize("W", [1, 2, 3, 4])
@pytest.mark.parametrize("N", [1024, 1025, 1039, 4097, 20000, 100003])
def test_streaming_decode_kernel_ragged_every_row(W, N):
    """The cache-hit kernel proper (bf16, head dimension 128, at most four query rows, history of
    1024 rows or more): partition tails of every residue, automatic and forced partition counts,
    values and log-sum-exp of every row."""
    w = ti.Workload(f"stream_decode_{W}_{N}", 2, 5, 128, N, W, ti.BF16, 1.0, 60601 + 31 * W + N)
    host = ti.make(w, which=("Q", "Kh", "Vh"))
    dev = upload(host, w.dtype)
    ro, rl = oracle.history(host["Q"], host["Kh"], host["Vh"], w.dtype, w.scale)
    for s in (0, 1, 3, 16):
        o, lse = tl.tlin_history_attn(dev["Q"], dev["Kh"], dev["Vh"], scale=w.scale, num_splits=s, return_lse=True)
        assert_close(o, ro, w.dtype, f"{w.name} splits {s}")
        np.testing.assert_allclose(to_host64(lse), rl, rtol=1e-6, atol=lse_atol(w.dtype, rl))
    o32 = tl.tlin_history_attn(dev["Q"], dev["Kh"], dev["Vh"], scale=w.scale, out_dtype=torch.float32)
    assert_close(o32, ro, w.dtype, f"{w.name} f32 out")


@pytest.mark.parametrize("dtype,D", [(ti.BF16, 64), (ti.F32, 128), (ti.F32, 64), (ti.BF16, 36), (ti.BF16, 100),
                                     (ti.F32, 36), (ti.F32, 100), (ti.BF16, 8), (ti.F32, 12)])
@pytest.mark.parametrize("W", [1, 2, 3, 4, 5, 8])
@pytest.mark.parametrize("N", [1025, 1039, 4097, 20011])
def test_cache_hit_shapes_dtypes_and_head_dimensions(dtype, D, W, N):
    """Few query rows over histories of 1024 rows and more, for fp32 inputs (the streaming kernel
    with fp32 arithmetic, up to eight rows) and for every kind of head dimension the library takes
    (native sizes and sizes in between, with NaNs in the rows' padding); automatic and forced
    partition counts."""
    w = ti.Workload(f"stream_decode_{dtype}_{D}_{W}_{N}", 2, 3, D, N, W, dtype, 1.0, 70701 + 131 * D + 31 * W + N)
    host = ti.make(w, which=("Q", "Kh", "Vh"))
    dev = {k: padded(v, w.dtype) for k, v in host.items()}
    ro, rl = oracle.history(host["Q"], host["Kh"], host["Vh"], w.dtype, w.scale)
    for s in (0, 1, 5):
        o, lse = tl.tlin_history_attn(dev["Q"], dev["Kh"], dev["Vh"], scale=w.scale, num_splits=s, return_lse=True)
        assert o.shape[-1] == D
        assert_close(o, ro, w.dtype, f"{w.name} splits {s}")
        np.testing.assert_allclose(to_host64(lse), rl, rtol=1e-6, atol=lse_atol(w.dtype, rl))


@pytest.mark.parametrize("dtype,D", [(ti.F32, 128), (ti.BF16, 64), (ti.BF16, 36)])
def test_streaming_decode_kernel_full_size_other_shapes(dtype, D):
    """One query row over 131072 history rows of 32 heads, fp32 inputs and smaller head dimensions:
    the launch configuration the bench times for these shapes."""
    w = ti.Workload(f"stream_decode_full_{dtype}_{D}", 1, 32, D, 131072, 1, dtype, 1.0, 80801 + D + dtype)
    host = ti.make(w, which=("Q", "Kh", "Vh"))
    dev = {k: padded(v, w.dtype) for k, v in host.items()}
    o, lse = tl.tlin_history_attn(dev["Q"], dev["Kh"], dev["Vh"], scale=w.scale, return_lse=True)
    ro, rl = oracle.history(host["Q"], host["Kh"], host["Vh"], w.dtype, w.scale)
    assert_close(o, ro, w.dtype, w.name)
    np.testing.assert_allclose(to_host64(lse), rl, rtol=1e-6, atol=lse_atol(w.dtype, rl))


def test_streaming_decode_kernel_peaky_keys_and_strided_layout():
    """Keys of very different sizes (one row in a hundred eight times larger: the reference point
    of the online softmax moves late and far), on an interleaved-head layout."""
    w = ti.Workload("stream_decode_peaky", 1, 6, 128, 30011, 2, ti.BF16, 1.0, 60707, peaky_mod=100, peaky_factor=8.0)
    host = ti.make(w, which=("Q", "Kh", "Vh"))
    dev = upload(host, w.dtype)

    def interleave(t):
        return t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    Q, Kh, Vh = (interleave(dev[k]) for k in ("Q", "Kh", "Vh"))
    o, lse = tl.tlin_history_attn(Q, Kh, Vh, scale=w.scale, return_lse=True)
    ro, rl = oracle.history(host["Q"], host["Kh"], host["Vh"], w.dtype, w.scale)
    assert_close(o, ro, w.dtype, w.name)
    np.testing.assert_allclose(to_host64(lse), rl, rtol=1e-6, atol=lse_atol(w.dtype, rl))


def test_decode_shape_at_the_papers_maximum_length():
    """Cache-hit step over 2^20 history rows (Section 6.4 runs sequences beyond one million
    tokens), 32 heads of dimension 128: 16 GiB of keys and values, every output row compared; then
    the layer call of a 512-row window over the same history."""
    w = ti.decode_point(1048576, 1)
    host = ti.make(w, which=("Q", "Kh", "Vh"))
    dev = upload(host, w.dtype)
    o, lse = tl.tlin_history_attn(dev["Q"], dev["Kh"], dev["Vh"], scale=w.scale, return_lse=True)
    ro, rl = oracle.history(host["Q"], host["Kh"], host["Vh"], w.dtype, w.scale)
    assert_close(o, ro, w.dtype, w.name)
    np.testing.assert_allclose(to_host64(lse), rl, rtol=1e-6, atol=lse_atol(w.dtype, rl))
    # the cache-miss layer call of a 512-row window over the same history (partitions of 4096 key
    # tiles; the window blocks ride on partition 0), first and last row of every 32-row block
    w2 = ti.Workload("layer_N1048576_W512", w.B, w.H, w.D, w.N, 512, w.dtype, 1.0, w.seed + 1)
    win = ti.make(w2, which=("Q", "Kw", "Vw"))
    dwin = upload(win, w.dtype)
    rows = stratified_rows(512)
    idx = torch.from_numpy(rows).long().cuda()
    for mode, omode in ((tl.TLIN_COMBINE_SUM, oracle.SUM), (tl.TLIN_COMBINE_JOINT, oracle.JOINT)):
        o = tl.tlin_layer_attn(dwin["Q"], dev["Kh"], dev["Vh"], dwin["Kw"], dwin["Vw"], combine=mode, scale=w.scale)
        ro = oracle.layer(win["Q"], host["Kh"], host["Vh"], win["Kw"], win["Vw"], w.dtype, w.scale, omode, rows)
        assert_close(o[:, :, idx], ro, w.dtype, f"{w2.name} mode {mode}")


@pytest.mark.parametrize("dtype", [ti.F32, ti.BF16])
@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("W,N", [(1, 63), (1, 4097), (2, 1000), (3, 129), (5, 8191), (8, 2048)])
def test_decode_shapes_ragged(dtype, D, W, N):
    w = ti.Workload(f"decode_{dtype}_{D}_{W}_{N}", 2, 3, D, N, W, dtype, 1.0, 991 + W * 17 + N)
    run_all(w)


def test_restoration_shape_full_size_sampled_rows():
    """Last layer of the context path (Section 3): every history row queries the W_oh = 256
    compressed rows.  Many query blocks, one partition of four key tiles."""
    w = ti.restore_point(131072, 256)
    host = ti.make(w, which=("Q", "Kh", "Vh"))
    dev = upload(host, w.dtype)
    rows = sample_rows(w.W, 40, seed=11)
    o, lse = tl.tlin_history_attn(dev["Q"], dev["Kh"], dev["Vh"], scale=w.scale, return_lse=True)
    ro, rl = oracle.history(host["Q"], host["Kh"], host["Vh"], w.dtype, w.scale, rows)
    idx = torch.from_numpy(rows).long().cuda()
    assert_close(o[:, :, idx], ro, w.dtype, w.name)
    np.testing.assert_allclose(to_host64(lse[:, :, idx]), rl, rtol=1e-6, atol=lse_atol(w.dtype, rl))


@pytest.mark.parametrize("dtype", [ti.F32, ti.BF16])
@pytest.mark.parametrize("n_queries,w_oh", [(5000, 256), (3001, 200), (1025, 64)])
def test_restoration_shape_reduced_every_row(dtype, n_queries, w_oh):
    w = ti.shrink(ti.restore_point(n_queries, w_oh), H=2, dtype=dtype)
    host = ti.make(w, which=("Q", "Kh", "Vh"))
    dev = upload(host, w.dtype)
    o = tl.tlin_history_attn(dev["Q"], dev["Kh"], dev["Vh"], scale=w.scale)
    ro, _ = oracle.history(host["Q"], host["Kh"], host["Vh"], w.dtype, w.scale, None)
    assert_close(o, ro, w.dtype, w.name)


@pytest.mark.parametrize("D,n_queries,w_oh", [(128, 33017, 256), (128, 32768, 200), (128, 40000, 1), (64, 33017, 512),
                                               (64, 36000, 333), (128, 33001, 128), (128, 34000, 100), (128, 33333, 192),
                                               (100, 33017, 250), (36, 40000, 256)])
def test_restoration_shape_keys_resident_in_lds_every_row(D, n_queries, w_oh):
    """Enough query blocks per compute unit that the library keeps the whole key/value side in
    LDS and lets every workgroup walk over several query blocks; ragged query and key tails."""
    w = ti.shrink(ti.restore_point(n_queries, w_oh), H=8, D=D)
    host = ti.make(w, which=("Q", "Kh", "Vh"))
    dev = upload(host, w.dtype) if D % 8 == 0 else {k: padded(v, w.dtype) for k, v in host.items()}
    o, lse = tl.tlin_history_attn(dev["Q"], dev["Kh"], dev["Vh"], scale=w.scale, return_lse=True)
    ro, rl = oracle.history(host["Q"], host["Kh"], host["Vh"], w.dtype, w.scale, None)
    assert_close(o, ro, w.dtype, w.name)
    np.testing.assert_allclose(to_host64(lse), rl, rtol=1e-6, atol=lse_atol(w.dtype, rl))
    o32 = tl.tlin_history_attn(dev["Q"], dev["Kh"], dev["Vh"], scale=w.scale, out_dtype=torch.float32)
    assert_close(o32, ro, w.dtype, w.name + " f32 out")


# ---------------------------------------------------------------- sliding schedule over a whole sequence
def run_slide(w: ti.Workload, chunk, rows=None, num_splits=0, shared=False):
    """tlin_slide_layer_attn against the oracle; w.N is the sequence length (w.W unused)."""
    L = w.N
    shape = (w.B, w.H, L, w.D)
    host = {name: ti.normal(shape, w.dtype, w.seed, tag, w.mul) for name, tag in
            (("Q", ti.TAG_Q), ("Kh", ti.TAG_KH), ("Vh", ti.TAG_VH), ("Kw", ti.TAG_KW), ("Vw", ti.TAG_VW))}
    if shared:
        host["Kw"], host["Vw"] = host["Kh"], host["Vh"]
    dev = upload(host, w.dtype)
    if shared:
        dev["Kw"], dev["Vw"] = dev["Kh"], dev["Vh"]
    for mode, omode in ((tl.TLIN_COMBINE_SUM, oracle.SUM), (tl.TLIN_COMBINE_JOINT, oracle.JOINT)):
        o = tl.tlin_slide_layer_attn(dev["Q"], dev["Kh"], dev["Vh"], dev["Kw"], dev["Vw"], chunk, combine=mode,
                                     scale=w.scale, num_splits=num_splits)
        ro = oracle.slide(host["Q"], host["Kh"], host["Vh"], host["Kw"], host["Vw"], w.dtype, w.scale, chunk, omode,
                          rows)
        g = o if rows is None else o[:, :, torch.from_numpy(rows).long().cuda()]
        assert_close(g, ro, w.dtype, f"{w.name} slide chunk {chunk} mode {mode}")
    return o


@pytest.mark.parametrize("dtype", [ti.F32, ti.BF16])
@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("L,chunk", [(1000, 128), (1024, 256), (777, 64), (300, 512), (130, 1), (2100, 300), (4096, 512)])
def test_slide_every_row(dtype, D, L, chunk):
    w = ti.Workload(f"slide_{dtype}_{D}_{L}_{chunk}", 2, 2, D, L, chunk, dtype, 1.0, 4242 + L + chunk)
    run_slide(w, chunk)


@pytest.mark.parametrize("num_splits", [1, 3, 7])
def test_slide_partition_count_does_not_change_the_result_class(num_splits):
    w = ti.Workload("slide_splits", 1, 3, 128, 3000, 256, ti.BF16, 1.0, 5151)
    run_slide(w, 256, num_splits=num_splits)


def test_slide_joint_with_shared_keys_is_causal_attention():
    """One K/V tensor in both roles and one softmax: the sliding schedule is plain causal
    attention over the sequence; compared with the library's own window causal kernel run on
    the whole sequence as one window, and with the oracle."""
    w = ti.Workload("slide_shared", 1, 4, 128, 2048, 256, ti.BF16, 1.0, 6161)
    o = run_slide(w, 256, shared=True)       # returns the JOINT result
    host = {name: ti.normal((w.B, w.H, w.N, w.D), w.dtype, w.seed, tag, w.mul) for name, tag in
            (("Q", ti.TAG_Q), ("K", ti.TAG_KH), ("V", ti.TAG_VH))}
    dev = upload(host, w.dtype)
    ref = tl.tlin_window_causal_attn(dev["Q"], dev["K"], dev["V"], scale=w.scale)
    assert_close(o, to_host64(ref), w.dtype, "slide JOINT vs one causal window")


def test_slide_full_size_stratified_rows():
    """The sequence length of the largest fixed workload cut into its window length: 256 chunks
    of 512 rows, 32 heads, in the launch configuration the bench times.  Compared: first and last
    row of every 32-row wave block of the first two chunks (empty and one-chunk history), a
    middle chunk and the last chunk, plus the rows around the middle of the sequence."""
    w = ti.Workload("slide_bf16_L131072_W512", 1, 32, 128, 131072, 512, ti.BF16, 1.0, 7171)
    block = stratified_rows(512)
    rows = np.concatenate([c * 512 + block for c in (0, 1, 100, 255)] + [np.array([65535, 65536, 100000])])
    run_slide(w, 512, rows=np.unique(rows).astype(np.int32))


@pytest.mark.parametrize("dtype", [ti.BF16, ti.F32])
@pytest.mark.parametrize("D", [128, 64, 36])
@pytest.mark.parametrize("W", [40, 128, 300, 512])
@pytest.mark.parametrize("N,splits", [(20000, 2), (20000, 5), (40001, 0), (9000, 3)])
def test_layer_call_whose_window_blocks_ride_on_partition_0(dtype, D, W, N, splits):
    """Layer calls with partitions long enough that no window block is launched: the workgroup of
    partition 0 also computes the window's causal block, and every partition's bounds are shifted
    by that block's cost.  Every row, both combine modes, forced and automatic partition counts,
    one and two query blocks per head, a ragged last key tile."""
    w = ti.Workload(f"fused_{dtype}_{D}_{W}_{N}_{splits}", 1, 2, D, N, W, dtype, 1.0, 515151 + D + 7 * W + N + splits + dtype)
    host = ti.make(w)
    dev = {k: padded(v, w.dtype) for k, v in host.items()}
    for mode, omode in ((tl.TLIN_COMBINE_SUM, oracle.SUM), (tl.TLIN_COMBINE_JOINT, oracle.JOINT)):
        o = tl.tlin_layer_attn(dev["Q"], dev["Kh"], dev["Vh"], dev["Kw"], dev["Vw"], combine=mode, scale=w.scale,
                               num_splits=splits)
        ro = oracle.layer(host["Q"], host["Kh"], host["Vh"], host["Kw"], host["Vw"], w.dtype, w.scale, omode)
        assert_close(o, ro, w.dtype, f"{w.name} mode {mode}")


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_shapes_through_every_entry_point(seed):
    """Eighty seeded random problems per seed: input type, head dimension (native sizes and sizes in
    between, NaN padding), batch and heads, history length 1 ... 400000 and window 1 ... 600
    (log-uniform), automatic and forced partition counts, a quarter of the bf16 ones with peaky keys;
    history, window and both layer modes against the oracle (all rows, or a sample when the problem
    is large)."""
    import math
    import random
    rng = random.Random(424200 + seed)
    for case in range(80):
        dtype = rng.choice([ti.BF16, ti.BF16, ti.F32])
        D = rng.choice([128, 128, 64, 64, 36, 8, 12, 40, 48, 96, 100, 120, 16, 32])
        B, H = rng.choice([1, 1, 2]), rng.choice([1, 2, 3, 5])
        N = int(round(math.exp(rng.uniform(0, math.log(400000)))))
        W = int(round(math.exp(rng.uniform(0, math.log(600)))))
        splits = rng.choice([0, 0, 0, 1, 2, 3, 5, 17])
        peaky = dtype == ti.BF16 and rng.random() < 0.25
        w = ti.Workload(f"random{seed}_{case}", B, H, D, N, W, dtype, 1.0, 9000000 + 1000 * seed + case,
                        peaky_mod=50 if peaky else 0, peaky_factor=6.0 if peaky else 1.0)
        what = f"{w.name}: dtype {dtype} B{B} H{H} D{D} N{N} W{W} splits {splits} peaky {peaky}"
        host = ti.make(w)
        dev = {k: padded(v, w.dtype) for k, v in host.items()}
        rows = None if W * N <= 3_000_000 else sample_rows(W, max(4, 3_000_000 // N), seed=case)
        sel = (lambda t: t) if rows is None else (lambda t: t[:, :, torch.from_numpy(rows).long().cuda()])
        o, lse = tl.tlin_history_attn(dev["Q"], dev["Kh"], dev["Vh"], scale=w.scale, num_splits=splits, return_lse=True)
        ro, rl = oracle.history(host["Q"], host["Kh"], host["Vh"], w.dtype, w.scale, rows)
        assert_close(sel(o), ro, w.dtype, f"{what} history")
        np.testing.assert_allclose(to_host64(sel(lse.unsqueeze(-1)))[..., 0], rl, rtol=1e-6, atol=lse_atol(w.dtype, rl), err_msg=what)
        o = tl.tlin_window_causal_attn(dev["Q"], dev["Kw"], dev["Vw"], scale=w.scale)
        ro, _ = oracle.window_causal(host["Q"], host["Kw"], host["Vw"], w.dtype, w.scale, rows)
        assert_close(sel(o), ro, w.dtype, f"{what} window")
        for mode, omode in ((tl.TLIN_COMBINE_SUM, oracle.SUM), (tl.TLIN_COMBINE_JOINT, oracle.JOINT)):
            o = tl.tlin_layer_attn(dev["Q"], dev["Kh"], dev["Vh"], dev["Kw"], dev["Vw"], combine=mode, scale=w.scale,
                                   num_splits=splits)
            ro = oracle.layer(host["Q"], host["Kh"], host["Vh"], host["Kw"], host["Vw"], w.dtype, w.scale, omode, rows)
            assert_close(sel(o), ro, w.dtype, f"{what} layer mode {mode}")


# ---------------------------------------------------------------- head dimensions between the native sizes
def padded(a: np.ndarray, dtype: int) -> torch.Tensor:
    """Device tensor whose rows are padded to whole 16-byte pieces; the padding holds NaNs (it
    must be ignored), the view handed to the library has the logical head dimension."""
    t = to_device_any(a, dtype)
    per16 = 16 // t.element_size()
    D = t.shape[-1]
    row = (D + per16 - 1) // per16 * per16
    buf = torch.full(t.shape[:-1] + (row,), float("nan"), dtype=t.dtype, device=t.device)
    buf[..., :D] = t
    return buf[..., :D]


def to_device_any(a, dtype):
    from helpers import to_device
    return to_device(a, dtype)


@pytest.mark.parametrize("dtype", [ti.F32, ti.BF16])
@pytest.mark.parametrize("D", [36, 8, 12, 60, 96, 100])
@pytest.mark.parametrize("W,N", [(1, 700), (70, 333), (256, 2100), (300, 64)])
def test_head_dimensions_between_the_native_sizes(dtype, D, W, N):
    """The paper's own model has head dimension 36 (432 / 12, Section 6.2)."""
    w = ti.Workload(f"hd_{dtype}_{D}_{W}_{N}", 1, 3, D, N, W, dtype, 1.0, 3636 + D + W + N)
    host = ti.make(w)
    dev = {k: padded(v, w.dtype) for k, v in host.items()}
    o, lse = tl.tlin_history_attn(dev["Q"], dev["Kh"], dev["Vh"], scale=w.scale, return_lse=True)
    ro, rl = oracle.history(host["Q"], host["Kh"], host["Vh"], w.dtype, w.scale)
    assert o.shape[-1] == D
    assert_close(o, ro, w.dtype, f"{w.name} history")
    np.testing.assert_allclose(to_host64(lse), rl, rtol=1e-6, atol=lse_atol(w.dtype, rl))
    o = tl.tlin_window_causal_attn(dev["Q"], dev["Kw"], dev["Vw"], scale=w.scale)
    ro, _ = oracle.window_causal(host["Q"], host["Kw"], host["Vw"], w.dtype, w.scale)
    assert_close(o, ro, w.dtype, f"{w.name} window")
    for mode, omode in ((tl.TLIN_COMBINE_SUM, oracle.SUM), (tl.TLIN_COMBINE_JOINT, oracle.JOINT)):
        o = tl.tlin_layer_attn(dev["Q"], dev["Kh"], dev["Vh"], dev["Kw"], dev["Vw"], combine=mode, scale=w.scale)
        ro = oracle.layer(host["Q"], host["Kh"], host["Vh"], host["Kw"], host["Vw"], w.dtype, w.scale, omode)
        assert_close(o, ro, w.dtype, f"{w.name} layer mode {mode}")


@pytest.mark.parametrize("N", [131072, 999754])
def test_paper_model_shape_head_dimension_36_full_size_stratified_rows(N):
    """12 heads of dimension 36, windows of 256 rows (Sections 5.1 and 6.2), over 131072 history
    rows and over the history of a sequence just beyond one million tokens (Section 6.4: 999754
    history rows + the 256-row window; ragged last key tile)."""
    w = ti.Workload(f"paper_hd36_N{N}", 1, 12, 36, N, 256, ti.BF16, 1.0, 36036 + N)
    host = ti.make(w)
    dev = {k: padded(v, w.dtype) for k, v in host.items()}
    rows = stratified_rows(w.W)
    idx = torch.from_numpy(rows).long().cuda()
    for mode, omode in ((tl.TLIN_COMBINE_SUM, oracle.SUM), (tl.TLIN_COMBINE_JOINT, oracle.JOINT)):
        o = tl.tlin_layer_attn(dev["Q"], dev["Kh"], dev["Vh"], dev["Kw"], dev["Vw"], combine=mode, scale=w.scale)
        ro = oracle.layer(host["Q"], host["Kh"], host["Vh"], host["Kw"], host["Vw"], w.dtype, w.scale, omode, rows)
        assert_close(o[:, :, idx], ro, w.dtype, f"{w.name} mode {mode}")
    # cache-hit step and restoration shape of the same model
    q1 = dev["Q"][:, :, -1:, :]
    o = tl.tlin_history_attn(q1, dev["Kh"], dev["Vh"], scale=w.scale)
    ro, _ = oracle.history(host["Q"][:, :, -1:, :], host["Kh"], host["Vh"], w.dtype, w.scale)
    assert_close(o, ro, w.dtype, "paper_hd36 cache-hit step")
    o = tl.tlin_history_attn(dev["Kh"][:, :, :40000], dev["Kw"], dev["Vw"], scale=w.scale)     # many queries x 256 keys
    rr = sample_rows(40000, 24, seed=37)
    ro, _ = oracle.history(host["Kh"][:, :, :40000], host["Kw"], host["Vw"], w.dtype, w.scale, rr)
    assert_close(o[:, :, torch.from_numpy(rr).long().cuda()], ro, w.dtype, "paper_hd36 restoration")


# ---------------------------------------------------------------- shapes, tails, degenerate cases
@pytest.mark.parametrize("dtype", [ti.F32, ti.BF16])
@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("W,N", [(1, 1), (1, 200), (31, 63), (33, 65), (64, 64), (100, 1000), (129, 129),
                                 (257, 300), (300, 2049)])
def test_ragged_shapes(dtype, D, W, N):
    w = ti.Workload(f"ragged_{dtype}_{D}_{W}_{N}", 1, 2, D, N, W, dtype, 1.0, 77 + W * 131 + N)
    run_all(w)


@pytest.mark.parametrize("dtype", [ti.F32, ti.BF16])
def test_split_count_invariance_and_determinism(dtype):
    w = ti.Workload(f"splits_{dtype}", 1, 2, 128, 3000, 96, dtype, 1.0, 4242)
    host = ti.make(w)
    dev = upload(host, w.dtype)
    ro, _ = oracle.history(host["Q"], host["Kh"], host["Vh"], w.dtype, w.scale)
    outs = []
    for s in (1, 2, 3, 7, 47, 1000):
        o = tl.tlin_history_attn(dev["Q"], dev["Kh"], dev["Vh"], scale=w.scale, num_splits=s, out_dtype=torch.float32)
        assert_close(o, ro, w.dtype, f"num_splits={s}")
        o2 = tl.tlin_history_attn(dev["Q"], dev["Kh"], dev["Vh"], scale=w.scale, num_splits=s, out_dtype=torch.float32)
        assert torch.equal(o, o2), "run-to-run results differ"
        outs.append(to_host64(o))
    for o in outs[1:]:
        assert np.abs(o - outs[0]).max() <= (1e-5 if dtype == ti.F32 else 5e-3)


def test_strided_views_and_f32_output_for_bf16_inputs():
    w = ti.Workload("strided", 2, 3, 128, 500, 70, ti.BF16, 1.0, 999)
    host = ti.make(w)
    dev = upload(host, w.dtype)
    # [B, rows, H, D] storage viewed as [B, H, rows, D]: head stride D, row stride H*D
    def interleave(t):
        return t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    Q, Kh, Vh, Kw, Vw = (interleave(dev[k]) for k in ("Q", "Kh", "Vh", "Kw", "Vw"))
    assert not Q.is_contiguous()
    o = tl.tlin_layer_attn(Q, Kh, Vh, Kw, Vw, combine=tl.TLIN_COMBINE_JOINT, scale=w.scale, out_dtype=torch.float32)
    ro = oracle.layer(host["Q"], host["Kh"], host["Vh"], host["Kw"], host["Vw"], w.dtype, w.scale, oracle.JOINT)
    assert o.dtype == torch.float32
    assert_close(o, ro, w.dtype, "strided joint")
    o = tl.tlin_history_attn(Q, Kh, Vh, scale=w.scale)
    ro, _ = oracle.history(host["Q"], host["Kh"], host["Vh"], w.dtype, w.scale)
    assert_close(o, ro, w.dtype, "strided history")


@pytest.mark.parametrize("dtype", [ti.F32, ti.BF16])
def test_invariants_hold_on_the_gpu_result(dtype):
    w = ti.Workload(f"inv_{dtype}", 1, 2, 64, 777, 50, dtype, 1.0, 31337)
    dev = upload(ti.make(w), w.dtype)
    Q, Kh, Vh, Kw, Vw = (dev[k] for k in ("Q", "Kh", "Vh", "Kw", "Vw"))
    ones_h, ones_w = torch.ones_like(Vh), torch.ones_like(Vw)
    tol = 1e-5 if dtype == ti.F32 else 8e-3
    o = tl.tlin_history_attn(Q, Kh, ones_h, scale=w.scale, out_dtype=torch.float32)
    assert (o - 1).abs().max().item() <= tol          # rows are convex combinations
    o = tl.tlin_layer_attn(Q, Kh, ones_h, Kw, ones_w, combine=tl.TLIN_COMBINE_SUM, scale=w.scale, out_dtype=torch.float32)
    assert (o - 2).abs().max().item() <= 2 * tol
    o = tl.tlin_layer_attn(Q, Kh, ones_h, Kw, ones_w, combine=tl.TLIN_COMBINE_JOINT, scale=w.scale, out_dtype=torch.float32)
    assert (o - 1).abs().max().item() <= tol
    # history is a set: a joint permutation of its rows changes nothing beyond rounding
    perm = torch.randperm(w.N, generator=torch.Generator().manual_seed(1)).cuda()
    o1 = tl.tlin_history_attn(Q, Kh, Vh, scale=w.scale, out_dtype=torch.float32)
    o2 = tl.tlin_history_attn(Q, Kh[:, :, perm].contiguous(), Vh[:, :, perm].contiguous(), scale=w.scale, out_dtype=torch.float32)
    assert (o1 - o2).abs().max().item() <= (2e-6 if dtype == ti.F32 else 1e-2)
    # causal row 0 is the first value row
    o = tl.tlin_window_causal_attn(Q, Kw, Vw, scale=w.scale)
    assert torch.equal(o[:, :, 0], Vw[:, :, 0])


def test_errors_are_reported_not_raised_by_the_gpu():
    w = ti.Workload("err", 1, 1, 64, 128, 16, ti.BF16, 1.0, 5)
    dev = upload(ti.make(w), w.dtype)
    with pytest.raises(tl.TlinError) as e:
        tl.tlin_history_attn(dev["Q"], dev["Kh"], dev["Vh"], scale=-1.0)
    assert e.value.status == tl.binding.TLIN_ERR_INVALID_ARG
    with pytest.raises(ValueError):
        tl.tlin_history_attn(dev["Q"].cpu(), dev["Kh"], dev["Vh"])


# ---------------------------------------------------------------- running maximum, streams, many heads
@pytest.mark.parametrize("dtype,amp", [(ti.F32, 20.0), (ti.F32, 60.0), (ti.BF16, 600.0)])
@pytest.mark.parametrize("direction", [1.0, -1.0])
def test_scores_that_climb_or_fall_along_the_history(dtype, amp, direction):
    """Keys whose scores grow (or shrink) steadily with the row index, by 10 or 30 (fp32) or 300
    (bf16) powers of two over the history: the running maximum of the online softmax keeps moving
    (or never moves after the first tile), partitions differ by more than the reference-point
    threshold (bf16: by more than the fp32 exponent range), and almost all the weight sits on the
    rows at one end.  The fp32 path rounds each logit to a few 2^-24 of its size, which the
    exponential turns into relative error of the weight: the 1e-5 bound holds for logits up to 10
    nats (amp 20: 7 nats), beyond that the documented envelope grows by 1e-6 per nat (amp 60: 21
    nats, bound 2.1e-5; measured 1.2e-5)."""
    B, H, D, N, W = 1, 2, 128, 3000, 70
    w = ti.Workload(f"climb_{dtype}_{direction}", B, H, D, N, W, dtype, 1.0, 8642)
    host = ti.make(w)
    rng = np.random.default_rng(5)
    u = rng.standard_normal(D).astype(np.float32)
    u /= np.linalg.norm(u)

    def rounded(a):          # the generator's arrays are float32 for fp32 and bf16 bit patterns (uint16) for bf16
        if dtype == ti.F32:
            return a.astype(np.float32)
        t = torch.from_numpy(a.astype(np.float32)).to(torch.bfloat16)
        return t.view(torch.int16).numpy().view(host["Q"].dtype)

    q = 4.0 * u[None, None, None, :] + 0.1 * rng.standard_normal((B, H, W, D))
    ramp = direction * (np.arange(N, dtype=np.float64) / N)[None, None, :, None]
    # scale * <q, k_j> = 4 * amp * ramp_j / sqrt(128) nats: 0.51 powers of two per unit of amp
    kh = amp * ramp * u[None, None, None, :] + 0.1 * rng.standard_normal((B, H, N, D))
    host = dict(host, Q=rounded(q), Kh=rounded(kh))
    bound = f32_rel_bound(4.0 * amp / np.sqrt(D))
    dev = upload(host, dtype)
    for s in (1, 4, 11):
        o, lse = tl.tlin_history_attn(dev["Q"], dev["Kh"], dev["Vh"], scale=w.scale, num_splits=s, return_lse=True)
        ro, rl = oracle.history(host["Q"], host["Kh"], host["Vh"], dtype, w.scale)
        assert_close(o, ro, dtype, f"climb {direction} splits {s}", f32_rel=bound)
        np.testing.assert_allclose(to_host64(lse), rl, rtol=2e-6, atol=lse_atol(dtype, rl))
    for mode, omode in ((tl.TLIN_COMBINE_SUM, oracle.SUM), (tl.TLIN_COMBINE_JOINT, oracle.JOINT)):
        o = tl.tlin_layer_attn(dev["Q"], dev["Kh"], dev["Vh"], dev["Kw"], dev["Vw"], combine=mode, scale=w.scale)
        ro = oracle.layer(host["Q"], host["Kh"], host["Vh"], host["Kw"], host["Vw"], dtype, w.scale, omode)
        assert_close(o, ro, dtype, f"climb {direction} layer {mode}", f32_rel=bound)


def test_calls_on_a_stream_of_the_callers():
    w = ti.Workload("stream", 1, 4, 128, 5000, 256, ti.BF16, 1.0, 1717)
    host = ti.make(w)
    dev = upload(host, w.dtype)
    ro = oracle.layer(host["Q"], host["Kh"], host["Vh"], host["Kw"], host["Vw"], w.dtype, w.scale, oracle.SUM)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        outs = [tl.tlin_layer_attn(*(dev[k] for k in ("Q", "Kh", "Vh", "Kw", "Vw")), scale=w.scale) for _ in range(3)]
    side.synchronize()
    for o in outs:
        assert_close(o, ro, w.dtype, "side stream")
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])


@pytest.mark.parametrize("dtype", [ti.F32, ti.BF16])
def test_many_small_heads(dtype):
    # thousands of independent (batch, head) problems, each a fraction of a tile
    w = ti.Workload(f"heads_{dtype}", 8, 300, 64, 100, 9, dtype, 1.0, 2323)
    run_all(w, check_lse=True)


def test_bf16_output_for_fp32_inputs():
    """fp32 arithmetic, result rounded to bf16 at the store: within half a unit in the last place of
    bf16 (8 significant bits: relative 2^-8) plus the fp32 path's own bound, for the direct, merged
    and layer paths."""
    w = ti.Workload("f32_bf16out", 1, 3, 128, 1500, 200, ti.F32, 1.0, 6161)
    host = ti.make(w)
    dev = upload(host, w.dtype)
    Q, Kh, Vh, Kw, Vw = (dev[k] for k in ("Q", "Kh", "Vh", "Kw", "Vw"))

    def check(o, ref, what):
        assert o.dtype == torch.bfloat16
        g = to_host64(o)
        rms = float(np.sqrt(np.mean(ref * ref)))
        err = np.abs(g - ref) / np.maximum(np.abs(ref), rms)
        assert err.max() <= 2.0 ** -8 + 1e-5, f"{what}: {err.max():.3e}"

    for s in (1, 5):
        o = tl.tlin_history_attn(Q, Kh, Vh, scale=w.scale, num_splits=s, out_dtype=torch.bfloat16)
        check(o, oracle.history(host["Q"], host["Kh"], host["Vh"], w.dtype, w.scale)[0], f"history splits {s}")
    o = tl.tlin_window_causal_attn(Q, Kw, Vw, scale=w.scale, out_dtype=torch.bfloat16)
    check(o, oracle.window_causal(host["Q"], host["Kw"], host["Vw"], w.dtype, w.scale)[0], "window")
    o = tl.tlin_layer_attn(Q, Kh, Vh, Kw, Vw, combine=tl.TLIN_COMBINE_JOINT, scale=w.scale, out_dtype=torch.bfloat16)
    check(o, oracle.layer(host["Q"], host["Kh"], host["Vh"], host["Kw"], host["Vw"], w.dtype, w.scale, oracle.JOINT), "layer")


@pytest.mark.parametrize("dtype", [ti.F32, ti.BF16])
def test_layer_call_replays_from_a_hip_graph(dtype):
    """The library only enqueues kernels on the caller's stream (no allocation, no memset, no
    synchronisation), so a call can be captured into a HIP graph once its one-time set-up has run.
    The graph is replayed several times with new inputs written into the captured tensors and eager
    work in between; every replay must equal the eager call on the same inputs, and the oracle."""
    w = ti.Workload(f"graph_{dtype}", 2, 4, 128, 3000, 160, dtype, 1.0, 7373)
    names = ("Q", "Kh", "Vh", "Kw", "Vw")
    hosts = [ti.make(ti.Workload(w.name, w.B, w.H, w.D, w.N, w.W, dtype, 1.0, w.seed + i)) for i in range(3)]
    devs = [upload(h, dtype) for h in hosts]
    static = {k: devs[0][k].clone() for k in names}
    ws = tl.Workspace()

    def call(t):
        return tl.tlin_layer_attn(*(t[k] for k in names), combine=tl.TLIN_COMBINE_JOINT, scale=w.scale, workspace=ws)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call(static)                                   # one-time set-up and workspace allocation, outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        out = call(static)
    for rep in range(5):
        i = rep % 3
        for k in names:
            static[k].copy_(devs[i][k])
        graph.replay()
        torch.cuda.synchronize()
        got = out.clone()
        eager = call(devs[i])                          # the program's own eager work between replays
        torch.cuda.synchronize()
        assert torch.equal(got, eager), f"replay {rep} differs from the eager call"
        if rep < 3:
            ro = oracle.layer(*(hosts[i][k] for k in names), dtype, w.scale, oracle.JOINT)
            assert_close(got, ro, dtype, f"graph replay {rep}")


@pytest.mark.parametrize("dtype", [ti.F32, ti.BF16])
def test_slide_on_interleaved_head_layout(dtype):
    """The sliding schedule on tensors stored [B, L, H, D] (what a fused projection writes) and
    viewed as [B, H, L, D]: head stride D, row stride H*D; K and V of both roles are one tensor each."""
    B, H, L, D, chunk = 2, 3, 700, 64, 96
    w = ti.Workload(f"slide_strided_{dtype}", B, H, D, L, chunk, dtype, 1.0, 9191)
    shape = (B, H, L, D)
    host = {n: ti.normal(shape, dtype, w.seed, tag, w.mul) for n, tag in (("Q", ti.TAG_Q), ("K", ti.TAG_KH), ("V", ti.TAG_VH))}
    dev = upload(host, dtype)

    def interleave(t):
        return t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    Q, K, V = (interleave(dev[k]) for k in ("Q", "K", "V"))
    assert not Q.is_contiguous()
    for mode, omode in ((tl.TLIN_COMBINE_SUM, oracle.SUM), (tl.TLIN_COMBINE_JOINT, oracle.JOINT)):
        o = tl.tlin_slide_layer_attn(Q, K, V, K, V, chunk, combine=mode, scale=w.scale)
        ro = oracle.slide(host["Q"], host["K"], host["V"], host["K"], host["V"], dtype, w.scale, chunk, omode)
        assert_close(o, ro, dtype, f"strided slide mode {mode}")
