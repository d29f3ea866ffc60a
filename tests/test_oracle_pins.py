"""Pins for the CPU oracle: every check compares it with something that is not the oracle
itself - a library attention routine, a closed form, an invariance, a hand-derived example."""
import math
import os

import numpy as np
import pytest
import torch
from scipy.special import logsumexp

import oracle
import tlin_inputs as ti

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def rnd(shape, seed, tag, mul=1.0, dtype=ti.F32):
    return ti.normal(shape, dtype, seed, tag, mul)


def sdpa64(Q, K, V, scale, causal=False, mask=None):
    """Library scaled-dot-product attention on the CPU in fp64."""
    q, k, v = (torch.from_numpy(np.asarray(x, dtype=np.float64)) for x in (Q, K, V))
    m = None if mask is None else torch.from_numpy(mask)
    return torch.nn.functional.scaled_dot_product_attention(
        q, k, v, attn_mask=m, is_causal=causal, scale=scale).numpy()


# ---------------------------------------------------------------- library pins
@pytest.mark.parametrize("dtype", [ti.F32, ti.BF16])
@pytest.mark.parametrize("B,H,W,N,D", [(1, 1, 5, 19, 8), (2, 3, 17, 70, 16), (1, 2, 33, 129, 64)])
def test_history_matches_library_attention(dtype, B, H, W, N, D):
    Q, K, V = (rnd((B, H, r, D), 11, t, 0.7, dtype) for t, r in ((1, W), (2, N), (3, N)))
    scale = 1.0 / math.sqrt(D)
    O, lse = oracle.history(Q, K, V, dtype, scale)
    q, k, v = (ti.to_f64(x, dtype) for x in (Q, K, V))
    np.testing.assert_allclose(O, sdpa64(q, k, v, scale), rtol=0, atol=1e-13)
    s = scale * np.einsum("bhid,bhjd->bhij", q, k)
    np.testing.assert_allclose(lse, logsumexp(s, axis=-1), rtol=0, atol=1e-12)


@pytest.mark.parametrize("dtype", [ti.F32, ti.BF16])
@pytest.mark.parametrize("B,H,W,D", [(1, 1, 7, 8), (2, 2, 40, 16), (1, 3, 65, 64)])
def test_window_causal_matches_library_causal_attention(dtype, B, H, W, D):
    Q, K, V = (rnd((B, H, W, D), 12, t, 0.9, dtype) for t in (1, 4, 5))
    scale = 1.0 / math.sqrt(D)
    O, lse = oracle.window_causal(Q, K, V, dtype, scale)
    q, k, v = (ti.to_f64(x, dtype) for x in (Q, K, V))
    np.testing.assert_allclose(O, sdpa64(q, k, v, scale, causal=True), rtol=0, atol=1e-13)
    s = scale * np.einsum("bhid,bhjd->bhij", q, k)
    s = np.where(np.tril(np.ones((W, W), dtype=bool)), s, -np.inf)
    np.testing.assert_allclose(lse, logsumexp(s, axis=-1), rtol=0, atol=1e-12)


@pytest.mark.parametrize("dtype", [ti.F32, ti.BF16])
@pytest.mark.parametrize("N", [1, 5, 48, 100])
def test_joint_layer_is_tail_of_causal_attention_over_concatenation(dtype, N):
    """Figure 2(b): a window node has full edges from the history and causal edges inside the
    window, so JOINT equals rows [N, N+W) of library causal attention over [hist; window],
    for every split point."""
    B, H, W, D = 2, 2, 23, 16
    Q, Kw, Vw = (rnd((B, H, W, D), 13, t, 0.8, dtype) for t in (1, 4, 5))
    Kh, Vh = (rnd((B, H, N, D), 13, t, 0.8, dtype) for t in (2, 3))
    scale = 0.31
    O = oracle.layer(Q, Kh, Vh, Kw, Vw, dtype, scale, oracle.JOINT)
    q, kh, vh, kw, vw = (ti.to_f64(x, dtype) for x in (Q, Kh, Vh, Kw, Vw))
    qpad = np.concatenate([np.full((B, H, N, D), 123.0), q], axis=2)   # first N rows are irrelevant
    ref = sdpa64(qpad, np.concatenate([kh, kw], 2), np.concatenate([vh, vw], 2), scale, causal=True)
    np.testing.assert_allclose(O, ref[:, :, N:], rtol=0, atol=1e-13)


@pytest.mark.parametrize("dtype", [ti.F32, ti.BF16])
def test_sum_layer_is_sum_of_library_parts(dtype):
    B, H, W, N, D = 1, 3, 19, 37, 8
    Q, Kw, Vw = (rnd((B, H, W, D), 14, t, 1.0, dtype) for t in (1, 4, 5))
    Kh, Vh = (rnd((B, H, N, D), 14, t, 1.0, dtype) for t in (2, 3))
    scale = 0.4
    O = oracle.layer(Q, Kh, Vh, Kw, Vw, dtype, scale, oracle.SUM)
    q, kh, vh, kw, vw = (ti.to_f64(x, dtype) for x in (Q, Kh, Vh, Kw, Vw))
    ref = sdpa64(q, kh, vh, scale) + sdpa64(q, kw, vw, scale, causal=True)
    np.testing.assert_allclose(O, ref, rtol=0, atol=1e-13)


@pytest.mark.parametrize("combine", [oracle.SUM, oracle.JOINT])
def test_empty_history_layer_is_standard_causal_attention(combine):
    """First chunk of the sliding schedule (Section 5.1) has no history: the layer is then
    plain causal attention of length W."""
    B, H, W, D = 1, 2, 50, 16
    Q, Kw, Vw = (rnd((B, H, W, D), 15, t) for t in (1, 4, 5))
    scale = 0.25
    O = oracle.layer(Q, None, None, Kw, Vw, ti.F32, scale, combine)
    ref = sdpa64(Q, Kw, Vw, scale, causal=True)
    np.testing.assert_allclose(O, ref, rtol=0, atol=1e-13)


# ---------------------------------------------------------------- sliding schedule (Section 5.1)
@pytest.mark.parametrize("dtype", [ti.F32, ti.BF16])
@pytest.mark.parametrize("L,W", [(37, 8), (64, 16), (50, 50), (23, 40), (41, 1)])
def test_slide_joint_with_shared_keys_is_causal_attention_over_the_sequence(dtype, L, W):
    """History = all earlier chunks in full, window = causal inside the chunk: with one key/value
    tensor for both, one softmax over the two sets is plain causal attention of length L,
    whatever the chunk size."""
    B, H, D = 2, 2, 16
    Q, K, V = (rnd((B, H, L, D), 21, t, 0.8, dtype) for t in (1, 2, 3))
    scale = 0.29
    O = oracle.slide(Q, K, V, K, V, dtype, scale, W, oracle.JOINT)
    q, k, v = (ti.to_f64(x, dtype) for x in (Q, K, V))
    np.testing.assert_allclose(O, sdpa64(q, k, v, scale, causal=True), rtol=0, atol=1e-13)


@pytest.mark.parametrize("combine", [oracle.SUM, oracle.JOINT])
@pytest.mark.parametrize("L,W", [(45, 10), (32, 8), (9, 20)])
def test_slide_chunks_are_library_attention_per_chunk(combine, L, W):
    """Distinct history and window projections.  Chunk c against the library: SUM = unmasked
    attention over rows [0, cW) of Kh/Vh plus causal attention over the chunk's Kw/Vw; JOINT =
    tail rows of causal attention over [Kh[:cW]; Kw[chunk]].  Chunk 0 has no history."""
    B, H, D = 1, 3, 8
    Q, Kh, Vh, Kw, Vw = (rnd((B, H, L, D), 22, t, 0.9) for t in (1, 2, 3, 4, 5))
    scale = 0.37
    O = oracle.slide(Q, Kh, Vh, Kw, Vw, ti.F32, scale, W, combine)
    for c0 in range(0, L, W):
        c1 = min(c0 + W, L)
        q, kw, vw = Q[:, :, c0:c1], Kw[:, :, c0:c1], Vw[:, :, c0:c1]
        if combine == oracle.SUM:
            ref = sdpa64(q, kw, vw, scale, causal=True)
            if c0:
                ref = ref + sdpa64(q, Kh[:, :, :c0], Vh[:, :, :c0], scale)
        else:
            qpad = np.concatenate([np.zeros((B, H, c0, D)), q], axis=2)
            ref = sdpa64(qpad, np.concatenate([Kh[:, :, :c0], kw], 2), np.concatenate([Vh[:, :, :c0], vw], 2),
                         scale, causal=True)[:, :, c0:]
        np.testing.assert_allclose(O[:, :, c0:c1], ref, rtol=0, atol=1e-13)


def test_slide_row_subset_and_bad_arguments():
    B, H, L, W, D = 1, 2, 30, 7, 8
    Q, Kh, Vh, Kw, Vw = (rnd((B, H, L, D), 23, t) for t in (1, 2, 3, 4, 5))
    full = oracle.slide(Q, Kh, Vh, Kw, Vw, ti.F32, 0.3, W, oracle.SUM)
    rows = np.array([0, 6, 7, 13, 29], dtype=np.int32)
    sub = oracle.slide(Q, Kh, Vh, Kw, Vw, ti.F32, 0.3, W, oracle.SUM, rows)
    np.testing.assert_array_equal(sub, full[:, :, rows])
    with pytest.raises(RuntimeError):
        oracle.slide(Q, Kh, Vh, Kw, Vw, ti.F32, 0.3, 0, oracle.SUM)
    with pytest.raises(RuntimeError):
        oracle.slide(Q, Kh, Vh, Kw, Vw, ti.F32, 0.3, W, 7)
    with pytest.raises(RuntimeError):
        oracle.slide(Q, Kh, Vh, Kw, Vw, ti.F32, 0.3, W, oracle.SUM, np.array([30], dtype=np.int32))


# ---------------------------------------------------------------- hand-derived example
def _golden():
    rows = {}
    with open(os.path.join(GOLD, "rational_weights.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            key, *vals = line.split()
            rows.setdefault(key, []).append([float(v) for v in vals])
    return {k: np.array(v) for k, v in rows.items()}


def test_rational_weight_worked_example():
    g = _golden()
    Q1 = g["Q"].astype(np.float32).reshape(1, 1, 1, 2)
    K = g["K"].astype(np.float32).reshape(1, 1, 3, 2)
    V = g["V"].astype(np.float32).reshape(1, 1, 3, 2)
    tol = dict(rtol=0, atol=2e-7)   # ln 2, ln 3 are rounded to fp32 on input
    O, lse = oracle.history(Q1, K, V, ti.F32, 1.0)
    np.testing.assert_allclose(O[0, 0], g["O_full"], **tol)
    np.testing.assert_allclose(lse[0, 0], g["LSE_full"][0], **tol)
    Q3 = np.repeat(Q1, 3, axis=2)
    O, lse = oracle.window_causal(Q3, K, V, ti.F32, 1.0)
    np.testing.assert_allclose(O[0, 0], g["O_causal"], **tol)
    np.testing.assert_allclose(lse[0, 0], g["LSE_causal"][0], **tol)
    Oj = oracle.layer(Q1, K[:, :, :2], V[:, :, :2], K[:, :, 2:], V[:, :, 2:], ti.F32, 1.0, oracle.JOINT)
    np.testing.assert_allclose(Oj[0, 0], g["O_joint"], **tol)
    Os = oracle.layer(Q1, K[:, :, :2], V[:, :, :2], K[:, :, 2:], V[:, :, 2:], ti.F32, 1.0, oracle.SUM)
    np.testing.assert_allclose(Os[0, 0], g["O_sum"], **tol)


# ---------------------------------------------------------------- closed forms
def test_two_keys_is_a_sigmoid():
    D = 4
    Q = rnd((1, 1, 6, D), 21, 1)
    K = rnd((1, 1, 2, D), 21, 2)
    V = rnd((1, 1, 2, D), 21, 3)
    scale = 0.7
    O, _ = oracle.history(Q, K, V, ti.F32, scale)
    q, k, v = Q.astype(np.float64)[0, 0], K.astype(np.float64)[0, 0], V.astype(np.float64)[0, 0]
    for i in range(6):
        dlt = scale * (q[i] @ k[0] - q[i] @ k[1])
        w0 = 1.0 / (1.0 + math.exp(-dlt))
        np.testing.assert_allclose(O[0, 0, i], w0 * v[0] + (1 - w0) * v[1], rtol=0, atol=1e-14)


def test_zero_query_gives_mean_of_values_and_prefix_means_when_causal():
    B, H, W, N, D = 1, 2, 9, 31, 8
    Q = np.zeros((B, H, W, D), np.float32)
    K, V = rnd((B, H, N, D), 22, 2), rnd((B, H, N, D), 22, 3)
    O, lse = oracle.history(Q, K, V, ti.F32, 0.5)
    np.testing.assert_allclose(O, np.broadcast_to(V.astype(np.float64).mean(2, keepdims=True), O.shape), atol=1e-14)
    np.testing.assert_allclose(lse, math.log(N), atol=1e-14)
    Kw, Vw = rnd((B, H, W, D), 22, 4), rnd((B, H, W, D), 22, 5)
    O, _ = oracle.window_causal(Q, Kw, Vw, ti.F32, 0.5)
    pref = np.cumsum(Vw.astype(np.float64), axis=2) / np.arange(1, W + 1)[None, None, :, None]
    np.testing.assert_allclose(O, pref, atol=1e-14)


def test_single_history_row_is_copied():
    Q, K, V = rnd((2, 2, 5, 8), 23, 1), rnd((2, 2, 1, 8), 23, 2), rnd((2, 2, 1, 8), 23, 3)
    O, lse = oracle.history(Q, K, V, ti.F32, 0.3)
    np.testing.assert_array_equal(O, np.broadcast_to(V.astype(np.float64), O.shape))
    s = 0.3 * np.einsum("bhid,bhjd->bhi", Q.astype(np.float64), K.astype(np.float64))
    np.testing.assert_allclose(lse, s, atol=1e-15)


def test_causal_row0_is_first_value_row_and_rows_are_prefix_history_calls():
    B, H, W, D = 1, 2, 12, 8
    Q, K, V = (rnd((B, H, W, D), 24, t) for t in (1, 4, 5))
    O, lse = oracle.window_causal(Q, K, V, ti.F32, 0.35)
    np.testing.assert_array_equal(O[:, :, 0], V.astype(np.float64)[:, :, 0])
    for i in (0, 3, 11):
        Oi, li = oracle.history(Q[:, :, i:i + 1], K[:, :, :i + 1], V[:, :, :i + 1], ti.F32, 0.35)
        np.testing.assert_allclose(O[:, :, i], Oi[:, :, 0], atol=1e-15)
        np.testing.assert_allclose(lse[:, :, i], li[:, :, 0], atol=1e-15)


def test_rows_are_convex_combinations():
    B, H, W, N, D = 1, 2, 7, 40, 8
    Q, K, V = rnd((B, H, W, D), 25, 1, 2.0), rnd((B, H, N, D), 25, 2, 2.0), rnd((B, H, N, D), 25, 3)
    ones = np.ones_like(V)
    O, _ = oracle.history(Q, K, ones, ti.F32, 0.5)
    np.testing.assert_allclose(O, 1.0, atol=1e-14)
    const = np.broadcast_to(np.arange(D, dtype=np.float32) - 3, V.shape).copy()
    O, _ = oracle.history(Q, K, const, ti.F32, 0.5)
    np.testing.assert_allclose(O, np.broadcast_to(np.arange(D) - 3.0, O.shape), atol=1e-13)
    O, _ = oracle.history(Q, K, V, ti.F32, 0.5)
    v = V.astype(np.float64)
    assert (O <= v.max(2, keepdims=True) + 1e-14).all() and (O >= v.min(2, keepdims=True) - 1e-14).all()
    Kw, Vw = rnd((B, H, W, D), 25, 4), np.ones((B, H, W, D), np.float32)
    np.testing.assert_allclose(oracle.layer(Q, K, ones, Kw, Vw, ti.F32, 0.5, oracle.SUM), 2.0, atol=1e-14)
    np.testing.assert_allclose(oracle.layer(Q, K, ones, Kw, Vw, ti.F32, 0.5, oracle.JOINT), 1.0, atol=1e-14)
    np.testing.assert_allclose(oracle.layer(Q, None, None, Kw, Vw, ti.F32, 0.5, oracle.SUM), 1.0, atol=1e-14)


# ---------------------------------------------------------------- invariances
def test_history_is_a_set_joint_row_permutation_changes_nothing():
    B, H, W, N, D = 1, 2, 6, 50, 8
    Q, K, V = rnd((B, H, W, D), 26, 1), rnd((B, H, N, D), 26, 2), rnd((B, H, N, D), 26, 3)
    perm = np.random.default_rng(0).permutation(N)
    O1, l1 = oracle.history(Q, K, V, ti.F32, 0.4)
    O2, l2 = oracle.history(Q, K[:, :, perm].copy(), V[:, :, perm].copy(), ti.F32, 0.4)
    np.testing.assert_allclose(O1, O2, atol=1e-14)
    np.testing.assert_allclose(l1, l2, atol=1e-14)
    # permuting K alone (not V) must change the result: the pairing matters
    O3, _ = oracle.history(Q, K[:, :, perm].copy(), V, ti.F32, 0.4)
    assert np.abs(O3 - O1).max() > 1e-3


def test_key_shift_invariance_and_lse_shift():
    B, H, W, N, D = 1, 1, 5, 30, 8
    rng = np.random.default_rng(1)
    Q = rng.integers(-3, 4, (B, H, W, D)).astype(np.float32)
    K = rng.integers(-3, 4, (B, H, N, D)).astype(np.float32)
    V = rnd((B, H, N, D), 27, 3)
    c = rng.integers(-2, 3, (D,)).astype(np.float32)
    O1, l1 = oracle.history(Q, K, V, ti.F32, 0.25)
    O2, l2 = oracle.history(Q, K + c, V, ti.F32, 0.25)    # integer data: the shift is exact
    np.testing.assert_allclose(O1, O2, atol=1e-14)
    np.testing.assert_allclose(l2 - l1, 0.25 * (Q.astype(np.float64) @ c.astype(np.float64)), atol=1e-13)


def test_scale_multiplies_logits():
    """Doubling the scale equals doubling Q (exact in binary floating point); scale 0 gives the
    mean; a large scale selects the arg-max key."""
    B, H, W, N, D = 1, 1, 4, 25, 8
    Q, K, V = rnd((B, H, W, D), 28, 1), rnd((B, H, N, D), 28, 2), rnd((B, H, N, D), 28, 3)
    O1, _ = oracle.history(Q, K, V, ti.F32, 0.6)
    O2, _ = oracle.history(2 * Q, K, V, ti.F32, 0.3)
    np.testing.assert_allclose(O1, O2, atol=1e-15)
    O0, _ = oracle.history(Q, K, V, ti.F32, 0.0)
    np.testing.assert_allclose(O0, np.broadcast_to(V.astype(np.float64).mean(2, keepdims=True), O0.shape), atol=1e-14)
    Ob, _ = oracle.history(Q, K, V, ti.F32, 1e4)
    best = np.einsum("bhid,bhjd->bhij", Q.astype(np.float64), K.astype(np.float64)).argmax(-1)
    np.testing.assert_allclose(Ob[0, 0], V.astype(np.float64)[0, 0, best[0, 0]], atol=1e-12)


def test_lse_merge_identity_over_history_partitions():
    """Attention over [K_a; K_b] equals the log-sum-exp weighted merge of the two parts."""
    B, H, W, D = 1, 2, 5, 8
    Q = rnd((B, H, W, D), 29, 1)
    K, V = rnd((B, H, 60, D), 29, 2), rnd((B, H, 60, D), 29, 3)
    O, L = oracle.history(Q, K, V, ti.F32, 0.5)
    for cut in (1, 17, 59):
        Oa, La = oracle.history(Q, K[:, :, :cut].copy(), V[:, :, :cut].copy(), ti.F32, 0.5)
        Ob, Lb = oracle.history(Q, K[:, :, cut:].copy(), V[:, :, cut:].copy(), ti.F32, 0.5)
        Lm = np.logaddexp(La, Lb)
        np.testing.assert_allclose(Lm, L, atol=1e-13)
        wa, wb = np.exp(La - Lm)[..., None], np.exp(Lb - Lm)[..., None]
        np.testing.assert_allclose(wa + wb, 1.0, atol=1e-14)
        np.testing.assert_allclose(wa * Oa + wb * Ob, O, atol=1e-13)


# ---------------------------------------------------------------- indexing
def test_heads_and_batches_are_independent_problems_and_row_subsets_match():
    B, H, W, N, D = 2, 3, 9, 21, 8
    Q, Kw, Vw = (rnd((B, H, W, D), 30, t) for t in (1, 4, 5))
    Kh, Vh = (rnd((B, H, N, D), 30, t) for t in (2, 3))
    O, L = oracle.history(Q, Kh, Vh, ti.F32, 0.3)
    Oc, Lc = oracle.window_causal(Q, Kw, Vw, ti.F32, 0.3)
    Oj = oracle.layer(Q, Kh, Vh, Kw, Vw, ti.F32, 0.3, oracle.JOINT)
    for b in range(B):
        for h in range(H):
            sl = (slice(b, b + 1), slice(h, h + 1))
            o1, l1 = oracle.history(Q[sl].copy(), Kh[sl].copy(), Vh[sl].copy(), ti.F32, 0.3)
            np.testing.assert_array_equal(o1[0, 0], O[b, h])
            np.testing.assert_array_equal(l1[0, 0], L[b, h])
            o2, _ = oracle.window_causal(Q[sl].copy(), Kw[sl].copy(), Vw[sl].copy(), ti.F32, 0.3)
            np.testing.assert_array_equal(o2[0, 0], Oc[b, h])
    rows = [8, 0, 3]
    o, l = oracle.history(Q, Kh, Vh, ti.F32, 0.3, rows=rows)
    np.testing.assert_array_equal(o, O[:, :, rows])
    np.testing.assert_array_equal(l, L[:, :, rows])
    o, l = oracle.window_causal(Q, Kw, Vw, ti.F32, 0.3, rows=rows)
    np.testing.assert_array_equal(o, Oc[:, :, rows])
    o = oracle.layer(Q, Kh, Vh, Kw, Vw, ti.F32, 0.3, oracle.JOINT, rows=rows)
    np.testing.assert_array_equal(o, Oj[:, :, rows])


def test_bf16_inputs_are_widened_exactly():
    B, H, W, N, D = 1, 1, 4, 13, 8
    Qb, Kb, Vb = rnd((B, H, W, D), 31, 1, 1.0, ti.BF16), rnd((B, H, N, D), 31, 2, 1.0, ti.BF16), rnd((B, H, N, D), 31, 3, 1.0, ti.BF16)
    O1, _ = oracle.history(Qb, Kb, Vb, ti.BF16, 0.5)
    O2, _ = oracle.history(ti.bf16_bits_to_f32(Qb), ti.bf16_bits_to_f32(Kb), ti.bf16_bits_to_f32(Vb), ti.F32, 0.5)
    np.testing.assert_array_equal(O1, O2)


def test_bad_arguments_are_rejected():
    Q, K = rnd((1, 1, 4, 8), 32, 1), rnd((1, 1, 6, 8), 32, 2)
    with pytest.raises(RuntimeError):
        oracle.history(Q, K, K, ti.F32, 0.5, rows=[4])
    with pytest.raises(TypeError):
        oracle.history(Q.astype(np.float64), K, K, ti.F32, 0.5)
