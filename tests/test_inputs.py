"""The seeded input generator: determinism, distribution, bf16 rounding, peaky rows."""
import numpy as np
import torch

import tlin_inputs as ti


def test_deterministic_and_counter_based():
    a = ti.normal((3, 50, 16), ti.F32, 7, ti.TAG_KH)
    b = ti.normal((3, 50, 16), ti.F32, 7, ti.TAG_KH)
    np.testing.assert_array_equal(a, b)
    # a prefix of a longer draw is the same stream: values depend on (seed, tag, index) only
    c = ti.normal((6, 50, 16), ti.F32, 7, ti.TAG_KH)
    np.testing.assert_array_equal(a, c[:3])
    assert not np.array_equal(a, ti.normal((3, 50, 16), ti.F32, 8, ti.TAG_KH))
    assert not np.array_equal(a, ti.normal((3, 50, 16), ti.F32, 7, ti.TAG_VH))


def test_standard_normal_moments():
    a = ti.normal((1 << 20,), ti.F32, 3, 1).astype(np.float64)
    assert abs(a.mean()) < 5e-3 and abs(a.std() - 1) < 5e-3
    assert abs((a ** 3).mean()) < 2e-2 and abs((a ** 4).mean() - 3) < 5e-2
    assert np.isfinite(a).all()
    b = ti.normal((1 << 16,), ti.F32, 3, 1, 0.5)
    np.testing.assert_array_equal(b, a[: 1 << 16].astype(np.float32) * np.float32(0.5))


def test_bf16_is_round_to_nearest_even_of_the_f32_stream():
    a = ti.normal((4096, 8), ti.F32, 5, 2)
    b = ti.normal((4096, 8), ti.BF16, 5, 2)
    ref = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(b, ref)
    np.testing.assert_array_equal(ti.f32_to_bf16_bits(a), ref)
    np.testing.assert_array_equal(ti.bf16_bits_to_f32(b), torch.from_numpy(a).to(torch.bfloat16).float().numpy())


def test_peaky_rows_are_about_one_percent_and_scaled_by_eight():
    plain = ti.normal((2, 5000, 16), ti.F32, 9, ti.TAG_KH)
    peaky = ti.normal((2, 5000, 16), ti.F32, 9, ti.TAG_KH, 1.0, 100, 8.0)
    ratio = peaky / plain
    is8 = np.isclose(ratio, 8.0).all(-1)
    is1 = np.isclose(ratio, 1.0).all(-1)
    assert (is8 | is1).all()
    assert 0.005 < is8.mean() < 0.015


def test_workload_table():
    w = ti.config(3)
    assert (w.B, w.H, w.D, w.N, w.W, w.dtype) == (1, 32, 128, 131072, 512, ti.BF16)
    assert abs(w.flops_history() - 1.0995e12) < 1e9
    assert ti.config(0).dtype == ti.F32 and ti.config(2).peaky_mod == 100
    small = ti.shrink(ti.config(2), B=1, H=1, N=256, W=32)
    t = ti.make(small)
    assert t["Kh"].shape == (1, 1, 256, 128) and t["Q"].shape == (1, 1, 32, 128) and t["Kh"].dtype == np.uint16
    assert len(ti.sweep_points()) == 8 and ti.degenerate_causal().N == 0


def test_points_after_the_fixed_configs():
    d, r, p, f = ti.decode_point(131072, 1), ti.restore_point(131072, 256), ti.paper_model_point(1000000), ti.f32_point(32768)
    assert (d.W, d.N, d.dtype) == (1, 131072, ti.BF16)
    assert (r.W, r.N) == (131072, 256)                      # the query side is the long one
    assert (p.H, p.D, p.W) == (12, 36, 256)                 # the paper's model: width 432 in 12 heads
    assert (f.H, f.D, f.N, f.W, f.dtype) == (32, 128, 32768, 512, ti.F32)
    assert len({w.seed for w in (d, r, p, f, ti.config(3))}) == 5
