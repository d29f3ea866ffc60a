"""Shared helpers for the GPU parity tests: upload seeded inputs, compare with the oracle."""
import numpy as np
import torch

import tlin_inputs as ti

# Tolerances.  fp32 path: max |g-r| / max(|r|, rms(r)) <= 1e-5 (outputs are averages and can be
# arbitrarily close to zero, so the denominator is floored at the tensor's rms).  bf16 path
# (bf16 inputs, fp32 accumulation, bf16 weights and outputs): max abs <= 2e-2, mean abs <= 5e-3.
F32_REL = 1e-5
BF16_MAX_ABS = 2e-2
BF16_MEAN_ABS = 5e-3
# The absolute bounds say little when the outputs themselves are tiny (near-uniform softmax over
# small values), so the bf16 path must also meet a scale-free bound: rms error <= 1% of the rms
# of the reference.  Rounding the weights and the output to bf16 (relative error up to 2^-8 each,
# random sign) gives about 0.2-0.4%.
BF16_REL_RMS = 1e-2


def to_device(a: np.ndarray, dtype: int) -> torch.Tensor:
    if dtype == ti.F32:
        return torch.from_numpy(a).cuda()
    return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)


def upload(host: dict, dtype: int) -> dict:
    return {k: to_device(v, dtype) for k, v in host.items()}


def to_host64(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def rel_err_f32(g: np.ndarray, r: np.ndarray) -> float:
    rms = float(np.sqrt(np.mean(r * r)))
    return float(np.max(np.abs(g - r) / np.maximum(np.abs(r), rms)))


def f32_rel_bound(max_logit_nats: float) -> float:
    """Accuracy envelope of the fp32 path.  A logit is a 128-term fp32 sum and carries an
    absolute rounding error of a few 2^-24 of its own size (measured: up to 3 units of
    2^-24 * sum|q_i k_i|), which the exponential turns into the same amount of RELATIVE error in
    the weight.  Up to 10 nats of logit magnitude that stays inside 1e-5; beyond, the bound
    grows with the magnitude: 1e-6 per nat."""
    return F32_REL * max(1.0, max_logit_nats / 10.0)


def assert_close(g, r, dtype: int, what: str = "", lse: bool = False, f32_rel: float = F32_REL):
    g = to_host64(g) if isinstance(g, torch.Tensor) else np.asarray(g, dtype=np.float64)
    assert g.shape == r.shape, (g.shape, r.shape)
    assert np.isfinite(g).all(), f"{what}: non-finite output"
    if dtype == ti.F32:
        e = rel_err_f32(g, r)
        big = np.abs(r) > np.sqrt(np.mean(r * r))
        plain = float(np.max(np.abs(g - r)[big] / np.abs(r[big]))) if big.any() else 0.0
        assert e <= f32_rel, (f"{what}: fp32 relative error {e:.3e} > {f32_rel} (denominator floored at the rms; "
                              f"unfloored over |r| > rms: {plain:.3e})")
        assert plain <= f32_rel, f"{what}: fp32 relative error over |r| > rms {plain:.3e} > {f32_rel}"
    else:
        d = np.abs(g - r)
        assert d.max() <= BF16_MAX_ABS, f"{what}: bf16 max abs error {d.max():.3e} > {BF16_MAX_ABS}"
        assert d.mean() <= BF16_MEAN_ABS, f"{what}: bf16 mean abs error {d.mean():.3e} > {BF16_MEAN_ABS}"
        rr = float(np.sqrt(np.mean(d * d)) / max(np.sqrt(np.mean(r * r)), 1e-30))
        assert rr <= BF16_REL_RMS, f"{what}: bf16 rms error is {rr:.3e} of the reference rms > {BF16_REL_RMS}"


def sample_rows(W: int, k: int, seed: int = 0) -> np.ndarray:
    """First, last and k-2 seeded rows (sorted, unique)."""
    rng = np.random.default_rng(seed)
    rows = {0, W - 1}
    while len(rows) < min(k, W):
        rows.add(int(rng.integers(0, W)))
    return np.array(sorted(rows), dtype=np.int32)


def stratified_rows(W: int, block: int = 32) -> np.ndarray:
    """First and last row of every `block`-row group of the window.  A wave of the matrix-core
    kernels owns 32 consecutive query rows, so this looks at every wave of every query block of
    the launch (W = 512: 32 rows)."""
    rows = set()
    for r0 in range(0, W, block):
        rows.add(r0)
        rows.add(min(r0 + block, W) - 1)
    return np.array(sorted(rows), dtype=np.int32)
