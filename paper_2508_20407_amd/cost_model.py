"""The paper's cost model (Section 4, Appendix A), in its own unit: one unit = one length-D
multiply-accumulate row, so an attention of `q` query rows over `k` key rows costs D*q*k.

Real flops of the library's kernels are 4 units' worth per (query, key) pair and head dimension
element: two products (Q K^T and P V) at two flops per multiply-accumulate.
"""
from __future__ import annotations


def cache_miss_parts(N: int, W_oh: int, W_og: int, H: int, D: int) -> dict:
    """Terms of a full forward pass of one block (Appendix A, cache miss).  N is the total
    sequence length; the history has N - W_og rows."""
    hist = N - W_og
    return {
        # context window ("left")
        "context_focused_over_history": D * hist * W_oh,          # first layer: W_oh queries x history
        "context_self": H * D * W_oh * W_oh,                      # H intermediate layers
        "context_restoration": D * hist * W_oh,                   # last layer: history queries x W_oh keys
        # generation window ("right")
        "generation_cross_over_history": D * W_og * hist,         # first cross attention
        "generation_cross_over_context": (H + 1) * D * W_og * W_oh,
        "generation_causal": (H + 2) * D * W_og * W_og,
    }


def cache_miss_total(N: int, W_oh: int, W_og: int, H: int, D: int) -> int:
    """Closed form of the cache-miss cost (Section 4.1, equation (4))."""
    return D * (N * (2 * W_oh + W_og) + H * (W_oh * W_oh + W_og * W_og + W_og * W_oh) + W_og * W_og - W_og * W_oh)


def slope_intercept(W_oh: int, W_og: int, H: int, D: int) -> tuple:
    """C_1 and C_0 of Total = C_1 * N + C_0 (Section 4.1, equations (2) and (3))."""
    return (D * (2 * W_oh + W_og),
            D * (H * (W_oh * W_oh + W_og * W_og + W_og * W_oh) + W_og * W_og - W_og * W_oh))


def cache_hit_total(N: int, W_oh: int, W_og: int, H: int, D: int) -> int:
    """Cost of a step that reuses the cached context (Section 4.2, equation (5)): only the newest
    row queries the history and the context."""
    return D * N - D * W_og + (H + 1) * D * W_oh + (H + 2) * D * W_og * W_og


def history_flops(B: int, heads: int, W: int, N_hist: int, head_dim: int) -> float:
    """Flops of tlin_history_attn: the D*W*N_hist term of the model with D = heads * head_dim,
    four flops per unit."""
    return 4.0 * B * heads * head_dim * W * N_hist
