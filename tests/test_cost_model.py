"""The cost model of Section 4 / Appendix A: the closed forms equal the sums of their parts, the
cost is exactly linear in N, and the library's flop accounting is the model's N-dependent term."""
import random

import tlin_inputs as ti
from paper_2508_20407_amd import cost_model as cm


def cases():
    rng = random.Random(2508)
    out = [(1_000_000, 256, 256, 2, 432), (4096, 512, 512, 0, 64), (513, 1, 512, 3, 8)]
    for _ in range(50):
        W_og = rng.randint(1, 700)
        out.append((W_og + rng.randint(0, 100000), rng.randint(1, 700), W_og, rng.randint(0, 6), rng.randint(1, 512)))
    return out


def test_cache_miss_closed_form_is_the_sum_of_the_appendix_terms():
    for N, W_oh, W_og, H, D in cases():
        parts = cm.cache_miss_parts(N, W_oh, W_og, H, D)
        assert sum(parts.values()) == cm.cache_miss_total(N, W_oh, W_og, H, D)
        left = parts["context_focused_over_history"] + parts["context_self"] + parts["context_restoration"]
        assert left == 2 * D * (N - W_og) * W_oh + H * D * W_oh * W_oh            # Appendix A, C_left


def test_cost_is_linear_in_N_with_the_stated_slope_and_intercept():
    for N, W_oh, W_og, H, D in cases():
        c1, c0 = cm.slope_intercept(W_oh, W_og, H, D)
        assert cm.cache_miss_total(N, W_oh, W_og, H, D) == c1 * N + c0
        assert cm.cache_miss_total(N + 10_000, W_oh, W_og, H, D) - cm.cache_miss_total(N, W_oh, W_og, H, D) == 10_000 * c1


def test_cache_hit_is_the_last_row_only_and_its_slope_is_D():
    for N, W_oh, W_og, H, D in cases():
        hit = cm.cache_hit_total(N, W_oh, W_og, H, D)
        assert hit == D * (N - W_og) + (H + 1) * D * W_oh + (H + 2) * D * W_og * W_og   # Appendix A, C_right
        assert cm.cache_hit_total(N + 1, W_oh, W_og, H, D) - hit == D
        c1, _ = cm.slope_intercept(W_oh, W_og, H, D)
        assert c1 == D * (2 * W_oh + W_og) and c1 >= 3 * D        # a miss costs 2 W_oh + W_og times more per row


def test_library_flop_accounting_is_the_history_term_of_the_model():
    w = ti.config(3)                                               # 32 heads x 128, W = 512, 131072 history rows
    D_model = w.H * w.D
    parts = cm.cache_miss_parts(w.N + w.W, 256, w.W, 2, D_model)
    assert cm.history_flops(w.B, w.H, w.W, w.N, w.D) == 4.0 * w.B * parts["generation_cross_over_history"]
    assert w.flops_history() == cm.history_flops(w.B, w.H, w.W, w.N, w.D)
    # the three N-dependent terms are exactly the shapes the library serves: W_oh or W_og queries over
    # the history (tlin_history_attn) and the history's rows over W_oh keys (the restoration shape)
    n_terms = parts["context_focused_over_history"] + parts["context_restoration"] + parts["generation_cross_over_history"]
    c1, _ = cm.slope_intercept(256, w.W, 2, D_model)
    assert n_terms == c1 * w.N
