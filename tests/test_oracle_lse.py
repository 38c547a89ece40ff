"""Pins of the oracle's one-sweep scores from a given row log-sum-exp (the by-product of a
flash-style prefill attention kernel)."""
import numpy as np
import torch

from oracle import ta_oracle as ora


def _rand(rng, shape):
    t = torch.tensor(rng.standard_normal(shape).astype(np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16), t.to(torch.float64)


def test_row_lse_equals_torch_logsumexp_with_the_causal_mask():
    rng = np.random.default_rng(1)
    G, W, n, d = 2, 5, 37, 16
    Qb, Q = _rand(rng, (G, W, d))
    Kb, K = _rand(rng, (n, d))
    S = torch.einsum("gwd,nd->gwn", Q, K) / d ** 0.5
    for causal in (True, False):
        ref = torch.empty(G, W, dtype=torch.float64)
        for w in range(W):
            last = n - W + w if causal else n - 1
            ref[:, w] = torch.logsumexp(S[:, w, :last + 1], dim=-1)
        assert np.allclose(ora.row_lse(Qb, Kb, causal), ref.numpy(), rtol=0, atol=1e-6)
    # a window longer than the context: the first rows see nothing
    lse = ora.row_lse(Qb, Kb[:3], True)
    assert np.all(np.isneginf(lse[:, :2])) and np.all(np.isfinite(lse[:, 2:]))


def test_scores_from_lse_agree_with_the_two_pass_scores_and_sum_to_the_row_count():
    rng = np.random.default_rng(2)
    G, W, n, d = 4, 8, 300, 128
    Qb, _ = _rand(rng, (G, W, d))
    Kb, _ = _rand(rng, (n, d))
    for causal in (True, False):
        A = ora.score(Qb, Kb, causal)
        A2 = ora.score_lse(Qb, Kb, ora.row_lse(Qb, Kb, causal), causal)
        # the only difference is the rounding of lse to fp32: |lse| * 2^-24 relative
        assert np.all(np.abs(A2 - A) <= 2e-6 * np.abs(A) + 1e-12)
        assert abs(float(A2.astype(np.float64).sum()) - G * W) < 1e-3


def test_closed_form_equal_keys_and_shifted_lse():
    # all keys equal: every visible key gets 1 / (visible count); lse = s + log(count)
    G, W, n, d = 1, 3, 10, 8
    one = np.full((n, d), 0x3F80, np.uint16)                   # 1.0
    q = np.full((G, W, d), 0x3F80, np.uint16)
    lse = ora.row_lse(q, one, True)
    s = d / np.sqrt(d)
    assert np.allclose(lse[0], [s + np.log(8), s + np.log(9), s + np.log(10)], atol=1e-6)
    A = ora.score_lse(q, one, lse, True)
    expect = np.array([1 / 8 + 1 / 9 + 1 / 10] * 8 + [1 / 9 + 1 / 10, 1 / 10])
    assert np.allclose(A, expect, atol=1e-6)
    # an lse that is larger by log 2 halves every weight (the normaliser is taken, not recomputed)
    A_half = ora.score_lse(q, one, lse + np.float32(np.log(2.0)), True)
    assert np.allclose(A_half, expect / 2, atol=1e-6)
