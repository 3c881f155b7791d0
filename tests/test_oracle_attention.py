"""Pins of oracle/attention.py: facts the definition fixes, none of them a re-typing of its formula."""
import numpy as np

from oracle import attention as A
from oracle import nets
from synth import CONFIGS, make_workload


def _rand(B, T, H, dh, seed):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((B, T, 3 * H * dh))


def test_probabilities_sum_to_one_and_constant_values_pass_through():
    B, T, H, dh = 2, 7, 3, 4
    qkv = _rand(B, T, H, dh, 0)
    D = H * dh
    qkv[..., 2 * D:] = np.arange(D)[None, None, :]          # every token carries the same value vector
    out, lse, p = A.attention_forward(qkv, H)
    np.testing.assert_allclose(p.sum(axis=-1), 1.0, rtol=0, atol=1e-14)
    np.testing.assert_allclose(out, np.broadcast_to(np.arange(D, dtype=float), out.shape), rtol=0, atol=1e-12)


def test_equal_keys_give_the_mean_of_the_values_and_lse_of_log_T():
    B, T, H, dh = 1, 5, 2, 4
    qkv = _rand(B, T, H, dh, 1)
    D = H * dh
    qkv[..., D:2 * D] = 0.0                                 # all scores zero: uniform attention
    out, lse, _ = A.attention_forward(qkv, H)
    np.testing.assert_allclose(out, np.broadcast_to(qkv[..., 2 * D:].mean(axis=1, keepdims=True), out.shape), atol=1e-13)
    np.testing.assert_allclose(lse, np.log(T), atol=1e-13)


def test_one_dominant_key_is_selected_and_lse_is_its_score():
    B, T, H, dh = 1, 4, 1, 4
    qkv = np.zeros((B, T, 3 * dh))
    qkv[0, :, 0] = 1.0                                      # every query = e0
    qkv[0, 2, dh] = 400.0                                   # key 2 = 400 e0, others 0: score 200 against 0
    qkv[0, :, 2 * dh:] = np.arange(T * dh).reshape(T, dh)
    out, lse, _ = A.attention_forward(qkv, 1)
    np.testing.assert_allclose(out[0], np.broadcast_to(qkv[0, 2, 2 * dh:], (T, dh)), atol=1e-12)
    np.testing.assert_allclose(lse, 200.0, atol=1e-12)


def test_backward_matches_central_differences():
    B, T, H, dh = 2, 5, 2, 4
    qkv = _rand(B, T, H, dh, 2)
    rng = np.random.default_rng(3)
    dout = rng.standard_normal((B, T, H * dh))
    g = A.attention_backward(qkv, dout, H)
    f = lambda z: float((A.attention_forward(z, H)[0] * dout).sum())
    h = 1e-6
    for idx in [(0, 0, 0), (1, 4, 7), (0, 2, 8), (1, 1, 15), (0, 3, 16), (1, 0, 23), (0, 4, 11), (1, 2, 3)]:
        zp, zm = qkv.copy(), qkv.copy()
        zp[idx] += h
        zm[idx] -= h
        fd = (f(zp) - f(zm)) / (2 * h)
        assert abs(fd - g[idx]) <= 1e-7 * max(1.0, abs(fd)), (idx, fd, g[idx])


def test_backward_of_a_sum_over_queries_sends_nothing_to_the_scores_when_values_are_constant():
    # with identical value rows the output does not depend on Q or K at all
    B, T, H, dh = 1, 6, 2, 4
    qkv = _rand(B, T, H, dh, 4)
    D = H * dh
    qkv[..., 2 * D:] = 3.0
    g = A.attention_backward(qkv, np.ones((B, T, D)), H)
    np.testing.assert_allclose(g[..., :2 * D], 0.0, atol=1e-13)
    # and every value row receives the column sums of the probabilities: they add up to T per head dimension
    np.testing.assert_allclose(g[..., 2 * D:].sum(axis=1), T, atol=1e-12)


def test_agrees_with_the_attention_inside_the_vit_oracle():
    cfg = CONFIGS["vit_tiny"]
    wl = make_workload(cfg, seed=0, init="random")
    _, c = nets.vit_forward(cfg, wl.weights, wl.x, wl.y)
    blk = c["blocks"][0]
    B, T, D, H, dh, L, scale = c["dims"]
    merge = lambda a: a.transpose(0, 2, 1, 3).reshape(B, T, D)
    qkv = np.concatenate([merge(blk[n]) for n in ("q", "k", "v")], axis=-1)
    out, _, p = A.attention_forward(qkv, H)
    np.testing.assert_allclose(out, blk["o"], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(p, blk["p"], rtol=1e-12, atol=1e-15)
