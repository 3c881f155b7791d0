"""Pins of the oracle's tensor importance (Eq. 2) against the Taylor expansion it
approximates (Eq. 6), a library norm, and additivity."""
import numpy as np
import pytest

from oracle import importance as imp
from oracle import nets
from synth import CONFIGS, make_workload


@pytest.mark.parametrize("name", ["mlp_tiny", "vit_tiny"])
def test_first_order_taylor_term(name):
    """sum_k I_k equals L(w + dw) - L(w) up to a second-order remainder: halving dw
    divides the gap by four."""
    cfg = CONFIGS[name]
    wl = make_workload(cfg, seed=11, init="random")
    W = [w.astype(np.float64) for w in wl.weights]
    rng = np.random.default_rng(1)
    # the ReLU net is only piecewise smooth: stay inside one linear region
    base = 0.004 if cfg.kind == "vit" else 0.001
    D = [base * rng.standard_normal(w.shape) for w in W]
    L0, _ = nets.forward(cfg, W, wl.x, wl.y)
    gaps = []
    for scale in (1.0, 0.5, 0.25):
        snap = [w + scale * d for w, d in zip(W, D)]
        I, _ = imp.importance(cfg, W, snap, wl.x, wl.y)
        L1, _ = nets.forward(cfg, snap, wl.x, wl.y)
        gaps.append(abs((L1 - L0) - I.sum()))
    assert 3.0 < gaps[0] / gaps[1] < 6.0 and 3.0 < gaps[1] / gaps[2] < 6.0, gaps


def test_descent_step_gives_minus_lr_times_squared_norm():
    cfg = CONFIGS["vit_tiny"]
    wl = make_workload(cfg, seed=4, init="random")
    W = [w.astype(np.float64) for w in wl.weights]
    g = nets.step(cfg, W, wl.x, wl.y, [1] * len(W))["grads"]
    lr = 1e-3
    snap = [w - lr * gk for w, gk in zip(W, g)]
    I, _ = imp.importance(cfg, W, snap, wl.x, wl.y)
    ref = np.array([-lr * np.linalg.norm(gk.ravel()) ** 2 for gk in g])
    np.testing.assert_allclose(I, ref, rtol=1e-9, atol=1e-18)


def test_sign_reading_positive_when_snapshot_is_the_pre_update_point():
    """With the snapshot taken before a loss-reducing step, importance is positive
    and approximates the loss that undoing the step would give back."""
    cfg = CONFIGS["mlp_tiny"]
    wl = make_workload(cfg, seed=9)
    W0 = [w.astype(np.float64) for w in wl.weights]
    g0 = nets.step(cfg, W0, wl.x, wl.y, [1] * len(W0))["grads"]
    W1 = [w - 1e-3 * g for w, g in zip(W0, g0)]            # the recent update
    I, _ = imp.importance(cfg, W1, W0, wl.x, wl.y)          # snapshot = weights before it
    L0, _ = nets.forward(cfg, W0, wl.x, wl.y)
    L1, _ = nets.forward(cfg, W1, wl.x, wl.y)
    assert np.all(I > 0)
    assert abs(I.sum() - (L0 - L1)) < 0.05 * (L0 - L1)


def test_additivity_over_a_split_tensor():
    rng = np.random.default_rng(3)
    g, w, s = (rng.standard_normal(1000) for _ in range(3))
    whole = imp.importance_from_grads([g], [w], [s])[0]
    parts = imp.importance_from_grads([g[:300], g[300:]], [w[:300], w[300:]], [s[:300], s[300:]])
    assert abs(whole - parts.sum()) <= 1e-12 * imp.abs_importance_from_grads([g], [w], [s])[0]
    perm = rng.permutation(1000)
    assert abs(whole - imp.importance_from_grads([g[perm]], [w[perm]], [s[perm]])[0]) <= 1e-11


def test_magnitude_metrics_are_l1_norms():
    rng = np.random.default_rng(5)
    tensors = [rng.standard_normal((7, 5)), rng.standard_normal(11) * 3.0, np.zeros(4)]
    want = [np.linalg.norm(t.ravel(), 1) for t in tensors]
    assert np.allclose(imp.weight_magnitude(tensors), want, rtol=1e-14, atol=0)
    assert np.allclose(imp.grad_magnitude(tensors), want, rtol=1e-14, atol=0)
    # not additive in the sense of Section 4: the sign of an update does not matter to them
    assert np.array_equal(imp.weight_magnitude([-t for t in tensors]), imp.weight_magnitude(tensors))
