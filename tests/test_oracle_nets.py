"""Pins of the oracle's forward/backward pass against things other than itself:
central finite differences of its own loss, PyTorch's CPU autograd over library
ops, and the invariants of selective training (Section 2.2)."""
import itertools

import numpy as np
import pytest
import torch

from oracle import nets
from synth import CONFIGS, make_workload, tensor_specs


def _fd(cfg, wl, k, idx, h=1e-5):
    W = [w.astype(np.float64) for w in wl.weights]
    W[k] = W[k].copy()
    old = W[k][idx]
    W[k][idx] = old + h
    lp, _ = nets.forward(cfg, W, wl.x, wl.y)
    W[k][idx] = old - h
    lm, _ = nets.forward(cfg, W, wl.x, wl.y)
    return (lp - lm) / (2 * h)


@pytest.mark.parametrize("name", ["mlp_tiny", "vit_tiny"])
def test_gradients_match_finite_differences(name):
    cfg = CONFIGS[name]
    wl = make_workload(cfg, seed=3, init="random")
    N = len(wl.weights)
    r = nets.step(cfg, wl.weights, wl.x, wl.y, [1] * N)
    rng = np.random.default_rng(0)
    for k in range(N):
        g = r["grads"][k]
        assert g.shape == wl.weights[k].shape
        for _ in range(6):
            idx = tuple(int(rng.integers(0, s)) for s in g.shape)
            fd = _fd(cfg, wl, k, idx)
            assert abs(fd - g[idx]) <= 1e-6 * max(1.0, abs(fd)), (wl.names[k], idx, fd, g[idx])


def _torch_vit_loss(cfg, W, x, y):
    """The same network built from PyTorch library ops (float64, autograd)."""
    F = torch.nn.functional
    B, T, D, H, dh = x.shape[0], cfg.tokens, cfg.width, cfg.heads, cfg.head_dim
    e = F.linear(x, W[0], W[1])
    h = torch.cat([W[2].expand(B, 1, D), e], dim=1) + W[3]
    for l in range(cfg.blocks):
        g1, b1, Wqkv, bqkv, Wo, bo, g2, b2, W1, c1, W2, c2 = W[4 + 12 * l: 16 + 12 * l]
        a = F.layer_norm(h, (D,), g1, b1, cfg.ln_eps)
        q, k, v = F.linear(a, Wqkv, bqkv).reshape(B, T, 3, H, dh).permute(2, 0, 3, 1, 4)
        o = F.scaled_dot_product_attention(q, k, v).transpose(1, 2).reshape(B, T, D)
        h = h + F.linear(o, Wo, bo)
        a = F.layer_norm(h, (D,), g2, b2, cfg.ln_eps)
        h = h + F.linear(F.gelu(F.linear(a, W1, c1)), W2, c2)
    z = F.layer_norm(h[:, 0], (D,), W[-4], W[-3], cfg.ln_eps)
    return F.cross_entropy(F.linear(z, W[-2], W[-1]), y)


@pytest.mark.parametrize("name", ["vit_tiny", "vit_small"])
def test_vit_matches_torch_autograd(name):
    cfg = CONFIGS[name]
    wl = make_workload(cfg, seed=5, init="random")
    N = len(wl.weights)
    r = nets.step(cfg, wl.weights, wl.x, wl.y, [1] * N)
    W = [torch.tensor(w, dtype=torch.float64, requires_grad=True) for w in wl.weights]
    loss = _torch_vit_loss(cfg, W, torch.tensor(wl.x, dtype=torch.float64), torch.tensor(wl.y, dtype=torch.long))
    loss.backward()
    assert abs(loss.item() - r["loss"]) <= 1e-12 * abs(loss.item())
    for k in range(N):
        ref = W[k].grad.numpy()
        err = np.linalg.norm(r["grads"][k] - ref) / max(np.linalg.norm(ref), 1e-300)
        assert err <= 1e-10, (wl.names[k], err)


def test_mlp_matches_torch_autograd():
    cfg = CONFIGS["mlp"]
    wl = make_workload(cfg, seed=0)
    r = nets.step(cfg, wl.weights, wl.x, wl.y, [1] * 4)
    W = [torch.tensor(w, dtype=torch.float64, requires_grad=True) for w in wl.weights]
    a = torch.tensor(wl.x, dtype=torch.float64)
    for i, w in enumerate(W):
        a = a @ w.T
        if i < 3:
            a = torch.relu(a)
    loss = torch.nn.functional.cross_entropy(a, torch.tensor(wl.y, dtype=torch.long))
    loss.backward()
    assert abs(loss.item() - r["loss"]) <= 1e-12
    for k in range(4):
        np.testing.assert_allclose(r["grads"][k], W[k].grad.numpy(), rtol=1e-10, atol=1e-14)


def test_all_16_masks_of_the_mlp():
    """A selected tensor's gradient does not depend on what else is selected; the
    all-ones mask is full backpropagation; the empty mask does no backward work."""
    cfg = CONFIGS["mlp"]
    wl = make_workload(cfg, seed=0)
    full = nets.step(cfg, wl.weights, wl.x, wl.y, [1, 1, 1, 1])
    assert sorted(full["work"]) == sorted([("dw", j) for j in range(4)] + [("dy", j) for j in (1, 2, 3)])
    for mask in itertools.product([0, 1], repeat=4):
        r = nets.step(cfg, wl.weights, wl.x, wl.y, mask)
        assert r["loss"] == full["loss"]
        for k in range(4):
            if mask[k]:
                assert np.array_equal(r["grads"][k], full["grads"][k])
            else:
                assert r["grads"][k] is None
        if not any(mask):
            assert r["work"] == []


def test_section_2_2_worked_example():
    """Five layers, only layer 3 selected: the executed backward work is the weight
    gradient of layer 3 and the gradient passing of layers 4 and 5, nothing else."""
    cfg = CONFIGS["mlp5"]
    wl = make_workload(cfg, seed=1)
    r = nets.step(cfg, wl.weights, wl.x, wl.y, [0, 0, 1, 0, 0])
    assert sorted(r["work"]) == [("dw", 2), ("dy", 3), ("dy", 4)]


def test_executed_work_is_selected_dw_plus_dy_after_the_input_most_selected():
    cfg = CONFIGS["vit_tiny"]
    wl = make_workload(cfg, seed=2, init="random")
    N = len(wl.weights)
    assert N == len(tensor_specs(cfg)) == 4 + 12 * cfg.blocks + 4
    full = nets.step(cfg, wl.weights, wl.x, wl.y, [1] * N)
    rng = np.random.default_rng(7)
    for _ in range(25):
        mask = (rng.random(N) < rng.choice([0.05, 0.3, 0.8])).astype(int)
        r = nets.step(cfg, wl.weights, wl.x, wl.y, mask)
        sel = [j for j in range(N) if mask[j]]
        dw = sorted(j for op, j in r["work"] if op == "dw")
        dy = sorted(j for op, j in r["work"] if op == "dy")
        assert dw == sel
        assert dy == (list(range(sel[0] + 1, N)) if sel else [])
        for j in sel:
            assert np.array_equal(r["grads"][j], full["grads"][j])
