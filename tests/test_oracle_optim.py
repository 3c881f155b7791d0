"""Pins of the oracle's optimizer formulas against PyTorch's optimizers and closed forms."""
import numpy as np
import torch

from oracle import optim


def test_adam_matches_torch():
    rng = np.random.default_rng(0)
    w0 = rng.standard_normal(50)
    p = torch.tensor(w0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([p], lr=1e-2, betas=(0.9, 0.999), eps=1e-8)
    w, m, v = w0.copy(), np.zeros(50), np.zeros(50)
    for t in range(1, 6):
        g = rng.standard_normal(50)
        p.grad = torch.tensor(g)
        opt.step()
        w, m, v = optim.adam(w, m, v, g, 1e-2, 0.9, 0.999, 1e-8, t)
        np.testing.assert_allclose(w, p.detach().numpy(), rtol=1e-12, atol=1e-15)


def test_sgdw_momentum_matches_torch_and_decay_closed_form():
    rng = np.random.default_rng(1)
    w0 = rng.standard_normal(40)
    p = torch.tensor(w0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([p], lr=1e-2, momentum=0.9)
    w, m = w0.copy(), np.zeros(40)
    for _ in range(5):
        g = rng.standard_normal(40)
        p.grad = torch.tensor(g)
        opt.step()
        w, m = optim.sgdw(w, m, g, 1e-2, 0.9, 0.0)
        np.testing.assert_allclose(w, p.detach().numpy(), rtol=1e-12, atol=1e-15)
    # zero gradient: pure decoupled decay, w_t = w_0 (1 - lr wd)^t
    w, m = w0.copy(), np.zeros(40)
    for _ in range(7):
        w, m = optim.sgdw(w, m, np.zeros(40), 0.1, 0.9, 0.05)
    np.testing.assert_allclose(w, w0 * (1 - 0.1 * 0.05) ** 7, rtol=1e-13)


def test_masked_update_leaves_unselected_alone():
    rng = np.random.default_rng(2)
    W = [rng.standard_normal(5) for _ in range(3)]
    S = [(np.zeros(5), np.zeros(5)) for _ in range(3)]
    G = [rng.standard_normal(5) for _ in range(3)]
    nw, ns = optim.masked_update("adam", [1, 0, 1], W, S, G, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, step=1)
    assert nw[1] is W[1] and ns[1] is S[1]
    assert not np.array_equal(nw[0], W[0]) and not np.array_equal(nw[2], W[2])
    # first Adam step moves every weight by lr * sign(g) (up to eps)
    np.testing.assert_allclose(nw[0], W[0] - 1e-3 * np.sign(G[0]), atol=1e-9)
