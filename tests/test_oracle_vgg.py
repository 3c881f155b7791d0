"""Pins of the oracle's plain convolution stack (VGG family): finite differences, PyTorch CPU autograd
over library convolution / pooling / linear ops, and the executed-work invariants of selective training."""
import numpy as np
import pytest
import torch

from oracle import nets
from oracle import resnet as R
from oracle import vgg as V
from synth import CONFIGS, make_workload, tensor_specs


def test_tensor_count_of_vgg16():
    specs = tensor_specs(CONFIGS["vgg16"])
    assert len(specs) == 32                                    # 13 convolutions + 3 linear layers, Kernel and Bias each
    assert specs[26] == ("fc0.W", (4096, 7 * 7 * 512))


def test_gradients_match_finite_differences():
    cfg = CONFIGS["vgg_tiny"]
    wl = make_workload(cfg, seed=3, init="random")
    N = len(wl.weights)
    r = nets.step(cfg, wl.weights, wl.x, wl.y, [1] * N)
    rng = np.random.default_rng(0)
    h = 1e-6
    ok = total = 0
    for k in range(N):
        g = r["grads"][k]
        assert g.shape == wl.weights[k].shape
        for _ in range(6):
            idx = tuple(rng.integers(0, s) for s in g.shape)
            wp = [w.astype(np.float64).copy() for w in wl.weights]
            wm = [w.astype(np.float64).copy() for w in wl.weights]
            wp[k][idx] += h
            wm[k][idx] -= h
            fd = (nets.forward(cfg, wp, wl.x, wl.y)[0] - nets.forward(cfg, wm, wl.x, wl.y)[0]) / (2 * h)
            total += 1
            ok += abs(fd - g[idx]) <= 1e-6 * max(1.0, abs(fd))
    assert ok >= 0.95 * total, (ok, total)                     # a step across a ReLU / pooling kink may miss


def _torch_grads(cfg, wl):
    import torch.nn.functional as F
    W = [torch.tensor(w, dtype=torch.float64, requires_grad=True) for w in wl.weights]
    h = torch.tensor(wl.x, dtype=torch.float64).permute(0, 3, 1, 2)
    t = 0
    for n in cfg.convs:
        for _ in range(n):
            h = F.relu(F.conv2d(h, W[t].permute(0, 3, 1, 2), W[t + 1], padding=1))
            t += 2
        h = F.max_pool2d(h, 2)
    a = h.permute(0, 2, 3, 1).reshape(h.shape[0], -1)          # (h, w, c) order
    n_fc = len(cfg.fc) + 1
    for j in range(n_fc):
        a = F.linear(a, W[t], W[t + 1])
        if j + 1 < n_fc:
            a = F.relu(a)
        t += 2
    loss = F.cross_entropy(a, torch.tensor(wl.y, dtype=torch.long))
    loss.backward()
    return float(loss), [w.grad.numpy() for w in W], a.detach().numpy()


@pytest.mark.parametrize("name,seed", [("vgg_tiny", 0), ("vgg_small", 1)])
def test_matches_torch_autograd(name, seed):
    cfg = CONFIGS[name]
    wl = make_workload(cfg, seed=seed, init="random")
    N = len(wl.weights)
    r = nets.step(cfg, wl.weights, wl.x, wl.y, [1] * N)
    loss, grads, logits = _torch_grads(cfg, wl)
    assert abs(r["loss"] - loss) <= 1e-12 * abs(loss)
    assert np.allclose(r["logits"], logits, rtol=1e-11, atol=1e-12)
    for k in range(N):
        scale = np.abs(grads[k]).max() + 1e-300
        assert np.abs(r["grads"][k] - grads[k]).max() <= 1e-10 * scale, wl.names[k]


def test_masks_skip_work_and_keep_values():
    cfg = CONFIGS["vgg_tiny"]
    wl = make_workload(cfg, seed=2, init="random")
    N = len(wl.weights)
    full = nets.step(cfg, wl.weights, wl.x, wl.y, [1] * N)
    assert full["work"] == [op for j in range(N - 1, -1, -1) for op in ([("dw", j)] + ([("dy", j)] if j > 0 else []))]
    assert nets.step(cfg, wl.weights, wl.x, wl.y, [0] * N)["work"] == []
    rng = np.random.default_rng(1)
    for _ in range(12):
        mask = (rng.random(N) < 0.4).astype(int)
        if not mask.any():
            continue
        r = nets.step(cfg, wl.weights, wl.x, wl.y, mask)
        jstar = int(np.argmax(mask))
        assert set(r["work"]) == {("dw", j) for j in range(N) if mask[j]} | {("dy", j) for j in range(jstar + 1, N)}
        for j in range(N):
            if mask[j]:
                assert np.array_equal(r["grads"][j], full["grads"][j])
            else:
                assert r["grads"][j] is None


def test_store_hook():
    cfg = CONFIGS["vgg_small"]
    wl = make_workload(cfg, seed=4, init="random")
    N = len(wl.weights)
    exact = V.vgg_step(cfg, wl.weights, wl.x, wl.y, [1] * N)
    same = V.vgg_step(cfg, wl.weights, wl.x, wl.y, [1] * N, store=lambda a: a)
    for a, b in zip(exact["grads"], same["grads"]):
        assert np.array_equal(a, b)
    stored = V.vgg_step(cfg, wl.weights, wl.x, wl.y, [1] * N, store=R.round_bf16)
    errs = [np.linalg.norm(a - b) / np.linalg.norm(a) for a, b in zip(exact["grads"], stored["grads"])]
    assert 1e-4 < max(errs) < 0.3                              # a bf16 evaluation, not a rounding of the exact gradient


def test_maxpool_takes_the_first_maximum():
    x = np.zeros((1, 2, 2, 2))
    x[0, :, :, 1] = [[1.0, 3.0], [3.0, 2.0]]
    p, arg = V.maxpool_2x2(x)
    assert p[0, 0, 0].tolist() == [0.0, 3.0] and arg[0, 0, 0].tolist() == [0, 1]
    d = np.ones((1, 1, 1, 2))
    back = V.maxpool_2x2_backward(d, arg, x.shape)
    assert back[0, :, :, 0].tolist() == [[1.0, 0.0], [0.0, 0.0]] and back[0, :, :, 1].tolist() == [[0.0, 1.0], [0.0, 0.0]]


def test_batch_mean_gradient_is_the_mean_over_chunks_also_with_storage_rounding():
    """Used by the full-size golden writer: chunks of a batch (count a power of two) average to the batch result."""
    cfg = CONFIGS["vgg_small"]
    wl = make_workload(cfg, seed=11, init="random", batch=4)
    N = len(wl.weights)
    for store in (None, R.round_bf16):
        whole = V.vgg_step(cfg, wl.weights, wl.x, wl.y, [1] * N, store=store)
        parts = [V.vgg_step(cfg, wl.weights, wl.x[i:i + 2], wl.y[i:i + 2], [1] * N, store=store) for i in (0, 2)]
        assert abs(whole["loss"] - 0.5 * (parts[0]["loss"] + parts[1]["loss"])) < 1e-13
        for k in range(N):
            np.testing.assert_allclose(whole["grads"][k], 0.5 * (parts[0]["grads"][k] + parts[1]["grads"][k]),
                                       rtol=1e-11, atol=1e-15)


def test_rounding_noise_moves_the_gradients_of_a_deep_plain_stack_by_per_cent():
    """Why the full-size VGG16 comparison allows 0.25: thirteen ReLU convolutions without shortcuts.  Noise of
    3e-7 (fp32 summation order) ahead of the bf16 storage rounding flips some roundings; every flip perturbs all
    later activations at the 2^-9 level, ReLU decisions next to zero flip with them, and each flipped decision
    drops or passes a whole gradient element.  The disagreement grows from the output side to the input side."""
    from synth.configs import VGGConfig
    cfg = VGGConfig("vgg16_img32", 1, 32, 3, (64, 128, 256, 512, 512), (2, 2, 3, 3, 3), (256,), 40)
    wl = make_workload(cfg, seed=0)
    N = len(wl.weights)
    rng = np.random.default_rng(123)

    def noisy(a):
        a = np.asarray(a, dtype=np.float64)
        return R.round_bf16(a * (1.0 + 3e-7 * rng.standard_normal(a.shape)))

    a = V.vgg_step(cfg, wl.weights, wl.x, wl.y, [1] * N, store=R.round_bf16)
    b = V.vgg_step(cfg, wl.weights, wl.x, wl.y, [1] * N, store=noisy)
    diff = [np.linalg.norm((a["grads"][k] - b["grads"][k]).ravel()) / np.linalg.norm(a["grads"][k].ravel())
            for k in range(N)]
    assert diff[0] > 0.03, diff[0]                 # conv0.W: several per cent from 3e-7 of noise
    assert diff[N - 2] < 0.5 * diff[0]             # the last linear layer sees far less of it
