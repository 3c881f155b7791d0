"""Pins of the oracle's inverted-residual network (MobileNetV2 family): finite differences, PyTorch CPU autograd
over library convolution (dense and grouped) / hardtanh / pooling / linear ops, the depthwise convolution against
a dense convolution with a block-diagonal weight, and the executed-work invariants of selective training."""
import numpy as np
import pytest
import torch

from oracle import mobilenet as MB
from oracle import nets
from oracle import resnet as R
from synth import CONFIGS, make_workload, mobilenet_blocks, tensor_specs


def test_tensor_count_and_size_of_mobilenetv2():
    specs = tensor_specs(CONFIGS["mobilenetv2"])
    assert len(specs) == 158                                   # 52 convolutions x (W, g, b) + head W, b
    assert sum(int(np.prod(s)) for _, s in specs) == 2480072
    assert specs[3] == ("b0.dw.W", (32, 3, 3, 1))              # the first block has no expansion
    assert sum(sc for *_, sc in mobilenet_blocks(CONFIGS["mobilenetv2"])) == 10   # blocks with a shortcut


def test_depthwise_is_a_dense_convolution_with_a_block_diagonal_weight():
    rng = np.random.default_rng(0)
    for stride in (1, 2):
        x = rng.standard_normal((2, 7, 6, 5))
        w = rng.standard_normal((5, 3, 3, 1))
        d = rng.standard_normal((2, (7 - 1) // stride + 1, (6 - 1) // stride + 1, 5))
        dense = np.zeros((5, 3, 3, 5))
        for c in range(5):
            dense[c, :, :, c] = w[c, :, :, 0]
        a, b = MB.Depthwise(x, w, stride), R.Conv(x, dense, stride)
        assert a.out.shape == d.shape
        np.testing.assert_allclose(a.out, b.out, rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(a.dx(d), b.dx(d), rtol=1e-12, atol=1e-13)
        full = b.dw(d)
        for c in range(5):
            np.testing.assert_allclose(a.dw(d)[c, :, :, 0], full[c, :, :, c], rtol=1e-12, atol=1e-13)


def test_gradients_match_finite_differences():
    cfg = CONFIGS["mobilenet_tiny"]
    wl = make_workload(cfg, seed=3, init="random")
    N = len(wl.weights)
    r = nets.step(cfg, wl.weights, wl.x, wl.y, [1] * N)
    rng = np.random.default_rng(0)
    h = 1e-6
    ok = total = 0
    for k in range(N):
        g = r["grads"][k]
        assert g.shape == wl.weights[k].shape
        for _ in range(4):
            idx = tuple(rng.integers(0, s) for s in g.shape)
            wp = [w.astype(np.float64).copy() for w in wl.weights]
            wm = [w.astype(np.float64).copy() for w in wl.weights]
            wp[k][idx] += h
            wm[k][idx] -= h
            fd = (nets.forward(cfg, wp, wl.x, wl.y)[0] - nets.forward(cfg, wm, wl.x, wl.y)[0]) / (2 * h)
            total += 1
            ok += abs(fd - g[idx]) <= 1e-6 * max(1.0, abs(fd))
    assert ok >= 0.95 * total, (ok, total)                     # a step across a ReLU6 kink may miss


def _torch_grads(cfg, wl):
    import torch.nn.functional as F
    W = [torch.tensor(w, dtype=torch.float64, requires_grad=True) for w in wl.weights]
    aff = lambda z, t: z * W[t + 1].view(1, -1, 1, 1) + W[t + 2].view(1, -1, 1, 1)
    cw = lambda t: W[t].permute(0, 3, 1, 2)
    h = torch.tensor(wl.x, dtype=torch.float64).permute(0, 3, 1, 2)
    h = F.hardtanh(aff(F.conv2d(h, cw(0), stride=2, padding=1), 0), 0.0, 6.0)
    t = 3
    for (cin, hid, cout, stride, expand, shortcut) in mobilenet_blocks(cfg):
        a = h
        if expand:
            a = F.hardtanh(aff(F.conv2d(a, cw(t)), t), 0.0, 6.0)
            t += 3
        a = F.hardtanh(aff(F.conv2d(a, cw(t), stride=stride, padding=1, groups=hid), t), 0.0, 6.0)
        p = aff(F.conv2d(a, cw(t + 3)), t + 3)
        h = h + p if shortcut else p
        t += 6
    h = F.hardtanh(aff(F.conv2d(h, cw(t)), t), 0.0, 6.0)
    p = h.mean(dim=(2, 3))
    logits = F.linear(p, W[t + 3], W[t + 4])
    loss = F.cross_entropy(logits, torch.tensor(wl.y, dtype=torch.long))
    loss.backward()
    return float(loss.detach()), [w.grad.numpy() for w in W], logits.detach().numpy()


@pytest.mark.parametrize("name,seed", [("mobilenet_tiny", 0), ("mobilenet_small", 1)])
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


def test_selected_gradients_do_not_depend_on_the_mask_and_work_follows_the_time_model():
    cfg = CONFIGS["mobilenet_small"]
    wl = make_workload(cfg, seed=2, init="random")
    N = len(wl.weights)
    full = nets.step(cfg, wl.weights, wl.x, wl.y, [1] * N)
    rng = np.random.default_rng(5)
    assert nets.step(cfg, wl.weights, wl.x, wl.y, [0] * N)["work"] == []
    for _ in range(6):
        mask = (rng.random(N) < 0.3).astype(int)
        mask[rng.integers(0, N)] = 1
        r = nets.step(cfg, wl.weights, wl.x, wl.y, mask)
        jstar = int(np.argmax(mask))
        expect = {("dw", j) for j in range(N) if mask[j]} | {("dy", j) for j in range(jstar + 1, N)}
        assert set(r["work"]) == expect
        for j in range(N):
            if mask[j]:
                assert np.array_equal(r["grads"][j], full["grads"][j])
            else:
                assert r["grads"][j] is None


def test_storage_hook():
    cfg = CONFIGS["mobilenet_small"]
    wl = make_workload(cfg, seed=4, init="random")
    N = len(wl.weights)
    a = MB.mobilenet_step(cfg, wl.weights, wl.x, wl.y, [1] * N)
    b = MB.mobilenet_step(cfg, wl.weights, wl.x, wl.y, [1] * N, store=lambda v: v)
    c = MB.mobilenet_step(cfg, wl.weights, wl.x, wl.y, [1] * N, store=R.round_bf16)
    for k in range(N):
        assert np.array_equal(a["grads"][k], b["grads"][k])
    err = max(np.linalg.norm((a["grads"][k] - c["grads"][k]).ravel()) / np.linalg.norm(a["grads"][k].ravel()) for k in range(N))
    assert 1e-4 < err < 0.5, err                                # rounding is applied, and it is a perturbation


def test_rounding_noise_moves_the_gradients_of_the_deep_network_by_tens_of_per_cent():
    """Why the full-size MobileNetV2 comparison is informative only at the output side: 52 convolutions, ReLU6
    clamping on both sides, random weights and no normalisation.  Noise of 3e-7 (fp32 summation order) ahead of
    the bf16 storage rounding changes the gradients of the input-side tensors by tens of per cent, those of the
    head by a few per cent."""
    from dataclasses import replace
    cfg = replace(CONFIGS["mobilenetv2"], name="mobilenetv2_img64", batch=2, image=64)
    wl = make_workload(cfg, seed=0)
    N = len(wl.weights)
    rng = np.random.default_rng(123)

    def noisy(a):
        a = np.asarray(a, dtype=np.float64)
        return R.round_bf16(a * (1.0 + 3e-7 * rng.standard_normal(a.shape)))

    a = MB.mobilenet_step(cfg, wl.weights, wl.x, wl.y, [1] * N, store=R.round_bf16)
    b = MB.mobilenet_step(cfg, wl.weights, wl.x, wl.y, [1] * N, store=noisy)
    diff = [np.linalg.norm((a["grads"][k] - b["grads"][k]).ravel()) / np.linalg.norm(a["grads"][k].ravel())
            for k in range(N)]
    print("first tensors", np.round(diff[:6], 3), "last tensors", np.round(diff[-5:], 3))
    assert np.median(diff[:30]) > 0.1
    assert diff[N - 2] < 0.3 * np.median(diff[:30])
