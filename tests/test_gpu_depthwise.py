"""Depthwise 3x3 kernels (forward with affine + ReLU6, input gradient with addend and ReLU6 mask, weight
gradient) against the oracle's depthwise convolution on the same bf16 inputs, through the C ABI: small ragged
shapes and the shapes of the MobileNetV2 workload (two images of its largest layers)."""
import numpy as np
import pytest

from oracle import mobilenet as MB
from synth import bf16_round

pytestmark = pytest.mark.gpu

SHAPES = [(2, 7, 6, 8, 1), (2, 7, 6, 16, 2), (3, 9, 9, 24, 2), (1, 16, 16, 40, 1),
          (2, 112, 112, 96, 2), (2, 112, 112, 32, 1), (2, 56, 56, 144, 1), (2, 14, 14, 576, 2), (4, 7, 7, 960, 1)]


def _setup(batch, H, W, C, stride, seed):
    import torch
    rng = np.random.default_rng(seed)
    Ho, Wo = (H - 1) // stride + 1, (W - 1) // stride + 1
    x = bf16_round(rng.standard_normal((batch, H, W, C)).astype(np.float32))
    w = bf16_round((rng.standard_normal((C, 3, 3, 1)) / 3.0).astype(np.float32))
    d = bf16_round(rng.standard_normal((batch, Ho, Wo, C)).astype(np.float32))
    to = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0").to(torch.bfloat16)
    return x, w, d, to, (Ho, Wo)


@pytest.mark.parametrize("batch,H,W,C,stride", SHAPES)
def test_depthwise_forward(batch, H, W, C, stride):
    import torch
    from paper_2312_14227_amd import binding as et
    x, w, d, to, (Ho, Wo) = _setup(batch, H, W, C, stride, seed=C + stride)
    rng = np.random.default_rng(1)
    gain = bf16_round((1.0 + 0.3 * rng.standard_normal(C)).astype(np.float32))
    shift = bf16_round((0.5 * rng.standard_normal(C)).astype(np.float32))
    dwc = MB.Depthwise(x.astype(np.float64), w.astype(np.float64), stride)
    z = dwc.out
    xt, wt, gt, st = to(x), to(w.reshape(C, 9)), to(gain), to(shift)
    zt = torch.full((batch, Ho, Wo, C), float("nan"), device="cuda:0", dtype=torch.bfloat16)
    yt = torch.full_like(zt, float("nan"))
    assert et.et_debug_depthwise3x3(0, xt.data_ptr(), wt.data_ptr(), gt.data_ptr(), st.data_ptr(), zt.data_ptr(), yt.data_ptr(),
                                    0, batch, H, W, C, stride, torch.cuda.current_stream().cuda_stream) == 0
    torch.cuda.synchronize()
    zg = zt.float().cpu().numpy().astype(np.float64)
    assert np.all(np.abs(zg - z) <= 2.0 ** -8 * np.abs(z) + 1e-5)
    # y is computed from the rounded z the kernel stored
    y_ref = MB.relu6(zg * gain.astype(np.float64) + shift.astype(np.float64))
    yg = yt.float().cpu().numpy().astype(np.float64)
    assert np.all(np.abs(yg - y_ref) <= 2.0 ** -8 * np.abs(y_ref) + 1e-6)
    # z not kept: y alone
    y2 = torch.full_like(zt, float("nan"))
    assert et.et_debug_depthwise3x3(0, xt.data_ptr(), wt.data_ptr(), gt.data_ptr(), st.data_ptr(), 0, y2.data_ptr(), 0, batch, H,
                                    W, C, stride, torch.cuda.current_stream().cuda_stream) == 0
    torch.cuda.synchronize()
    assert torch.equal(y2, yt)


@pytest.mark.parametrize("with_add,with_mask", [(0, 0), (1, 1), (0, 1)])
@pytest.mark.parametrize("batch,H,W,C,stride", SHAPES)
def test_depthwise_input_gradient(batch, H, W, C, stride, with_add, with_mask):
    import torch
    from paper_2312_14227_amd import binding as et
    x, w, d, to, (Ho, Wo) = _setup(batch, H, W, C, stride, seed=C + 7 * stride)
    rng = np.random.default_rng(2)
    add = bf16_round(rng.standard_normal(x.shape).astype(np.float32))
    act = bf16_round(np.clip(4.0 * rng.standard_normal(x.shape) + 3.0, 0.0, 6.0).astype(np.float32))   # zeros, sixes, in between
    dwc = MB.Depthwise(x.astype(np.float64), w.astype(np.float64), stride)
    ref = dwc.dx(d.astype(np.float64))
    scale = MB.Depthwise(x.astype(np.float64), np.abs(w).astype(np.float64), stride).dx(np.abs(d).astype(np.float64))
    if with_add:
        ref = ref + add
        scale = scale + np.abs(add)
    if with_mask:
        ref = ref * MB.relu6_mask(act)
    dt, wt, at, mt = to(d), to(w.reshape(C, 9)), to(add), to(act)
    out = torch.full(x.shape, float("nan"), device="cuda:0", dtype=torch.bfloat16)
    assert et.et_debug_depthwise3x3(1, dt.data_ptr(), wt.data_ptr(), at.data_ptr() if with_add else 0,
                                    mt.data_ptr() if with_mask else 0, out.data_ptr(), 0, 0, batch, H, W, C, stride,
                                    torch.cuda.current_stream().cuda_stream) == 0
    torch.cuda.synchronize()
    got = out.float().cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref) + 2e-6 * scale + 1e-6)


@pytest.mark.parametrize("batch,H,W,C,stride", SHAPES)
def test_depthwise_weight_gradient(batch, H, W, C, stride):
    import torch
    from paper_2312_14227_amd import binding as et
    x, w, d, to, (Ho, Wo) = _setup(batch, H, W, C, stride, seed=C + 13 * stride)
    dwc = MB.Depthwise(x.astype(np.float64), w.astype(np.float64), stride)
    ref = dwc.dw(d.astype(np.float64)).reshape(C, 9)
    scale = MB.Depthwise(np.abs(x).astype(np.float64), w.astype(np.float64), stride).dw(np.abs(d).astype(np.float64)).reshape(C, 9)
    xt, dt = to(x), to(d)
    n = et.et_debug_depthwise3x3_ws_floats(batch, H, W, C, stride)
    assert n > 0
    ws = torch.empty(n, device="cuda:0", dtype=torch.float32)
    out = torch.full((C, 9), float("nan"), device="cuda:0", dtype=torch.float32)
    assert et.et_debug_depthwise3x3(2, dt.data_ptr(), xt.data_ptr(), 0, 0, out.data_ptr(), 0, ws.data_ptr(), batch, H, W, C, stride,
                                    torch.cuda.current_stream().cuda_stream) == 0
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - ref) <= 2e-6 * scale * np.sqrt(batch * Ho * Wo) + 1e-6)


def test_depthwise_rejects_bad_arguments():
    import torch
    from paper_2312_14227_amd import binding as et
    t = torch.zeros(1 << 16, device="cuda:0", dtype=torch.bfloat16)
    p = t.data_ptr()
    assert et.et_debug_depthwise3x3(0, p, p, p, p, p, p, 0, 1, 8, 8, 12, 1) == -1     # channels not a multiple of 8
    assert et.et_debug_depthwise3x3(0, p, p, p, p, p, p, 0, 1, 8, 8, 8, 3) == -1      # stride
    assert et.et_debug_depthwise3x3(2, p, p, 0, 0, p, 0, 0, 1, 8, 8, 8, 1) == -1      # no scratch
    assert et.et_debug_depthwise3x3(5, p, p, p, p, p, p, 0, 1, 8, 8, 8, 1) == -1
    assert et.et_debug_depthwise3x3_ws_floats(1, 8, 8, 12, 1) == 0
