"""Implicit-GEMM 3x3 convolution kernel (the im2col matrix is gathered from the activation, never written)
against the oracle's convolution (explicit im2col and a float64 matrix product) on the same bf16 inputs,
through the C ABI; all four tile shapes, images smaller and larger than a tile, ragged row and column tails."""
import numpy as np
import pytest

from oracle import resnet as R
from synth import bf16_round

pytestmark = pytest.mark.gpu


def _case(batch, H, W, C, N, mode, tile, seed):
    import torch
    from paper_2312_14227_amd import binding as et
    rng = np.random.default_rng(seed)
    x = bf16_round(rng.standard_normal((batch, H, W, C)).astype(np.float32))
    w = bf16_round((rng.standard_normal((N, 3, 3, C)) / np.sqrt(9 * C)).astype(np.float32))
    bias = bf16_round(rng.standard_normal(N).astype(np.float32))
    u = bf16_round(rng.standard_normal((batch * H * W, N)).astype(np.float32))
    cv = R.Conv(x.astype(np.float64), w.astype(np.float64), 1)
    ref = cv.out.reshape(batch * H * W, N)
    scale = (np.abs(cv.cols.reshape(batch * H * W, -1)) @ np.abs(cv.wm).T)
    if mode == 1:
        ref = np.maximum(ref + bias.astype(np.float64), 0.0)
    if mode == 2:
        ref = ref * (u > 0)
    dev = "cuda:0"
    to = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev).to(torch.bfloat16)
    xt, wt, bt, ut = to(x), to(w), to(bias), to(u)
    out = torch.full((batch * H * W, N), float("nan"), device=dev, dtype=torch.bfloat16)
    st = et.et_debug_conv3x3(xt.data_ptr(), wt.data_ptr(), out.data_ptr(), batch, H, W, C, N, bt.data_ptr(), ut.data_ptr(),
                             mode, tile, torch.cuda.current_stream().cuda_stream)
    assert st == 0
    torch.cuda.synchronize()
    got = out.float().cpu().numpy().astype(np.float64)
    # fp32 accumulation of exact bf16 products, then one rounding of the output
    bound = 2e-6 * scale * np.sqrt(9 * C) + 1e-6 + 2.0 ** -8 * np.abs(ref)
    if mode == 1:
        bound = bound + 2.0 ** -8 * np.abs(bias)
    bad = np.abs(got - ref) > bound
    assert not bad.any(), (int(bad.sum()), float(np.abs(got - ref).max()))


@pytest.mark.parametrize("tile", [0, 11, 13, 15, 17])
@pytest.mark.parametrize("batch,H,W,C,N", [(2, 14, 14, 64, 64), (1, 28, 28, 128, 72), (3, 7, 9, 64, 264), (1, 40, 24, 192, 128)])
def test_conv3x3_plain(batch, H, W, C, N, tile):
    _case(batch, H, W, C, N, 0, tile, seed=tile + H)


@pytest.mark.parametrize("mode", [1, 2])
@pytest.mark.parametrize("batch,H,W,C,N,tile", [(2, 14, 14, 64, 64, 17), (1, 28, 28, 128, 128, 15), (3, 7, 9, 64, 264, 11),
                                                (2, 16, 16, 64, 200, 13), (2, 16, 16, 256, 512, 0)])
def test_conv3x3_epilogues(batch, H, W, C, N, tile, mode):
    _case(batch, H, W, C, N, mode, tile, seed=mode * 100 + tile)


# layer shapes of the VGG16 and ResNet-50 workloads (a few images; the weight gradient needs a multiple of 64 pixels)
REAL = [(2, 224, 224, 64, 64), (2, 112, 112, 128, 128), (2, 56, 56, 256, 256), (4, 28, 28, 512, 512), (16, 14, 14, 512, 512),
        (2, 56, 56, 64, 64), (16, 14, 14, 256, 256)]


@pytest.mark.parametrize("batch,H,W,C,N", REAL)
def test_conv3x3_workload_shapes(batch, H, W, C, N):
    """Forward with bias + ReLU, gradient passing with the ReLU mask, weight gradient with the planned tile and split."""
    _case(batch, H, W, C, N, 1, 0, seed=H + C)
    _case(batch, H, W, C, N, 2, 0, seed=H + C + 1)
    _case_dw(batch, H, W, C, N, 0, 0, seed=H + C + 2)


def test_conv3x3_rejects_bad_arguments():
    import torch
    from paper_2312_14227_amd import binding as et
    t = torch.zeros(1 << 16, device="cuda:0", dtype=torch.bfloat16)
    p = t.data_ptr()
    assert et.et_debug_conv3x3(p, p, p, 1, 8, 8, 48, 64) == -1        # channels not a multiple of 64
    assert et.et_debug_conv3x3(p, p, p, 0, 8, 8, 64, 64) == -1
    assert et.et_debug_conv3x3(p + 2, p, p, 1, 8, 8, 64, 64) == -1    # misaligned


def _case_dw(batch, H, W, C, N, split, tile, seed):
    import torch
    from paper_2312_14227_amd import binding as et
    rng = np.random.default_rng(seed)
    x = bf16_round(rng.standard_normal((batch, H, W, C)).astype(np.float32))
    d = bf16_round(rng.standard_normal((batch, H, W, N)).astype(np.float32))
    cv = R.Conv(x.astype(np.float64), np.zeros((N, 3, 3, C)), 1)
    ref = cv.dw(d.astype(np.float64)).reshape(N, 9 * C)
    scale = np.abs(d.reshape(-1, N).astype(np.float64)).T @ np.abs(cv.cols.reshape(batch * H * W, -1))
    dev = "cuda:0"
    to = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev).to(torch.bfloat16)
    xt, dt = to(x), to(d)
    out = torch.full((N, 9 * C), float("nan"), device=dev, dtype=torch.float32)
    part = torch.empty(N * 9 * C * 256, device=dev, dtype=torch.float32)
    st = et.et_debug_conv3x3_dw(xt.data_ptr(), dt.data_ptr(), out.data_ptr(), batch, H, W, C, N, split, part.data_ptr(),
                                tile, torch.cuda.current_stream().cuda_stream)
    assert st == 0
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    bound = 2e-6 * scale * np.sqrt(batch * H * W) + 1e-6
    bad = ~(np.abs(got - ref) <= bound)
    assert not bad.any(), (int(bad.sum()), float(np.nanmax(np.abs(got - ref))))


@pytest.mark.parametrize("tile", [11, 13, 19, 21])
@pytest.mark.parametrize("batch,H,W,C,N,split", [(1, 8, 8, 8, 8, 1), (2, 16, 16, 64, 64, 1), (4, 8, 8, 24, 40, 2), (1, 32, 24, 64, 128, 3),
                                                 (2, 14, 16, 128, 264, 1), (3, 7, 64, 16, 520, 5)])
def test_conv3x3_weight_gradient(batch, H, W, C, N, split, tile):
    _case_dw(batch, H, W, C, N, split, tile, seed=tile + H + N)


@pytest.mark.parametrize("batch,H,W,C,N", [(2, 32, 32, 64, 64), (2, 16, 16, 128, 128), (4, 16, 16, 256, 512)])
def test_conv3x3_weight_gradient_planned(batch, H, W, C, N):
    _case_dw(batch, H, W, C, N, 0, 0, seed=C + N)


def test_conv3x3_weight_gradient_rejects_bad_arguments():
    import torch
    from paper_2312_14227_amd import binding as et
    t = torch.zeros(1 << 20, device="cuda:0", dtype=torch.float32)
    p = t.data_ptr()
    assert et.et_debug_conv3x3_dw(p, p, p, 1, 8, 8, 12, 64) == -1     # channels not a multiple of 8
    assert et.et_debug_conv3x3_dw(p, p, p, 1, 5, 5, 8, 64) == -1      # pixels not a multiple of 64
    assert et.et_debug_conv3x3_dw(p, p, p, 1, 8, 8, 8, 64, 2, 0) == -1  # split without partials


def _case_split(batch, H, W, C, N, mode, split, tile, seed):
    import torch
    from paper_2312_14227_amd import binding as et
    rng = np.random.default_rng(seed)
    x = bf16_round(rng.standard_normal((batch, H, W, C)).astype(np.float32))
    w = bf16_round((rng.standard_normal((N, 3, 3, C)) / np.sqrt(9 * C)).astype(np.float32))
    bias = bf16_round(rng.standard_normal(N).astype(np.float32))
    gain = bf16_round((1.0 + 0.3 * rng.standard_normal(N)).astype(np.float32))
    u = bf16_round(rng.standard_normal((batch * H * W, N)).astype(np.float32))
    cv = R.Conv(x.astype(np.float64), w.astype(np.float64), 1)
    z = cv.out.reshape(batch * H * W, N)
    scale = (np.abs(cv.cols.reshape(batch * H * W, -1)) @ np.abs(cv.wm).T)
    dev = "cuda:0"
    to = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev).to(torch.bfloat16)
    xt, wt, bt, gt, ut = to(x), to(w), to(bias), to(gain), to(u)
    out = torch.full((batch * H * W, N), float("nan"), device=dev, dtype=torch.bfloat16)
    zt = torch.full_like(out, float("nan"))
    part = torch.empty(batch * H * W * N * 18, device=dev, dtype=torch.float32)
    st = et.et_debug_conv3x3_split(xt.data_ptr(), wt.data_ptr(), out.data_ptr(), zt.data_ptr() if mode == 3 else 0, batch, H, W, C, N,
                                   bt.data_ptr(), gt.data_ptr(), ut.data_ptr(), mode, split, part.data_ptr(), tile,
                                   torch.cuda.current_stream().cuda_stream)
    assert st == 0
    torch.cuda.synchronize()
    got = out.float().cpu().numpy().astype(np.float64)
    acc = 2e-6 * scale * np.sqrt(9 * C) + 1e-6
    if mode == 0:
        ref, bound = z, acc + 2.0 ** -8 * np.abs(z)
    elif mode == 1:
        ref = np.maximum(z + bias, 0.0)
        bound = acc + 2.0 ** -8 * (np.abs(ref) + np.abs(bias))
    elif mode == 2:
        ref = z * (u > 0)
        bound = acc + 2.0 ** -8 * np.abs(ref)
    else:
        zg = zt.float().cpu().numpy().astype(np.float64)
        assert np.all(np.abs(zg - z) <= acc + 2.0 ** -8 * np.abs(z))
        ref = np.minimum(np.maximum(zg * gain + bias, 0.0), 6.0)        # from the rounded z the kernel stored
        bound = 2.0 ** -8 * np.abs(ref) + 1e-6
    bad = ~(np.abs(got - ref) <= bound)
    assert not bad.any(), (int(bad.sum()), float(np.nanmax(np.abs(got - ref))))


@pytest.mark.parametrize("mode", [0, 1, 2, 3])
@pytest.mark.parametrize("batch,H,W,C,N,split,tile", [(2, 7, 7, 64, 64, 3, 17), (2, 7, 7, 128, 72, 9, 15), (3, 14, 14, 64, 264, 2, 11),
                                                      (2, 7, 9, 192, 128, 5, 13), (32, 7, 7, 512, 512, 0, 0), (32, 14, 14, 256, 256, 0, 0)])
def test_conv3x3_split_reduction(batch, H, W, C, N, split, tile, mode):
    _case_split(batch, H, W, C, N, mode, split, tile, seed=mode * 31 + H + N)


def _case_gathered(batch, H, W, C, N, taps, stride, tile, seed, split=1):
    """Forward product and weight gradient of a gathered convolution with `taps` per side and `stride` against the
    oracle's convolution (explicit im2col, float64)."""
    import torch
    from paper_2312_14227_amd import binding as et
    rng = np.random.default_rng(seed)
    x = bf16_round(rng.standard_normal((batch, H, W, C)).astype(np.float32))
    w = bf16_round((rng.standard_normal((N, taps, taps, C)) / np.sqrt(taps * taps * C)).astype(np.float32))
    cv = R.Conv(x.astype(np.float64), w.astype(np.float64), stride)
    Ho, Wo = cv.out.shape[1:3]
    assert (Ho, Wo) == ((H - 1) // stride + 1, (W - 1) // stride + 1)
    rows, kk = batch * Ho * Wo, taps * taps * C
    d = bf16_round(rng.standard_normal((batch, Ho, Wo, N)).astype(np.float32))
    dev = "cuda:0"
    to = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev).to(torch.bfloat16)
    xt, wt, dt = to(x), to(w), to(d)
    stream = torch.cuda.current_stream().cuda_stream
    cols = cv.cols.reshape(rows, kk)
    if C % 64 == 0:
        out = torch.full((rows, N), float("nan"), device=dev, dtype=torch.bfloat16)
        assert et.et_debug_conv_gathered(0, xt.data_ptr(), wt.data_ptr(), out.data_ptr(), batch, H, W, C, N, taps, stride,
                                         1, 0, tile, stream) == 0
        torch.cuda.synchronize()
        ref = cv.out.reshape(rows, N)
        got = out.float().cpu().numpy().astype(np.float64)
        bound = 2e-6 * (np.abs(cols) @ np.abs(cv.wm).T) * np.sqrt(kk) + 1e-6 + 2.0 ** -8 * np.abs(ref)
        bad = ~(np.abs(got - ref) <= bound)
        assert not bad.any(), ("forward", int(bad.sum()), float(np.nanmax(np.abs(got - ref))))
    if rows % 64 == 0:
        dw = torch.full((N, kk), float("nan"), device=dev, dtype=torch.float32)
        part = torch.empty(N * kk * max(split, 1) if split else N * kk * 256, device=dev, dtype=torch.float32)
        assert et.et_debug_conv_gathered(1, xt.data_ptr(), dt.data_ptr(), dw.data_ptr(), batch, H, W, C, N, taps, stride,
                                         split, part.data_ptr(), tile if tile in (0, 11, 13) else 0, stream) == 0
        torch.cuda.synchronize()
        ref = cv.dw(d.astype(np.float64)).reshape(N, kk)
        got = dw.cpu().numpy().astype(np.float64)
        bound = 2e-6 * (np.abs(d.reshape(rows, N).astype(np.float64)).T @ np.abs(cols)) * np.sqrt(rows) + 1e-6
        bad = ~(np.abs(got - ref) <= bound)
        assert not bad.any(), ("dw", int(bad.sum()), float(np.nanmax(np.abs(got - ref))))


# (batch, H, W, C, N, taps, stride): images smaller and larger than a 64-pixel slice, odd sizes (the last input row and
# column are then read by the centre tap), output rows that do and do not divide a slice, the ResNet-50 stage shapes
STRIDED = [(2, 16, 16, 64, 64, 3, 2), (1, 32, 32, 128, 72, 3, 2), (4, 15, 17, 64, 136, 3, 2), (2, 56, 56, 128, 128, 3, 2),
           (8, 14, 14, 512, 512, 3, 2), (2, 16, 16, 64, 128, 1, 2), (4, 15, 17, 64, 264, 1, 2), (2, 56, 56, 256, 512, 1, 2),
           (64, 3, 3, 64, 64, 3, 2), (2, 16, 16, 64, 64, 3, 1), (2, 16, 16, 8, 16, 3, 2), (2, 16, 16, 24, 16, 1, 2)]


@pytest.mark.parametrize("batch,H,W,C,N,taps,stride", STRIDED)
@pytest.mark.parametrize("tile", [0, 11, 13, 15])
def test_gathered_convolution_with_stride(batch, H, W, C, N, taps, stride, tile):
    _case_gathered(batch, H, W, C, N, taps, stride, tile, seed=H * 7 + C + taps + tile)


@pytest.mark.parametrize("split", [0, 2, 3])
def test_gathered_strided_weight_gradient_split(split):
    _case_gathered(4, 28, 28, 64, 64, 3, 2, 0, seed=split, split=split)
    _case_gathered(4, 28, 28, 64, 96, 1, 2, 0, seed=split + 10, split=split)


def test_gathered_convolution_rejects_bad_arguments():
    import torch
    from paper_2312_14227_amd import binding as et
    t = torch.zeros(1 << 18, device="cuda:0", dtype=torch.float32)
    p = t.data_ptr()
    assert et.et_debug_conv_gathered(0, p, p, p, 1, 8, 8, 64, 64, 2, 1) == -1     # taps
    assert et.et_debug_conv_gathered(0, p, p, p, 1, 8, 8, 64, 64, 3, 3) == -1     # stride
    assert et.et_debug_conv_gathered(0, p, p, p, 1, 8, 8, 48, 64, 3, 2) == -1     # channels
    assert et.et_debug_conv_gathered(1, p, p, p, 1, 10, 10, 8, 64, 3, 2) == -1    # 25 output pixels
    assert et.et_debug_conv_gathered(2, p, p, p, 1, 8, 8, 64, 64, 3, 2) == -1     # op


def _case_stem(batch, H, W, C, N, seed):
    """The stem convolution (7x7, stride 2, zero padding 3) and its weight gradient through the padded-image GEMM."""
    import torch
    from paper_2312_14227_amd import binding as et
    rng = np.random.default_rng(seed)
    x = bf16_round(rng.standard_normal((batch, H, W, C)).astype(np.float32))
    w = bf16_round((rng.standard_normal((N, 7, 7, C)) / np.sqrt(49 * C)).astype(np.float32))
    cv = R.Conv(x.astype(np.float64), w.astype(np.float64), 2)
    Ho, Wo = cv.out.shape[1:3]
    rows, kk = batch * Ho * Wo, 49 * C
    d = bf16_round(rng.standard_normal((batch, Ho, Wo, N)).astype(np.float32))
    dev = "cuda:0"
    to = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev).to(torch.bfloat16)
    xt, wt, dt = to(x), to(w), to(d)
    nbytes = et.et_debug_stem_ws_bytes(batch, H, W, C, N)
    assert nbytes > 0
    ws = torch.empty(nbytes, device=dev, dtype=torch.uint8)
    stream = torch.cuda.current_stream().cuda_stream
    cols = cv.cols.reshape(rows, kk)
    out = torch.full((rows, N), float("nan"), device=dev, dtype=torch.float32)
    assert et.et_debug_stem(0, xt.data_ptr(), wt.data_ptr(), out.data_ptr(), ws.data_ptr(), batch, H, W, C, N, stream) == 0
    torch.cuda.synchronize()
    ref = cv.out.reshape(rows, N)
    got = out.cpu().numpy().astype(np.float64)
    bound = 2e-6 * (np.abs(cols) @ np.abs(cv.wm).T) * np.sqrt(kk) + 1e-6
    bad = ~(np.abs(got - ref) <= bound)
    assert not bad.any(), ("forward", int(bad.sum()), float(np.nanmax(np.abs(got - ref))))
    if rows % 64 == 0:
        dw = torch.full((N, kk), float("nan"), device=dev, dtype=torch.float32)
        assert et.et_debug_stem(1, xt.data_ptr(), dt.data_ptr(), dw.data_ptr(), ws.data_ptr(), batch, H, W, C, N, stream) == 0
        torch.cuda.synchronize()
        ref = cv.dw(d.astype(np.float64)).reshape(N, kk)
        got = dw.cpu().numpy().astype(np.float64)
        bound = 2e-6 * (np.abs(d.reshape(rows, N).astype(np.float64)).T @ np.abs(cols)) * np.sqrt(rows) + 1e-6
        bad = ~(np.abs(got - ref) <= bound)
        assert not bad.any(), ("dw", int(bad.sum()), float(np.nanmax(np.abs(got - ref))))


# even and odd image sizes, 1 to 4 channels, images smaller than the window, one ResNet-50 sized image pair
@pytest.mark.parametrize("batch,H,W,C,N", [(2, 32, 32, 3, 16), (4, 16, 16, 3, 64), (1, 33, 31, 3, 24), (3, 5, 9, 1, 8), (2, 64, 48, 4, 64),
                                           (1, 15, 17, 2, 72), (2, 224, 224, 3, 64)])
def test_stem_convolution(batch, H, W, C, N):
    _case_stem(batch, H, W, C, N, seed=H + W + C)


def test_stem_convolution_rejects_bad_arguments():
    from paper_2312_14227_amd import binding as et
    assert et.et_debug_stem_ws_bytes(1, 32, 32, 5, 16) == 0     # channels
    assert et.et_debug_stem_ws_bytes(1, 32, 32, 3, 12) == 0     # output channels not a multiple of 8
    assert et.et_debug_stem_ws_bytes(0, 32, 32, 3, 16) == 0
