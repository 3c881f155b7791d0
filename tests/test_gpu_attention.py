"""The fused attention kernels against the oracle's definition, for every number of 32-key tiles the kernels are
instantiated for, ragged last tiles included."""
import numpy as np
import pytest

from gpu_util import rel_l2
from oracle import attention as oatt

pytestmark = pytest.mark.gpu


def _bf16(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16)


def _run(B, T, H, seed, q_gain=1.0):
    import torch
    from paper_2312_14227_amd import binding as et
    D = 64 * H
    rng = np.random.default_rng(seed)
    qkv = rng.standard_normal((B, T, 3 * D))
    qkv[..., :D] *= q_gain
    dout = rng.standard_normal((B, T, D))
    qkv_t, dout_t = _bf16(qkv).cuda(), _bf16(dout).cuda()
    out_t = torch.full((B, T, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    lse_t = torch.full((B, H, T), float("nan"), dtype=torch.float32, device="cuda")
    dqkv_t = torch.full((B, T, 3 * D), float("nan"), dtype=torch.bfloat16, device="cuda")
    assert et.et_debug_attention(0, qkv_t.data_ptr(), out_t.data_ptr(), lse_t.data_ptr(), 0, 0, B, T, H) == 0
    assert et.et_debug_attention(1, qkv_t.data_ptr(), out_t.data_ptr(), lse_t.data_ptr(), dout_t.data_ptr(), dqkv_t.data_ptr(),
                                 B, T, H) == 0
    torch.cuda.synchronize()
    qkv64 = qkv_t.float().cpu().numpy().astype(np.float64)          # the same bit patterns, widened
    dout64 = dout_t.float().cpu().numpy().astype(np.float64)
    out_ref, lse_ref, _ = oatt.attention_forward(qkv64, H)
    g_ref = oatt.attention_backward(qkv64, dout64, H)
    return (out_t.float().cpu().numpy(), lse_t.cpu().numpy(), dqkv_t.float().cpu().numpy()), (out_ref, lse_ref, g_ref), D


@pytest.mark.parametrize("T", [1, 5, 31, 32, 33, 64, 65, 100, 128, 150, 160, 192, 197, 223, 224])
def test_attention_matches_the_definition(T):
    (out, lse, g), (out_ref, lse_ref, g_ref), D = _run(2, T, 3, seed=T)
    assert np.isfinite(out).all() and np.isfinite(lse).all() and np.isfinite(g).all()
    # probabilities and results are rounded to bf16 once each: 2^-9 relative per element
    assert rel_l2(out, out_ref) <= 6e-3, rel_l2(out, out_ref)
    np.testing.assert_allclose(lse, lse_ref, rtol=0, atol=2e-5 * max(1.0, np.abs(lse_ref).max()))
    for i, name in enumerate(("dq", "dk", "dv")):
        a, b = g[..., i * D:(i + 1) * D], g_ref[..., i * D:(i + 1) * D]
        if T == 1 and i < 2:                       # one key: the softmax is constant, dQ = dK = 0 exactly
            assert np.abs(a).max() <= 1e-6 * np.abs(g_ref).max(), name
            continue
        assert rel_l2(a, b) <= 1e-2, (name, rel_l2(a, b))


def test_attention_with_peaked_scores():
    # queries four times larger: score standard deviation 4, a few keys dominate each row
    (out, lse, g), (out_ref, lse_ref, g_ref), D = _run(3, 197, 2, seed=11, q_gain=4.0)
    assert rel_l2(out, out_ref) <= 6e-3
    np.testing.assert_allclose(lse, lse_ref, rtol=0, atol=2e-5 * np.abs(lse_ref).max())
    for i in range(3):
        assert rel_l2(g[..., i * D:(i + 1) * D], g_ref[..., i * D:(i + 1) * D]) <= 1e-2, i


def test_attention_at_the_benchmark_shape_on_sampled_heads():
    import torch
    from paper_2312_14227_amd import binding as et
    B, T, H = 64, 197, 12
    D = 64 * H
    g = torch.Generator(device="cpu").manual_seed(5)
    qkv_t = torch.randn((B, T, 3 * D), generator=g).to(torch.bfloat16).cuda()
    dout_t = torch.randn((B, T, D), generator=g).to(torch.bfloat16).cuda()
    out_t = torch.empty((B, T, D), dtype=torch.bfloat16, device="cuda")
    lse_t = torch.empty((B, H, T), dtype=torch.float32, device="cuda")
    dqkv_t = torch.empty((B, T, 3 * D), dtype=torch.bfloat16, device="cuda")
    assert et.et_debug_attention(0, qkv_t.data_ptr(), out_t.data_ptr(), lse_t.data_ptr(), 0, 0, B, T, H) == 0
    assert et.et_debug_attention(1, qkv_t.data_ptr(), out_t.data_ptr(), lse_t.data_ptr(), dout_t.data_ptr(), dqkv_t.data_ptr(),
                                 B, T, H) == 0
    torch.cuda.synchronize()
    for b, h in ((0, 0), (63, 11), (17, 5), (40, 8)):
        cols = np.concatenate([np.arange(i * D + h * 64, i * D + h * 64 + 64) for i in range(3)])
        sub = qkv_t[b:b + 1][..., torch.from_numpy(cols).cuda()].float().cpu().numpy().astype(np.float64)
        do = dout_t[b:b + 1, :, h * 64:(h + 1) * 64].float().cpu().numpy().astype(np.float64)
        out_ref, lse_ref, _ = oatt.attention_forward(sub, 1)
        g_ref = oatt.attention_backward(sub, do, 1)
        assert rel_l2(out_t[b:b + 1, :, h * 64:(h + 1) * 64].float().cpu().numpy(), out_ref) <= 6e-3, (b, h)
        np.testing.assert_allclose(lse_t[b, h].cpu().numpy(), lse_ref[0, 0], rtol=0, atol=2e-5 * np.abs(lse_ref).max())
        got = dqkv_t[b:b + 1][..., torch.from_numpy(cols).cuda()].float().cpu().numpy()
        for i in range(3):
            assert rel_l2(got[..., i * 64:(i + 1) * 64], g_ref[..., i * 64:(i + 1) * 64]) <= 1e-2, (b, h, i)


def test_attention_rejects_what_it_does_not_cover():
    import torch
    from paper_2312_14227_amd import binding as et
    buf = torch.zeros(1 << 16, dtype=torch.float32, device="cuda")
    p = buf.data_ptr()
    assert et.et_debug_attention(0, p, p, p, 0, 0, 1, 225, 1) == -1      # longer than the fused kernels hold on chip
    assert et.et_debug_attention(0, p, p, p, 0, 0, 1, 0, 1) == -1
    assert et.et_debug_attention(0, p, p, p, 0, 0, 0, 8, 1) == -1
    assert et.et_debug_attention(1, p, p, p, 0, 0, 1, 8, 1) == -1        # backward without dout / dqkv
    assert et.et_debug_attention(2, p, p, p, p, p, 1, 8, 1) == -1
    assert et.et_debug_attention(0, p + 2, p, p, 0, 0, 1, 8, 1) == -1    # misaligned
