"""bf16 MFMA GEMM kernel against a float64 matmul of the same bf16 inputs, through the C ABI."""
import numpy as np
import pytest

from synth import bf16_round

pytestmark = pytest.mark.gpu

CASES = [
    # (M, N, K, a_t, b_t) : several tiles and ragged tails in every dimension
    (197, 197, 64, 0, 0), (197, 64, 197, 0, 1), (197, 64, 197, 1, 1), (200, 768, 64, 1, 1),
    (300, 200, 136, 0, 0), (300, 136, 200, 0, 1), (136, 200, 300, 1, 1),
    (1000, 768, 768, 0, 0), (1000, 768, 3072, 0, 1), (768, 768, 5000, 1, 1), (64, 200, 768, 0, 0),
    (3, 8, 8, 0, 0), (129, 129 + 7, 72, 0, 1),
]


def _run(M, N, K, a_t, b_t, c_f32, bias, residual, split_k, tile, seed):
    import torch
    from paper_2312_14227_amd import binding as et
    rng = np.random.default_rng(seed)
    K8, M8, N8 = (K + 7) // 8 * 8, (M + 7) // 8 * 8, (N + 7) // 8 * 8
    A = np.zeros((K, M8) if a_t else (M, K8), dtype=np.float32)
    B = np.zeros((K, N8) if b_t else (N, K8), dtype=np.float32)
    if a_t:
        A[:, :M] = bf16_round(rng.standard_normal((K, M)).astype(np.float32))
    else:
        A[:, :K] = bf16_round(rng.standard_normal((M, K)).astype(np.float32))
    if b_t:
        B[:, :N] = bf16_round(rng.standard_normal((K, N)).astype(np.float32))
    else:
        B[:, :K] = bf16_round(rng.standard_normal((N, K)).astype(np.float32))
    Am = A[:, :M].T.astype(np.float64) if a_t else A[:, :K].astype(np.float64)
    Bm = B[:, :N].T.astype(np.float64) if b_t else B[:, :K].astype(np.float64)
    ref = Am @ Bm.T
    scale = np.abs(Am) @ np.abs(Bm).T
    dev = "cuda:0"
    At = torch.from_numpy(A).to(dev).to(torch.bfloat16)
    Bt = torch.from_numpy(B).to(dev).to(torch.bfloat16)
    ldc = N8 if not split_k > 1 else N
    Ct = torch.full((M, ldc), float("nan"), device=dev, dtype=torch.float32 if c_f32 else torch.bfloat16)
    bias_t = res_t = None
    if bias:
        b = bf16_round(rng.standard_normal(N).astype(np.float32))
        bias_t = torch.from_numpy(b).to(dev).to(torch.bfloat16)
        ref = ref + b.astype(np.float64)
    if residual:
        r = rng.standard_normal((M, ldc)).astype(np.float32)       # same leading dimension as C
        res_t = torch.from_numpy(r).to(dev)
        ref = ref + r[:, :N].astype(np.float64)
    part = torch.empty(M * N * split_k, device=dev, dtype=torch.float32) if split_k > 1 else None
    st = et.et_debug_gemm_bf16(At.data_ptr(), Bt.data_ptr(), Ct.data_ptr(), M, N, K, A.shape[1], B.shape[1], ldc, a_t,
                               b_t, c_f32, 1.0, bias_t.data_ptr() if bias else 0, res_t.data_ptr() if residual else 0,
                               split_k, part.data_ptr() if part is not None else 0, tile,
                               torch.cuda.current_stream().cuda_stream)   # (plain epilogue)
    assert st == 0
    torch.cuda.synchronize()
    got = Ct.float().cpu().numpy().astype(np.float64)[:, :N]
    # fp32 accumulation of exact bf16 products, then one rounding of the output
    bound = 2e-6 * scale * np.sqrt(K) + 1e-6 + (0 if c_f32 else 2.0 ** -8 * np.abs(ref))
    bad = np.abs(got - ref) > bound
    assert not bad.any(), (int(bad.sum()), float(np.abs(got - ref).max()))
    if ldc > N and not c_f32:
        assert torch.isnan(Ct[:, N:].float()).all()        # nothing written outside the N columns


@pytest.mark.parametrize("M,N,K,a_t,b_t", CASES)
def test_gemm_layouts_fp32_out(M, N, K, a_t, b_t):
    _run(M, N, K, a_t, b_t, 1, False, False, 1, 0, seed=M + N + K)


@pytest.mark.parametrize("M,N,K,a_t,b_t", CASES[:8])
def test_gemm_bf16_out_bias(M, N, K, a_t, b_t):
    _run(M, N, K, a_t, b_t, 0, True, False, 1, 0, seed=7 + M)


@pytest.mark.parametrize("M,N,K", [(197, 197, 64), (300, 200, 136), (1000, 768, 768), (64, 200, 768)])
def test_gemm_fp32_out_bias_residual(M, N, K):
    _run(M, N, K, 0, 0, 1, True, True, 1, 0, seed=11 + M)


@pytest.mark.parametrize("tile", [1, 3])
@pytest.mark.parametrize("M,N,K,a_t,b_t", [(300, 200, 136, 0, 0), (300, 136, 200, 0, 1), (136, 200, 300, 1, 1)])
def test_gemm_every_tile_shape(M, N, K, a_t, b_t, tile):
    _run(M, N, K, a_t, b_t, 1, True, False, 1, tile, seed=tile)


@pytest.mark.parametrize("tile", [5, 7])
@pytest.mark.parametrize("M,N,K,a_t,b_t", [(700, 520, 160, 0, 0), (700, 160, 512, 0, 1), (520, 264, 704, 1, 1),
                                           (1000, 768, 768, 0, 0), (200, 768, 64, 1, 1), (3, 8, 32, 0, 0)])
def test_gemm_direct_to_lds_tiles(M, N, K, a_t, b_t, tile):
    _run(M, N, K, a_t, b_t, 1, True, a_t == 0 and b_t == 0, 1, tile, seed=tile + M)
    _run(M, N, K, a_t, b_t, 0, True, False, 1, tile, seed=tile + N)


@pytest.mark.parametrize("M,N,K,a_t,b_t", [(700, 520, 192, 0, 0), (700, 192, 512, 0, 1), (520, 264, 704, 1, 1),
                                           (1000, 768, 768, 0, 0), (200, 768, 64, 1, 1), (3, 8, 64, 0, 0),
                                           (513, 300, 128, 0, 0), (260, 257, 256, 0, 1)])
@pytest.mark.parametrize("tile", [11, 13, 15, 17])
def test_gemm_two_group_tile(M, N, K, a_t, b_t, tile):
    """Slices of 64 through registers into two LDS stages: one, two, three and many slices."""
    _run(M, N, K, a_t, b_t, 1, True, a_t == 0 and b_t == 0, 1, tile, seed=tile + M)
    _run(M, N, K, a_t, b_t, 0, True, False, 1, tile, seed=tile + N)


@pytest.mark.parametrize("tile", [11, 13, 15, 17, 19, 21])
def test_gemm_two_group_tile_split_k(tile):
    _run(768, 520, 4992, 1, 1, 1, False, False, 6, tile, seed=3)


@pytest.mark.parametrize("split", [2, 5, 16, 40, 200])
def test_gemm_split_k_weight_gradient(split):
    if split > 32:      # many chunks: the reduction that shares one output among 16 lanes
        _run(24, 40, 64 * 4 * split + 64, 1, 1, 1, False, False, split, 0, seed=split)
        return
    _run(768, 200, 5000, 1, 1, 1, False, False, split, 0, seed=split)
    _run(136, 200, 300, 1, 1, 1, False, False, split, 0, seed=split + 1)


def test_gemm_rejects_bad_arguments():
    import torch
    from paper_2312_14227_amd import binding as et
    t = torch.zeros(64 * 64, device="cuda:0", dtype=torch.bfloat16)
    c = torch.zeros(64 * 64, device="cuda:0", dtype=torch.float32)
    assert et.et_debug_gemm_bf16(t.data_ptr(), t.data_ptr(), c.data_ptr(), 16, 16, 16, 12, 16, 16, 0, 0, 1) == et.ET_EINVAL
    assert et.et_debug_gemm_bf16(t.data_ptr() + 2, t.data_ptr(), c.data_ptr(), 16, 16, 16, 16, 16, 16, 0, 0, 1) == et.ET_EINVAL
    assert et.et_debug_gemm_bf16(t.data_ptr(), t.data_ptr(), c.data_ptr(), 16, 16, 16, 16, 16, 16, 1, 0, 1) == et.ET_EINVAL
    assert et.et_debug_gemm_bf16(0, t.data_ptr(), c.data_ptr(), 16, 16, 16, 16, 16, 16, 0, 0, 1) == et.ET_EINVAL


@pytest.mark.parametrize("tile", [0, 1, 7, 11, 13])
@pytest.mark.parametrize("M,N,K", [(700, 520, 192), (1000, 768, 768), (513, 300, 128), (77, 136, 64)])
def test_gemm_gelu_epilogues(M, N, K, tile):
    """The fused GELU epilogues against the oracle's erf-form GELU and its derivative: forward (two outputs), forward
    without the derivative, and the backward product that multiplies by the stored derivative."""
    import torch
    from oracle import nets
    from paper_2312_14227_amd import binding as et
    rng = np.random.default_rng(1000 * tile + M)
    N8 = (N + 7) // 8 * 8
    dev = "cuda:0"
    stream = torch.cuda.current_stream().cuda_stream
    A = bf16_round(rng.standard_normal((M, K)).astype(np.float32) * 0.3)
    B = bf16_round(rng.standard_normal((N, K)).astype(np.float32) * 0.3)
    b = bf16_round(rng.standard_normal(N).astype(np.float32))
    At, Bt = torch.from_numpy(A).to(dev).to(torch.bfloat16), torch.from_numpy(B).to(dev).to(torch.bfloat16)
    bt = torch.from_numpy(b).to(dev).to(torch.bfloat16)
    u = A.astype(np.float64) @ B.astype(np.float64).T + b.astype(np.float64)
    slack = 2e-6 * (np.abs(A).astype(np.float64) @ np.abs(B).astype(np.float64).T) * np.sqrt(K) + 1e-5   # fp32 sum, erf approximation
    for epi in (1, 3):
        C1 = torch.full((M, N8), float("nan"), device=dev, dtype=torch.bfloat16)
        C2 = torch.full((M, N8), float("nan"), device=dev, dtype=torch.bfloat16)
        st = et.et_debug_gemm_bf16(At.data_ptr(), Bt.data_ptr(), C1.data_ptr(), M, N, K, K, K, N8, 0, 0, 0, 1.0, bt.data_ptr(), 0, 1, 0,
                                   tile, stream, epilogue=epi, aux=C2.data_ptr() if epi == 1 else 0)
        assert st == 0
        torch.cuda.synchronize()
        got1 = C1.float().cpu().numpy().astype(np.float64)[:, :N]
        want1 = nets.gelu_grad(u) if epi == 1 else nets.gelu(u)
        # |d gelu / du| <= 1.13 and |d gelu' / du| <= 1: an error of the sum passes through at most unchanged
        assert (np.abs(got1 - want1) <= 1.2 * slack + 2.0 ** -8 * np.abs(want1)).all(), float(np.abs(got1 - want1).max())
        if epi == 1:
            got2 = C2.float().cpu().numpy().astype(np.float64)[:, :N]
            assert (np.abs(got2 - nets.gelu(u)) <= 1.2 * slack + 2.0 ** -8 * np.abs(nets.gelu(u))).all()
            if N8 > N:
                assert torch.isnan(C2[:, N:].float()).all() and torch.isnan(C1[:, N:].float()).all()
    # backward: dU = (dY W) * gelu'(u) with the stored derivative as second operand; here A [M][K] W [K][N] (b_t)
    W = bf16_round(rng.standard_normal((K, N8)).astype(np.float32) * 0.3)
    W[:, N:] = 0
    U = bf16_round(rng.standard_normal((M, N8)).astype(np.float32))
    Wt, Ut = torch.from_numpy(W).to(dev).to(torch.bfloat16), torch.from_numpy(U).to(dev).to(torch.bfloat16)
    C3 = torch.full((M, N8), float("nan"), device=dev, dtype=torch.bfloat16)
    st = et.et_debug_gemm_bf16(At.data_ptr(), Wt.data_ptr(), C3.data_ptr(), M, N, K, K, N8, N8, 0, 1, 0, 1.0, 0, 0, 1, 0, tile, stream,
                               epilogue=2, aux=Ut.data_ptr())
    assert st == 0
    torch.cuda.synchronize()
    want = (A.astype(np.float64) @ W[:, :N].astype(np.float64)) * U[:, :N].astype(np.float64)
    sl = (2e-6 * (np.abs(A).astype(np.float64) @ np.abs(W[:, :N]).astype(np.float64)) * np.sqrt(K) + 1e-6) * np.abs(U[:, :N])
    got = C3.float().cpu().numpy().astype(np.float64)[:, :N]
    assert (np.abs(got - want) <= sl + 2.0 ** -8 * np.abs(want)).all(), float(np.abs(got - want).max())
