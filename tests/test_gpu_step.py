"""Parity of the HIP training step with the fp64 oracle, through the C ABI, element by element
on the same seeded inputs; plus the invariants of selective training."""
import itertools

import numpy as np
import pytest

from gpu_util import rel_l2, sample_masks, tol_for
from oracle import nets
from synth import CONFIGS, make_workload

pytestmark = pytest.mark.gpu


def _session(cfg, wl, **kw):
    from paper_2312_14227_amd.session import Session
    return Session(cfg, wl.weights, **kw)


def _check_step(s, cfg, wl, xt, yt, mask, ref_full, tol):
    import torch
    for g in s.grad:
        g.fill_(float("nan"))
    loss = s.train_step(xt, yt, mask)
    torch.cuda.synchronize()
    assert abs(loss - ref_full["loss"]) <= tol * abs(ref_full["loss"]), (loss, ref_full["loss"])
    worst = 0.0
    for j in range(s.n):
        g = s.grad[j].cpu().numpy()
        if mask[j]:
            assert np.isfinite(g).all(), wl.names[j]
            err = rel_l2(g, ref_full["grads"][j])
            worst = max(worst, err)
            assert err <= tol, (wl.names[j], err, list(mask))
        else:
            assert np.isnan(g).all(), ("unselected gradient buffer was written", wl.names[j])
    return worst


def test_mlp_all_16_masks():
    cfg = CONFIGS["mlp"]
    wl = make_workload(cfg, seed=0)
    ref = nets.step(cfg, wl.weights, wl.x, wl.y, [1] * 4)
    s = _session(cfg, wl)
    xt, yt = s.put_input(wl.x, wl.y)
    for mask in itertools.product([0, 1], repeat=4):
        _check_step(s, cfg, wl, xt, yt, np.array(mask, dtype=np.uint8), ref, tol_for(cfg))
        fwd, bwd, upd = s.launch_counts()
        sel = [j for j in range(4) if mask[j]]
        assert fwd == 6 and upd == 0      # 4 GEMMs + the two cross-entropy launches
        assert bwd == (len(sel) + (3 - sel[0]) if sel else 0)      # dw per selected + dy after the first selected
    s.close()


@pytest.mark.parametrize("name,seed", [("vit_small", 0), ("vit_small", 1), ("vit_mid", 2), ("vit_t230", 3),
                                       ("vit_t40", 4), ("vit_w256", 5), ("vit_w512", 6), ("vit_w1280", 7),
                                       ("vit_w1536", 8), ("vit_w2048", 9)])
def test_vit_masks_match_oracle(name, seed):
    cfg = CONFIGS[name]
    wl = make_workload(cfg, seed=seed, init="random")
    N = len(wl.weights)
    ref = nets.step(cfg, wl.weights, wl.x, wl.y, [1] * N)
    s = _session(cfg, wl)
    xt, yt = s.put_input(wl.x, wl.y)
    rng = np.random.default_rng(seed)
    worst = 0.0
    for mask in sample_masks(N, rng, extra=(4, 6, 8, 10, 14, 15)):
        worst = max(worst, _check_step(s, cfg, wl, xt, yt, mask, ref, tol_for(cfg)))
    print("worst relative L2 error over tensors and masks: %.3e" % worst)
    s.close()


def test_vit_empty_mask_is_forward_only():
    cfg = CONFIGS["vit_small"]
    wl = make_workload(cfg, seed=0, init="random")
    N = len(wl.weights)
    loss_ref, _ = nets.forward(cfg, wl.weights, wl.x, wl.y)
    s = _session(cfg, wl)
    xt, yt = s.put_input(wl.x, wl.y)
    for g in s.grad:
        g.fill_(float("nan"))
    loss = s.train_step(xt, yt, np.zeros(N, dtype=np.uint8))
    fwd, bwd, upd = s.launch_counts()
    assert bwd == 0 and upd == 0 and fwd > 0
    assert abs(loss - loss_ref) <= 2e-2 * abs(loss_ref)
    for g in s.grad:
        assert bool(g.isnan().all())
    # the head alone: two weight-gradient launches' worth of work, no gradient passing
    m = np.zeros(N, dtype=np.uint8)
    m[N - 1] = 1
    s.train_step(xt, yt, m)
    assert s.launch_counts()[1] == 2
    s.close()


def test_step_is_deterministic():
    import torch
    cfg = CONFIGS["vit_small"]
    wl = make_workload(cfg, seed=3, init="random")
    N = len(wl.weights)
    s = _session(cfg, wl)
    xt, yt = s.put_input(wl.x, wl.y)
    ones = np.ones(N, dtype=np.uint8)
    l1 = s.train_step(xt, yt, ones)
    g1 = [g.clone() for g in s.grad]
    l2 = s.train_step(xt, yt, ones)
    assert l1 == l2
    for a, b in zip(g1, s.grad):
        assert torch.equal(a, b)
    s.close()


def test_kernel_timing_records_every_launch_and_its_own_overhead():
    """Measurement support: with timing enabled, a step's GEMM launches are all recorded with their algorithmic work,
    the summed durations are plausible, and the event-pair overhead measured beside them is a few microseconds."""
    from paper_2312_14227_amd import binding as et
    cfg = CONFIGS["vit_small"]
    wl = make_workload(cfg, seed=1, init="random")
    N = len(wl.weights)
    s = _session(cfg, wl)
    xt, yt = s.put_input(wl.x, wl.y)
    ones = np.ones(N, dtype=np.uint8)
    s.train_step(xt, yt, ones)
    with pytest.raises(RuntimeError):
        et.et_kernel_timing_overhead(s.ctx)          # nothing measured while timing is off
    et.et_kernel_timing(s.ctx, 1)
    s.train_step(xt, yt, ones)
    pair_ns = et.et_kernel_timing_overhead(s.ctx)
    assert 100.0 < pair_ns < 1e5, pair_ns
    n_fwd, ns_fwd, flop_fwd = et.et_kernel_timing_read(s.ctx, 0)
    n_dx, ns_dx, _ = et.et_kernel_timing_read(s.ctx, 1)
    n_dw, ns_dw, _ = et.et_kernel_timing_read(s.ctx, 2)
    # forward products: patch embedding, four per block, the head
    assert n_fwd == 4 * cfg.blocks + 2 and n_dw >= 4 * cfg.blocks and n_dx >= 4 * cfg.blocks - 1
    M = cfg.batch * cfg.tokens
    want = 2.0 * M * cfg.width * (3 * cfg.width + cfg.width + 2 * cfg.mlp) * cfg.blocks
    assert flop_fwd > want and flop_fwd < 1.5 * want
    for n, ns in ((n_fwd, ns_fwd), (n_dx, ns_dx), (n_dw, ns_dw)):
        assert ns > n * 0.5 * pair_ns and ns < n * 1e6      # every launch spans at least most of a pair, none a millisecond
    et.et_kernel_timing(s.ctx, 0)
    s.close()
