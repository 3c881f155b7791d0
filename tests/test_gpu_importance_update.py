"""Importance (Eq. 2), the masked optimizer update, the profiler and the selection on
GPU-produced inputs, against the oracle."""
import numpy as np
import pytest

from gpu_util import rel_l2, tol_for
from oracle import importance as oimp
from oracle import nets
from oracle import optim as oopt
from oracle import select as osel
from synth import CONFIGS, make_workload

pytestmark = pytest.mark.gpu


def _session(cfg, wl, **kw):
    from paper_2312_14227_amd.session import Session
    return Session(cfg, wl.weights, **kw)


@pytest.mark.parametrize("name", ["mlp", "vit_small"])
def test_importance_matches_oracle(name):
    cfg = CONFIGS[name]
    wl = make_workload(cfg, seed=0, init="random")
    N = len(wl.weights)
    I_ref, r = oimp.importance(cfg, wl.weights, wl.snapshot, wl.x, wl.y)
    A_ref = oimp.abs_importance_from_grads(r["grads"], wl.weights, wl.snapshot)
    s = _session(cfg, wl)
    xt, yt = s.put_input(wl.x, wl.y)
    snap = s.put_snapshot(wl.snapshot)
    I = s.importance(xt, yt, snap)
    tol = tol_for(cfg)
    worst = 0.0
    for k in range(N):
        # I_k is a cancelling signed sum: a gradient within tol (relative L2) moves g.dw by at most
        # tol |g| |dw| (Cauchy-Schwarz), so the error is judged against the larger of |I_k| and that
        gn = np.linalg.norm(r["grads"][k].ravel())
        dwn = np.linalg.norm((wl.snapshot[k].astype(np.float64) - wl.weights[k].astype(np.float64)).ravel())
        bound = tol * max(abs(I_ref[k]), gn * dwn)
        worst = max(worst, abs(I[k] - I_ref[k]) / bound)
        assert abs(I[k] - I_ref[k]) <= bound, (wl.names[k], I[k], I_ref[k], A_ref[k])
    print("worst importance error / bound: %.3f" % worst)
    # the reduction in isolation: same gradients (read back from the device) on both sides
    g_dev = [s.grads_host(k).reshape(wl.weights[k].shape) for k in range(N)]
    I_iso = oimp.importance_from_grads(g_dev, wl.weights, wl.snapshot)
    A_iso = oimp.abs_importance_from_grads(g_dev, wl.weights, wl.snapshot)
    for k in range(N):
        assert abs(I[k] - I_iso[k]) <= 1e-5 * A_iso[k] + 1e-300, (wl.names[k], I[k], I_iso[k])
    # a second call gives the same bits (fixed reduction order)
    assert np.array_equal(I, s.importance(xt, yt, snap))
    s.close()


@pytest.mark.parametrize("name,kind", [("mlp", "sgdw"), ("vit_small", "adam"), ("vit_small", "sgdw")])
def test_masked_update(name, kind):
    import torch
    from paper_2312_14227_amd.session import make_opt
    cfg = CONFIGS[name]
    wl = make_workload(cfg, seed=1, init="random")
    N = len(wl.weights)
    s = _session(cfg, wl)
    xt, yt = s.put_input(wl.x, wl.y)
    rng = np.random.default_rng(5)
    mask = (rng.random(N) < 0.5).astype(np.uint8)
    mask[0], mask[N - 1] = 1, 0
    # the C ABI carries the hyper-parameters as float32: give the oracle the same values
    hp = {k: float(np.float32(v)) for k, v in dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, momentum=0.9,
                                                    wd=5e-2).items()}
    w_ref = [w.astype(np.float64) for w in wl.weights]
    st_ref = [(np.zeros(w.shape), np.zeros(w.shape)) if kind == "adam" else (np.zeros(w.shape),) for w in wl.weights]
    bf16 = cfg.dtype == "bf16"
    for step in (1, 2, 3):
        before_w = [w.clone() for w in s.w]
        before_s = [[t.clone() for t in slots] for slots in s.state]
        s.train_step(xt, yt, mask, make_opt(kind, step=step, **hp))
        torch.cuda.synchronize()
        assert s.launch_counts()[2] == 1
        grads = [s.grads_host(k).reshape(wl.weights[k].shape) if mask[k] else None for k in range(N)]
        w_ref, st_ref = oopt.masked_update(kind, mask, w_ref, st_ref, grads, step=step, **hp)
        for k in range(N):
            if not mask[k]:
                assert torch.equal(s.w[k], before_w[k]), wl.names[k]
                for a, b in zip(s.state[k], before_s[k]):
                    assert torch.equal(a, b), wl.names[k]
                continue
            fp = (s.state[k][0] if bf16 else s.w[k]).cpu().numpy().astype(np.float64).reshape(w_ref[k].shape)
            np.testing.assert_allclose(fp, w_ref[k], rtol=2e-6, atol=step * 2e-3 * hp["lr"], err_msg=wl.names[k])
            m_dev = s.state[k][1 if bf16 else 0].cpu().numpy().astype(np.float64).reshape(w_ref[k].shape)
            np.testing.assert_allclose(m_dev, st_ref[k][0], rtol=1e-5, atol=1e-6 * np.abs(st_ref[k][0]).max() + 1e-30,
                                       err_msg=wl.names[k])
            if kind == "adam":
                v_dev = s.state[k][2 if bf16 else 1].cpu().numpy().astype(np.float64).reshape(w_ref[k].shape)
                np.testing.assert_allclose(v_dev, st_ref[k][1], rtol=1e-5, atol=1e-6 * np.abs(st_ref[k][1]).max() + 1e-30,
                                           err_msg=wl.names[k])
            if bf16:     # the bf16 copy is the rounded master weight
                assert torch.equal(s.w[k].reshape(-1), s.state[k][0].to(torch.bfloat16)), wl.names[k]
    s.close()


@pytest.mark.parametrize("name", ["mlp", "vit_small"])
def test_profile_and_select_bit_exact_on_device_inputs(name):
    from paper_2312_14227_amd import binding as et
    cfg = CONFIGS[name]
    wl = make_workload(cfg, seed=0, init="random")
    N = len(wl.weights)
    s = _session(cfg, wl)
    xt, yt = s.put_input(wl.x, wl.y)
    w_before = [w.clone() for w in s.w]
    t_fwd, t_dw, t_dy = s.profile(xt, yt, warmup=1, reps=3)
    import torch
    for a, b in zip(w_before, s.w):
        assert torch.equal(a, b)                       # profiling leaves the weights alone
    assert t_fwd > 0 and (t_dw > 0).all()
    names = wl.names
    for k in range(N):
        leaf = names[k].split(".")[-1]
        if cfg.kind == "vit" and (leaf == "b" or names[k] in ("pos", "patch.b")):
            assert t_dy[k] == 0, names[k]              # biases and shifts pass gradients for free
    assert t_dy[0] == 0                                 # never passed
    snap = s.put_snapshot(wl.snapshot)
    I = s.importance(xt, yt, snap)
    for rho in (300_000, 400_000, 500_000, 600_000, 700_000, 1_000_000):
        for Tq in (1000, 10_000):
            st, mask, pred = et.et_select(I, t_dw, t_dy, t_fwd, rho, Tq)
            want = osel.select(I, t_dw, t_dy, t_fwd, rho, Tq)
            assert st == want["status"]
            assert list(mask) == list(want["mask"]), (rho, Tq)
            assert pred == want["predicted_ns"]
    s.close()


def test_importance_from_master_weights():
    """Full-precision weight updates: float32 snapshots against the float32 master weights."""
    import torch
    from paper_2312_14227_amd import binding as et
    from paper_2312_14227_amd.session import make_opt
    cfg = CONFIGS["vit_small"]
    wl = make_workload(cfg, seed=2, init="random")
    N = len(wl.weights)
    s = _session(cfg, wl)
    xt, yt = s.put_input(wl.x, wl.y)
    snap = [st[0].clone() for st in s.state]
    ones = np.ones(N, dtype=np.uint8)
    for step in (1, 2, 3):
        s.train_step(xt, yt, ones, make_opt("adam", lr=1e-5, step=step))
    I = s.importance_master(xt, yt, snap)
    torch.cuda.synchronize()
    g = [s.grads_host(k) for k in range(N)]
    w = [s.state[k][0].cpu().numpy().astype(np.float64) for k in range(N)]
    sn = [t.cpu().numpy().astype(np.float64) for t in snap]
    I_ref = oimp.importance_from_grads(g, w, sn)
    A_ref = oimp.abs_importance_from_grads(g, w, sn)
    for k in range(N):
        assert abs(I[k] - I_ref[k]) <= 1e-5 * A_ref[k] + 1e-300, (wl.names[k], I[k], I_ref[k])
    assert (I > 0).sum() > N // 2                       # undoing descent steps raises the loss
    # the bf16 copies barely move at this learning rate: their delta w is mostly rounding noise
    I16 = s.importance(xt, yt, [t.to(torch.bfloat16) for t in snap])
    assert np.abs(I16 - I).max() > 0
    with pytest.raises(et.EtError):
        mlp = CONFIGS["mlp"]
        wl2 = make_workload(mlp, seed=0)
        s2 = _session(mlp, wl2)
        x2, y2 = s2.put_input(wl2.x, wl2.y)
        s2.importance_master(x2, y2, [w.clone() for w in s2.w])
    s.close()


def test_weight_and_gradient_magnitude_metrics():
    """The ablation's two metrics through the same segmented reduction, against the oracle's L1 norms."""
    from oracle import importance as oimp
    from paper_2312_14227_amd import binding as et
    cfg = CONFIGS["vit_small"]
    wl = make_workload(cfg, seed=4, init="random")
    N = len(wl.weights)
    ref = nets.step(cfg, wl.weights, wl.x, wl.y, [1] * N)
    s = _session(cfg, wl)
    xt, yt = s.put_input(wl.x, wl.y)
    wm = s.tensor_metric(None, None, et.ET_METRIC_WEIGHT_L1)
    want = oimp.weight_magnitude(wl.weights)
    assert np.all(np.abs(wm - want) <= 1e-5 * want + 1e-30), np.abs(wm / want - 1).max()   # same values, fp32 terms
    gm = s.tensor_metric(xt, yt, et.ET_METRIC_GRAD_L1)
    want = oimp.grad_magnitude(ref["grads"])
    assert np.all(np.abs(gm - want) <= tol_for(cfg) * want), np.abs(gm / want - 1).max()
    # selection runs on them like on importances
    t_fwd, t_dw, t_dy = s.profile(xt, yt, warmup=1, reps=3)
    for metric in (wm, gm):
        st, mask, pred = et.et_select(metric, t_dw, t_dy, t_fwd, 600_000, 1000)
        want_sel = osel.select(metric, [int(t) for t in t_dw], [int(t) for t in t_dy], int(t_fwd), 600_000, 1000)
        assert st == want_sel["status"] and list(mask) == list(want_sel["mask"])
    s.close()


def _bf16_storage_step(cfg, wl):
    """Oracle step with bf16 storage rounding for the convolutional families (see tests/test_gpu_resnet.py)."""
    from oracle import mobilenet as MB
    from oracle import resnet as R
    from oracle import vgg as V
    ones = [1] * len(wl.weights)
    if cfg.kind == "resnet":
        return R.resnet_step(cfg, wl.weights, wl.x, wl.y, ones, store=R.round_bf16)
    if cfg.kind == "vgg":
        return V.vgg_step(cfg, wl.weights, wl.x, wl.y, ones, store=R.round_bf16)
    return MB.mobilenet_step(cfg, wl.weights, wl.x, wl.y, ones, store=R.round_bf16)


@pytest.mark.parametrize("name", ["resnet_small", "vgg_small", "mobilenet_small"])
def test_importance_profile_and_selection_on_the_convolutional_families(name):
    """Eq. 2 importance against the oracle's (same storage rounding on both sides), the attribution of the profiled
    times (shifts and biases pass gradients for free) and bit-exact selection from the device's own numbers."""
    from paper_2312_14227_amd import binding as et
    cfg = CONFIGS[name]
    wl = make_workload(cfg, seed=7, init="random")
    N = len(wl.weights)
    r = _bf16_storage_step(cfg, wl)
    I_ref = oimp.importance_from_grads(r["grads"], wl.weights, wl.snapshot)
    s = _session(cfg, wl)
    xt, yt = s.put_input(wl.x, wl.y)
    snap = s.put_snapshot(wl.snapshot)
    I = s.importance(xt, yt, snap)
    tol = 0.1 * tol_for(cfg)
    for k in range(N):
        gn = np.linalg.norm(r["grads"][k].ravel())
        dwn = np.linalg.norm((wl.snapshot[k].astype(np.float64) - wl.weights[k].astype(np.float64)).ravel())
        assert abs(I[k] - I_ref[k]) <= tol * max(abs(I_ref[k]), gn * dwn), (wl.names[k], I[k], I_ref[k])
    t_fwd, t_dw, t_dy = s.profile(xt, yt, warmup=1, reps=3)
    assert t_fwd > 0 and (t_dw > 0).all() and t_dy[0] == 0
    for k in range(N):
        if wl.names[k].endswith(".b"):
            assert t_dy[k] == 0, wl.names[k]
    for rho in (400_000, 500_000, 700_000, 1_000_000):
        st, mask, pred = et.et_select(I, t_dw, t_dy, t_fwd, rho, 10_000)
        want = osel.select(I, t_dw, t_dy, t_fwd, rho, 10_000)
        assert st == want["status"] and list(mask) == list(want["mask"]) and pred == want["predicted_ns"], rho
    s.close()


def test_masked_update_sgd_on_a_convolutional_model():
    import torch
    from paper_2312_14227_amd.session import make_opt
    cfg = CONFIGS["mobilenet_small"]
    wl = make_workload(cfg, seed=3, init="random")
    N = len(wl.weights)
    s = _session(cfg, wl)
    xt, yt = s.put_input(wl.x, wl.y)
    rng = np.random.default_rng(9)
    mask = (rng.random(N) < 0.5).astype(np.uint8)
    mask[N - 1] = 1
    hp = {k: float(np.float32(v)) for k, v in dict(lr=1e-2, beta1=0.9, beta2=0.999, eps=1e-8, momentum=0.9, wd=5e-3).items()}
    w_ref = [w.astype(np.float64) for w in wl.weights]
    st_ref = [(np.zeros(w.shape),) for w in wl.weights]
    for step in (1, 2):
        before = [w.clone() for w in s.w]
        s.train_step(xt, yt, mask, make_opt("sgdw", step=step, **hp))
        torch.cuda.synchronize()
        grads = [s.grads_host(k).reshape(wl.weights[k].shape) if mask[k] else None for k in range(N)]
        w_ref, st_ref = oopt.masked_update("sgdw", mask, w_ref, st_ref, grads, step=step, **hp)
        for k in range(N):
            if not mask[k]:
                assert torch.equal(s.w[k], before[k]), wl.names[k]
                continue
            fp = s.state[k][0].cpu().numpy().astype(np.float64).reshape(w_ref[k].shape)
            np.testing.assert_allclose(fp, w_ref[k], rtol=2e-6, atol=step * 2e-3 * hp["lr"], err_msg=wl.names[k])
            assert torch.equal(s.w[k].reshape(-1), s.state[k][0].to(torch.bfloat16)), wl.names[k]
    s.close()


@pytest.mark.parametrize("name,micro", [("vit_small", 1), ("mlp", 4), ("mlp", 8)])
def test_importance_aggregated_over_micro_batches(name, micro):
    """Section 4: the importance may be evaluated on micro-batches and aggregated.  The loss is a mean over the
    samples, so Eq. 2 is additive: the mean of et_importance over the micro-batches of a batch must be the oracle's
    importance of the whole batch, at the importance tolerance, and must select the same tensors."""
    from paper_2312_14227_amd import binding as et
    cfg = CONFIGS[name]
    wl = make_workload(cfg, seed=11, init="random")
    N, B = len(wl.weights), cfg.batch
    assert B % micro == 0
    I_ref, r = oimp.importance(cfg, wl.weights, wl.snapshot, wl.x, wl.y)
    s = _session(cfg, wl)
    xt, yt = s.put_input(wl.x, wl.y)
    t_fwd, t_dw, t_dy = s.profile(xt, yt, warmup=1, reps=3)
    I_full = s.importance(xt, yt, s.put_snapshot(wl.snapshot))
    sm = _session(cfg, wl, batch=micro, with_state=False)
    snap = sm.put_snapshot(wl.snapshot)
    agg = np.zeros(N)
    for i in range(0, B, micro):
        xm, ym = sm.put_input(wl.x[i:i + micro], wl.y[i:i + micro])
        agg += sm.importance(xm, ym, snap)
    agg /= B // micro
    tol = tol_for(cfg)
    worst = 0.0
    for k in range(N):
        gn = np.linalg.norm(r["grads"][k].ravel())
        dwn = np.linalg.norm((wl.snapshot[k].astype(np.float64) - wl.weights[k].astype(np.float64)).ravel())
        bound = tol * max(abs(I_ref[k]), gn * dwn)
        worst = max(worst, abs(agg[k] - I_ref[k]) / bound)
        assert abs(agg[k] - I_ref[k]) <= bound, (wl.names[k], agg[k], I_ref[k])
    print("aggregated over %d micro-batches of %d: worst importance error / bound %.3f; max |agg - full| / max |I| %.2e"
          % (B // micro, micro, worst, np.abs(agg - I_full).max() / np.abs(I_full).max()))
    # Eq. 3 on the aggregated importances: the library and the oracle agree bit for bit on identical inputs
    for rho in (400_000, 600_000, 800_000):
        st, mask, pred = et.et_select(agg, t_dw, t_dy, t_fwd, rho, 10_000)
        want = osel.select(agg, [int(t) for t in t_dw], [int(t) for t in t_dy], int(t_fwd), rho, 10_000)
        assert st == want["status"] and list(mask) == list(want["mask"]) and pred == want["predicted_ns"]
    sm.close()
    s.close()
