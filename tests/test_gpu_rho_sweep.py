"""The rho sweep of the ViT-B workload: profile on the device, importance and selection re-run every
10 steps with the weights of 10 steps earlier as the snapshot; masks bit-identical to the oracle on
the device-produced inputs, measured step time against the time model's prediction."""
import time

import numpy as np
import pytest

from oracle import select as osel
from synth import CONFIGS, make_workload

pytestmark = pytest.mark.gpu


def _timed(s, xt, yt, mask, mk, first_step, n):
    import torch
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(n):
        s.train_step(xt, yt, mask, mk(first_step + i), want_loss=False)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / n


def test_vit_b_rho_sweep_time_model_and_masks():
    import torch
    from paper_2312_14227_amd import binding as et
    from paper_2312_14227_amd.session import Session, make_opt
    cfg = CONFIGS["vit_b"]
    wl = make_workload(cfg, seed=0)
    N = len(wl.weights)
    s = Session(cfg, wl.weights)
    xt, yt = s.put_input(wl.x, wl.y)
    # a learning rate small enough for ten Adam steps on this random-init model to descend, so
    # that undoing them would raise the loss (positive importance) for most tensors
    mk = lambda step: make_opt("adam", lr=1e-5, step=step)
    t_fwd, t_dw, t_dy = s.profile(xt, yt, warmup=3, reps=7)
    t_full = int(t_fwd) + int(t_dw.sum()) + int(t_dy[1:].sum())
    step = 1
    ones = np.ones(N, dtype=np.uint8)
    rows = []
    for rho in (0.3, 0.4, 0.5, 0.6, 0.7):
        # a period starts with ten full steps; their weight update is what the importance judges
        snap = [w.clone() for w in s.w]                       # snapshot = weights 10 steps earlier
        losses = []
        for _ in range(10):
            losses.append(s.train_step(xt, yt, ones, mk(step)))
            step += 1
        assert losses[-1] < losses[0], losses
        imp = s.importance(xt, yt, snap)
        assert (imp > 0).sum() >= N // 8                      # undoing a descending update raises the loss
        status, mask, pred = et.et_select(imp, t_dw, t_dy, t_fwd, int(rho * 1e6), 10_000)
        want = osel.select(imp, t_dw, t_dy, t_fwd, int(rho * 1e6), 10_000)
        assert status == want["status"] and list(mask) == list(want["mask"]) and pred == want["predicted_ns"], rho
        if status == et.ET_INFEASIBLE:
            assert not mask.any() and rho * t_full < t_fwd
            rows.append((rho, None, None, 0))
            continue
        assert mask.any(), "nothing selected although the budget allows backward work"
        assert pred <= rho * t_full * 1.02                    # the quantised model is optimistic by at most (#terms)/Tq
        _timed(s, xt, yt, mask, mk, step, 3)
        step += 3
        dt = min(_timed(s, xt, yt, mask, mk, step + 10 * r, 10) for r in range(3))
        step += 30
        rows.append((rho, dt * 1e9, pred, int(mask.sum())))
        assert abs(dt * 1e9 - pred) <= 0.10 * pred, (rho, dt * 1e9, pred)
    feasible = [r for r in rows if r[1] is not None]
    assert len(feasible) >= 3
    # (the importances are re-evaluated before every rho, so the predicted time need not grow with the budget)
    print("rho, measured ms, predicted ms, selected:", [(r[0], None if r[1] is None else round(r[1] / 1e6, 3),
                                                          None if r[2] is None else round(r[2] / 1e6, 3), r[3]) for r in rows])
    s.close()
