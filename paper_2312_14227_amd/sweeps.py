"""Measurement sweeps around the selective step (run on the GPU):

  python -m paper_2312_14227_amd.sweeps --what tq         time resolution T_q of Eq. 8 (Section 6.3, Figure 10):
                                                           table sizes with and without pruning, selection time,
                                                           predicted and measured step time per T_q and rho
  python -m paper_2312_14227_amd.sweeps --what baselines  fixed masks (full training, head only, norms and biases)
                                                           and the three importance metrics of the ablation
  python -m paper_2312_14227_amd.sweeps --what schedule   cost of the importance evaluation: full batch against
                                                           aggregated micro-batches of 4 (Section 4), and its share
                                                           of the training time for several evaluation periods

Inputs are the seeded synthetic workload of the benchmark.  Everything runs through the C ABI.
"""
import argparse
import time

import numpy as np


def _timed(s, xt, yt, mask, mk, n, warm=3):
    import torch
    for i in range(warm):
        s.train_step(xt, yt, mask, mk(1 + i), want_loss=False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(n):
        s.train_step(xt, yt, mask, mk(1 + warm + i), want_loss=False)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / n * 1e3


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--what", choices=["tq", "baselines", "schedule"], required=True)
    ap.add_argument("--config", default="vit_b")
    ap.add_argument("--steps", type=int, default=10)
    a = ap.parse_args()

    import torch
    from . import binding as et
    from .session import Session, make_opt
    from synth import CONFIGS, make_workload

    cfg = CONFIGS[a.config]
    wl = make_workload(cfg, seed=0)
    N = len(wl.weights)
    s = Session(cfg, wl.weights)
    xt, yt = s.put_input(wl.x, wl.y)
    snap = s.put_snapshot(wl.snapshot)
    kind = "adam" if cfg.kind == "vit" else "sgdw"
    mk = lambda step: make_opt(kind, step=step, lr=1e-5)
    t_fwd, t_dw, t_dy = s.profile(xt, yt, warmup=3, reps=7)
    imp = s.importance(xt, yt, snap)
    ones = np.ones(N, dtype=np.uint8)
    t_full_model = int(t_fwd) + int(t_dw.sum()) + int(t_dy[1:].sum())
    # (the schedule sweep compares importances of identical weights, so it trains only at its end)
    full_ms = _timed(s, xt, yt, ones, mk, a.steps) if a.what != "schedule" else float("nan")
    print("# %s: batch %d, %d tensors; profiled T_fwd %.3f ms, T_full (model) %.3f ms%s"
          % (cfg.name, cfg.batch, N, t_fwd / 1e6, t_full_model / 1e6,
             "" if a.what == "schedule" else ", measured full step %.3f ms" % full_ms))

    if a.what == "tq":
        print("%8s %5s %9s %12s %12s %12s %9s %8s %10s %10s %9s" % (
            "Tq", "rho", "select_ms", "cells_table", "cells_pruned", "cells_knap", "selected", "first", "pred/full", "meas/full", "meas/pred"))
        for tq in (100, 1000, 10_000, 100_000, 1_000_000):
            for rho in (0.4, 0.5, 0.6):
                t0 = time.perf_counter()
                st, mask, pred, cnt = et.et_select_stats(imp, t_dw, t_dy, t_fwd, int(rho * 1e6), tq)
                sel_ms = (time.perf_counter() - t0) * 1e3
                if st != et.ET_OK:
                    print("%8d %5.2f %9.3f   infeasible (the forward pass alone exceeds the budget)" % (tq, rho, sel_ms))
                    continue
                ms = _timed(s, xt, yt, mask, mk, a.steps)
                print("%8d %5.2f %9.3f %12d %12d %12d %9d %8d %10.3f %10.3f %9.3f" % (
                    tq, rho, sel_ms, cnt["cells_table"], cnt["cells_pruned"], cnt["cells_knapsack"], int(mask.sum()),
                    int(np.argmax(mask)), pred / t_full_model, ms / full_ms, ms / (pred / 1e6)))

    if a.what == "baselines":
        rows = [("full training", ones)]
        head = np.zeros(N, dtype=np.uint8)
        head[-2:] = 1
        rows.append(("head only", head))
        leaf = [n.split(".")[-1] for n in wl.names]
        nb = np.array([1 if (l in ("g", "b") or wl.names[i] in ("cls", "pos")) else 0 for i, l in enumerate(leaf)], dtype=np.uint8)
        nb[-2:] = 1
        rows.append(("norms, biases and head", nb))
        wmag = s.tensor_metric(None, None, et.ET_METRIC_WEIGHT_L1)
        gmag = s.tensor_metric(xt, yt, et.ET_METRIC_GRAD_L1)
        for name, metric in (("selected, Eq. 2 importance", imp), ("selected, weight magnitude", wmag),
                             ("selected, gradient magnitude", gmag)):
            st, mask, pred = et.et_select(metric, t_dw, t_dy, t_fwd, 500_000, 10_000)
            rows.append((name + " (rho 0.5)", mask))
        print("%-42s %9s %8s %10s %10s" % ("mask", "selected", "first", "ms/step", "vs full"))
        for name, mask in rows:
            ms = _timed(s, xt, yt, mask, mk, a.steps)
            print("%-42s %9d %8d %10.3f %10.3f" % (name, int(mask.sum()), int(np.argmax(mask)), ms, ms / full_ms))

    if a.what == "schedule":
        micro = 4
        sm = Session(cfg, wl.weights, batch=micro, with_state=False)
        snap_m = sm.put_snapshot(wl.snapshot)
        parts = []
        for i in range(0, cfg.batch, micro):
            parts.append(sm.put_input(wl.x[i:i + micro], wl.y[i:i + micro]))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        agg = np.zeros(N)
        for (xm, ym) in parts:
            agg += sm.importance(xm, ym, snap_m)
        agg /= len(parts)
        t_micro_all = (time.perf_counter() - t0) * 1e3
        t0 = time.perf_counter()
        one = sm.importance(*parts[0], snap_m)
        t_micro_one = (time.perf_counter() - t0) * 1e3
        t0 = time.perf_counter()
        full_imp = s.importance(xt, yt, snap)
        t_full = (time.perf_counter() - t0) * 1e3
        scale = np.abs(full_imp).max()
        print("importance evaluation: full batch %d: %.3f ms; one micro-batch of %d: %.3f ms; %d aggregated micro-batches: %.3f ms"
              % (cfg.batch, t_full, micro, t_micro_one, len(parts), t_micro_all))
        print("aggregated micro-batches against the full batch (the loss is a mean, so Eq. 2 is additive over samples): "
              "max |difference| / max |I| = %.3e" % (np.abs(agg - full_imp).max() / scale))
        sel = {}
        for name, v in (("full batch", full_imp), ("aggregated micro-batches", agg), ("one micro-batch", one)):
            st, mask, pred = et.et_select(v, t_dw, t_dy, t_fwd, 500_000, 10_000)
            sel[name] = mask
        base = sel["full batch"]
        for name, m in sel.items():
            inter, union = int((m & base).sum()), int((m | base).sum())
            print("selection at rho 0.5 from %-26s: %3d tensors, Jaccard with the full-batch selection %.3f" % (name, int(m.sum()), inter / max(union, 1)))
        st, mask, pred = et.et_select(full_imp, t_dw, t_dy, t_fwd, 500_000, 10_000)
        step_ms = _timed(s, xt, yt, mask, mk, a.steps)
        t0 = time.perf_counter()
        et.et_select(full_imp, t_dw, t_dy, t_fwd, 500_000, 10_000)
        sel_ms = (time.perf_counter() - t0) * 1e3
        print("selective step at rho 0.5: %.3f ms; selection %.3f ms" % (step_ms, sel_ms))
        print("%-28s %10s %10s" % ("evaluation period (steps)", "full batch", "one micro"))
        for period in (10, 100, 1000):
            print("%-28d %9.2f%% %9.2f%%" % (period, 100 * (t_full + sel_ms) / (period * step_ms),
                                             100 * (t_micro_one + sel_ms) / (period * step_ms)))
        sm.close()
    s.close()


if __name__ == "__main__":
    main()
