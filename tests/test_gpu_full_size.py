"""Parity at the full size of the benchmark workloads (ViT-B shape at batch 64, ViT-L shape at batch
32, ResNet-50 shape at batch 32, VGG16 shape at batch 32), in the launch configuration bench.py times, against oracle values stored by tests/golden/make_full_size_golden.py
(per tensor 512 uniformly drawn gradient elements plus its 512 largest ones, gradient norms, loss,
importance)."""
import os

import numpy as np
import pytest

from gpu_util import rel_l2
from synth import CONFIGS, make_workload

pytestmark = pytest.mark.gpu
GOLD_DIR = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


# Tolerance.  ViT: the 2e-2 of the workload definition, against the exact oracle.  ResNet-50: the stored
# reference is the oracle with bf16 storage rounding (see oracle/resnet.py), and the bound is 2e-2 as well,
# except for the tensors for which the ORACLE ITSELF, evaluated twice with summation-order noise (3e-7) ahead of
# the storage rounding, is further apart than that: the golden writer stores that distance per tensor
# (`spread`), and such a tensor is bounded by twice its spread.  The mechanism (a flipped rounding perturbs
# everything behind it, a ReLU mask bit that changes drops or passes a whole gradient element, so two correct
# bf16 evaluations differ by per cent on the input side of a 50-layer ReLU network) is pinned on the CPU at the
# workload's own depth in tests/test_oracle_resnet.py; the small ResNet cases, where no rounding flips, agree
# to 2e-6 (tests/test_gpu_resnet.py).  The distance to the exact float64 gradient is printed beside it.
# VGG16: the same kind of reference and the same mechanism, but thirteen ReLU convolutions in a row with no
# shortcut to carry the gradient past them: the disagreement of two correct bf16 evaluations grows towards the
# input side, to 3-30 % at the first layers (CPU pin: noise of 3e-7 ahead of the storage rounding, in
# tests/test_oracle_vgg.py; observed here: median 3 %, worst 18 % at conv0.W).  A wrong kernel shows as an
# error of order one; the kernels themselves are compared element by element, layer by layer, in
# tests/test_gpu_conv3x3.py and tests/test_gpu_gemm.py, and the small cases, where no rounding flips, agree
# to 1e-7 (tests/test_gpu_vgg.py).
# MobileNetV2: 52 convolutions, ReLU6 clamping on both sides, random weights without normalisation: the same
# mechanism makes two correct bf16 evaluations agree to 0.3-2 % over the last eight tensors and disagree by
# 30-55 % from the middle of the network to its input (CPU pin: noise of 3e-7 on the oracle alone gives 26-85 % at
# batch 2, tests/test_oracle_mobilenet.py).  The end-to-end comparison at full size is therefore informative only
# at the output side (bound 5e-2 there; 0.75 elsewhere, which still rejects zero, sign-flipped or unrelated
# gradients); the depthwise kernels are compared with the oracle at the full-size shapes in
# tests/test_gpu_depthwise.py, the GEMMs in tests/test_gpu_gemm.py, and the small cases agree to 1e-7
# (tests/test_gpu_mobilenet.py).
# rho of the workload's configuration (0.5; ViT-L 0.4): Eq. 3 on the importances and the times the device itself
# produced at the full size must give the oracle's mask bit for bit
RHO_PPM = {"vit_b": 500_000, "vit_l": 400_000, "resnet50": 500_000, "vgg16": 500_000, "mobilenetv2": 500_000}


# tol: the workload tolerance (relative L2 per tensor, bf16 inputs with fp32 accumulation).  cap: the widest bound a
# tensor may get where the bf16-storage ORACLE itself, evaluated twice with summation-order noise, is further apart
# than tol (`spread`, stored per tensor by the golden writer): bound = max(tol, min(cap, 2 spread)).
@pytest.mark.parametrize("name,first,tol,cap", [("vit_b", 87, 2e-2, 2e-2), ("vit_l", 200, 2e-2, 2e-2), ("resnet50", 80, 2e-2, 0.1),
                                                ("vgg16", 11, 2e-2, 0.25), ("mobilenetv2", 60, 2e-2, 0.75)])
def test_full_size_gradients_importance_and_masks(name, first, tol, cap):
    import torch
    from oracle import select as osel
    from paper_2312_14227_amd import binding as et
    from paper_2312_14227_amd.session import Session
    G = np.load(os.path.join(GOLD_DIR, "%s_seed0.npz" % name))
    cfg = CONFIGS[name]
    assert int(G["batch"]) == cfg.batch
    wl = make_workload(cfg, seed=int(G["seed"]))
    N = len(wl.weights)
    s = Session(cfg, wl.weights, with_state=False)
    xt, yt = s.put_input(wl.x, wl.y)
    snap = s.put_snapshot(wl.snapshot)
    bounds = {n: tol for n in wl.names}
    if "spread" in G.files:
        # the convolutional workloads: where two bf16-storage evaluations of the ORACLE that differ by summation-order
        # noise are further apart than the workload tolerance (CPU pins of the mechanism in tests/test_oracle_resnet.py,
        # test_oracle_vgg.py, test_oracle_mobilenet.py), that distance, doubled, is the bound of the tensor, up to cap
        bounds = {n: max(tol, min(cap, 2.0 * float(G["spread"][k]))) for k, n in enumerate(wl.names)}
    errs, els = {}, {}
    I = s.importance(xt, yt, snap)                 # full backward, gradients stay in the buffers
    torch.cuda.synchronize()
    full = [g.clone() for g in s.grad]
    worst, worst_i, worst_el = 0.0, 0.0, 0.0
    for k in range(N):
        idx = torch.from_numpy(G["idx_%d" % k].astype(np.int64)).to(s.dev)
        got = full[k][idx].cpu().numpy()
        err = rel_l2(got, G["g_%d" % k])
        worst = max(worst, err)
        errs[wl.names[k]] = err
        # element by element on the sample: no element is off by more than tol of the tensor's largest one
        el = float(np.max(np.abs(got - G["g_%d" % k])) / max(float(np.max(np.abs(G["g_%d" % k]))), 1e-30))
        worst_el = max(worst_el, el)
        els[wl.names[k]] = el
        nrm = float(torch.linalg.vector_norm(full[k].double()))
        assert abs(nrm - G["gnorm"][k]) <= bounds[wl.names[k]] * G["gnorm"][k], (wl.names[k], nrm, G["gnorm"][k])
        # a gradient within tol (relative L2) moves g.dw by at most tol |g| |dw| (Cauchy-Schwarz)
        dwn = float(np.linalg.norm((wl.snapshot[k].astype(np.float64) - wl.weights[k].astype(np.float64)).ravel()))
        bound = bounds[wl.names[k]] * max(abs(G["importance"][k]), G["gnorm"][k] * dwn)
        if bound > 0.0:
            worst_i = max(worst_i, abs(I[k] - G["importance"][k]) / bound)
        assert abs(I[k] - G["importance"][k]) <= bound, (wl.names[k], I[k], G["importance"][k])
    if name in ("vgg16", "mobilenetv2"):
        print("per tensor:", [(n, round(e, 4)) for n, e in errs.items()])
    if name == "mobilenetv2":
        # 52 convolutions with ReLU6 on random weights: two correct bf16 evaluations agree only near the output
        # (CPU pin in tests/test_oracle_mobilenet.py); there the workload-level agreement is required
        print("output side:", [(n, round(e, 4)) for n, e in list(errs.items())[-8:]])
        assert all(e <= 5e-2 for e in list(errs.values())[-8:]), list(errs.items())[-8:]
    if name == "vgg16":
        # the linear layers, which see the least of the disagreement, keep the workload tolerance
        assert all(e <= 2e-2 for n, e in errs.items() if n.startswith("fc")), errs
    if "spread" in G.files:
        wide = {n: round(b, 4) for n, b in bounds.items() if b > tol}
        print("%d of %d tensors bounded by the oracle's own spread instead of %.0e:" % (len(wide), N, tol), wide)
    if "gx_0" in G.files:
        ex = {n: rel_l2(full[k][torch.from_numpy(G["idx_%d" % k].astype(np.int64)).to(s.dev)].cpu().numpy(), G["gx_%d" % k])
              for k, n in enumerate(wl.names)}
        print("distance to the exact float64 gradient: median %.4f, worst %s; the bf16-storage oracle's own distance to it: "
              "median %.4f" % (float(np.median(list(ex.values()))), max(ex.items(), key=lambda kv: kv[1]),
                               float(np.median([rel_l2(G["g_%d" % k], G["gx_%d" % k]) for k in range(N)]))))
    top = sorted(errs.items(), key=lambda kv: -kv[1])[:6]
    print("largest sampled gradient errors:", [(n, round(e, 4)) for n, e in top],
          "| tensors above 2e-2:", sum(e > 2e-2 for e in errs.values()), "of", N, "| median %.4f" % float(np.median(list(errs.values()))))
    assert all(e <= bounds[n] for n, e in errs.items()), [(n, e, bounds[n]) for n, e in errs.items() if e > bounds[n]]
    top_el = sorted(els.items(), key=lambda kv: -kv[1])[:6]
    print("largest element errors / largest element:", [(n, round(e, 4)) for n, e in top_el])
    # (a tensor bounded by the oracle's spread: its worst element may be off by twice that L2 bound; where the bound
    # itself is of order one a single element says nothing)
    el_bound = {n: (b if b <= tol else 2.0 * b) for n, b in bounds.items()}
    assert all(e <= el_bound[n] for n, e in els.items() if bounds[n] <= 0.1), [(n, e, el_bound[n]) for n, e in els.items() if e > el_bound[n]]
    print("worst sampled relative L2 gradient error at full size: %.3e; worst element error / largest element: %.3e; "
          "worst importance error / bound: %.3f" % (worst, worst_el, worst_i))
    # Eq. 3 on what the device produced: times profiled in place, the importances just computed
    t_fwd, t_dw, t_dy = s.profile(xt, yt, warmup=1, reps=3)
    st, sel, pred = et.et_select(I, t_dw, t_dy, t_fwd, RHO_PPM[name], 10_000)
    want = osel.select(I, [int(t) for t in t_dw], [int(t) for t in t_dy], int(t_fwd), RHO_PPM[name], 10_000)
    assert st == want["status"] and list(sel) == list(want["mask"]) and pred == want["predicted_ns"], name
    print("rho %.2f: status %d, %d of %d tensors selected, first %d, predicted %.3f ms (full %.3f ms)"
          % (RHO_PPM[name] / 1e6, st, int(sel.sum()), N, int(np.argmax(sel)) if sel.any() else -1, pred / 1e6,
             osel.t_full(int(t_fwd), [int(t) for t in t_dw], [int(t) for t in t_dy]) / 1e6))
    # a selective step: selected gradients are the very same numbers, the rest is not written
    rng = np.random.default_rng(0)
    mask = np.zeros(N, dtype=np.uint8)
    mask[first:] = rng.random(N - first) < 0.3
    mask[first] = 1
    for g in s.grad:
        g.fill_(float("nan"))
    loss = s.train_step(xt, yt, mask)
    assert abs(loss - float(G["loss"])) <= tol * float(G["loss"])
    for k in range(N):
        if mask[k]:
            assert torch.equal(s.grad[k], full[k]), wl.names[k]
        else:
            assert bool(s.grad[k].isnan().all()), wl.names[k]
    s.close()


def test_full_size_importance_from_micro_batches():
    """Section 4 at the benchmark's size: Eq. 2 evaluated on 16 micro-batches of 4 and averaged is the importance of
    the batch of 64 (the loss is a mean over samples), against the oracle's stored full-batch importance at the
    importance tolerance; the selection from the aggregated values is the oracle's on the same numbers, and the
    full-batch selection is reported beside it."""
    import torch
    from oracle import select as osel
    from paper_2312_14227_amd import binding as et
    from paper_2312_14227_amd.session import Session
    name, micro, tol = "vit_b", 4, 2e-2
    G = np.load(os.path.join(GOLD_DIR, "%s_seed0.npz" % name))
    cfg = CONFIGS[name]
    wl = make_workload(cfg, seed=int(G["seed"]))
    N = len(wl.weights)
    s = Session(cfg, wl.weights, with_state=False)
    xt, yt = s.put_input(wl.x, wl.y)
    t_fwd, t_dw, t_dy = s.profile(xt, yt, warmup=1, reps=3)
    I_full = s.importance(xt, yt, s.put_snapshot(wl.snapshot))
    s.close()
    sm = Session(cfg, wl.weights, batch=micro, with_state=False)
    snap = sm.put_snapshot(wl.snapshot)
    agg = np.zeros(N)
    for i in range(0, cfg.batch, micro):
        xm, ym = sm.put_input(wl.x[i:i + micro], wl.y[i:i + micro])
        agg += sm.importance(xm, ym, snap)
    agg /= cfg.batch // micro
    sm.close()
    worst = 0.0
    for k in range(N):
        dwn = float(np.linalg.norm((wl.snapshot[k].astype(np.float64) - wl.weights[k].astype(np.float64)).ravel()))
        bound = tol * max(abs(G["importance"][k]), G["gnorm"][k] * dwn)
        worst = max(worst, abs(agg[k] - G["importance"][k]) / bound)
        assert abs(agg[k] - G["importance"][k]) <= bound, (wl.names[k], agg[k], G["importance"][k])
    st, mask, pred = et.et_select(agg, t_dw, t_dy, t_fwd, RHO_PPM[name], 10_000)
    want = osel.select(agg, [int(t) for t in t_dw], [int(t) for t in t_dy], int(t_fwd), RHO_PPM[name], 10_000)
    assert st == want["status"] and list(mask) == list(want["mask"]) and pred == want["predicted_ns"]
    _, mask_full, _ = et.et_select(I_full, t_dw, t_dy, t_fwd, RHO_PPM[name], 10_000)
    print("16 micro-batches of 4: worst importance error / bound %.3f; max |agg - full| / max |I| %.2e; "
          "mask equal to the full-batch selection: %s (%d vs %d tensors)"
          % (worst, np.abs(agg - I_full).max() / np.abs(I_full).max(), bool(np.array_equal(mask, mask_full)),
             int(mask.sum()), int(mask_full.sum())))
