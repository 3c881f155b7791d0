"""Pins of the oracle's time model and selection: the worked example of Section 2.2,
a definition-level pure-Python search, enumeration against the Section 6 recurrence
(with and without the Section 6.3 pruning), and the properties the optimum must have."""
import itertools

import numpy as np
import pytest

from oracle import select as sel


def test_time_model_worked_example():
    t_dw = [1, 2, 4, 8, 16]
    t_dy = [32, 64, 128, 256, 512]
    # only layer 3 (index 2) of 5 selected: t_dw(3) + t_dy(4) + t_dy(5)
    assert sel.t_selective([0, 0, 1, 0, 0], 1000, t_dw, t_dy) == 1000 + 4 + 256 + 512
    assert sel.t_selective([0, 0, 0, 0, 0], 1000, t_dw, t_dy) == 1000
    # full training never charges the input-most tensor's gradient passing
    assert sel.t_full(1000, t_dw, t_dy) == 1000 + 31 + (64 + 128 + 256 + 512)
    assert sel.t_selective([0, 0, 0, 1, 1, 0, 0], 0, [1] * 7, [10] * 7) == 2 + 30


def _random_instance(rng, N):
    style = rng.integers(0, 4)
    imp = rng.standard_normal(N) * (10.0 ** rng.integers(-6, 3))
    if style == 1:
        imp = np.round(imp / np.abs(imp).max() * 3)         # many ties and zeros
    if style == 2:
        imp[rng.random(N) < 0.3] = 0.0
    if style == 3:
        imp = np.abs(imp)
    t_dw = rng.integers(0, 50, N)
    t_dy = rng.integers(0, 50, N)
    t_dw[rng.random(N) < 0.15] = 0
    t_dy[rng.random(N) < 0.3] = 0
    t_fwd = int(rng.integers(0, 200))
    rho = int(rng.integers(150_000, 1_050_000))
    Tq = int(rng.choice([0, 7, 25, 60, 10_000]))
    return imp, [int(t) for t in t_dw], [int(t) for t in t_dy], t_fwd, rho, Tq


def _definition_search(imp, t_dw, t_dy, t_fwd, rho, Tq):
    """Pure-Python statement of the optimum on the quantised integers."""
    N = len(t_dw)
    iq = sel.quantise_importance(imp)
    a, b, budget = sel.quantise_times(t_fwd, t_dw, t_dy, rho, Tq)
    if budget < 0:
        return [0] * N
    best_key, best = None, None
    for mask in itertools.product([0, 1], repeat=N):
        if sel.t_selective(mask, 0, a, b) > budget:
            continue
        key = (-sum(i for i, m in zip(iq, mask) if m), mask)      # larger value, then smaller binary number
        if best_key is None or key < best_key:
            best_key, best = key, mask
    return list(best)


def test_enumeration_matches_pure_python_definition():
    rng = np.random.default_rng(0)
    for _ in range(300):
        inst = _random_instance(rng, int(rng.integers(1, 8)))
        got = sel.select_enumerate(*inst)
        assert list(got["mask"]) == _definition_search(*inst), inst


@pytest.mark.parametrize("seed", range(4))
def test_recurrence_matches_enumeration(seed):
    rng = np.random.default_rng(100 + seed)
    for _ in range(400):
        inst = _random_instance(rng, int(rng.integers(1, 13)))
        want = sel.select_enumerate(*inst)
        for prune in (True, False):
            got = sel.select_recurrence(*inst, prune=prune)
            assert got["status"] == want["status"]
            assert list(got["mask"]) == list(want["mask"]), (inst, prune)
            assert got["value_q"] == want["value_q"]
            assert got["predicted_ns"] == want["predicted_ns"]


def test_recurrence_at_sixteen_tensors():
    rng = np.random.default_rng(5)
    for _ in range(6):
        inst = _random_instance(rng, 16)
        assert list(sel.select_recurrence(*inst)["mask"]) == list(sel.select_enumerate(*inst)["mask"])


def test_pruning_skips_cells_without_changing_the_mask():
    rng = np.random.default_rng(8)
    N = 60
    imp = np.abs(rng.standard_normal(N))
    t_dw = [int(t) for t in rng.integers(1, 2000, N)]
    t_dy = [int(t) for t in rng.integers(1, 2000, N)]
    full = sel.select_recurrence(imp, t_dw, t_dy, 20000, 500_000, 1000, prune=False)
    pruned = sel.select_recurrence(imp, t_dw, t_dy, 20000, 500_000, 1000, prune=True)
    assert list(full["mask"]) == list(pruned["mask"])
    assert pruned["cells"] < full["cells"] / 2


def test_properties_of_the_optimum():
    rng = np.random.default_rng(2)
    for _ in range(60):
        imp, t_dw, t_dy, t_fwd, _, Tq = _random_instance(rng, 10)
        iq = sel.quantise_importance(imp)
        # rho = 100 %: exactly the tensors with positive importance
        r = sel.select_enumerate(imp, t_dw, t_dy, t_fwd, 1_000_000, Tq)
        assert list(r["mask"]) == [1 if q > 0 else 0 for q in iq]
        # the optimum value never decreases with rho; the predicted time respects the budget when unquantised
        last = -1
        for rho in (200_000, 400_000, 600_000, 800_000, 1_000_000):
            r = sel.select_enumerate(imp, t_dw, t_dy, t_fwd, rho, 0)
            if r["status"] == sel.INFEASIBLE:
                assert not r["mask"].any()
                assert rho * sel.t_full(t_fwd, t_dw, t_dy) // 1_000_000 < t_fwd
                continue
            assert r["value_q"] >= last
            last = r["value_q"]
            assert r["predicted_ns"] <= rho * sel.t_full(t_fwd, t_dw, t_dy) // 1_000_000
            # tensors of non-positive importance are never taken
            assert all(q > 0 for q, m in zip(iq, r["mask"]) if m)


def test_importance_quantisation():
    q = sel.quantise_importance([1.0, -0.5, 0.25, 0.0])
    assert q == [2 ** 39, -(2 ** 38), 2 ** 37, 0]
    assert sel.quantise_importance([0.0, 0.0]) == [0, 0]
    # max 3.0 = 0.75 * 2^2, so the scale is 2^38; halves go to the even neighbour
    q = sel.quantise_importance([3.0, 1.5 * 2.0 ** -38, 2.5 * 2.0 ** -38, -3.5 * 2.0 ** -38])
    assert q == [3 * 2 ** 38, 2, 2, -4]
    with pytest.raises(ValueError):
        sel.quantise_importance([1.0, float("nan")])
