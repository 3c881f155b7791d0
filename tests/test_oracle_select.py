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


def test_time_quantisation_by_hand():
    """Eq. 8 with every integer worked out by hand: t~ = floor(t * T_q / T_b), T_b the full backward time, in which
    the input-most tensor's gradient passing is never charged (Section 2.2, Eq. 7)."""
    t_dw, t_dy, t_fwd = [7, 13, 5, 11], [1000, 9, 17, 3], 20
    # T_b = (7 + 13 + 5 + 11) + (9 + 17 + 3) = 65, not 1065; T_full = 85
    assert sel.t_full(t_fwd, t_dw, t_dy) == 85
    # rho = 0.7: floor(59.5) - 20 = 39 ns (a ceiling would give 40)
    a, b, budget = sel.quantise_times(t_fwd, t_dw, t_dy, 700_000, 0)
    assert (a, b, budget) == (t_dw, t_dy, 39)
    # T_q = 10: 70/65, 130/65, 50/65, 110/65 -> 1, 2, 0, 1 (ceilings: 2, 2, 1, 2; with t_dy[0] in T_b all four
    # would be 0); 10000/65, 90/65, 170/65, 30/65 -> 153, 1, 2, 0; budget 390/65 = 6 exactly
    a, b, budget = sel.quantise_times(t_fwd, t_dw, t_dy, 700_000, 10)
    assert (a, b, budget) == ([1, 2, 0, 1], [153, 1, 2, 0], 6)
    # rho = 0.69: floor(58.65) - 20 = 38 -> 380/65 = 5.85 -> 5
    assert sel.quantise_times(t_fwd, t_dw, t_dy, 690_000, 10)[2] == 5
    # T_q = 64 is still below T_b = 65: 448/65, 832/65, 320/65, 704/65 -> 6, 12, 4, 10
    a, b, budget = sel.quantise_times(t_fwd, t_dw, t_dy, 700_000, 64)
    assert (a, b[1:], budget) == ([6, 12, 4, 10], [8, 16, 2], 38)
    # T_q >= T_b keeps nanoseconds
    for Tq in (65, 66, 10_000):
        assert sel.quantise_times(t_fwd, t_dw, t_dy, 700_000, Tq) == (t_dw, t_dy, 39)
    # the budget: rho * T_full below T_fwd is infeasible; exactly T_fwd leaves a budget of zero
    assert sel.quantise_times(t_fwd, t_dw, t_dy, 235_294, 10)[2] == -1     # floor(19.99999) = 19 < 20
    assert sel.quantise_times(t_fwd, t_dw, t_dy, 235_295, 10)[2] == 0      # floor(20.000075) = 20
    assert sel.quantise_times(t_fwd, t_dw, t_dy, 235_295, 0)[2] == 0
    # and the search uses exactly these integers: at T_q = 10 and budget 6 tensors 1 and 2 (a = 2 + 0, passing
    # b[2] + b[3] = 2) fit together with tensor 3 (a = 1): cost 2 + 0 + 1 + 2 = 5 <= 6, while adding tensor 0 would
    # charge b[1] = 1 and a[0] = 1 more: 7 > 6
    imp = [1.0, 1.0, 1.0, 1.0]
    for method in ("enumerate", "recurrence"):
        r = sel.select(imp, t_dw, t_dy, t_fwd, 700_000, 10, method=method)
        assert list(r["mask"]) == [0, 1, 1, 1] and r["status"] == sel.OK
        # in nanoseconds tensor 1..3 cost 13 + 5 + 11 + 17 + 3 = 49 > 39: the unquantised search must drop some
        r0 = sel.select(imp, t_dw, t_dy, t_fwd, 700_000, 0, method=method)
        assert sel.t_selective(r0["mask"], 0, t_dw, t_dy) <= 39 and int(r0["mask"].sum()) == 2
