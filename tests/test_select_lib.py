"""et_select (host code of the library, runs without a GPU) against the oracle: bit-identical
masks on identical inputs, by enumeration for N <= 16 and by the paper's recurrence beyond."""
import numpy as np
import pytest

from oracle import select as osel
from paper_2312_14227_amd import binding as et
from test_oracle_select import _random_instance


def _lib(inst):
    imp, t_dw, t_dy, t_fwd, rho, Tq = inst
    return et.et_select(imp, t_dw, t_dy, t_fwd, rho, Tq)


@pytest.mark.parametrize("seed", range(4))
def test_masks_match_enumeration(seed):
    rng = np.random.default_rng(1000 + seed)
    for _ in range(500):
        inst = _random_instance(rng, int(rng.integers(1, 15)))
        want = osel.select_enumerate(*inst)
        st, mask, pred = _lib(inst)
        assert st == want["status"], inst
        assert list(mask) == list(want["mask"]), inst
        assert pred == want["predicted_ns"]


def test_sixteen_tensors_enumerated():
    rng = np.random.default_rng(77)
    for _ in range(12):
        inst = _random_instance(rng, 16)
        want = osel.select_enumerate(*inst)
        st, mask, pred = _lib(inst)
        assert (st, list(mask), pred) == (want["status"], list(want["mask"]), want["predicted_ns"])


def _profile_like(rng, N, scale_ns):
    """Times shaped like a profiled transformer: matrices cost much more than vectors, vector
    tensors pass gradients for free."""
    kind = rng.integers(0, 3, N)
    t_dw = np.where(kind == 0, rng.integers(20, 80, N), rng.integers(1, 6, N)) * scale_ns
    t_dy = np.where(kind == 0, rng.integers(20, 120, N), np.where(kind == 1, 0, rng.integers(2, 30, N))) * scale_ns
    imp = rng.standard_normal(N) * np.exp(rng.standard_normal(N))
    t_fwd = int(0.5 * (t_dw.sum() + t_dy.sum()))
    return imp, [int(t) for t in t_dw], [int(t) for t in t_dy], t_fwd


@pytest.mark.parametrize("N,Tq", [(40, 500), (152, 1000), (152, 10_000), (296, 10_000)])
def test_masks_match_the_paper_recurrence_on_large_instances(N, Tq):
    rng = np.random.default_rng(N + Tq)
    imp, t_dw, t_dy, t_fwd = _profile_like(rng, N, 1000)
    for rho in (300_000, 400_000, 500_000, 600_000, 700_000, 1_000_000):
        want = osel.select_recurrence(imp, t_dw, t_dy, t_fwd, rho, Tq)
        st, mask, pred = et.et_select(imp, t_dw, t_dy, t_fwd, rho, Tq)
        assert st == want["status"]
        assert list(mask) == list(want["mask"]), (N, Tq, rho)
        assert pred == want["predicted_ns"]
        if st == et.ET_OK and rho < 1_000_000:
            # the quantised model is optimistic by at most one unit per charged term
            assert pred <= rho * osel.t_full(t_fwd, t_dw, t_dy) // 1_000_000 + 2 * N * (sum(t_dw) + sum(t_dy[1:])) // Tq


def test_error_paths():
    assert et.et_select([1.0, 2.0], [5, 5], [5, 5], 1000, 100_000, 0)[0] == et.ET_INFEASIBLE
    with pytest.raises(et.EtError) as e:
        et.et_select([1.0, float("nan")], [5, 5], [5, 5], 10, 500_000, 0)
    assert e.value.status == et.ET_ENAN
    with pytest.raises(et.EtError) as e:
        et.et_select([], [], [], 10, 500_000, 0)
    assert e.value.status == et.ET_EINVAL
    with pytest.raises(et.EtError) as e:       # nanosecond resolution on a long step: table too large
        et.et_select([1.0] * 200, [10 ** 8] * 200, [10 ** 8] * 200, 10 ** 9, 900_000, 0)
    assert e.value.status == et.ET_ENOMEM
    # all-zero importance and all-zero times are fine
    st, mask, _ = et.et_select([0.0, 0.0], [0, 0], [0, 0], 0, 500_000, 1000)
    assert st == et.ET_OK and not mask.any()
    st, mask, _ = et.et_select([1.0, 2.0], [0, 0], [0, 0], 0, 500_000, 1000)
    assert st == et.ET_OK and list(mask) == [1, 1]


@pytest.mark.parametrize("N,Tq", [(12, 50), (40, 500), (152, 1000)])
def test_table_sizes_match_the_cells_the_recurrence_visits(N, Tq):
    """et_select_stats: same mask as et_select, and the cell counts of Section 6.3 equal what the oracle's
    recurrence actually evaluates with and without pruning."""
    rng = np.random.default_rng(7 * N + Tq)
    imp, t_dw, t_dy, t_fwd = _profile_like(rng, N, 1000)
    for rho in (350_000, 500_000, 800_000):
        pruned = osel.select_recurrence(imp, t_dw, t_dy, t_fwd, rho, Tq, prune=True)
        full = osel.select_recurrence(imp, t_dw, t_dy, t_fwd, rho, Tq, prune=False)
        st, mask, pred, cnt = et.et_select_stats(imp, t_dw, t_dy, t_fwd, rho, Tq)
        st2, mask2, pred2 = et.et_select(imp, t_dw, t_dy, t_fwd, rho, Tq)
        assert (st, list(mask), pred) == (st2, list(mask2), pred2)
        assert list(mask) == list(pruned["mask"]) == list(full["mask"])
        if st != et.ET_OK:
            assert all(v == 0 for v in cnt.values())
            continue
        a, b, budget = osel.quantise_times(t_fwd, t_dw, t_dy, rho, Tq)
        assert cnt["budget_q"] == budget and cnt["backward_q"] == sum(a) + sum(b[1:])
        assert cnt["cells_pruned"] == pruned["cells"]
        assert cnt["cells_table"] == full["cells"]
        assert cnt["cells_knapsack"] == N * (budget + 1)
        assert cnt["cells_pruned"] <= cnt["cells_knapsack"] <= cnt["cells_table"]


def test_time_quantisation_by_hand():
    """The library's Eq. 8 integers for the instance worked out by hand in tests/test_oracle_select.py: the
    quantised full backward time and budget as et_select_stats reports them, and the masks that follow."""
    t_dw, t_dy, t_fwd = [7, 13, 5, 11], [1000, 9, 17, 3], 20
    imp = [1.0, 1.0, 1.0, 1.0]
    st, mask, pred, counts = et.et_select_stats(imp, t_dw, t_dy, t_fwd, 700_000, 10)
    # a = 1, 2, 0, 1 and b[1:] = 1, 2, 0: backward 7, budget floor(39 * 10 / 65) = 6
    assert st == 0 and counts["backward_q"] == 7 and counts["budget_q"] == 6
    assert list(mask) == [0, 1, 1, 1] and pred == 20 + 13 + 5 + 11 + 17 + 3
    st, mask, pred, counts = et.et_select_stats(imp, t_dw, t_dy, t_fwd, 700_000, 0)
    assert st == 0 and counts["backward_q"] == 65 and counts["budget_q"] == 39 and pred <= 20 + 39
    st, mask, pred, counts = et.et_select_stats(imp, t_dw, t_dy, t_fwd, 700_000, 64)
    assert counts["backward_q"] == 6 + 12 + 4 + 10 + 8 + 16 + 2 and counts["budget_q"] == 38
    assert et.et_select(imp, t_dw, t_dy, t_fwd, 235_294, 10)[0] == 1      # ET_INFEASIBLE
    # budget 0: at T_q = 10 tensor 2 costs a[2] + b[3] = 0 + 0 and is selected; in nanoseconds nothing is free
    st, mask, _ = et.et_select(imp, t_dw, t_dy, t_fwd, 235_295, 10)
    assert st == 0 and list(mask) == [0, 0, 1, 0]
    st, mask, _ = et.et_select(imp, t_dw, t_dy, t_fwd, 235_295, 0)
    assert st == 0 and not any(mask)
