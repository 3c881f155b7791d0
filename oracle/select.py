"""Oracle time model and tensor selection.  TEST INFRASTRUCTURE ONLY.

Problem (Eq. 3): choose the binary mask M over the N tensors that maximises
M . I subject to  T_fwd + M . t_dw + f(M) . t_dy <= rho * T_full.

Readings (the paper is ambiguous or silent; index 0 is the input-most tensor):
  * f(M): t_dy of every tensor strictly output-side of the input-most selected
    tensor j*.  The worked example of Section 2.2 (only layer 3 of 5 selected
    costs t_dw(3) + t_dy(4) + t_dy(5)) and Eq. 7 (the sum stops at k-1) leave
    out t_dy(j*); the f(M) example of Section 3.3 would include it.  Two
    passages against one, and the hardware indeed stops there: excluded.
  * Times are unsigned integer nanoseconds.  Quantisation (Eq. 8):
    T_b = sum t_dw + sum_{j>=1} t_dy (the full backward time); if Tq == 0 or
    Tq >= T_b times are kept; else every time becomes floor(t * Tq / T_b).
  * Budget: B = floor(rho_ppm * T_full / 1e6) - T_fwd in nanoseconds, rho given
    in parts per million; B < 0 means nothing is feasible (empty mask,
    status INFEASIBLE); the budget is quantised by the same floor.
  * Importance is made an integer: with max|I| = m * 2^e (0.5 <= m < 1),
    Iq = rint(I * 2^(40 - e)), ties to even; all-zero importance stays zero.
  * Among feasible masks the best is the one with (1) the largest sum of Iq,
    (2) on ties the smallest mask read as a binary number whose most
    significant bit is tensor 0.
The oracle for N <= ~20 is enumeration of all masks.  The dynamic programme of
Section 6 (subproblems by backward depth, Eq. 7, with and without the pruning
of Section 6.3) is the oracle for larger N and is itself tested against
enumeration.
"""
import math

import numpy as np

OK, INFEASIBLE = 0, 1
_NEG = np.iinfo(np.int64).min // 4


def t_selective(mask, t_fwd, t_dw, t_dy):
    """Training time of one iteration under mask M (Section 2.2 time model)."""
    sel = [j for j, m in enumerate(mask) if m]
    if not sel:
        return int(t_fwd)
    jstar = sel[0]
    return int(t_fwd) + sum(int(t_dw[j]) for j in sel) + sum(int(t_dy[j]) for j in range(jstar + 1, len(mask)))


def t_full(t_fwd, t_dw, t_dy):
    return t_selective([1] * len(t_dw), t_fwd, t_dw, t_dy)


def quantise_importance(importance):
    imp = np.asarray(importance, dtype=np.float64)
    if not np.all(np.isfinite(imp)):
        raise ValueError("importance is not finite")
    imax = float(np.max(np.abs(imp))) if imp.size else 0.0
    if imax == 0.0:
        return [0] * imp.size
    _, e = math.frexp(imax)
    return [int(v) for v in np.rint(np.ldexp(imp, 40 - e))]


def quantise_times(t_fwd, t_dw, t_dy, rho_ppm, Tq):
    """Integer (a, b, budget) fed to the search; budget < 0 means infeasible."""
    t_dw = [int(t) for t in t_dw]
    t_dy = [int(t) for t in t_dy]
    T_b = sum(t_dw) + sum(t_dy[1:])
    budget_ns = (int(rho_ppm) * t_full(t_fwd, t_dw, t_dy)) // 1_000_000 - int(t_fwd)
    if budget_ns < 0:
        return t_dw, t_dy, -1
    if Tq == 0 or Tq >= T_b:
        return t_dw, t_dy, budget_ns
    a = [(t * Tq) // T_b for t in t_dw]
    b = [(t * Tq) // T_b for t in t_dy]
    return a, b, (budget_ns * Tq) // T_b


def _result(mask, status, t_fwd, t_dw, t_dy, **extra):
    out = dict(mask=np.asarray(mask, dtype=np.uint8), status=status,
               predicted_ns=t_selective(mask, t_fwd, t_dw, t_dy))
    out.update(extra)
    return out


def select_enumerate(importance, t_dw, t_dy, t_fwd, rho_ppm, Tq):
    """All 2^N masks; the definition of the optimum."""
    N = len(t_dw)
    assert N <= 22
    iq = quantise_importance(importance)
    a, b, budget = quantise_times(t_fwd, t_dw, t_dy, rho_ppm, Tq)
    if budget < 0:
        return _result([0] * N, INFEASIBLE, t_fwd, t_dw, t_dy, value_q=0)
    m = np.arange(1 << N, dtype=np.int64)
    bits = ((m[:, None] >> (N - 1 - np.arange(N))[None, :]) & 1).astype(np.int64)   # column j = tensor j
    value = bits @ np.asarray(iq, dtype=np.int64)
    cost = bits @ np.asarray(a, dtype=np.int64)
    after = np.concatenate([np.cumsum(np.asarray(b, dtype=np.int64)[::-1])[::-1][1:], [0]])  # sum_{j>k} b_j
    jstar = np.argmax(bits, axis=1)                    # first selected tensor (0 for the empty mask)
    cost = cost + np.where(m > 0, after[jstar], 0)
    value = np.where(cost <= budget, value, _NEG)
    best = int(np.argmax(value))                        # first maximum = smallest binary number
    return _result(list(bits[best]), OK, t_fwd, t_dw, t_dy, value_q=int(value[best]))


def select_recurrence(importance, t_dw, t_dy, t_fwd, rho_ppm, Tq, prune=True):
    """The dynamic programme of Section 6 on the quantised integers.

    Depth d = 1..N counts tensors from the output (tensor j has depth N - j).
    Q[d][t]: best summed importance with the tensor at depth d selected and no
    deeper tensor selected, backward time at most t.  Selecting depth d costs
    its own t_dw plus the t_dy of passing the gradient from the closest
    selected shallower tensor e down to d (Eq. 7), or, when d is the only
    selected tensor, from the output down to d.  P[d][t] = max(P[d-1][t],
    Q[d][t]) (cases 1 and 2).  With prune=True only cells that are neither
    invalid (t above the budget) nor redundant (t below the time of merely
    reaching depth d) are evaluated (Section 6.3); otherwise t runs over the
    whole backward time.
    """
    N = len(t_dw)
    iq = quantise_importance(importance)
    a, b, budget = quantise_times(t_fwd, t_dw, t_dy, rho_ppm, Tq)
    if budget < 0:
        return _result([0] * N, INFEASIBLE, t_fwd, t_dw, t_dy, value_q=0, cells=0)
    # by depth (index 0 unused)
    A = [0] + [a[N - d] for d in range(1, N + 1)]
    Bq = [0] + [b[N - d] for d in range(1, N + 1)]
    I = [0] + [iq[N - d] for d in range(1, N + 1)]
    reach = [0] * (N + 2)                               # reach[d] = sum_{e<d} b_e
    for d in range(2, N + 2):
        reach[d] = reach[d - 1] + Bq[d - 1]
    T = budget if prune else max(budget, sum(A) + reach[N])
    Q = np.full((N + 1, T + 1), _NEG, dtype=np.int64)
    pred = np.full((N + 1, T + 1), -1, dtype=np.int32)  # -1: infeasible, 0: alone, e: closest selected
    cells = 0
    for d in range(1, N + 1):
        lo = reach[d] + A[d]                            # cheapest mask with deepest tensor d
        if prune and lo > budget:
            continue
        if lo > T:
            continue
        cells += (T - (reach[d] if prune else 0) + 1)
        q, p = Q[d], pred[d]
        q[lo:] = I[d]
        p[lo:] = 0
        for e in range(1, d):
            shift = A[d] + (reach[d] - reach[e])        # t_dw(d) + sum_{j=e}^{d-1} t_dy(j)
            if shift > T:
                continue
            cand = Q[e][: T + 1 - shift]
            ok = cand > _NEG
            val = np.where(ok, cand + I[d], _NEG)
            better = val > q[shift:]
            q[shift:][better] = val[better]
            p[shift:][better] = e
    top = Q[1:, budget]
    best = int(top.max()) if N else _NEG
    mask = [0] * N
    if best > 0:                                        # otherwise the empty mask (value 0) wins
        d = int(np.argmax(top)) + 1                     # first maximum = shallowest deepest tensor
        t = budget
        while True:
            mask[N - d] = 1
            e = int(pred[d][t])
            assert e >= 0
            if e == 0:
                break
            t -= A[d] + (reach[d] - reach[e])
            d = e
    return _result(mask, OK, t_fwd, t_dw, t_dy, value_q=max(best, 0), cells=cells)


def select(importance, t_dw, t_dy, t_fwd, rho_ppm, Tq, method=None):
    if method is None:
        method = "enumerate" if len(t_dw) <= 16 else "recurrence"
    f = select_enumerate if method == "enumerate" else select_recurrence
    return f(importance, t_dw, t_dy, t_fwd, rho_ppm, Tq)
