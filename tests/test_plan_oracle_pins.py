"""Pins of oracle/plan_oracle.py (Eq. 2) against hand-worked cases, a MILP library and properties."""
import os

import numpy as np
import pytest

from oracle import plan_oracle as P

HERE = os.path.dirname(os.path.abspath(__file__))
L_FULL, LAT = 10.0, [4.0, 0.0]


def hand_cases():
    for line in open(os.path.join(HERE, "golden", "plan_hand_cases.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        head, rows, want = (p.strip() for p in line.split("|"))
        delta, c = (float(x) for x in head.split())
        infl = [[float(x) for x in r.split()] for r in rows.split(";")]
        yield delta, c, infl, float(want)


def test_hand_worked_cases():
    cases = list(hand_cases())
    assert len(cases) >= 7
    for delta, c, infl, want in cases:
        best, assigns = P.solve(infl, LAT, L_FULL, delta, c)
        assert best == want, (delta, c, infl, best, want)
        for a in assigns:       # every reported optimum is feasible and has that latency
            tot_i = sum(infl[h][m] for h, m in enumerate(a) if m >= 0)
            tot_l = sum(L_FULL if m < 0 else LAT[m] for m in a)
            assert tot_i <= delta and tot_l == want
            assert all(m < 0 or infl[h][m] <= c / len(infl) * delta for h, m in enumerate(a))


def milp_optimum(infl, lat, l_full, delta, c):
    """The same problem handed to scipy's MILP solver (HiGHS)."""
    from scipy.optimize import Bounds, LinearConstraint, milp
    infl = np.asarray(infl, dtype=np.float64)
    H, M = infl.shape
    cost = np.tile(np.asarray(lat, dtype=np.float64) - l_full, H)          # x[h*M + m]
    rows = [infl.reshape(-1)]
    ub = [delta]
    for h in range(H):                                                   # at most one method per head
        r = np.zeros(H * M)
        r[h * M:(h + 1) * M] = 1.0
        rows.append(r)
        ub.append(1.0)
    upper = (infl.reshape(-1) <= c / H * delta).astype(np.float64)        # the per-head cap switches variables off
    res = milp(cost, constraints=LinearConstraint(np.array(rows), -np.inf, np.array(ub)),
               integrality=np.ones(H * M), bounds=Bounds(np.zeros(H * M), upper))
    assert res.success
    return H * l_full + res.fun


@pytest.mark.parametrize("seed", range(12))
def test_brute_force_agrees_with_a_milp_library(seed):
    g = np.random.Generator(np.random.PCG64(seed))
    H, M = int(g.integers(2, 6)), int(g.integers(1, 4))
    infl = g.uniform(0.01, 1.0, size=(H, M)) * np.linspace(0.3, 1.5, M)[None, :]
    lat = list(np.sort(g.uniform(0.0, 8.0, size=M))[::-1])                # more influence, less latency
    delta, c = float(g.uniform(0.2, 2.5)), float(g.uniform(0.8, 3.0))
    best, _ = P.solve(infl.tolist(), lat, 10.0, delta, c)
    assert abs(best - milp_optimum(infl, lat, 10.0, delta, c)) <= 1e-9


def test_limits_and_monotonicity():
    g = np.random.Generator(np.random.PCG64(99))
    infl = g.uniform(0.05, 1.0, size=(4, 3)).tolist()
    lat = [6.0, 3.0, 0.0]
    # no budget: every head keeps full attention
    best, assigns = P.solve(infl, lat, 10.0, 0.0, 4.0)
    assert best == 40.0 and assigns == [(-1, -1, -1, -1)]
    # unlimited budget and cap: every head takes the fastest method
    best, assigns = P.solve(infl, lat, 10.0, 1e9, 4.0)
    assert best == 0.0 and assigns == [(2, 2, 2, 2)]
    # more budget never costs latency
    prev = None
    for delta in (0.1, 0.3, 0.6, 1.0, 1.5, 2.5, 4.0):
        best, _ = P.solve(infl, lat, 10.0, delta, 4.0)
        assert prev is None or best <= prev
        prev = best
    # a tighter cap never helps
    assert P.solve(infl, lat, 10.0, 1.5, 1.0)[0] >= P.solve(infl, lat, 10.0, 1.5, 4.0)[0]
