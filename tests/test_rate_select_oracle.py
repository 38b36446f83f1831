"""Pins for the block-rate selection oracle (Sec. 3.3): hand-worked cases, an independent ILP solver,
invariants, and planted mistakes that must be caught."""
import itertools
import os

import numpy as np
import pytest

from oracle import rate_select_oracle as RO

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "rate_select_cases.txt")


def golden_cases():
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, cost, err, budget, choice, total = [f.strip() for f in line.split("|")]
        rows = lambda s: [[float(x) for x in blk.split()] for blk in s.split(";")]
        yield name, rows(cost), rows(err), float(budget), (None if choice == "infeasible" else tuple(int(x) for x in choice.split())), total


@pytest.mark.parametrize("case", list(golden_cases()), ids=lambda c: c[0])
def test_hand_worked_cases(case):
    _, cost, err, budget, choice, total = case
    got = RO.select_rates_bruteforce(cost, err, budget)
    if choice is None:
        assert got is None
    else:
        assert got is not None and got[0] == choice and got[2] == float(total)
        assert got[1] == sum(cost[i][r] for i, r in enumerate(choice))


def random_instance(rng, n_blocks, n_rates, integer=True):
    cost = np.sort(rng.integers(1, 20, size=(n_blocks, n_rates)), axis=1)[:, ::-1].astype(float)
    err = np.sort(rng.integers(0, 30, size=(n_blocks, n_rates)), axis=1).astype(float)
    if not integer:
        cost += rng.random(cost.shape)
        err += rng.random(err.shape)
    return cost.tolist(), err.tolist()


def milp_optimum(cost, err, budget):
    """The same integer program handed to SciPy's MILP solver (HiGHS): min e.z, c.z <= beta, one z per block."""
    from scipy.optimize import milp, LinearConstraint, Bounds
    c = np.asarray(cost)
    e = np.asarray(err)
    nb, nr = c.shape
    A = np.zeros((nb + 1, nb * nr))
    A[0] = c.ravel()
    for i in range(nb):
        A[1 + i, i * nr:(i + 1) * nr] = 1.0
    lo = np.concatenate([[-np.inf], np.ones(nb)])
    hi = np.concatenate([[budget], np.ones(nb)])
    res = milp(e.ravel(), constraints=LinearConstraint(A, lo, hi), integrality=np.ones(nb * nr), bounds=Bounds(0, 1))
    return None if res.status != 0 else float(res.fun)


@pytest.mark.parametrize("seed", range(12))
def test_matches_an_independent_ilp_solver(seed):
    rng = np.random.default_rng(seed)
    nb, nr = int(rng.integers(2, 7)), int(rng.integers(2, 5))
    cost, err = random_instance(rng, nb, nr)
    lo = sum(min(c) for c in cost)
    hi = sum(max(c) for c in cost)
    for budget in (lo - 1, lo, (lo + hi) // 2, hi, hi + 5):
        got = RO.select_rates_bruteforce(cost, err, float(budget))
        ref = milp_optimum(cost, err, float(budget))
        if ref is None:
            assert got is None
        else:
            assert got is not None and abs(got[2] - ref) < 1e-9
            assert got[1] <= budget and got[1] == sum(cost[i][r] for i, r in enumerate(got[0]))


def test_invariants():
    rng = np.random.default_rng(99)
    cost, err = random_instance(rng, 5, 4, integer=False)
    # a budget that admits everything: every block takes its smallest error
    big = RO.select_rates_bruteforce(cost, err, 1e9)
    assert big[0] == tuple(int(np.argmin(e)) for e in err)
    # the tightest feasible budget: every block takes its cheapest candidate
    tight = RO.select_rates_bruteforce(cost, err, sum(min(c) for c in cost))
    assert tight[0] == tuple(int(np.argmin(c)) for c in cost)
    assert RO.select_rates_bruteforce(cost, err, sum(min(c) for c in cost) - 1e-6) is None
    # the optimum never gets worse when the budget grows
    prev = np.inf
    for budget in np.linspace(sum(min(c) for c in cost), sum(max(c) for c in cost), 25):
        cur = RO.select_rates_bruteforce(cost, err, float(budget))[2]
        assert cur <= prev + 1e-12
        prev = cur
    # a single candidate per block ("homogeneous" selection) leaves no choice
    one = RO.select_rates_bruteforce([[3.0], [4.0]], [[1.0], [2.0]], 7.0)
    assert one == ((0, 0), 7.0, 3.0)


def _variant(kind):
    """The oracle with one planted mistake."""
    def f(cost, error, budget):
        nb, nr = len(cost), len(cost[0])
        best = None
        choices = itertools.product(range(nr), repeat=nb)
        for ch in choices:
            tc = sum(cost[i][r] for i, r in enumerate(ch))
            te = sum(error[i][r] for i, r in enumerate(ch))
            if kind == "strict_budget" and tc >= budget:
                continue
            if kind != "strict_budget" and tc > budget:
                continue
            if kind == "swapped_tables":
                tc, te = te, tc
            key = (-te if kind == "maximise" else te, tc, ch)
            if best is None or key < best:
                best = key
        return None if best is None else (best[2], best[1], abs(best[0]))
    return f


@pytest.mark.parametrize("kind", ["strict_budget", "maximise", "swapped_tables"])
def test_planted_mistakes_fail_the_hand_worked_cases(kind):
    bad = _variant(kind)
    failures = 0
    for _, cost, err, budget, choice, total in golden_cases():
        got = bad(cost, err, budget)
        ok = (got is None) if choice is None else (got is not None and got[0] == choice and got[2] == float(total))
        failures += not ok
    assert failures > 0
