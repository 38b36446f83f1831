"""The library's block-rate selection (Sec. 3.3) against the enumeration oracle: host code only, so
these run without a GPU, through the C ABI."""
import ctypes
import os

import numpy as np
import pytest

from oracle import rate_select_oracle as RO
from paper_2509_24899_amd import hybrid_attn as ha
from tests.test_rate_select_oracle import golden_cases, random_instance


@pytest.fixture(scope="module", autouse=True)
def lib():
    if not os.path.exists(ha.LIB_PATH):
        from paper_2509_24899_amd.build import build_library
        build_library()
    return ha._lib()


@pytest.mark.parametrize("case", list(golden_cases()), ids=lambda c: c[0])
def test_hand_worked_cases(case):
    _, cost, err, budget, choice, total = case
    got = ha.hybrid_attn_select_rates(cost, err, budget)
    if choice is None:
        assert got is None
    else:
        assert got[0] == choice and got[2] == float(total)


@pytest.mark.parametrize("seed", range(40))
@pytest.mark.parametrize("integer", (True, False))
def test_equals_enumeration(seed, integer):
    """Integer tables are full of ties (the tie-break convention is exercised); real-valued tables have
    unique optima.  Choice vector, total cost and total error must be identical, bit for bit."""
    rng = np.random.default_rng(1000 + seed)
    nb, nr = int(rng.integers(1, 8)), int(rng.integers(1, 5))
    cost, err = random_instance(rng, nb, nr, integer=integer)
    lo, hi = sum(min(c) for c in cost), sum(max(c) for c in cost)
    for budget in (lo - 0.5, lo, lo + 0.37 * (hi - lo), lo + 0.71 * (hi - lo), hi, hi + 3):
        ref = RO.select_rates_bruteforce(cost, err, float(budget))
        got = ha.hybrid_attn_select_rates(cost, err, float(budget))
        if ref is None:
            assert got is None
        else:
            assert got is not None
            assert got[2] == ref[2] and got[1] == ref[1] and tuple(got[0]) == tuple(ref[0])


def test_model_sized_instance_is_valid_and_beats_simple_rules():
    """30 blocks x 4 rates (the paper's setting: rates 1, 2, 4, 8): too large to enumerate, so check what
    holds at any size: the assignment is feasible, its sums are the sums of its entries, and no single-block
    change that stays within budget lowers the error; it is at least as good as every homogeneous choice."""
    rng = np.random.default_rng(7)
    nb, nr = 30, 4
    cost = np.tile(np.array([5.41, 3.02, 1.72, 1.08]), (nb, 1)) * (1 + 0.02 * rng.random((nb, nr)))
    err = np.abs(rng.lognormal(0, 1, size=(nb, 1))) * np.array([0.0, 0.2, 0.55, 1.0])
    budget = 0.45 * cost[:, 0].sum()
    choice, tc, te = ha.hybrid_attn_select_rates(cost.tolist(), err.tolist(), budget)
    assert tc <= budget
    assert tc == sum(cost[i][r] for i, r in enumerate(choice)) or abs(tc - sum(cost[i, r] for i, r in enumerate(choice))) < 1e-9
    assert abs(te - sum(err[i, r] for i, r in enumerate(choice))) < 1e-9
    for i in range(nb):
        for r in range(nr):
            c2 = tc - cost[i, choice[i]] + cost[i, r]
            e2 = te - err[i, choice[i]] + err[i, r]
            assert not (c2 <= budget and e2 < te - 1e-12)
    for r in range(nr):
        if cost[:, r].sum() <= budget:
            assert te <= err[:, r].sum() + 1e-12


def test_argument_errors(lib):
    f = lib.hybrid_attn_select_rates
    one = (ctypes.c_double * 2)(1.0, 2.0)
    bad = (ctypes.c_double * 2)(1.0, -2.0)
    nan = (ctypes.c_double * 2)(1.0, float("nan"))
    ch = (ctypes.c_int * 1)()
    tc, te = ctypes.c_double(), ctypes.c_double()
    assert f(1, 2, None, one, 5.0, ch, ctypes.byref(tc), ctypes.byref(te)) == ha.HA_ERR_NULL
    assert f(1, 2, one, one, 5.0, None, ctypes.byref(tc), ctypes.byref(te)) == ha.HA_ERR_NULL
    assert f(0, 2, one, one, 5.0, ch, ctypes.byref(tc), ctypes.byref(te)) == ha.HA_ERR_SHAPE
    assert f(1, 0, one, one, 5.0, ch, ctypes.byref(tc), ctypes.byref(te)) == ha.HA_ERR_SHAPE
    assert f(1, 2, bad, one, 5.0, ch, ctypes.byref(tc), ctypes.byref(te)) == ha.HA_ERR_SHAPE
    assert f(1, 2, one, nan, 5.0, ch, ctypes.byref(tc), ctypes.byref(te)) == ha.HA_ERR_SHAPE
    assert f(1, 2, one, one, float("inf"), ch, ctypes.byref(tc), ctypes.byref(te)) == ha.HA_ERR_SHAPE
    assert f(1, 2, one, one, 0.5, ch, ctypes.byref(tc), ctypes.byref(te)) == ha.HA_ERR_INFEASIBLE
    assert f(1, 2, one, one, 1.0, ch, ctypes.byref(tc), ctypes.byref(te)) == ha.HA_OK and ch[0] == 0
