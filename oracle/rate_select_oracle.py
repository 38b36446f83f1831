"""Oracle for the block-rate selection of Sec. 3.3 ("Heterogeneous Block-Rate Optimization").

TEST INFRASTRUCTURE ONLY: imported by tests/ (and by bench.py's reporting of a reference answer on
tiny instances); the library never calls it.

The paper states the selection as a multiple-choice knapsack: block i takes exactly one candidate
rate r, with pre-computed cost c_ir and error e_ir; minimise the summed error subject to the summed
cost staying within the budget beta.  The oracle is that definition written out: it enumerates every
assignment (n_rates ** n_blocks of them, so tiny instances only) and keeps the best feasible one.
Where several assignments reach the minimum error the paper does not say which to take; the oracle
reports the minimum error (unique) and, as a convention, the cheapest such assignment, then the
lexicographically smallest.
"""
from __future__ import annotations

import itertools
from typing import Optional, Sequence, Tuple


def select_rates_bruteforce(cost: Sequence[Sequence[float]], error: Sequence[Sequence[float]],
                            budget: float) -> Optional[Tuple[Tuple[int, ...], float, float]]:
    """Returns (choice per block, total cost, total error) of the best assignment, or None when even
    the cheapest assignment exceeds the budget.  cost[i][r], error[i][r]: block i, candidate r."""
    n_blocks = len(cost)
    assert n_blocks == len(error) and n_blocks >= 1
    n_rates = len(cost[0])
    assert all(len(c) == n_rates for c in cost) and all(len(e) == n_rates for e in error)
    best = None
    for choice in itertools.product(range(n_rates), repeat=n_blocks):
        total_cost = 0.0
        total_error = 0.0
        for i, r in enumerate(choice):
            total_cost += cost[i][r]
            total_error += error[i][r]
        if total_cost > budget:
            continue
        key = (total_error, total_cost, choice)
        if best is None or key < best:
            best = key
    if best is None:
        return None
    return best[2], best[1], best[0]
