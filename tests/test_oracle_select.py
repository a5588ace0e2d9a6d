"""Pins for the victim-selection oracle (lowest importance first, section 3.4;
k lowest under a budget): numpy lexsort as brute force, ties, edge cases."""
import numpy as np
import pytest

RES, HOST, PROT, SCORED = 1, 2, 4, 8


def brute(prio, state, k):
    el = np.nonzero(((state & RES) != 0) & ((state & PROT) == 0) & ((state & SCORED) != 0))[0]
    p = prio[el].astype(np.float64)
    p[np.isnan(p)] = np.inf
    order = np.lexsort((el, p))            # primary key p, ties by uid
    return np.sort(el[order[:k]])


def random_case(rng, n, levels=None):
    prio = rng.random(n).astype(np.float32)
    if levels:                              # few distinct values -> many ties
        prio = (np.floor(prio * levels) / levels).astype(np.float32)
    state = rng.choice(np.array([0, RES, RES | SCORED, RES | SCORED | PROT, HOST | SCORED, RES | SCORED],
                                np.uint8), size=n)
    return prio, state


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("levels", [None, 5])
def test_matches_brute_force(oracle, seed, levels):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 400))
    prio, state = random_case(rng, n, levels)
    n_el = int(np.sum(((state & RES) != 0) & ((state & PROT) == 0) & ((state & SCORED) != 0)))
    for k in {0, 1, n_el // 2, max(n_el - 1, 0), n_el}:
        got = oracle.select_victims(prio, state, k=k)
        np.testing.assert_array_equal(got, brute(prio, state, k))


def test_exhaustive_tiny(oracle):
    """Every subset of size k of 6 units: the chosen one minimises the sorted (prio, uid) list."""
    from itertools import combinations
    prio = np.array([0.3, 0.1, 0.3, 0.1, 0.2, 0.3], np.float32)
    state = np.full(6, RES | SCORED, np.uint8)
    for k in range(7):
        got = tuple(oracle.select_victims(prio, state, k=k))
        best = min(combinations(range(6), k), key=lambda c: sorted((float(prio[u]), u) for u in c))
        assert got == tuple(sorted(best))


def test_all_equal_takes_lowest_uids(oracle):
    prio = np.full(50, 0.25, np.float32)
    state = np.full(50, RES | SCORED, np.uint8)
    state[3] |= PROT
    got = oracle.select_victims(prio, state, k=10)
    np.testing.assert_array_equal(got, [0, 1, 2, 4, 5, 6, 7, 8, 9, 10])


def test_budget_rule_and_clipping(oracle):
    rng = np.random.default_rng(1)
    prio, state = random_case(rng, 300)
    n_res = int(np.sum((state & RES) != 0))
    n_el = int(np.sum(((state & RES) != 0) & ((state & PROT) == 0) & ((state & SCORED) != 0)))
    for budget in (n_res + 5, n_res, n_res - 1, n_res - n_el, 0):
        k = min(max(0, n_res - budget), n_el)
        got = oracle.select_victims(prio, state, k=-1, budget_units=budget)
        np.testing.assert_array_equal(got, brute(prio, state, k))
    assert len(oracle.select_victims(prio, state, k=10**6)) == n_el          # clipped to eligible
    got = oracle.select_victims(prio, state, k=40, victims_cap=7)             # clipped to capacity
    np.testing.assert_array_equal(got, brute(prio, state, 7))


def test_nan_and_inf_rank_last_and_zero_signs_tie(oracle):
    prio = np.array([np.nan, 0.5, np.inf, -0.0, 0.0, 0.1], np.float32)
    state = np.full(6, RES | SCORED, np.uint8)
    np.testing.assert_array_equal(oracle.select_victims(prio, state, k=1), [3])   # -0 == +0, lower uid wins
    np.testing.assert_array_equal(oracle.select_victims(prio, state, k=4), [1, 3, 4, 5])
    np.testing.assert_array_equal(oracle.select_victims(prio, state, k=5), [0, 1, 3, 4, 5])  # NaN == inf, uid 0 < 2


def test_empty_input(oracle):
    assert len(oracle.select_victims(np.zeros(0, np.float32), np.zeros(0, np.uint8), k=3)) == 0
