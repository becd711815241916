"""Pins of the taxonomy / budget oracle (Sec. 4.1-4.2; App. C.2)."""
import random
from fractions import Fraction

import pytest

from oracle import taxonomy as T


def adj_from_edges(n, edges):
    a = [[0] * n for _ in range(n)]
    for i, j in edges:
        a[i][j] = a[j][i] = 1
    return a


def test_star_and_leftovers_worked_by_hand():
    # head 0 is adjacent to 1, 2, 3; heads 4-5 are adjacent to each other; 6, 7 are isolated
    adj = adj_from_edges(8, [(0, 1), (0, 2), (0, 3), (4, 5)])
    s = [0.9, 0.9, 0.9, 0.9, 0.9, 0.9, 0.7, 0.3]
    role, rep, pivot = T.taxonomy(adj, s, 0.5)
    assert pivot == [True, False, False, False, True, False, False, False]          # 4 beats 5 by index
    assert rep == [-1, 0, 0, 0, -1, 4, -1, -1]
    assert role == [T.ROLE_FULL, T.ROLE_SATELLITE, T.ROLE_SATELLITE, T.ROLE_SATELLITE, T.ROLE_FULL, T.ROLE_SATELLITE,
                    T.ROLE_ANCHOR, T.ROLE_FULL]                                      # 6 stable -> anchor, 7 -> volatile


def test_effective_degree_counts_unassigned_neighbours_only():
    # path 0-1-2-3-4: degrees 1,2,2,2,1 -> head 1 first (lowest index among degree 2), absorbs 0 and 2;
    # then 3 and 4 have effective degree 1 each -> head 3 is the pivot of {4}
    adj = adj_from_edges(5, [(0, 1), (1, 2), (2, 3), (3, 4)])
    role, rep, pivot = T.taxonomy(adj, [1.0] * 5, 0.5)
    assert [i for i in range(5) if pivot[i]] == [1, 3]
    assert rep == [1, -1, 1, -1, 3]


@pytest.mark.parametrize("seed", range(20))
def test_invariants_on_random_graphs(seed):
    rng = random.Random(seed)
    n = rng.randint(1, 40)
    adj = adj_from_edges(n, [(i, j) for i in range(n) for j in range(i) if rng.random() < 0.15])
    s = [rng.uniform(0.05, 1.0) for _ in range(n)]
    role, rep, pivot = T.taxonomy(adj, s, 0.5)
    piv = [i for i in range(n) if pivot[i]]
    for i in range(n):
        if role[i] == T.ROLE_SATELLITE:
            assert pivot[rep[i]] and adj[i][rep[i]]                 # a star: every satellite is adjacent to its pivot
        else:
            assert rep[i] == -1
        if pivot[i]:
            assert any(rep[j] == i for j in range(n))                # a pivot has at least one satellite
    assert all(not adj[a][b] for a in piv for b in piv if a != b)   # pivots are pairwise non-adjacent
    for i in range(n):                                              # what is left over has no unassigned neighbour
        if role[i] != T.ROLE_SATELLITE and not pivot[i]:
            assert all(not adj[i][j] or role[j] == T.ROLE_SATELLITE or pivot[j] for j in range(n))
            assert role[i] == (T.ROLE_ANCHOR if s[i] >= 0.5 else T.ROLE_FULL)


def test_budget_closed_forms():
    # equal stability: every compressed head gets L_base = (rho N - N_full) L / N_comp (Eq. 7)
    role = [T.ROLE_FULL, T.ROLE_FULL] + [T.ROLE_SATELLITE] * 5 + [T.ROLE_ANCHOR]
    L, rho = 12000, Fraction(1, 2)
    out = T.budgets(role, [0.5] * 8, 1, 2, L)
    assert out[:2] == [L, L]
    assert out[2:] == [(rho * 8 - 2) * L // 6] * 6 == [4000] * 6
    # inverse-stability weights: budgets in the ratio 1/S, summing to the total of Eq. 7
    s = [1.0, 1.0, 0.25, 0.5, 0.5, 1.0, 1.0, 1.0]
    out = T.budgets(role, s, 1, 2, L)
    total = (rho * 8 - 2) * L
    assert sum(out[2:]) == total
    w = [1 / Fraction(x) for x in s[2:]]
    for o, wi in zip(out[2:], w):
        assert abs(o - total * wi / sum(w)) < 1
    # weights 4 : 2 : 2 : 1 : 1 : 1 of a total of 2 L = 22000: exact
    assert T.budgets(role, s, 1, 2, 11000)[2:] == [8000, 4000, 4000, 2000, 2000, 2000]


@pytest.mark.parametrize("seed", range(20))
def test_budgets_stay_within_one_slot_of_the_exact_shares(seed):
    """Every integer budget lies within one slot of the real-valued share of Eq. 8 (written out again here), and the
    budgets add up to the total of Eq. 7."""
    rng = random.Random(500 + seed)
    n = rng.randint(2, 48)
    role = [rng.choice([T.ROLE_FULL, T.ROLE_SATELLITE, T.ROLE_SATELLITE, T.ROLE_ANCHOR]) for _ in range(n)]
    if all(r == T.ROLE_FULL for r in role):
        role[0] = T.ROLE_ANCHOR
    s = [rng.uniform(0.3, 1.0) for _ in range(n)]
    n_full = sum(r == T.ROLE_FULL for r in role)
    num = rng.randint(1, 9)
    L = rng.choice([4096, 229376])
    total = Fraction(num * n - n_full * 10, 10) * L
    if total <= 0:
        return
    out = T.budgets(role, s, num, 10, L)
    comp = [i for i in range(n) if role[i] != T.ROLE_FULL]
    tot = min(int(total), len(comp) * L)
    assert sum(out[i] for i in comp) == tot and all(out[i] == L for i in range(n) if role[i] == T.ROLE_FULL)
    if max(out[i] for i in comp) < L:           # nobody was cut to L: plain proportional shares
        w = {i: 1 / Fraction(s[i]) for i in comp}
        sw = sum(w.values())
        for i in comp:
            assert abs(out[i] - tot * w[i] / sw) <= 1


def test_budget_rounding_and_clamping():
    role = [T.ROLE_FULL] + [T.ROLE_ANCHOR] * 3
    out = T.budgets(role, [1.0, 1.0, 1.0, 1.0], 1, 2, 100)         # total (2 - 1) * 100 = 100 over 3 heads
    assert out == [100, 34, 33, 33]                                           # the spare slot goes to the lowest index
    out = T.budgets(role, [1.0, 0.01, 1.0, 1.0], 3, 4, 100)        # total 200; head 1 would get 196 > L
    assert out == [100, 100, 50, 50]
    with pytest.raises(ValueError):
        T.budgets(role, [1.0] * 4, 1, 4, 100)                       # rho N = N_full: nothing left
