"""The library's host-side taxonomy and budget functions against the oracle (no GPU needed)."""
import ctypes as C
import random
from fractions import Fraction

import pytest

from oracle import taxonomy as T
from paper_2601_13684_amd import binding as hc


def adj_from_edges(n, edges):
    a = [[0] * n for _ in range(n)]
    for i, j in edges:
        a[i][j] = a[j][i] = 1
    return a


def lib_taxonomy(adj, s, tau):
    n = len(adj)
    a = (C.c_uint8 * (n * n))(*[1 if adj[i][j] else 0 for i in range(n) for j in range(n)])
    sv = (C.c_double * n)(*s)
    role, rep, piv = (C.c_int32 * n)(), (C.c_int32 * n)(), (C.c_int32 * n)()
    assert hc.lib().hc_taxonomy(n, a, sv, C.c_double(tau), role, rep, piv) == 0
    return list(role), list(rep), [bool(x) for x in piv]


def lib_budgets(role, s, rho_num, rho_den, L):
    n = len(role)
    out = (C.c_int32 * n)()
    st = hc.lib().hc_budgets(n, (C.c_int32 * n)(*role), (C.c_double * n)(*s), rho_num, rho_den, L, out)
    return st, list(out)


def check_budgets_against_exact(role, s, rho_num, rho_den, L, got, expect):
    """The library decides in double precision, the oracle in exact rationals (Eq. 8 is real-valued).  They must
    agree, except that double rounding may move ONE slot between two heads at an exact near-tie: then the sums
    are equal, no head differs by more than one slot, and every head that differs has an exact share whose
    fractional part is within 1e-9 of 0 or 1 (the floor went the other way), of another head's fractional part
    (the left-over slot went to the other head), or whose share is within 1e-9 L of L (the cut went the other
    way).  Returns the number of heads that differ."""
    if got == expect:
        return 0
    comp = [i for i in range(len(role)) if role[i] != T.ROLE_FULL]
    assert sum(got[i] for i in comp) == sum(expect[i] for i in comp), (got, expect)
    shares = T.exact_shares(role, s, rho_num, rho_den, L)
    fracs = {i: sh - sh.__floor__() for i, sh in shares.items()}
    eps = Fraction(1, 10 ** 9)
    differ = [i for i in comp if got[i] != expect[i]]
    for i in differ:
        assert abs(got[i] - expect[i]) == 1, (i, got[i], expect[i])
        assert i in shares, (i, "a head that was cut to L differs")
        f = fracs[i]
        near = f < eps or f > 1 - eps or abs(shares[i] - L) < eps * L or \
            any(j != i and abs(fracs[j] - f) < eps for j in fracs)
        assert near, (i, "differs from the exact share without a near-tie", float(shares[i]), got[i], expect[i])
    return len(differ)


def check_budget_invariants(role, s, rho_num, rho_den, L, got):
    """What Eq. 7-8 fix whatever the rounding: full heads keep L; the compressed heads' budgets add up to the
    total of Eq. 7 rounded down (capped by N_comp L); none exceeds L; a less stable head never gets fewer slots
    than a more stable one (up to the one left-over slot)."""
    n = len(role)
    comp = [i for i in range(n) if role[i] != T.ROLE_FULL]
    n_full = n - len(comp)
    total = ((Fraction(rho_num, rho_den) * n - n_full) * L).__floor__()
    assert all(got[i] == L for i in range(n) if role[i] == T.ROLE_FULL)
    assert sum(got[i] for i in comp) == min(total, len(comp) * L)
    assert all(0 <= got[i] <= L for i in comp)
    for a in comp:
        for b in comp:
            if s[a] < s[b]:
                assert got[a] >= got[b] - 1, (a, b, s[a], s[b], got[a], got[b])


@pytest.mark.parametrize("seed", range(60))
def test_library_taxonomy_and_budgets_equal_the_oracle(seed):
    rng = random.Random(1000 + seed)
    n = rng.randint(1, 64)
    adj = adj_from_edges(n, [(i, j) for i in range(n) for j in range(i) if rng.random() < rng.choice([0.02, 0.1, 0.4])])
    s = [rng.choice([0.125, 0.25, 0.5, 0.75, 1.0, rng.uniform(0.05, 1.0)]) for _ in range(n)]
    tau = rng.choice([0.4, 0.5])
    want = T.taxonomy(adj, s, tau)
    assert lib_taxonomy(adj, s, tau) == tuple(want) or lib_taxonomy(adj, s, tau) == want
    role = want[0]
    rho_num, rho_den, L = rng.randint(1, 9), 10, rng.choice([1000, 32768, 229376])
    try:
        expect = T.budgets(role, s, rho_num, rho_den, L)
    except ValueError:
        assert lib_budgets(role, s, rho_num, rho_den, L)[0] == hc.HC_EINVAL
        return
    st, got = lib_budgets(role, s, rho_num, rho_den, L)
    assert st == 0
    check_budget_invariants(role, s, rho_num, rho_den, L, got)
    assert check_budgets_against_exact(role, s, rho_num, rho_den, L, got, expect) <= 2


def test_library_budgets_at_an_exact_tie_of_the_left_over_slot():
    """Three equally stable heads share 100 slots: 33 1/3 each, the left-over slot goes to the lowest index on
    both sides (an exact tie of the fractional parts, which double precision reproduces)."""
    role = [T.ROLE_FULL] + [T.ROLE_ANCHOR] * 3
    st, got = lib_budgets(role, [1.0, 1.0, 1.0, 1.0], 1, 2, 100)
    assert st == 0 and got == [100, 34, 33, 33] == T.budgets(role, [1.0] * 4, 1, 2, 100)
    st, got = lib_budgets(role, [1.0, 0.01, 1.0, 1.0], 3, 4, 100)          # head 1 would get 196 > L: cut to L
    assert st == 0 and got == [100, 100, 50, 50] == T.budgets(role, [1.0, 0.01, 1.0, 1.0], 3, 4, 100)
