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


@pytest.mark.parametrize("seed", range(30))
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
    assert st == 0 and got == expect
