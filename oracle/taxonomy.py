"""Oracle of the offline head taxonomy and budget allocation (Sec. 4.1-4.2, Eq. 4-8; App. C.2; Algorithm 1
stages 1-2), in plain Python.  Test infrastructure only: the product's implementation is the C library's
hc_taxonomy / hc_budgets; only tests import this module.

Readings where the paper leaves a choice (the same ones the library documents):
  * Sec. 4.1 first splits heads by the similarity score and clusters the similar ones; App. C.2 clusters on the
    adjacency graph of all heads and classifies what is left over by stability.  They agree when "similar"
    means "has a neighbour in the graph"; App. C.2's procedure is the one written out here.
  * effective degree ties: the lowest head index wins; a head whose effective degree is 0 is never a pivot.
  * budgets are real numbers in Eq. 8; they are rounded down and the remaining slots go to the largest
    fractional parts (lowest index first), so that the sum is exactly the total of Eq. 7 rounded down;
    a budget above the sequence length is cut to it and the excess shared among the others in the same
    proportion.  Eq. 8 is real-valued: the shares here are exact rationals of the given floats.  (The library
    evaluates them in double precision; a test allows it the one-slot differences that double rounding can
    cause at exact near-ties, and nothing else.)
"""
from fractions import Fraction
from typing import List, Sequence, Tuple

ROLE_FULL, ROLE_SATELLITE, ROLE_ANCHOR = 0, 1, 2


def taxonomy(adj: Sequence[Sequence[int]], s_stable: Sequence[float], tau_stable: float) -> Tuple[List[int], List[int], List[bool]]:
    """Greedy star clustering by effective degree (App. C.2), then anchors / volatile heads by stability
    (Eq. 5).  Returns (role, rep, is_pivot) per head; pivots and volatile heads both keep their full cache
    (ROLE_FULL)."""
    n = len(adj)
    unassigned = set(range(n))
    role = [None] * n
    rep = [-1] * n
    pivot = [False] * n
    while True:
        best, best_deg = -1, 0
        for h in sorted(unassigned):
            deg = sum(1 for j in unassigned if j != h and adj[h][j])
            if deg > best_deg:
                best, best_deg = h, deg
        if best < 0:
            break
        members = [j for j in sorted(unassigned) if j != best and adj[best][j]]
        role[best], pivot[best] = ROLE_FULL, True
        unassigned.discard(best)
        for j in members:
            role[j], rep[j] = ROLE_SATELLITE, best
            unassigned.discard(j)
    for h in unassigned:
        role[h] = ROLE_ANCHOR if s_stable[h] >= tau_stable else ROLE_FULL
    return role, rep, pivot


def budgets(role: Sequence[int], s_stable: Sequence[float], rho_num: int, rho_den: int, L: int) -> List[int]:
    """Eq. 7-8: the total (rho N - N_full) L, rho = rho_num / rho_den, shared among the compressed heads in
    proportion to w_i = 1 / S_stable_i; full heads get L.  Exact rational arithmetic on the given floats
    (every float is a rational number; nothing is rounded before the final floor)."""
    n = len(role)
    comp = [i for i in range(n) if role[i] != ROLE_FULL]
    n_full = n - len(comp)
    total = (Fraction(rho_num, rho_den) * n - n_full) * L
    if total <= 0 or not comp:
        raise ValueError("no budget for compressed heads")
    total = min(total.__floor__(), len(comp) * L)
    if total <= 0:
        raise ValueError("no budget for compressed heads")
    w = {i: 1 / Fraction(s_stable[i]) for i in comp}
    out = {i: L for i in range(n)}
    free, left = list(comp), total
    while True:       # heads whose share exceeds L are cut to L; the rest share what is left
        sw = sum(w[i] for i in free)
        over = [i for i in free if left * w[i] / sw > L]
        if not over:
            break
        for i in over:
            out[i] = L
            free.remove(i)
            left -= L
        if not free:
            return [out[i] for i in range(n)]
    share = {i: left * w[i] / sw for i in free}
    for i in free:
        out[i] = share[i].__floor__()
    rest = left - sum(out[i] for i in free)            # 0 <= rest < len(free): the floors lose less than one slot each
    order = sorted(free, key=lambda i: (-(share[i] - out[i]), i))
    for i in order[:rest]:
        out[i] += 1
    return [out[i] for i in range(n)]


def exact_shares(role: Sequence[int], s_stable: Sequence[float], rho_num: int, rho_den: int, L: int):
    """The real-valued shares of Eq. 8 before rounding, as exact fractions, for the heads that are not cut to L
    ({head: share}); tests use them to tell a genuine difference from a double-rounding near-tie."""
    n = len(role)
    comp = [i for i in range(n) if role[i] != ROLE_FULL]
    n_full = n - len(comp)
    total = min(((Fraction(rho_num, rho_den) * n - n_full) * L).__floor__(), len(comp) * L)
    w = {i: 1 / Fraction(s_stable[i]) for i in comp}
    free, left = list(comp), total
    while free:
        sw = sum(w[i] for i in free)
        over = [i for i in free if left * w[i] / sw > L]
        if not over:
            return {i: left * w[i] / sw for i in free}
        for i in over:
            free.remove(i)
            left -= L
    return {}
