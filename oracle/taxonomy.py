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
    proportion.  The shares are evaluated in IEEE double precision in a fixed order (see budgets), the
    precision in which both sides take the integer decision.
"""
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
    proportion to w_i = 1 / S_stable_i; full heads get L.  The total is exact integer arithmetic; the shares
    are evaluated in IEEE double precision, w = 1.0 / S, sums in head order, share = (total * w) / sum(w),
    which is the precision in which the integer budgets are decided on both sides."""
    n = len(role)
    comp = [i for i in range(n) if role[i] != ROLE_FULL]
    n_full = n - len(comp)
    total = ((rho_num * n - n_full * rho_den) * L) // rho_den if rho_num * n > n_full * rho_den else 0
    if total <= 0 or not comp:
        raise ValueError("no budget for compressed heads")
    total = min(total, len(comp) * L)
    w = {i: 1.0 / float(s_stable[i]) for i in comp}
    out = {i: L for i in range(n)}
    free, left = list(comp), total
    while True:       # heads whose share exceeds L are cut to L; the rest share what is left
        sw = 0.0
        for i in free:
            sw += w[i]
        over = [i for i in free if (float(left) * w[i]) / sw > float(L)]
        if not over:
            break
        for i in over:
            out[i] = L
            free.remove(i)
            left -= L
        if not free:
            return [out[i] for i in range(n)]
    share = {i: (float(left) * w[i]) / sw for i in free}
    for i in free:
        out[i] = int(share[i] // 1.0)
    rest = left - sum(out[i] for i in free)
    order = sorted(free, key=lambda i: (-(share[i] - float(out[i])), i))
    for k in range(max(0, rest)):           # rounding noise can leave a slot more than there are heads: go round again
        out[order[k % len(order)]] += 1
    return [out[i] for i in range(n)]
