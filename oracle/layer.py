"""The oracle's own description of one layer of the heterogeneous cache: TEST INFRASTRUCTURE ONLY.

Which KV heads keep their whole context (pivots and volatile heads), which are compressed (satellites of a
pivot, or anchors), their budgets, and what follows from that under the readings the oracle takes:

  * a compressed head's budget is l = sink + recent + r: the first `sink` and the last `recent` positions are
    always resident, the other r slots hold retrieved positions (the synthetic configs split the budget this
    way; sink = recent = 0 is the paper's pure top-l_i of Sec. 4.3);
  * the candidates of a pivot's TopIndices_k (Algorithm 1) are the positions that are neither sink nor recent
    slots of its satellites, [sink, ctx - recent): a position that is always resident is never retrieved twice;
  * the monitored set size (L_base of Eq. 9) is a parameter of the pivot; left at 0 it is the largest r among
    the pivot's satellites, so that the monitored set contains every retrieval list.

Nothing here is shared with the HIP library, which derives the same quantities from its own head table.  The
description is built from any object that carries the plain fields (``RefSpec.of``), e.g. what the seeded input
generators hand out; none of that object's methods is used.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Tuple

ROLE_FULL, ROLE_SATELLITE, ROLE_ANCHOR = 0, 1, 2


@dataclass(frozen=True)
class RefHead:
    role: int
    rep: int          # satellite: KV-head index of its pivot (same sequence); else -1
    sink: int
    recent: int
    budget: int       # compressed: resident rows l = sink + recent + r
    k_mon: int        # pivot: size of the monitored set, 0 = largest r of its satellites


@dataclass
class RefSpec:
    B: int
    Hq: int
    Hkv: int
    D: int
    ctx: List[int]
    heads: List[List[RefHead]]
    window: int
    metric: int       # 0: overlap |K_t ∩ K_base| / L_base (Eq. 9); 1: Jaccard
    tau_num: int
    tau_den: int
    agg: int          # 0: mean of the group's softmax weights (App. C.1); 1: mean of scaled logits (test mode)
    window_mode: int  # 0 sliding (Eq. 10), 1 tumbling, 2 tumbling with re-scoring (Algorithm 1)

    @classmethod
    def of(cls, spec) -> "RefSpec":
        if isinstance(spec, cls):
            return spec
        heads = [[RefHead(int(h.role), int(h.rep), int(h.sink), int(h.recent), int(h.budget), int(h.k_mon))
                  for h in row] for row in spec.heads]
        return cls(int(spec.B), int(spec.Hq), int(spec.Hkv), int(spec.D), [int(n) for n in spec.ctx], heads,
                   int(spec.window), int(spec.metric), int(spec.tau_num), int(spec.tau_den), int(spec.agg),
                   int(spec.window_mode))

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    def r(self, b: int, h: int) -> int:
        hs = self.heads[b][h]
        return hs.budget - hs.sink - hs.recent

    def satellites(self, b: int, p: int) -> List[int]:
        return [h for h in range(self.Hkv) if self.heads[b][h].role == ROLE_SATELLITE and self.heads[b][h].rep == p]

    def reps(self, b: int) -> List[int]:
        """The pivots of sequence b: full heads that at least one satellite follows."""
        return [p for p in range(self.Hkv) if self.heads[b][p].role == ROLE_FULL and self.satellites(b, p)]

    def k_mon(self, b: int, p: int) -> int:
        k = self.heads[b][p].k_mon
        return k if k > 0 else max(self.r(b, s) for s in self.satellites(b, p))

    def cand_range(self, b: int, p: int, ctx: int) -> Tuple[int, int]:
        """Candidate positions [lo, hi) of pivot p's top-k when the sequence holds ctx tokens."""
        sats = self.satellites(b, p)
        s0 = self.heads[b][sats[0]]
        assert all(self.heads[b][s].sink == s0.sink and self.heads[b][s].recent == s0.recent for s in sats)
        return s0.sink, ctx - s0.recent
