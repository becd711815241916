"""CPU oracle of the prefill-time initialisation of a layer: TEST INFRASTRUCTURE ONLY.

What the state looks like when decoding starts (Sec. 4.3, first paragraphs; Algorithm 1, the lines of
stage 3 before the loop): full heads keep all of their K/V; every compressed head keeps the K/V of the
positions with its OWN top attention scores of the prefill stage; the pivots' baseline sets are their top
attended indices of the prefill stage; the satellites' whole K/V goes to the host tier.  "Attention scores
of the prefill stage" are those of the last prompt token (App. B.1, App. C.1): per KV head the mean over
its query group of the softmax weights (App. C.1), optionally smoothed by a 1-D average pooling over
positions before the top entries are taken (App. C.1).

Readings (the paper gives no formula for either): pooling is a centred window of odd size P, stride 1,
zero padding and divisor P (what a library average pooling with padding P // 2 computes); the budget of a
compressed head is split as in decoding (first `sink` and last `recent` positions always resident, the
other r = budget - sink - recent slots go to the r best of the remaining positions), and a pivot's
baseline is taken over its satellites' candidate positions, so that the first decode step compares like
with like.

Plain numpy on top of the attention oracle; decisions on fp32 scores like every other top-k here.
Pins: tests/test_oracle_prefill.py.
"""
from __future__ import annotations

from typing import Dict, Tuple

import numpy as np
import torch

from oracle import ref
from oracle.layer import ROLE_FULL, RefSpec


def avg_pool_loops(s: np.ndarray, P: int) -> np.ndarray:
    """out[j] = (1/P) * sum of s[j - P//2 .. j + P//2], positions outside the array counting as zero: the
    definition, one position and one term at a time (short arrays)."""
    assert P >= 1 and P % 2 == 1
    s = np.asarray(s, np.float64)
    out = np.zeros_like(s)
    h = P // 2
    for j in range(s.size):
        acc = 0.0
        for d in range(-h, h + 1):
            if 0 <= j + d < s.size:
                acc += s[j + d]
        out[j] = acc / P
    return out


def avg_pool(s: np.ndarray, P: int) -> np.ndarray:
    """The same sums, term by term in the same order (offset -P//2 first), each term added for all positions at
    once; no rearrangement of the arithmetic, so the result equals avg_pool_loops bit for bit."""
    assert P >= 1 and P % 2 == 1
    s = np.asarray(s, np.float64)
    n, h = s.size, P // 2
    acc = np.zeros_like(s)
    for d in range(-h, h + 1):
        lo, hi = max(0, -d), min(n, n - d)          # positions j with 0 <= j + d < n
        if lo < hi:
            acc[lo:hi] += s[lo + d:hi + d]
    return acc / P


def head_scores(q_bits: np.ndarray, K_bits: np.ndarray, agg: int, pool: int) -> np.ndarray:
    """Smoothed last-token score of every position of one KV head, fp64 [N]."""
    _, lse, lg = ref.attn(q_bits, K_bits, K_bits, None, True)        # the value rows do not matter here
    s = ref.scores(lg, lse, agg)
    return s if pool == 1 else avg_pool(s, pool)


def prefill_init(spec, data, q_last: torch.Tensor, pool: int = 1):
    """Returns (retrieved, base, scores): retrieved[(b, h)] = ascending int32 positions in the r refillable
    slots of compressed head h; base[(b, p)] = ascending int32 baseline set of pivot p; scores[(b, h)] =
    the fp64 smoothed scores the selection of head h was taken on."""
    spec = RefSpec.of(spec)
    G, D = spec.G, spec.D
    qb = ref._bits(q_last).reshape(spec.B, spec.Hq, D)
    retrieved: Dict[Tuple[int, int], np.ndarray] = {}
    base: Dict[Tuple[int, int], np.ndarray] = {}
    scores: Dict[Tuple[int, int], np.ndarray] = {}
    for b in range(spec.B):
        N = spec.ctx[b]
        pivots = spec.reps(b)
        for h in range(spec.Hkv):
            hs = spec.heads[b][h]
            if hs.role == ROLE_FULL and h not in pivots:
                continue                                   # a volatile head keeps everything and selects nothing
            s = head_scores(np.ascontiguousarray(qb[b, h * G:(h + 1) * G]), ref._bits(data.K[(b, h)]), spec.agg, pool)
            scores[(b, h)] = s
            s32 = s.astype(np.float32)
            if hs.role == ROLE_FULL:
                lo, hi = spec.cand_range(b, h, N)
                base[(b, h)] = ref.topk(s32, lo, hi, spec.k_mon(b, h))
            else:
                retrieved[(b, h)] = ref.topk(s32, hs.sink, N - hs.recent, spec.r(b, h))
    return retrieved, base, scores
