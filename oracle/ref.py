"""ctypes loader for the C oracle and the per-step state machine of one layer.

TEST INFRASTRUCTURE ONLY (see hc_oracle.h).  The step order follows Algorithm 1, stage 3:
attention over the resident cache, then for every representative head the aggregated
score, top-k, overlap with the baseline set, windowed-median trigger, and on a trigger the
refill of its satellites' retrieved slots plus the baseline update.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Tuple

import numpy as np
import torch

from oracle.layer import ROLE_FULL, RefSpec

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libhc_oracle.so")


class _Job(C.Structure):
    _fields_ = [("q", C.c_void_p), ("K", C.c_void_p), ("V", C.c_void_p), ("idx", C.c_void_p),
                ("n", C.c_int32), ("out", C.c_void_p), ("lse", C.c_void_p), ("logits", C.c_void_p)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            from oracle.build import build
            build()
        L = C.CDLL(_LIB_PATH)
        L.hc_ref_attn_jobs.argtypes = [C.POINTER(_Job), C.c_int32, C.c_int32, C.c_int32]
        L.hc_ref_attn_jobs.restype = C.c_int
        L.hc_ref_scores.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p]
        L.hc_ref_scores.restype = C.c_int
        L.hc_ref_topk.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p]
        L.hc_ref_topk.restype = C.c_int
        L.hc_ref_intersect.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32]
        L.hc_ref_intersect.restype = C.c_int32
        L.hc_ref_trigger.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32]
        L.hc_ref_trigger.restype = C.c_int32
        L.hc_ref_threads.restype = C.c_int32
        _lib = L
    return _lib


def _bits(t: torch.Tensor) -> np.ndarray:
    """bf16 tensor -> contiguous uint16 array of its bit patterns (host)."""
    assert t.dtype == torch.bfloat16
    return np.ascontiguousarray(t.detach().cpu().contiguous().view(torch.int16).numpy()).view(np.uint16)


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def attn(q_bits: np.ndarray, K_bits: np.ndarray, V_bits: np.ndarray, idx: Optional[np.ndarray] = None,
         want_logits: bool = False):
    """Attention of one KV head's G query heads over its resident set.
    q_bits [G,D], K_bits/V_bits [N,D] uint16 (bf16 patterns); idx int32 resident positions or
    None for all N.  Returns (out [G,D] f64, lse [G] f64, logits [G,n] f64 or None)."""
    return attn_many([(q_bits, K_bits, V_bits, idx, want_logits)])[0]


def attn_many(jobs):
    """Batch of `attn` jobs run in one C call (parallel over jobs x query heads)."""
    if not jobs:
        return []
    G, D = jobs[0][0].shape
    arr = (_Job * len(jobs))()
    keep, res = [], []
    for i, (q, K, V, idx, want) in enumerate(jobs):
        assert q.dtype == np.uint16 and K.dtype == np.uint16 and V.dtype == np.uint16
        assert q.shape == (G, D) and K.shape[1] == D and K.shape == V.shape
        assert q.flags.c_contiguous and K.flags.c_contiguous and V.flags.c_contiguous
        if idx is not None:
            idx = np.ascontiguousarray(idx, dtype=np.int32)
            assert idx.ndim == 1 and idx.size >= 1 and idx.min() >= 0 and idx.max() < K.shape[0]
            n = idx.size
        else:
            n = K.shape[0]
        out = np.empty((G, D), np.float64)
        lse = np.empty((G,), np.float64)
        logits = np.empty((G, n), np.float64) if want else None
        arr[i] = _Job(_ptr(q), _ptr(K), _ptr(V), _ptr(idx), n, _ptr(out), _ptr(lse), _ptr(logits))
        keep.append((q, K, V, idx))
        res.append((out, lse, logits))
    rc = lib().hc_ref_attn_jobs(arr, len(jobs), G, D)
    if rc != 0:
        raise ValueError("oracle attention: non-finite value or bad job")
    return res


def scores(logits: np.ndarray, lse: np.ndarray, agg: int = 0) -> np.ndarray:
    """Aggregated per-position score of a representative head, fp64 [N]."""
    logits = np.ascontiguousarray(logits, np.float64)
    lse = np.ascontiguousarray(lse, np.float64)
    G, N = logits.shape
    s = np.empty((N,), np.float64)
    rc = lib().hc_ref_scores(_ptr(logits), _ptr(lse), G, N, agg, _ptr(s))
    assert rc == 0
    return s


def topk(s32: np.ndarray, lo: int, hi: int, k: int) -> np.ndarray:
    """Ascending list of the k best candidates in [lo,hi): score descending, index ascending."""
    s32 = np.ascontiguousarray(s32, np.float32)
    out = np.empty((k,), np.int32)
    rc = lib().hc_ref_topk(_ptr(s32), lo, hi, k, _ptr(out))
    if rc != 0:
        raise ValueError("oracle topk: bad arguments or NaN score")
    return out


def intersect(a: np.ndarray, b: np.ndarray) -> int:
    a = np.ascontiguousarray(a, np.int32)
    b = np.ascontiguousarray(b, np.int32)
    return int(lib().hc_ref_intersect(_ptr(a), a.size, _ptr(b), b.size))


def trigger(window_inter, k: int, metric: int, tau_num: int, tau_den: int) -> int:
    w = np.ascontiguousarray(window_inter, np.int32)
    r = int(lib().hc_ref_trigger(_ptr(w), w.size, k, metric, tau_num, tau_den))
    assert r in (0, 1)
    return r


def threads() -> int:
    return int(lib().hc_ref_threads())


class RefLayer:
    """State of one layer across decode steps, as the oracle sees it.

    A compressed head is an index list into its master K/V: positions [0,sink), then
    [ctx-recent, ctx), then the r retrieved positions (slot order).  A refill decided at
    step t is used by the attention of step t+1.

    The context may grow (append): the paper's ModelForward returns an updated cache (Algorithm 1)
    without saying how the decode token enters compressed heads or the host tier.  Reading: every head's
    master K/V (for a satellite, its host tier) grows by the token's row at position ctx; full heads
    attend over all of it; a compressed head sees the token through its window of the last `recent`
    positions, and the position that thereby leaves the window becomes an ordinary candidate of the
    pivot's top-k, retrievable like any other.

    window_mode 2 is Algorithm 1's test as printed: the pivot's queries of the window are buffered, and at
    the step that fills the window every buffered query is scored again against the pivot's cache AS IT IS
    THEN (Attention(q_k, C_GPU) with the current C_GPU), its top-k taken over the current candidate range
    and compared with the baseline; the median of those W overlaps decides.  While the cache does not
    change inside a window this equals window_mode 1 (same query, same cache); with a growing context it
    does not (tokens appended since step k are in the softmax, and the candidate range has moved).
    """

    def __init__(self, spec, data,
                 retrieved: Dict[Tuple[int, int], torch.Tensor], base: Dict[Tuple[int, int], torch.Tensor]):
        """spec: a RefSpec or anything RefSpec.of accepts; data: the master K and V of every KV head
        (data.K[(b, h)], data.V[(b, h)]: bf16 [N_b, D])."""
        self.spec = spec = RefSpec.of(spec)
        self.ctx = list(spec.ctx)              # current context length per sequence (grows with append)
        self.Kb = {k: _bits(v) for k, v in data.K.items()}
        self.Vb = {k: _bits(v) for k, v in data.V.items()}
        self.retrieved = {k: np.asarray(v, dtype=np.int32).copy() for k, v in retrieved.items()}
        self.base = {k: np.asarray(v, dtype=np.int32).copy() for k, v in base.items()}
        self.ring: Dict[Tuple[int, int], List[int]] = {k: [] for k in self.base}
        self.qbuf: Dict[Tuple[int, int], List[np.ndarray]] = {k: [] for k in self.base}    # Q_buffer of Algorithm 1
        self.n_tests = 0
        self.n_triggers = 0

    def resident(self, b: int, h: int) -> Optional[np.ndarray]:
        hs = self.spec.heads[b][h]
        if hs.role == ROLE_FULL:
            return None
        N = self.ctx[b]
        return np.concatenate([np.arange(0, hs.sink, dtype=np.int32),
                               np.arange(N - hs.recent, N, dtype=np.int32),
                               self.retrieved[(b, h)]]).astype(np.int32)

    def cand_range(self, b: int, p: int) -> Tuple[int, int]:
        """Candidate positions [lo, hi) of pivot p's top-k at the current context length."""
        return self.spec.cand_range(b, p, self.ctx[b])

    def append(self, k_new: torch.Tensor, v_new: torch.Tensor) -> None:
        """k_new, v_new: bf16 [B, Hkv, D], the decode token's rows; they become position ctx_b of every
        head of sequence b, and ctx_b grows by one.  Call before the step that attends over them."""
        kb = _bits(k_new).reshape(self.spec.B, self.spec.Hkv, self.spec.D)
        vb = _bits(v_new).reshape(self.spec.B, self.spec.Hkv, self.spec.D)
        for b in range(self.spec.B):
            for h in range(self.spec.Hkv):
                self.Kb[(b, h)] = np.concatenate([self.Kb[(b, h)][:self.ctx[b]], kb[b, h][None, :]])
                self.Vb[(b, h)] = np.concatenate([self.Vb[(b, h)][:self.ctx[b]], vb[b, h][None, :]])
            self.ctx[b] += 1

    def slot_rows(self, b: int, h: int):
        """(K rows, V rows) as uint16 bit patterns in slot order: what HBM must hold."""
        idx = self.resident(b, h)
        return self.Kb[(b, h)][idx], self.Vb[(b, h)][idx]

    def step(self, q: torch.Tensor, monitor: bool = True) -> dict:
        sp = self.spec
        G, D = sp.G, sp.D
        qb = _bits(q).reshape(sp.B, sp.Hq, D)
        jobs, where = [], []
        for b in range(sp.B):
            reps = set(sp.reps(b)) if monitor else set()
            for h in range(sp.Hkv):
                jobs.append((np.ascontiguousarray(qb[b, h * G:(h + 1) * G]), self.Kb[(b, h)], self.Vb[(b, h)],
                             self.resident(b, h), h in reps))
                where.append((b, h))
        res = attn_many(jobs)
        out = np.empty((sp.B, sp.Hq, D), np.float64)
        lse = np.empty((sp.B, sp.Hq), np.float64)
        rec = {"out": out, "lse": lse, "scores": {}, "topk": {}, "inter": {}, "flag": {}, "logits": {}, "rescored": {}, "window": {}}
        for (b, h), (o, l, lg) in zip(where, res):
            out[b, h * G:(h + 1) * G] = o
            lse[b, h * G:(h + 1) * G] = l
            if lg is not None:
                rec["logits"][(b, h)] = lg
        if not monitor:
            return rec
        for b in range(sp.B):
            for p in sp.reps(b):
                lg = rec["logits"][(b, p)]
                s = scores(lg, lse[b, p * G:(p + 1) * G], sp.agg)
                rec["scores"][(b, p)] = s
                s32 = s.astype(np.float32)          # the decision is taken on fp32 scores
                lo, hi = self.cand_range(b, p)
                kmon = sp.k_mon(b, p)
                T = topk(s32, lo, hi, kmon)
                rec["topk"][(b, p)] = T
                for sat in sp.satellites(b, p):
                    rec["topk"][(b, sat)] = topk(s32, lo, hi, sp.r(b, sat))
                inter = intersect(T, self.base[(b, p)])
                rec["inter"][(b, p)] = inter
                ring = self.ring[(b, p)]
                ring.append(inter)
                if len(ring) > sp.window:
                    ring.pop(0)
                flag = 0
                tested = len(ring) == sp.window
                if sp.window_mode == 2:
                    qbuf = self.qbuf[(b, p)]
                    qbuf.append(np.ascontiguousarray(qb[b, p * G:(p + 1) * G]))
                    if tested:
                        # every buffered query but the current one (whose overlap was just computed against
                        # this same cache) is scored again over the pivot's whole current cache
                        again = []
                        for j, qk in enumerate(qbuf[:-1]):
                            _, lse_k, lg_k = attn(qk, self.Kb[(b, p)], self.Vb[(b, p)], None, True)
                            s_k = scores(lg_k, lse_k, sp.agg)
                            T_k = topk(s_k.astype(np.float32), lo, hi, kmon)
                            ring[j] = intersect(T_k, self.base[(b, p)])
                            again.append((s_k, T_k, ring[j]))
                        rec["rescored"][(b, p)] = again
                        qbuf.clear()
                if tested:
                    self.n_tests += 1
                    rec["window"][(b, p)] = list(ring)          # the W overlaps the decision is taken on
                    flag = trigger(ring, kmon, sp.metric, sp.tau_num, sp.tau_den)
                rec["flag"][(b, p)] = flag
                if flag:
                    self.n_triggers += 1
                    for sat in sp.satellites(b, p):
                        self.retrieved[(b, sat)] = rec["topk"][(b, sat)].copy()
                    self.base[(b, p)] = T.copy()
                    ring.clear()
                elif tested and sp.window_mode in (1, 2):
                    # Algorithm 1: the buffer of the window is emptied after every test (t mod W = 0),
                    # whether or not it led to a retrieval
                    ring.clear()
        return rec
