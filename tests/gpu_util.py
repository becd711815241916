"""Helpers of the GPU parity tests: tolerances and set-validity checks."""
import numpy as np
import torch

from oracle import prefill as oracle_prefill
from oracle import ref
from paper_2601_13684_amd import inputs as I
from paper_2601_13684_amd import runtime as R

# Tolerances of the attention outputs (bf16 inputs, fp32 accumulation against the fp64 oracle):
#   |gpu - ref| <= 2e-2 + 1e-2 |ref|                 the stated bar
#   max |gpu - ref| <= 1e-2 * rms(ref) per query head   (the stated bar is vacuous for diffuse attention,
#                                                        whose outputs are ~3e-3 at 224K)
#   |lse_gpu - lse_ref| <= 1e-4 + 1e-6 |lse_ref|
ATOL, RTOL, RMS_FRAC, LSE_ATOL = 2e-2, 1e-2, 1e-2, 1e-4


def check_attention(out_gpu: torch.Tensor, lse_gpu: torch.Tensor, rec: dict, where: str = ""):
    o = out_gpu.detach().cpu().double().numpy()
    l = lse_gpu.detach().cpu().double().numpy()
    ro, rl = rec["out"], rec["lse"]
    assert np.isfinite(o).all() and np.isfinite(l).all(), where
    err = np.abs(o - ro)
    assert (err <= ATOL + RTOL * np.abs(ro)).all(), (where, err.max())
    rms = np.sqrt((ro ** 2).mean(-1))                       # [B,Hq]
    worst = (err.max(-1) / np.maximum(rms, 1e-30)).max()
    assert worst <= RMS_FRAC, (where, "max err / rms(ref)", worst)
    lerr = np.abs(l - rl)
    assert (lerr <= LSE_ATOL + 1e-6 * np.abs(rl)).all(), (where, "lse", lerr.max())
    return float(worst), float(lerr.max())


def check_scores(s_gpu: np.ndarray, s_ref: np.ndarray, lo: int, hi: int, where: str = ""):
    """fp32 scores of the kernel against the fp64 scores: 1e-5 absolute + 1e-4 relative."""
    d = np.abs(s_gpu[lo:hi].astype(np.float64) - s_ref[lo:hi])
    assert (d <= 1e-5 + 1e-4 * np.abs(s_ref[lo:hi])).all(), (where, d.max())
    return float(d.max()), float((d / np.maximum(np.abs(s_ref[lo:hi]), 1e-300)).max())


def check_gpu_scores(gpu, b: int, pv: int, s_ref: np.ndarray, lo: int, hi: int, where: str = ""):
    """The scores pivot (b, pv)'s last monitor call decided on, against the fp64 scores.  Without the pivot-logit
    filter (or after a fallback) that is every candidate's score by position; with it, the scores of the rows the
    split pass kept, whose positions must be ascending candidates.  Returns (max abs difference, max relative)."""
    kept = gpu.kept_rows(b, pv)
    if kept is None:
        return check_scores(gpu.scores[gpu.rep_slot(b, pv)].cpu().numpy(), s_ref, lo, hi, where)
    pos, sc = kept[0].cpu().numpy(), kept[1].cpu().numpy().astype(np.float64)
    assert pos.size and (np.diff(pos) > 0).all() and pos[0] >= lo and pos[-1] < hi, (where, "kept positions")
    d = np.abs(sc - s_ref[pos])
    assert (d <= 1e-5 + 1e-4 * np.abs(s_ref[pos])).all(), (where, "kept scores", d.max())
    return float(d.max()), float((d / np.maximum(np.abs(s_ref[pos]), 1e-300)).max())


def band_of(dabs: float) -> float:
    """Width of the near-tie band around the k-th fp64 score inside which the GPU's set may differ from the
    oracle's: 4 times the largest difference between the GPU's fp32 scores and the fp64 scores of this very
    call.  (Both sides decide on fp32 scores; two candidates can change places only if their fp64 scores are
    closer than the two scores' errors together, 2 max|ds| for the GPU side and as much again for the oracle's
    own rounding of its fp64 scores to fp32.)"""
    return 4.0 * float(dabs)


NEAR_TIES = []      # every difference that was accepted inside the band: (where, index, |score - kth|, band)


def check_set_valid(T_gpu: np.ndarray, T_ref: np.ndarray, s_ref: np.ndarray, band: float, where: str = ""):
    """Both are k-subsets in ascending order.  They must agree except for candidates whose fp64 score lies within
    `band` (absolute, see band_of) of the k-th fp64 score: near-ties that the fp32 rounding of the scores may
    order either way.  Every accepted difference is printed and kept in NEAR_TIES.  Returns the size of the
    symmetric difference."""
    assert T_gpu.shape == T_ref.shape, where
    assert (np.diff(T_gpu) > 0).all(), (where, "list not strictly ascending")
    a, b = set(T_gpu.tolist()), set(T_ref.tolist())
    diff = sorted(a ^ b)
    if diff:
        kth = s_ref[T_ref].min()
        dev = np.abs(s_ref[diff] - kth)
        assert (dev <= band + 2.0 ** -23 * abs(kth)).all(), (where, "set differs outside the near-tie band", float(dev.max()), band, len(diff))
        for j, d in zip(diff, dev):
            NEAR_TIES.append((where, int(j), float(d), float(band)))
            print(f"  near-tie accepted: {where} index {j} |score - kth| {d:.3e} band {band:.3e} kth {kth:.3e}", flush=True)
    return len(diff)


class Pair:
    """One layer on the GPU and its oracle twin, fed the same inputs."""

    def __init__(self, spec, data, device="cuda:0", ctx=None, host_tier=True, wg_per_cu=None, delta_gather=True, growth=0,
                 filter_margin=0.0):
        self.spec, self.data = spec, data
        self.ctx0 = list(spec.ctx)
        retrieved, base = I.initial_lists(spec)
        self.own_ctx = ctx is None
        self.ctx = ctx or R.Context(R.make_config(spec, growth=growth), device, workgroups_per_cu=wg_per_cu,
                                    filter_margin=filter_margin)
        self.gpu = R.LayerRuntime(self.ctx, spec, data, retrieved, base, host_tier=host_tier, delta_gather=delta_gather, growth=growth)
        cpu = I.LayerData({k: v.cpu() for k, v in data.K.items()}, {k: v.cpu() for k, v in data.V.items()}, {})
        self.ref = ref.RefLayer(spec, cpu, retrieved, base)

    @classmethod
    def from_prefill(cls, spec, data, q_last, pool, device="cuda:0", growth=0, where="prefill", filter_margin=0.0):
        """The GPU side builds its initial state with hc_prefill_init, the oracle twin with oracle/prefill.py.  Scores
        and lists are compared here (a list may differ from the oracle's inside the near-tie band: the twin
        then starts from the GPU's list, so that everything downstream compares like with like).
        Returns (pair, number of lists that differed)."""
        self = cls.__new__(cls)
        self.spec, self.data = spec, data
        self.ctx0 = list(spec.ctx)
        self.own_ctx = True
        self.ctx = R.Context(R.make_config(spec, growth=growth), device, filter_margin=filter_margin)
        self.gpu = R.LayerRuntime(self.ctx, spec, data, None, None, growth=growth, prefill=(q_last, pool))
        torch.cuda.synchronize()
        cpu = I.LayerData({k: v.cpu() for k, v in data.K.items()}, {k: v.cpu() for k, v in data.V.items()}, {})
        retrieved, base, scores = oracle_prefill.prefill_init(spec, cpu, q_last.cpu(), pool)
        got_scores = self.gpu.prefill_scores()
        assert sorted(got_scores) == sorted(b * spec.Hkv + h for (b, h) in scores)
        topk = self.gpu.topk_idx.cpu().numpy()
        basei = self.gpu.base_idx.cpu().numpy()
        differed = 0
        for (b, h), s_ref in scores.items():
            row = b * spec.Hkv + h
            dabs, _ = check_scores(got_scores[row].cpu().numpy(), s_ref, 0, spec.ctx[b], f"{where} head {(b, h)}")
            want = base[(b, h)] if (b, h) in base else retrieved[(b, h)]
            got = topk[row, :want.size].copy()
            if check_set_valid(got, want, s_ref, band_of(dabs), f"{where} head {(b, h)}"):
                differed += 1
            if (b, h) in base:
                assert np.array_equal(basei[row, :want.size], got), (where, "baseline row is not the pivot's list")
                base[(b, h)] = got
            else:
                retrieved[(b, h)] = got
        self.ref = ref.RefLayer(spec, cpu, {k: torch.from_numpy(v) for k, v in retrieved.items()},
                                {k: torch.from_numpy(v) for k, v in base.items()})
        return self, differed

    def tier_equals_masters(self):
        """Every satellite's block of the host tier holds its whole K and V, K row then V row per position."""
        if self.gpu.tier is None:               # a layer without satellites has no host tier
            return all(h.role != I.ROLE_SATELLITE for row in self.spec.heads for h in row)
        tier = self.gpu.tier.view(torch.int16).numpy().view(np.uint16)
        for b in range(self.spec.B):
            for h in range(self.spec.Hkv):
                if self.spec.heads[b][h].role != I.ROLE_SATELLITE:
                    continue
                d = self.gpu.descs[b * self.spec.Hkv + h]
                N = self.spec.ctx[b]
                want = np.stack([ref._bits(self.data.K[(b, h)].cpu()), ref._bits(self.data.V[(b, h)].cpu())], axis=1).reshape(-1)
                if not np.array_equal(tier[d.tier_off:d.tier_off + N * 256], want):
                    return False
        return True

    def slots_equal_oracle(self):
        """Byte-exact comparison of every compressed head's K/V slots with the oracle's rows.  With a slot
        map the retrieved slots may be in any order: the map must be a permutation of the oracle's list,
        and every slot must hold the rows of the position the map names."""
        arena = self.gpu.arena.cpu().view(torch.int16).numpy().view(np.uint16)
        slot_pos = self.gpu.slot_pos.cpu().numpy() if self.gpu.slot_pos is not None else None
        ctx0 = getattr(self, "ctx0", self.spec.ctx)
        for b in range(self.spec.B):
            for h in range(self.spec.Hkv):
                hs = self.spec.heads[b][h]
                if hs.role == I.ROLE_FULL:
                    continue
                d = self.gpu.descs[b * self.spec.Hkv + h]
                Kr, Vr = self.ref.slot_rows(b, h)
                Kg = arena[d.k_off:d.k_off + d.len * 128].reshape(-1, 128)
                Vg = arena[d.v_off:d.v_off + d.len * 128].reshape(-1, 128)
                fixed = hs.sink + hs.recent
                r = d.len - fixed
                if hs.recent and self.ref.ctx[b] != ctx0[b]:
                    # after appends the recent slots are a ring: slot sink + (position - initial ctx) mod recent
                    pos = self.ref.resident(b, h)[hs.sink:fixed]
                    ring = np.argsort((pos - ctx0[b]) % hs.recent)           # oracle rows in GPU slot order
                    Kr = np.concatenate([Kr[:hs.sink], Kr[hs.sink:fixed][ring], Kr[fixed:]])
                    Vr = np.concatenate([Vr[:hs.sink], Vr[hs.sink:fixed][ring], Vr[fixed:]])
                if slot_pos is not None and hs.role == I.ROLE_SATELLITE and r > 0:
                    sp = slot_pos[b * self.spec.Hkv + h, :r]
                    order = np.argsort(sp, kind="stable")
                    if not np.array_equal(sp[order], self.ref.resident(b, h)[fixed:]):
                        return False
                    Kg = np.concatenate([Kg[:fixed], Kg[fixed:][order]])
                    Vg = np.concatenate([Vg[:fixed], Vg[fixed:][order]])
                if not (np.array_equal(Kg, Kr) and np.array_equal(Vg, Vr)):
                    return False
        return True

    def push_oracle_state_to_gpu(self, rec):
        """Re-synchronise after a near-tie disagreement: the oracle's lists, flags and baseline are
        written into the device tables and the gather is re-run from them (oracle -> GPU only)."""
        sp, g = self.spec, self.gpu
        for (b, h), T in rec["topk"].items():
            g.topk_idx[b * sp.Hkv + h, :T.size] = torch.from_numpy(T).to(g.topk_idx.device)
        for (b, p), f in rec["flag"].items():
            g.flag[b * sp.Hkv + p] = int(f)
            g.inter[b * sp.Hkv + p] = int(rec["inter"][(b, p)])
            base = self.ref.base[(b, p)]
            g.base_idx[b * sp.Hkv + p, :base.size] = torch.from_numpy(base).to(g.base_idx.device)
        torch.cuda.synchronize()
        if g.tier is not None:
            g.gather()
            torch.cuda.synchronize()

    def close(self):
        self.gpu.close()
        if self.own_ctx:
            self.ctx.close()
