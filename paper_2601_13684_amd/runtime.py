"""Device-side plumbing around the C ABI: lay a layer out in HBM and pinned host memory, and issue
the three hot-path calls of one decode step in order.  No arithmetic of the method lives here; every
value is produced by the HIP kernels behind ``binding``.

HBM layout of one layer (the "arena", bf16): for every (sequence, KV head) a K block [len][128]
followed by a V block [len][128], each starting on a 256-byte boundary.  A full head's blocks hold
all ctx positions; a compressed head's hold its slots: [0,sink) the first positions, then the
``recent`` last positions, then the r retrieved positions in ascending order.  The host tier (pinned)
holds, for every satellite, [ctx][2][128]: the K row then the V row of each position, 512 contiguous
bytes per position, so that one retrieved position is one contiguous host read.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Tuple

import torch

from . import binding as hc
from .inputs import ROLE_ANCHOR, ROLE_FULL, ROLE_SATELLITE, LayerData, LayerSpec

D = 128


def make_config(spec: LayerSpec, max_ctx: Optional[int] = None, max_k: Optional[int] = None, growth: int = 0) -> hc.hc_config:
    mc = max_ctx or (max(spec.ctx) + growth)
    mc = (mc + 63) // 64 * 64
    ks = [1]
    for b in range(spec.B):
        ks += [spec.r(b, h) for h in range(spec.Hkv) if spec.heads[b][h].role == ROLE_ANCHOR]     # selected once, at prefill
        for p in spec.reps(b):
            ks.append(spec.k_mon(b, p))
            ks += [spec.r(b, s) for s in spec.satellites(b, p)]
    return hc.hc_config(B=spec.B, Hq=spec.Hq, Hkv=spec.Hkv, D=spec.D, max_ctx=mc, max_k=max_k or max(ks),
                        window=spec.window, metric=spec.metric, tau_num=spec.tau_num, tau_den=spec.tau_den,
                        agg=spec.agg, window_mode=spec.window_mode)


def make_descs(spec: LayerSpec, growth: int = 0) -> Tuple[List[hc.hc_head_desc], int, int]:
    """Head table of a layer plus the arena and host-tier sizes in bf16 elements.  With ``growth`` the K / V
    blocks of full heads and the host-tier blocks of satellites have room for that many appended tokens."""
    descs: List[hc.hc_head_desc] = []
    off = 0
    tier_off = 0
    for b in range(spec.B):
        for h in range(spec.Hkv):
            hs = spec.heads[b][h]
            ln = spec.resident(b, h)
            rows = ln + growth if hs.role == ROLE_FULL else ln          # rows the K and V blocks are laid out for
            d = hc.hc_head_desc(k_off=off, v_off=off + rows * D, tier_off=0, ctx=spec.ctx[b], len=ln, role=hs.role,
                                rep=hs.rep if hs.role == ROLE_SATELLITE else -1, sink=hs.sink, recent=hs.recent,
                                k_mon=hs.k_mon if hs.role == ROLE_FULL else 0,
                                cap=spec.ctx[b] + growth if (growth and hs.role != ROLE_ANCHOR) else 0)
            off += 2 * rows * D
            if hs.role == ROLE_SATELLITE:
                d.tier_off = tier_off
                tier_off += (spec.ctx[b] + growth) * 2 * D
            descs.append(d)
    return descs, off, tier_off


class Context:
    """Owns an hc_ctx and the scratch that consecutive layers can share."""

    def __init__(self, cfg: hc.hc_config, device: str = "cuda:0", workgroups_per_cu: Optional[int] = None,
                 filter_margin: float = 0.0, filter_min_candidates: int = 0):
        self.cfg = cfg
        self.device = torch.device(device)
        with torch.cuda.device(self.device):
            self.handle = hc.hc_create(cfg)
        if workgroups_per_cu:
            hc.hc_set_split(self.handle, workgroups_per_cu)
        if filter_margin:
            hc.hc_set_logit_filter(self.handle, filter_margin, filter_min_candidates)
        self.G = cfg.Hq // cfg.Hkv
        self._scratch: Dict[int, Tuple[torch.Tensor, torch.Tensor]] = {}

    def scratch(self, n_reps: int) -> Tuple[torch.Tensor, torch.Tensor]:
        """(rep_logits [n_reps,max_ctx,G] f32, scores [n_reps,max_ctx] f32), shared by layers."""
        n = max(1, n_reps)
        if n not in self._scratch:
            self._scratch[n] = (torch.zeros((n, self.cfg.max_ctx, self.G), dtype=torch.float32, device=self.device),
                                torch.zeros((n, self.cfg.max_ctx), dtype=torch.float32, device=self.device))
        return self._scratch[n]

    def close(self):
        if self.handle:
            hc.hc_destroy(self.handle)
            self.handle = None


class LayerRuntime:
    def __init__(self, ctx: Context, spec: LayerSpec, data: LayerData,
                 retrieved: Dict[Tuple[int, int], torch.Tensor], base: Dict[Tuple[int, int], torch.Tensor],
                 host_tier: bool = True, own_scratch: bool = False, delta_gather: bool = True, growth: int = 0,
                 prefill: Optional[Tuple[torch.Tensor, int]] = None):
        """``prefill = (q_last, pool)``: ``retrieved`` and ``base`` are ignored (may be None) and the library builds
        the initial state itself from ``data`` and the last prompt token's queries (hc_prefill_init)."""
        self.ctx, self.spec = ctx, spec
        cfg, dev = ctx.cfg, ctx.device
        B, Hkv = spec.B, spec.Hkv
        descs, off, tier_off = make_descs(spec, growth)
        self.descs = descs
        # ---- arena ----
        self.arena = torch.zeros((off,), dtype=torch.bfloat16, device=dev)
        for b in range(B if prefill is None else 0):
            for h in range(Hkv):
                d = descs[b * Hkv + h]
                hs = spec.heads[b][h]
                K, V = data.K[(b, h)], data.V[(b, h)]
                if hs.role == ROLE_FULL:
                    Kr, Vr = K, V
                else:
                    N = spec.ctx[b]
                    idx = torch.cat([torch.arange(0, hs.sink), torch.arange(N - hs.recent, N),
                                     retrieved[(b, h)].long().cpu()]).to(K.device)
                    Kr, Vr = K[idx], V[idx]
                self.arena[d.k_off:d.k_off + d.len * D].copy_(Kr.reshape(-1))
                self.arena[d.v_off:d.v_off + d.len * D].copy_(Vr.reshape(-1))
        # ---- host tier (pinned): [ctx][2][D] per satellite ----
        self.tier = None
        if host_tier and tier_off > 0:
            self.tier = torch.empty((tier_off,), dtype=torch.bfloat16, pin_memory=True)
            if prefill is not None:
                self.tier.zero_()
            for b in range(B if prefill is None else 0):
                for h in range(Hkv):
                    if spec.heads[b][h].role == ROLE_SATELLITE:
                        d = descs[b * Hkv + h]
                        blk = torch.stack([data.K[(b, h)], data.V[(b, h)]], dim=1)      # [N,2,D]
                        self.tier[d.tier_off:d.tier_off + blk.numel()].copy_(blk.reshape(-1))
        # ---- monitor state tables ----
        nh = B * Hkv
        self.topk_idx = torch.full((nh, cfg.max_k), -1, dtype=torch.int32, device=dev)
        self.base_idx = torch.full((nh, cfg.max_k), -1, dtype=torch.int32, device=dev)
        for (b, p), lst in (base.items() if prefill is None else ()):
            self.base_idx[b * Hkv + p, :lst.numel()] = lst.to(dev, torch.int32)
        # which position every retrieved slot of a satellite holds (None: refills replace whole lists)
        self.slot_pos = None
        if delta_gather:
            self.slot_pos = torch.full((nh, cfg.max_k), -1, dtype=torch.int32, device=dev)
            for (b, h), lst in (retrieved.items() if prefill is None else ()):
                if spec.heads[b][h].role == ROLE_SATELLITE:
                    self.slot_pos[b * Hkv + h, :lst.numel()] = lst.to(dev, torch.int32)
        self.ring = torch.zeros((nh, cfg.window + 1), dtype=torch.int32, device=dev)
        self.inter = torch.zeros((nh,), dtype=torch.int32, device=dev)
        self.flag = torch.zeros((nh,), dtype=torch.int32, device=dev)
        self.out = torch.zeros((B, spec.Hq, D), dtype=torch.float32, device=dev)
        self.lse = torch.zeros((B, spec.Hq), dtype=torch.float32, device=dev)
        with torch.cuda.device(dev):
            self.handle = hc.hc_layer_create(ctx.handle, descs)
        self.n_reps = hc.hc_layer_num_reps(self.handle)
        if own_scratch:     # needed when this layer's monitor overlaps the next layer's attention
            n = max(1, self.n_reps)
            self.rep_logits = torch.zeros((n, cfg.max_ctx, ctx.G), dtype=torch.float32, device=dev)
            self.scores = torch.zeros((n, cfg.max_ctx), dtype=torch.float32, device=dev)
        else:
            self.rep_logits, self.scores = ctx.scratch(self.n_reps)
        # Algorithm 1's re-scored window: the buffer of the window's queries and the pass's work buffer
        self.q_window = self.rescore_work = None
        if cfg.window_mode == hc.HC_WINDOW_RESCORED:
            self.q_window = torch.zeros((cfg.window, B, spec.Hq, D), dtype=torch.bfloat16, device=dev)
            self.rescore_work = torch.zeros((hc.hc_rescore_work_bytes(ctx.handle, self.handle),), dtype=torch.uint8, device=dev)
        if prefill is not None:
            self.prefill_init(data, prefill[0], prefill[1])
        # torch creates the HIP event lazily at the first record: do it now, the C ABI needs the handle
        self.ev_topk = torch.cuda.Event()
        self.ev_done = torch.cuda.Event()
        with torch.cuda.device(dev):
            self.ev_topk.record()
            self.ev_done.record()
        self._side_pending = False

    def rep_slot(self, b: int, h: int) -> int:
        return hc.hc_layer_rep_slot(self.handle, b, h)

    def monitor_counts(self, b: int, h: int) -> dict:
        return hc.hc_layer_monitor_counts(self.handle, b, h)

    def kept_rows(self, b: int, h: int):
        """With the pivot-logit filter: (positions, scores) of the rows kept for pivot (b, h) at the last monitored
        step (device tensors, ascending positions), or None if that step fell back to the dense passes (then
        ``scores`` holds every candidate's score by position, as without the filter)."""
        pos_addr, need_addr = hc.hc_layer_filter_view(self.handle)
        if not pos_addr:
            return None
        slot, mc = self.rep_slot(b, h), self.ctx.cfg.max_ctx
        n = self.monitor_counts(b, h)["kept"]
        need = _view_i32(need_addr, self.n_reps, self.ctx.device)
        if n is None or int(need[slot]) != 0:
            return None
        pos = _view_i32(pos_addr + 4 * slot * mc, n, self.ctx.device)
        return pos, self.scores[slot, :n]

    # -- the three calls ------------------------------------------------------------------------
    def attn(self, q: torch.Tensor, monitor: bool = True, stream=None) -> None:
        hc.hc_decode_attn(self.ctx.handle, self.handle, self.arena, q, self.out, self.lse,
                          self.rep_logits if (monitor and self.n_reps) else None, stream)

    def monitor(self, scores_given: bool = False, stream=None) -> None:
        hc.hc_rep_topk_drift(self.ctx.handle, self.handle, self.rep_logits, self.lse, self.scores, scores_given,
                             self.topk_idx, self.base_idx, self.ring, self.inter, self.flag, stream)

    def stage_prefill(self, data: LayerData) -> None:
        """The prefill stage's K/V of every head in one device buffer (the caller's side of hc_prefill_init)."""
        spec, dev = self.spec, self.ctx.device
        self._k_src, self._v_src, parts, off = [], [], [], 0
        for b in range(spec.B):
            for h in range(spec.Hkv):
                for lst, t in ((self._k_src, data.K[(b, h)]), (self._v_src, data.V[(b, h)])):
                    lst.append(off)
                    parts.append(t.reshape(-1))
                    off += t.numel()
        self.kv_prefill = torch.cat([p.to(dev) for p in parts])
        self.prefill_work = torch.zeros((hc.hc_prefill_work_bytes(self.ctx.handle, self.handle),), dtype=torch.uint8, device=dev)

    def prefill_init(self, data: Optional[LayerData], q_last: torch.Tensor, pool: int = 1, stream=None) -> None:
        """The state decoding starts from, built by the library from the prefill stage's K/V (``data``; None: what
        stage_prefill left) and the last prompt token's queries (hc_prefill_init)."""
        if data is not None:
            self.stage_prefill(data)
        hc.hc_prefill_init(self.ctx.handle, self.handle, self.kv_prefill, self._k_src, self._v_src, q_last.to(self.ctx.device), pool,
                           self.arena, self.tier, self.topk_idx, self.base_idx, self.slot_pos, self.ring, self.prefill_work,
                           self.prefill_work.numel(), stream)

    def prefill_scores(self) -> dict:
        """{table row of a selecting head: view of the fp32 scores its selection was taken on}."""
        lay = hc.hc_prefill_work_layout(self.ctx.handle, self.handle, self.spec.B * self.spec.Hkv)
        mc = self.ctx.cfg.max_ctx
        n = len(lay["heads"])
        sc = self.prefill_work[lay["scores"]:lay["scores"] + n * mc * 4].view(torch.float32).view(n, mc)
        return {bh: sc[i] for i, bh in enumerate(lay["heads"])}

    def rescore(self, q: torch.Tensor, stream=None) -> None:
        """Buffer this step's queries; at the window's last step score the earlier ones again (hc_rescore_window).
        Call between attn and monitor, once per monitored step: the layer counts the steps of the window."""
        hc.hc_rescore_window(self.ctx.handle, self.handle, self.arena, q, self.q_window, self.base_idx,
                             self.ring, self.rescore_work, self.rescore_work.numel(), stream)

    def rescored(self, item: int) -> dict:
        """Views of what the last test step's first pass left in the work buffer for buffered query `item`."""
        lay = hc.hc_rescore_work_layout(self.ctx.handle, self.handle)
        cfg, n, w = self.ctx.cfg, max(1, self.n_reps), self.rescore_work
        assert 0 <= item < lay["items_per_pass"]

        def view(off, count, dtype, shape):
            size = count * 4
            return w[off + item * size:off + (item + 1) * size].view(dtype).view(shape)
        nr = self.n_reps
        return dict(logits=view(lay["logits"], nr * cfg.max_ctx * self.ctx.G, torch.float32, (nr, cfg.max_ctx, self.ctx.G)),
                    scores=view(lay["scores"], nr * cfg.max_ctx, torch.float32, (nr, cfg.max_ctx)),
                    lse=view(lay["lse"], cfg.B * cfg.Hq, torch.float32, (cfg.B, cfg.Hq)),
                    topk=view(lay["topk"], cfg.B * cfg.Hkv * cfg.max_k, torch.int32, (cfg.B * cfg.Hkv, cfg.max_k)))

    def tune(self, q: torch.Tensor, rounds: int = 4) -> None:
        """Measure the split pass's share weights on this device with this layer (hc_layer_tune)."""
        hc.hc_layer_tune(self.ctx.handle, self.handle, self.arena, q, self.out, self.lse,
                         self.rep_logits if self.n_reps else None, rounds)

    def append(self, k_new: torch.Tensor, v_new: torch.Tensor, stream=None) -> None:
        """The decode token's K/V rows (bf16 [B, Hkv, D] on the device) enter the cache (hc_append_kv)."""
        hc.hc_append_kv(self.ctx.handle, self.handle, k_new, v_new, self.arena, self.tier, stream)

    def context(self, b: int) -> int:
        return hc.hc_layer_context(self.handle, b)

    def gather(self, stream=None, wait_event=None, done_event=None) -> None:
        hc.hc_gather_retrieve(self.ctx.handle, self.handle, self.tier, self.topk_idx, self.flag, self.arena,
                              self.slot_pos, stream, wait_event, done_event)

    def step(self, q: torch.Tensor, side: Optional[torch.cuda.Stream] = None) -> None:
        """One decode step of this layer.  Attention runs on the current stream; with ``side`` the monitor
        and the gather run there (so that they overlap whatever the current stream does next), otherwise
        they follow on the current stream.  A refill decided now is visible to the next step's attention:
        that attention waits for this step's side-stream work first (which also protects rep_logits,
        scores and lse of this layer from being overwritten while the monitor reads them)."""
        main = torch.cuda.current_stream()
        if self._side_pending:
            main.wait_event(self.ev_done)
            self._side_pending = False
        self.attn(q)
        if not self.n_reps:
            return
        if side is None:
            if self.q_window is not None:
                self.rescore(q)
            self.monitor()
            if self.tier is not None:
                self.gather()
            return
        self.ev_topk.record(main)                   # attention of this layer is enqueued
        side.wait_event(self.ev_topk)
        if self.q_window is not None:
            self.rescore(q, stream=side)            # q must stay untouched until the side stream is through (ev_done)
        self.monitor(stream=side)
        if self.tier is not None:
            self.gather(stream=side, done_event=self.ev_done)
        else:
            self.ev_done.record(side)
        self._side_pending = True

    def close(self):
        if self.handle:
            hc.hc_layer_destroy(self.handle)
            self.handle = None


class _DeviceInts:
    """n int32 at a raw device address, in the form torch.as_tensor understands."""

    def __init__(self, addr: int, n: int):
        self.__cuda_array_interface__ = {"shape": (n,), "typestr": "<i4", "data": (addr, False), "version": 2}


def _view_i32(addr: int, n: int, device) -> torch.Tensor:
    """A copy of n int32 of library-owned device memory."""
    if n <= 0:
        return torch.empty((0,), dtype=torch.int32, device=device)
    return torch.as_tensor(_DeviceInts(addr, n), device=device).clone()


def make_step_io(layers: List[LayerRuntime], q_per_layer: torch.Tensor, monitor: bool = True):
    """ctypes array for hc_decode_step: q_per_layer [L,B,Hq,D] bf16 is a fixed device buffer the caller
    refills before every step."""
    arr = (hc.hc_layer_io * len(layers))()
    for l, lay in enumerate(layers):
        arr[l] = hc.hc_layer_io(layer=lay.handle, kv_arena=lay.arena.data_ptr(),
                                host_tier=lay.tier.data_ptr() if lay.tier is not None else None,
                                q=q_per_layer[l].data_ptr(), out=lay.out.data_ptr(), lse=lay.lse.data_ptr(),
                                rep_logits=lay.rep_logits.data_ptr(),
                                scores=lay.scores.data_ptr() if monitor else None,
                                topk_idx=lay.topk_idx.data_ptr(), base_idx=lay.base_idx.data_ptr(),
                                ring=lay.ring.data_ptr(), inter=lay.inter.data_ptr(), flag=lay.flag.data_ptr(),
                                slot_pos=lay.slot_pos.data_ptr() if lay.slot_pos is not None else None,
                                q_window=lay.q_window.data_ptr() if lay.q_window is not None else None,
                                rescore_work=lay.rescore_work.data_ptr() if lay.rescore_work is not None else None,
                                rescore_work_bytes=lay.rescore_work.numel() if lay.rescore_work is not None else 0)
    return arr
