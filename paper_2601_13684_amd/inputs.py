"""Seeded synthetic inputs for the HeteroCache decode hot path.

This module only *describes* a layer (which KV heads are full, which are
compressed, their budgets) and *draws* random tensors of the shapes the paper's
workloads have (Llama-3.1-8B-shaped layers: 32 query heads, 8 KV heads,
head_dim 128, contexts of 4K to 224K tokens, Sec. 5 and App. D).  It holds none of the
method's arithmetic: no softmax, no top-k, no overlap test.  Both the HIP path
and the CPU oracle consume what is generated here, and nothing else is shared
between them.

Everything is deterministic given (seed, device type).  Tensors are drawn with
``torch.Generator`` on the requested device; CPU and GPU generators produce
different streams, but both sides of a parity test always see copies of the
same bits.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import torch

ROLE_FULL = 0        # volatile or pivot head: whole context resident in HBM (Sec. 4.3)
ROLE_SATELLITE = 1   # compressed, refilled from the host tier under its pivot's guidance
ROLE_ANCHOR = 2      # compressed, statically (never refilled)

METRIC_OVERLAP = 0   # Eq. 9: |K_t ∩ K_base| / L_base
METRIC_JACCARD = 1   # |∩| / |∪| (the synthetic configs quote their threshold on this)

AGG_PROB = 0         # GQA aggregation = mean of post-softmax weights (App. C.1)
AGG_LOGIT = 1        # mean of scaled logits (test mode: exact in fp32 for integer inputs)


@dataclass(frozen=True)
class HeadSpec:
    """One KV head of one sequence."""
    role: int
    rep: int = -1          # satellite: KV-head index of its representative (pivot), same sequence
    sink: int = 0          # compressed: positions [0, sink) are always resident
    recent: int = 0        # compressed: positions [ctx-recent, ctx) are always resident
    budget: int = 0        # compressed: resident rows l = sink + recent + r; full: ignored
    k_mon: int = 0         # representative only: size of the monitored top-k set; 0 = max r of its cluster


@dataclass
class LayerSpec:
    B: int
    Hq: int
    Hkv: int
    D: int
    ctx: List[int]                     # context length N_b per sequence
    heads: List[List[HeadSpec]]        # [B][Hkv]
    window: int = 1                    # W of Eq. 10
    metric: int = METRIC_JACCARD
    tau_num: int = 4                   # drift threshold tau = tau_num / tau_den
    tau_den: int = 5
    agg: int = AGG_PROB
    window_mode: int = 0               # 0: sliding window (Eq. 10), 1: tumbling window (Algorithm 1), 2: tumbling with the
                                       # window's buffered queries scored again at the test step (Algorithm 1 as printed)

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    def resident(self, b: int, h: int) -> int:
        hs = self.heads[b][h]
        return self.ctx[b] if hs.role == ROLE_FULL else hs.budget

    def r(self, b: int, h: int) -> int:
        """Number of retrieved (refillable) slots of a compressed head."""
        hs = self.heads[b][h]
        return hs.budget - hs.sink - hs.recent

    def satellites(self, b: int, p: int) -> List[int]:
        return [h for h in range(self.Hkv)
                if self.heads[b][h].role == ROLE_SATELLITE and self.heads[b][h].rep == p]

    def reps(self, b: int) -> List[int]:
        return [p for p in range(self.Hkv) if self.satellites(b, p)]

    def k_mon(self, b: int, p: int) -> int:
        hs = self.heads[b][p]
        if hs.k_mon > 0:
            return hs.k_mon
        return max(self.r(b, s) for s in self.satellites(b, p))

    def cand_range(self, b: int, p: int) -> Tuple[int, int]:
        """Candidate positions [lo, hi) of a representative's top-k: everything that is
        not a sink or recent slot of its satellites (they all share sink/recent)."""
        s0 = self.satellites(b, p)[0]
        hs = self.heads[b][s0]
        return hs.sink, self.ctx[b] - hs.recent

    def kv_bytes(self) -> int:
        """Algorithmic K+V bytes one decode step of this layer has to read."""
        return sum(self.resident(b, h) * self.D * 2 * 2
                   for b in range(self.B) for h in range(self.Hkv))


@dataclass
class LayerData:
    """Master (full-length) K and V of every KV head; bf16 [N_b, D] each."""
    K: Dict[Tuple[int, int], torch.Tensor] = field(default_factory=dict)
    V: Dict[Tuple[int, int], torch.Tensor] = field(default_factory=dict)
    heavy: Dict[Tuple[int, int], torch.Tensor] = field(default_factory=dict)   # planted positions


def _gen(seed: int, device: str) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _randn(shape, g: torch.Generator, device: str, dtype=torch.float32) -> torch.Tensor:
    return torch.randn(shape, generator=g, device=device, dtype=dtype)


def draw_q(spec: LayerSpec, seed: int, device: str = "cpu") -> torch.Tensor:
    """Base query of a layer, fp64 [B, Hq, D] ~ N(0,1) (kept in fp64 so that schedules
    can rotate it without accumulating bf16 rounding)."""
    g = _gen(seed, device)
    return _randn((spec.B, spec.Hq, spec.D), g, device).double()


def draw_token(spec: LayerSpec, seed: int, device: str = "cpu", toward: Optional[torch.Tensor] = None,
               gain: float = 0.0) -> Tuple[torch.Tensor, torch.Tensor]:
    """K and V rows of one generated token for every (sequence, KV head): bf16 [B, Hkv, D] ~ N(0,1); with
    ``toward`` (a query [B, Hq, D]) and ``gain`` the key gets ``gain`` times the unit mean of the head's
    query group added (a planted heavy token)."""
    g = _gen(seed, device)
    k = _randn((spec.B, spec.Hkv, spec.D), g, device)
    v = _randn((spec.B, spec.Hkv, spec.D), g, device)
    if toward is not None and gain:
        u = toward.to(device).float().reshape(spec.B, spec.Hkv, spec.G, spec.D).mean(2)
        k = k + gain * u / u.norm(dim=-1, keepdim=True)
    return k.to(torch.bfloat16), v.to(torch.bfloat16)


def draw_layer(spec: LayerSpec, q0: torch.Tensor, seed: int, device: str = "cpu",
               heavy_frac: float = 0.0, heavy_count: Optional[int] = None,
               heavy_gain: float = 3.0, heavy_noise: float = 0.3,
               segments: int = 0) -> LayerData:
    """K, V ~ N(0,1) in bf16 for every (sequence, KV head), with planted heavy tokens.

    A heavy token's key is ``heavy_gain * u + heavy_noise * N(0,1)`` with ``u`` the unit
    vector along the mean of that KV head's query group (recipe of the synthetic
    configs).  Heavy positions are drawn without replacement from the positions that
    are neither sink nor recent slots; with ``segments > 0`` they form that many
    contiguous, non-overlapping runs instead.
    """
    data = LayerData()
    G = spec.G
    for b in range(spec.B):
        N = spec.ctx[b]
        for h in range(spec.Hkv):
            g = _gen(seed + 100000 * b + 10 * h + 1, device)
            K = _randn((N, spec.D), g, device)
            V = _randn((N, spec.D), g, device)
            n_heavy = heavy_count if heavy_count is not None else int(round(heavy_frac * N))
            pos = torch.empty(0, dtype=torch.long, device=device)
            if n_heavy > 0:
                lo, hi = _heavy_range(spec, b, h)
                if segments > 0:
                    pos = _segment_positions(lo, hi, n_heavy, segments, g, device)
                else:
                    perm = torch.randperm(hi - lo, generator=g, device=device)[:n_heavy]
                    pos = (perm + lo).sort().values
                u = q0[b, h * G:(h + 1) * G].mean(0).float().to(device)
                u = u / u.norm()
                K[pos] = heavy_gain * u[None, :] + heavy_noise * _randn((pos.numel(), spec.D), g, device)
            data.K[(b, h)] = K.to(torch.bfloat16).contiguous()
            data.V[(b, h)] = V.to(torch.bfloat16).contiguous()
            data.heavy[(b, h)] = pos
    return data


def _heavy_range(spec: LayerSpec, b: int, h: int) -> Tuple[int, int]:
    hs = spec.heads[b][h]
    if hs.role == ROLE_FULL:
        sats = spec.satellites(b, h)
        if sats:
            return spec.cand_range(b, h)
        return 0, spec.ctx[b]
    return hs.sink, spec.ctx[b] - hs.recent


def _segment_positions(lo: int, hi: int, n_heavy: int, segments: int,
                       g: torch.Generator, device: str) -> torch.Tensor:
    """``segments`` contiguous non-overlapping runs holding ``n_heavy`` positions in total,
    starts uniform: the range is cut into equal stripes and one run is placed uniformly
    inside each stripe."""
    base, extra = divmod(n_heavy, segments)
    stripe = (hi - lo) // segments
    out = []
    for s in range(segments):
        ln = base + (1 if s < extra else 0)
        off = int(torch.randint(0, max(1, stripe - ln + 1), (1,), generator=g, device=device).item())
        start = lo + s * stripe + off
        out.append(torch.arange(start, start + ln, device=device))
    return torch.cat(out)


class QuerySchedule:
    """Sequence of decode-step queries q_t, bf16 [B, Hq, D].

    ``step_deg``: every step each query head is rotated by this angle toward a fresh
    random direction orthogonal to it (keeps its norm).  ``jump_every``/``jump_deg``:
    additionally, at steps that are positive multiples of ``jump_every`` the head is
    rotated by ``jump_deg``; ``jump_prob`` instead makes the jump an independent
    Bernoulli event per sequence and step.  State is carried in fp64 and rounded to
    bf16 only on output.
    """

    def __init__(self, q0: torch.Tensor, seed: int, step_deg: float = 0.0,
                 jump_every: int = 0, jump_deg: float = 0.0, jump_prob: float = 0.0):
        self.device = str(q0.device)
        self.q = q0.clone().double()
        self.g = _gen(seed, self.device)
        self.step_deg, self.jump_every, self.jump_deg, self.jump_prob = step_deg, jump_every, jump_deg, jump_prob
        self.t = 0

    def _rotate(self, deg: torch.Tensor) -> None:
        # deg: [B, 1, 1] angles in degrees (0 = leave unchanged)
        q = self.q
        w = _randn(tuple(q.shape), self.g, self.device).double()
        qn = q.norm(dim=-1, keepdim=True)
        w = w - (w * q).sum(-1, keepdim=True) / (qn * qn) * q
        w = w / w.norm(dim=-1, keepdim=True) * qn
        th = deg * (math.pi / 180.0)
        self.q = torch.cos(th) * q + torch.sin(th) * w

    def next(self) -> torch.Tensor:
        B = self.q.shape[0]
        if self.t > 0:
            if self.step_deg:
                self._rotate(torch.full((B, 1, 1), float(self.step_deg), dtype=torch.float64, device=self.device))
            if self.jump_every and self.t % self.jump_every == 0:
                self._rotate(torch.full((B, 1, 1), float(self.jump_deg), dtype=torch.float64, device=self.device))
            elif self.jump_prob > 0.0:
                hit = torch.rand((B, 1, 1), generator=self.g, device=self.device) < self.jump_prob
                self._rotate(hit.double() * float(self.jump_deg))
        self.t += 1
        return self.q.to(torch.bfloat16).contiguous()


# --------------------------------------------------------------------------------------
# The five synthetic workloads (shapes: Llama-3.1-8B layer, contexts of App. D / Table 9).
# Every builder takes size overrides so that tests can run reduced copies of the same recipe.
# --------------------------------------------------------------------------------------

def _cluster_heads(budgets: Sequence[int], sink: int, recent: int, n_full: int = 2) -> List[HeadSpec]:
    """Heads 0..n_full-1 full; compressed head j (in order) follows full head j % n_full."""
    heads = [HeadSpec(ROLE_FULL) for _ in range(n_full)]
    for j, l in enumerate(budgets):
        heads.append(HeadSpec(ROLE_SATELLITE, rep=j % n_full, sink=sink, recent=recent, budget=l))
    return heads


def spec_tiny(N: int = 4096, budget: int = 512, sink: int = 64, recent: int = 128) -> LayerSpec:
    heads = [HeadSpec(ROLE_FULL), HeadSpec(ROLE_SATELLITE, rep=0, sink=sink, recent=recent, budget=budget)]
    return LayerSpec(B=1, Hq=8, Hkv=2, D=128, ctx=[N], heads=[heads])


def spec_llama(N: int, budgets: Sequence[int], sink: int = 64, recent: int = 256) -> LayerSpec:
    return LayerSpec(B=1, Hq=32, Hkv=8, D=128, ctx=[N], heads=[_cluster_heads(budgets, sink, recent)])


def spec_dense(N: int, B: int = 1, Hq: int = 32, Hkv: int = 8) -> LayerSpec:
    """Uncompressed comparison: every KV head full."""
    return LayerSpec(B=B, Hq=Hq, Hkv=Hkv, D=128, ctx=[N] * B,
                     heads=[[HeadSpec(ROLE_FULL) for _ in range(Hkv)] for _ in range(B)])


CONFIG_BUDGETS = {
    2: (4096, 2048, 2048, 1024, 1024, 512),
    3: (8192, 4096, 4096, 2048, 2048, 1024),
    4: (8192, 4096, 4096, 2048, 2048, 1024),
}
CONFIG_CTX = {1: 4096, 2: 32768, 3: 131072, 4: 229376}
CONFIG_LAYERS = {1: 1, 2: 1, 3: 32, 4: 32, 5: 8}
CONFIG_STEPS = {1: 8, 2: 64, 3: 128, 4: 64, 5: 64}


def spec_ragged(seed: int, B: int = 16, lo: int = 8192, hi: int = 131072,
                budgets: Sequence[int] = (512, 1024, 2048, 4096), n_full: int = 2,
                Hq: int = 32, Hkv: int = 8, sink: int = 64, recent: int = 256, ctx: Optional[Sequence[int]] = None) -> LayerSpec:
    """Batched ragged workload: contexts log-uniform in [lo, hi]; per sequence ``n_full`` of the
    KV heads are full (drawn uniformly), every compressed head follows a uniformly drawn full
    head and gets a budget drawn uniformly from ``budgets``.  ``ctx``: the sequences' lengths are these instead
    (the layers of one stack see the same batch; the roles are still drawn from ``seed``)."""
    g = _gen(seed, "cpu")
    u = torch.rand((B,), generator=g, dtype=torch.float64)
    if ctx is None:
        ctx = [int(round(math.exp(math.log(lo) + float(x) * (math.log(hi) - math.log(lo))))) for x in u]
    ctx = list(ctx)
    heads = []
    for b in range(B):
        full = sorted(torch.randperm(Hkv, generator=g)[:n_full].tolist())
        row = []
        for h in range(Hkv):
            if h in full:
                row.append(HeadSpec(ROLE_FULL))
            else:
                rep = full[int(torch.randint(0, n_full, (1,), generator=g).item())]
                l = budgets[int(torch.randint(0, len(budgets), (1,), generator=g).item())]
                row.append(HeadSpec(ROLE_SATELLITE, rep=rep, sink=sink, recent=recent, budget=min(l, ctx[b])))
        heads.append(row)
    return LayerSpec(B=B, Hq=Hq, Hkv=Hkv, D=128, ctx=ctx, heads=heads)


def layer_seed(config: int, layer: int) -> int:
    return 1000 * config + 10 * layer


@dataclass
class Workload:
    """One layer of one of the synthetic configs: description, tensors and query schedule."""
    spec: LayerSpec
    data: LayerData
    schedule: QuerySchedule
    steps: int


def make_workload(config: int, layer: int = 0, device: str = "cpu", N: Optional[int] = None,
                  scale: float = 1.0, steps: Optional[int] = None, **kw) -> Workload:
    """Build layer ``layer`` of synthetic config 1..5.  ``N`` overrides the context length and
    ``scale`` multiplies budgets (reduced copies for tests keep the recipe otherwise)."""
    seed = layer_seed(config, layer)
    if config == 1:
        spec = spec_tiny(N or CONFIG_CTX[1], **kw)
        q0 = draw_q(spec, seed, device)
        data = draw_layer(spec, q0, seed + 1, device, heavy_count=40)
        sched = QuerySchedule(q0, seed + 2, step_deg=5.0)
    elif config in (2, 3):
        budgets = [max(352, int(x * scale)) for x in CONFIG_BUDGETS[config]]
        spec = spec_llama(N or CONFIG_CTX[config], budgets)
        q0 = draw_q(spec, seed, device)
        data = draw_layer(spec, q0, seed + 1, device, heavy_frac=0.01)
        sched = QuerySchedule(q0, seed + 2, step_deg=5.0)
    elif config == 4:
        budgets = [max(352, int(x * scale)) for x in CONFIG_BUDGETS[4]]
        spec = spec_llama(N or CONFIG_CTX[4], budgets)
        q0 = draw_q(spec, seed, device)
        data = draw_layer(spec, q0, seed + 1, device, heavy_frac=0.005, segments=16)
        sched = QuerySchedule(q0, seed + 2, jump_every=16, jump_deg=kw.get("jump_deg", 15.0))
    elif config == 5:
        spec = spec_ragged(seed, B=kw.get("B", 16), lo=kw.get("lo", 8192), hi=kw.get("hi", 131072), ctx=kw.get("ctx"))
        q0 = draw_q(spec, seed, device)
        data = draw_layer(spec, q0, seed + 1, device, heavy_frac=0.01)
        sched = QuerySchedule(q0, seed + 2, jump_deg=15.0, jump_prob=1.0 / 16.0)
    else:
        raise ValueError(f"unknown config {config}")
    return Workload(spec, data, sched, steps or CONFIG_STEPS[config])


def initial_lists(spec: LayerSpec) -> Tuple[Dict[Tuple[int, int], torch.Tensor], Dict[Tuple[int, int], torch.Tensor]]:
    """Caller-supplied initial state: every compressed head's retrieved slots hold the first r
    candidate positions, and every representative's baseline set is the first k_mon candidates.
    (A positional fill; the first decode step then finds a low overlap and refills.)"""
    retrieved, base = {}, {}
    for b in range(spec.B):
        for h in range(spec.Hkv):
            hs = spec.heads[b][h]
            if hs.role != ROLE_FULL:
                retrieved[(b, h)] = torch.arange(hs.sink, hs.sink + spec.r(b, h), dtype=torch.int32)
        for p in spec.reps(b):
            lo, _ = spec.cand_range(b, p)
            base[(b, p)] = torch.arange(lo, lo + spec.k_mon(b, p), dtype=torch.int32)
    return retrieved, base
