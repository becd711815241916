"""Randomised layers through the whole path on the GPU against the oracle: roles, group sizes, ragged contexts,
sink / recent windows, budgets, window modes, metrics, prefill initialisation or positional fill, appended tokens.
Each case is small (the oracle takes milliseconds per step); together they reach shapes no hand-written case has."""
import os
import random

import pytest
import torch

from paper_2601_13684_amd import binding as hc
from paper_2601_13684_amd import inputs as I
from paper_2601_13684_amd import runtime as R

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def random_spec(rng: random.Random):
    B = rng.choice([1, 1, 2, 3])
    G = rng.choice([1, 2, 4, 4, 8])
    Hkv = rng.randint(2, 6)
    rows, ctx = [], []
    for b in range(B):
        N = rng.choice([rng.randint(150, 700), rng.randint(700, 6000)])
        ctx.append(N)
        n_full = rng.randint(1, max(1, Hkv // 2))
        full = sorted(rng.sample(range(Hkv), n_full))
        geometry = {p: (rng.choice([0, 1, 4, 16]), rng.choice([0, 1, 8, 24])) for p in full}     # shared by a pivot's satellites
        row = []
        for h in range(Hkv):
            if h in full:
                row.append(I.HeadSpec(I.ROLE_FULL))
                continue
            room = N - 64
            if rng.random() < 0.25:
                sink, recent = rng.choice([0, 2, 8]), rng.choice([0, 3, 8])
                row.append(I.HeadSpec(I.ROLE_ANCHOR, sink=sink, recent=recent,
                                      budget=sink + recent + rng.randint(0 if sink + recent else 1, min(200, room))))      # at least one resident row
            else:
                p = rng.choice(full)
                sink, recent = geometry[p]
                row.append(I.HeadSpec(I.ROLE_SATELLITE, rep=p, sink=sink, recent=recent,
                                      budget=sink + recent + rng.randint(1, min(300, room))))
        rows.append(row)
    spec = I.LayerSpec(B=B, Hq=Hkv * G, Hkv=Hkv, D=128, ctx=ctx, heads=rows,
                       metric=rng.choice([I.METRIC_OVERLAP, I.METRIC_JACCARD]), tau_num=rng.choice([1, 3, 4]), tau_den=5,
                       agg=rng.choice([I.AGG_PROB, I.AGG_PROB, I.AGG_LOGIT]))
    spec.window = rng.choice([1, 1, 2, 3, 4])
    spec.window_mode = rng.choice([0, 1, 2])
    return spec


@pytest.mark.parametrize("seed", list(range(int(os.environ.get("HC_RANDOM_CASES", "16")))))      # more cases on request
def test_random_layer(seed):
    import gpu_util as U
    import test_gpu_parity as T
    rng = random.Random(1000 + seed)
    spec = random_spec(rng)
    steps = rng.randint(5, 9) if not os.environ.get("HC_RANDOM_LONG") else rng.randint(60, 140)      # long runs cross plan rebalancings
    grow = rng.random() < 0.6
    use_prefill = rng.random() < 0.5
    side = torch.cuda.Stream() if rng.random() < 0.5 else None
    step_api = rng.random() < 0.4           # the layer's steps go through hc_decode_step instead of the three calls
    T.say(f"random layer {seed}: B {spec.B} G {spec.G} Hkv {spec.Hkv} ctx {spec.ctx} W {spec.window} mode {spec.window_mode} "
          f"agg {spec.agg} grow {grow} prefill {use_prefill} side {side is not None} decode_step {step_api}")
    q0 = I.draw_q(spec, 5000 + seed)
    data = I.draw_layer(spec, q0, 6000 + seed, heavy_count=12)
    growth = steps + 1 if grow else 0
    if use_prefill:
        p, _ = U.Pair.from_prefill(spec, data, q0.to(torch.bfloat16), rng.choice([1, 3, 7]), DEV, growth=growth)
        assert p.slots_equal_oracle() and p.tier_equals_masters()
    else:
        p = U.Pair(spec, data, DEV, growth=growth)
    sched = I.QuerySchedule(q0, 7000 + seed, step_deg=rng.choice([3.0, 10.0, 30.0]))
    stepper = None
    if step_api:
        q_cur = torch.zeros((1, spec.B, spec.Hq, 128), dtype=torch.bfloat16, device=DEV)
        io = R.make_step_io([p.gpu], q_cur)

        def stepper(q):
            q_cur[0].copy_(q)
            hc.hc_decode_step(p.ctx.handle, io, 1, None, side, rng.choice([1, 8]))
    resyncs, _ = T.run_steps(p, sched, steps, side=side, tag=f"random {seed}", append_seed=8000 + 100 * seed if grow else None,
                             token_gain=lambda t: 25.0 if t % 3 == 1 else 0.0, stepper=stepper)
    assert resyncs <= 2
    if grow:
        assert [p.gpu.context(b) for b in range(spec.B)] == p.ref.ctx
    p.close()
