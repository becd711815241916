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


def random_spec(rng: random.Random, B=None, G=None, Hkv=None, common=None):
    B = B or rng.choice([1, 1, 2, 3])
    G = G or rng.choice([1, 2, 4, 4, 8])
    Hkv = Hkv or rng.randint(2, 6)
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
    common = common or dict(metric=rng.choice([I.METRIC_OVERLAP, I.METRIC_JACCARD]), tau_num=rng.choice([1, 3, 4]), tau_den=5,
                            agg=rng.choice([I.AGG_PROB, I.AGG_PROB, I.AGG_LOGIT]), window=rng.choice([1, 1, 2, 3, 4]),
                            window_mode=rng.choice([0, 1, 2]))
    return I.LayerSpec(B=B, Hq=Hkv * G, Hkv=Hkv, D=128, ctx=ctx, heads=rows, **common)


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
    margin = random.Random(77 + seed).choice([0.0, 1.25, 1.02, 4.0])      # the pivot-logit filter: off, usual, tight, loose
    T.say(f"random layer {seed}: B {spec.B} G {spec.G} Hkv {spec.Hkv} ctx {spec.ctx} W {spec.window} mode {spec.window_mode} "
          f"agg {spec.agg} grow {grow} prefill {use_prefill} side {side is not None} decode_step {step_api} filter {margin}")
    q0 = I.draw_q(spec, 5000 + seed)
    data = I.draw_layer(spec, q0, 6000 + seed, heavy_count=12)
    growth = steps + 1 if grow else 0
    if use_prefill:
        p, _ = U.Pair.from_prefill(spec, data, q0.to(torch.bfloat16), rng.choice([1, 3, 7]), DEV, growth=growth, filter_margin=margin)
        assert p.slots_equal_oracle() and p.tier_equals_masters()
    else:
        # a third of these run on "8 or 16 compute units": few, long shares per workgroup, i.e. the weighted and
        # cost-charged split of the long passes, and rebalanced plans, at sizes the oracle still likes
        ctx = None
        if rng.random() < 0.35:
            ctx = R.Context(R.make_config(spec, growth=growth), DEV, filter_margin=margin)
            hc.hc_set_split(ctx.handle, 2, rng.choice([8, 16]))
        p = U.Pair(spec, data, DEV, ctx=ctx, growth=growth, filter_margin=margin)
        p.own_ctx = True
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
    assert resyncs <= 2, (resyncs, U.NEAR_TIES[-4:])
    if grow:
        assert [p.gpu.context(b) for b in range(spec.B)] == p.ref.ctx
    p.close()


@pytest.mark.parametrize("seed", list(range(int(os.environ.get("HC_RANDOM_STACKS", "6")))))
def test_random_stack_through_the_decode_step(seed):
    """2-9 layers that differ in everything a layer may differ in (roles, budgets, windows of recent positions) through
    hc_decode_step: batched monitor, gather and window re-scoring over unlike layers, appended tokens, random group size."""
    import gpu_util as U
    import test_gpu_parity as T
    rng = random.Random(3000 + seed)
    first = random_spec(rng)
    common = dict(metric=first.metric, tau_num=first.tau_num, tau_den=first.tau_den, agg=first.agg, window=first.window,
                  window_mode=first.window_mode)
    n_layers = rng.randint(2, 9)
    specs = [first] + [random_spec(rng, first.B, first.G, first.Hkv, common) for _ in range(n_layers - 1)]
    for sp in specs[1:]:
        sp.ctx = list(first.ctx)                # one batch: the sequences have the same lengths in every layer
        for b in range(sp.B):                   # ... so budgets drawn for another length are cut to fit
            sp.heads[b] = [h if h.role == I.ROLE_FULL else
                           I.HeadSpec(h.role, rep=h.rep, sink=min(h.sink, 4), recent=min(h.recent, 8),
                                      budget=min(h.sink, 4) + min(h.recent, 8) + max(1, min(h.budget - h.sink - h.recent, sp.ctx[b] - 64)))
                           for h in sp.heads[b]]
            for p in sp.reps(b):                # satellites of one pivot share sink and recent
                sats = sp.satellites(b, p)
                s0 = sp.heads[b][sats[0]]
                for si in sats[1:]:
                    h = sp.heads[b][si]
                    sp.heads[b][si] = I.HeadSpec(h.role, rep=h.rep, sink=s0.sink, recent=s0.recent,
                                                 budget=s0.sink + s0.recent + (h.budget - h.sink - h.recent))
    steps = rng.randint(5, 8)
    grow = rng.random() < 0.6
    growth = steps + 1 if grow else 0
    group = rng.choice([1, 2, 4, 8])
    side = torch.cuda.Stream() if rng.random() < 0.7 else None
    T.say(f"random stack {seed}: {n_layers} layers, B {first.B} G {first.G} Hkv {first.Hkv} ctx {first.ctx} W {first.window} "
          f"mode {first.window_mode} grow {grow} group {group} side {side is not None}")
    cfg = R.make_config(first, growth=growth, max_k=max(R.make_config(sp, growth=growth).max_k for sp in specs))
    ctx = R.Context(cfg, DEV, filter_margin=random.Random(99 + seed).choice([0.0, 1.25, 1.02]))
    pairs, scheds = [], []
    for l, sp in enumerate(specs):
        q0 = I.draw_q(sp, 3100 + 10 * seed + l)
        data = I.draw_layer(sp, q0, 3200 + 10 * seed + l, heavy_count=10)
        pr = U.Pair(sp, data, DEV, ctx=ctx, growth=growth)
        pr.gpu.rep_logits = torch.zeros_like(pr.gpu.rep_logits)      # own buffers: the layers' monitors run together
        pr.gpu.scores = torch.zeros_like(pr.gpu.scores)
        pairs.append(pr)
        scheds.append(I.QuerySchedule(q0, 3300 + 10 * seed + l, step_deg=rng.choice([5.0, 20.0])))
    B, Hq, Hkv = first.B, first.Hq, first.Hkv
    q_cur = torch.zeros((n_layers, B, Hq, 128), dtype=torch.bfloat16, device=DEV)
    k_cur = torch.zeros((n_layers, B, Hkv, 128), dtype=torch.bfloat16, device=DEV)
    v_cur = torch.zeros_like(k_cur)
    io = R.make_step_io([pr.gpu for pr in pairs], q_cur)
    if grow:
        for l in range(n_layers):
            io[l].k_new, io[l].v_new = k_cur[l].data_ptr(), v_cur[l].data_ptr()
    for t in range(steps):
        qs = [s.next() for s in scheds]
        torch.cuda.synchronize()
        for l in range(n_layers):
            q_cur[l].copy_(qs[l])
            if grow:
                kn, vn = I.draw_token(specs[l], 3400 + 100 * seed + 10 * t + l, toward=qs[l], gain=25.0 if t % 3 == 1 else 0.0)
                k_cur[l].copy_(kn)
                v_cur[l].copy_(vn)
                pairs[l].ref.append(kn, vn)
        hc.hc_decode_step(ctx.handle, io, n_layers, None, side, group)
        torch.cuda.synchronize()
        for l, pr in enumerate(pairs):
            sp = specs[l]
            rec = pr.ref.step(qs[l])
            U.check_attention(pr.gpu.out, pr.gpu.lse, rec, f"stack {seed} L{l} t{t}")
            same = True
            topk = pr.gpu.topk_idx.cpu().numpy()
            for (b, pv), s_ref in rec["scores"].items():
                lo, hi = pr.ref.cand_range(b, pv)
                dabs, _ = U.check_gpu_scores(pr.gpu, b, pv, s_ref, lo, hi, f"stack {seed} L{l} t{t}")
                for h in [pv] + sp.satellites(b, pv):
                    Tl = rec["topk"][(b, h)]
                    if U.check_set_valid(topk[b * Hkv + h, :Tl.size], Tl, s_ref, U.band_of(dabs), f"stack {seed} L{l} t{t} head {h}"):
                        same = False
                if (b, pv) in rec["rescored"]:
                    same &= T.check_rescored(pr, rec, b, pv, f"stack {seed} L{l} t{t}")
                gi, gf = int(pr.gpu.inter[b * Hkv + pv]), int(pr.gpu.flag[b * Hkv + pv])
                if gi != rec["inter"][(b, pv)] or gf != rec["flag"][(b, pv)]:
                    assert not same, (seed, l, t, "same sets but different inter / flag")
                    same = False
            if not same:
                T.resync(pr, rec)
            assert pr.slots_equal_oracle(), f"stack {seed}: slots differ, layer {l} step {t}"
    for pr in pairs:
        pr.close()
    ctx.close()
