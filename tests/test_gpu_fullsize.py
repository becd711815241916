"""GPU parity at the full sizes of the synthetic configs that test_gpu_parity.py covers only reduced: config 2
(32K context, many steps), config 3 (128K context, budgets doubled, a stack of layers), config 5 (16 ragged
sequences of 8K-128K tokens, roles drawn per sequence) and the uncompressed 224K layer that config 4 is compared
with.  Everything goes through the C ABI in the launch configuration bench.py times (hc_decode_step, groups of 8
layers, monitor and gather batched on a side stream) and is compared with the CPU oracle element by element:
attention outputs and lse, the pivots' scores, every index list (bit-exact except for near-ties shown to lie
inside the band of gpu_util.band_of), overlaps, flags, and byte for byte the K/V rows the refills left in HBM.
Run with `-m gpu` on an MI355X."""
import numpy as np
import pytest
import torch

from paper_2601_13684_amd import binding as hc
from paper_2601_13684_amd import inputs as I
from paper_2601_13684_amd import runtime as R

import gpu_util as U
import test_gpu_parity as T

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
say = T.say


def run_stack(ws, steps, group, tag, max_k=None, filter_margin=0.0, side_lds=0):
    """The layers of `ws` as one stack through hc_decode_step with a side stream; every layer and step against
    its oracle twin.  Returns (triggers per step, re-synchronisations, steps at which some set differed)."""
    cfg = R.make_config(ws[0].spec)
    if max_k:
        cfg.max_k = max_k
    ctx = R.Context(cfg, DEV, filter_margin=filter_margin)
    hc.hc_set_side_lds(ctx.handle, side_lds)
    pairs = [U.Pair(w.spec, w.data, DEV, ctx=ctx) for w in ws]
    for p in pairs:                                                    # own buffers: the layers' monitors run together
        p.gpu.rep_logits = torch.zeros_like(p.gpu.rep_logits)
        p.gpu.scores = torch.zeros_like(p.gpu.scores)
    sp0 = ws[0].spec
    q_cur = torch.zeros((len(ws), sp0.B, sp0.Hq, 128), dtype=torch.bfloat16, device=DEV)
    io = R.make_step_io([p.gpu for p in pairs], q_cur)
    side = torch.cuda.Stream()
    ties_before = len(U.NEAR_TIES)
    trig_per_step, resyncs = [], 0
    for t in range(steps):
        qs = [w.schedule.next() for w in ws]
        q_cur.copy_(torch.stack([q.to(DEV) for q in qs]))
        hc.hc_decode_step(ctx.handle, io, len(ws), None, side, group)
        torch.cuda.synchronize()
        trig = 0
        for l, (p, w) in enumerate(zip(pairs, ws)):
            sp = w.spec
            rec = p.ref.step(qs[l].cpu())
            worst, lerr = U.check_attention(p.gpu.out, p.gpu.lse, rec, f"{tag} L{l} step {t}")
            topk = p.gpu.topk_idx.cpu().numpy()
            same = True
            worst_s = 0.0
            for (b, pv), s_ref in rec["scores"].items():
                lo, hi = p.ref.cand_range(b, pv)
                dabs, drel = U.check_gpu_scores(p.gpu, b, pv, s_ref, lo, hi, f"{tag} L{l} step {t}")
                worst_s = max(worst_s, drel)
                for h in [pv] + sp.satellites(b, pv):
                    Tl = rec["topk"][(b, h)]
                    if U.check_set_valid(topk[b * sp.Hkv + h, :Tl.size], Tl, s_ref, U.band_of(dabs), f"{tag} L{l} step {t} head {(b, h)}"):
                        same = False
                gi, gf = int(p.gpu.inter[b * sp.Hkv + pv]), int(p.gpu.flag[b * sp.Hkv + pv])
                if gi != rec["inter"][(b, pv)] or gf != rec["flag"][(b, pv)]:
                    assert not same, (tag, l, t, "same sets but different overlap / flag", gi, rec["inter"][(b, pv)], gf, rec["flag"][(b, pv)])
                    same = False
                trig += rec["flag"][(b, pv)]
            if not same:
                resyncs += 1
                T.resync(p, rec)
            assert p.slots_equal_oracle(), f"{tag}: slots differ, layer {l} step {t}"
            say(f"  {tag} L{l} step {t}: err/rms {worst:.2e} lse {lerr:.1e} score rel err {worst_s:.1e} "
                f"triggers {sum(rec['flag'].values())}/{len(rec['flag'])} sets {'equal' if same else 'NEAR-TIE'}")
        trig_per_step.append(trig)
    ties = U.NEAR_TIES[ties_before:]
    assert resyncs <= len(ties), (tag, f"{resyncs} re-synchronisations but {len(ties)} near-ties logged")
    # the monitor's own counters (tests, triggers, filter fall-backs) summed over the stack, for the caller
    run_stack.counts = {k: sum(p.gpu.monitor_counts(b, pv)[k] for p in pairs for b in range(p.spec.B) for pv in p.spec.reps(b))
                        for k in ("tests", "triggers", "fallbacks")}
    for p in pairs:
        p.close()
    ctx.close()
    return trig_per_step, resyncs, ties


def test_config2_full_size_ten_steps():
    """32768 tokens, the stated budgets, every query head rotated by 5 degrees per step: the monitor fires every few
    steps (the bivariate-normal pin of the oracle says every 3-4), and every refill is checked row by row."""
    say("config 2 full size: 32K context, 10 steps")
    w = I.make_workload(2, device=DEV)
    assert w.spec.ctx == [32768] and [w.spec.heads[0][h].budget for h in range(2, 8)] == [4096, 2048, 2048, 1024, 1024, 512]
    trig, resyncs, ties = run_stack([w], 10, 8, "cfg2")
    say("  triggers per step", trig, "re-synchronisations", resyncs)
    assert trig[0] == 2                                  # the positional initial fill is replaced at once
    assert sum(trig[1:]) >= 4, trig                      # each pivot fires at least twice more in nine steps
    assert resyncs <= 1, (resyncs, ties)


@pytest.mark.parametrize("margin", [0.0, 1.25])
def test_config3_full_size_two_layers_five_steps(margin):
    """131072 tokens, budgets doubled (8192 ... 1024), two layers with independent seeds through one
    hc_decode_step, five steps that span the initial refill and at least one drift trigger; without and with the
    pivot-logit filter (bench.py runs this config with it)."""
    say("config 3 full size: 128K context, budgets x2, 2 layers, 5 steps, filter margin", margin)
    ws = [I.make_workload(3, layer=l, device=DEV) for l in range(2)]
    assert ws[0].spec.ctx == [131072] and [ws[0].spec.heads[0][h].budget for h in range(2, 8)] == [8192, 4096, 4096, 2048, 2048, 1024]
    trig, resyncs, ties = run_stack(ws, 5, 1, "cfg3", filter_margin=margin)              # two groups: the side stream is in use
    say("  triggers per step", trig, "re-synchronisations", resyncs)
    assert trig[0] == 4 and sum(trig[1:]) >= 2, trig
    assert resyncs <= 1, (resyncs, ties)


def test_config4_full_size_across_a_query_jump():
    """229376 tokens, two layers, 18 steps with the pivot-logit filter as bench.py runs it: the initial refill, fifteen
    quiet steps, and the step at which every query jumps by 15 degrees (every pivot fires, a quarter of every list
    is replaced, the filter's cut of the step before no longer fits the scores), then the step that attends over
    the refilled slots."""
    say("config 4 full size: 224K context, 2 layers, 18 steps across the jump at step 16")
    ws = [I.make_workload(4, layer=l, device=DEV) for l in range(2)]
    assert ws[0].spec.ctx == [229376]
    trig, resyncs, ties = run_stack(ws, 18, 1, "cfg4", filter_margin=1.25, side_lds=81 * 1024)      # as bench.py runs this config
    say("  triggers per step", trig, "re-synchronisations", resyncs, "counters", run_stack.counts)
    assert trig[0] == 4 and trig[16] == 4 and sum(trig) == 8, trig
    assert run_stack.counts["tests"] == 4 * 18 and run_stack.counts["triggers"] == 8
    assert run_stack.counts["fallbacks"] <= 4, run_stack.counts          # at most the jump step itself goes the long way
    assert resyncs <= 1, (resyncs, ties)


@pytest.mark.parametrize("margin", [0.0, 1.25])
def test_config5_full_size_batch_of_16(margin):
    """16 sequences of 8192 ... 131072 tokens, two of eight KV heads full per sequence, budgets from
    {512, ..., 4096}, every sequence with its own jump events: 128 ragged head rows in one split pass (the long-pass
    plan: weighted shares, boundary costs), 32 pivots in one monitor call, refills of single sequences; without and with
    the pivot-logit filter (lists of up to a third of a short sequence's positions)."""
    say("config 5 full size: B = 16, 2 layers, 4 steps, filter margin", margin)
    w = I.make_workload(5, device=DEV)
    sp = w.spec
    say("  contexts", sp.ctx)
    assert sp.B == 16 and min(sp.ctx) >= 8192 and max(sp.ctx) <= 131072
    w1 = I.make_workload(5, layer=1, device=DEV, ctx=sp.ctx)        # the same batch, the roles drawn again for the second layer
    assert w1.spec.ctx == sp.ctx and w1.spec.heads != sp.heads
    trig, resyncs, ties = run_stack([w, w1], 4, 1, "cfg5", max_k=4096 - 64 - 256, filter_margin=margin,
                                    side_lds=81 * 1024 if margin else 0)
    n_piv = sum(len(x.spec.reps(b)) for x in (w, w1) for b in range(sp.B))
    say("  pivots", n_piv, "triggers per step", trig, "re-synchronisations", resyncs)
    assert trig[0] == n_piv                              # initial fill replaced
    assert 0 < sum(trig[1:]) < 3 * n_piv, trig           # some sequences jumped and refilled, not all of them every step
    assert resyncs <= 2, (resyncs, ties)


def test_dense_224k_layer_against_the_oracle():
    """The uncompressed comparison of config 4: all eight KV heads hold 229376 tokens (939.5 MB per layer), through
    the same split and combine kernels."""
    say("dense 224K layer, 1 step")
    w = I.make_workload(4, device=DEV)
    spec = I.spec_dense(229376)
    ctx = R.Context(R.make_config(spec), DEV)
    p = U.Pair(spec, w.data, DEV, ctx=ctx, host_tier=False)
    assert hc.hc_layer_num_workgroups(p.gpu.handle) == 512 and hc.hc_layer_num_reps(p.gpu.handle) == 0
    q_cur = torch.zeros((1, 1, 32, 128), dtype=torch.bfloat16, device=DEV)
    io = R.make_step_io([p.gpu], q_cur)
    for t in range(2):
        q = w.schedule.next()
        q_cur[0].copy_(q.to(DEV))
        hc.hc_decode_step(ctx.handle, io, 1, None, torch.cuda.Stream(), 8)
        torch.cuda.synchronize()
        rec = p.ref.step(q.cpu(), monitor=False)
        worst, lerr = U.check_attention(p.gpu.out, p.gpu.lse, rec, f"dense step {t}")
        say(f"  step {t}: err/rms {worst:.2e} lse {lerr:.1e} partials {hc.hc_layer_num_partials(p.gpu.handle)}")
    p.close()
    ctx.close()
