"""GPU parity with the pivot-logit filter on (hc_set_logit_filter): the split pass stores only the rows of a pivot's
logits that can reach a list, the monitor selects among them, checks on the device that no dropped row could have
mattered, and otherwise redoes the pivot from all of its logits.  Whatever path a step takes, lists, overlaps, flags
and refilled rows must be those of the oracle (which knows nothing of any filter).  Run with `-m gpu`."""
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


def counts(p):
    sp = p.spec
    return {(b, pv): p.gpu.monitor_counts(b, pv) for b in range(sp.B) for pv in sp.reps(b)}


@pytest.mark.parametrize("margin", [1.25, 1.0, 8.0])
def test_filtered_tiny_config_multi_step(margin):
    say("filter, config 1, 12 steps, margin", margin)
    w = I.make_workload(1)
    p = U.Pair(w.spec, w.data, DEV, filter_margin=margin)
    resyncs, triggers = T.run_steps(p, w.schedule, 12, side=torch.cuda.Stream(), tag=f"filter {margin}")
    c = counts(p)[(0, 0)]
    lo, hi = p.ref.cand_range(0, 0)
    say("  counters", c, "candidates", hi - lo, "triggers", triggers, "resyncs", resyncs)
    assert c["tests"] == 12 and c["triggers"] == triggers >= 2
    assert resyncs <= 1, (resyncs, U.NEAR_TIES[-4:])
    if margin == 1.25:
        assert c["fallbacks"] == 0 and c["kept"] is not None and 320 <= c["kept"] < (hi - lo) // 2
    if margin == 8.0:
        assert c["fallbacks"] == 0 and c["kept"] is not None
    p.close()


def test_filter_first_step_keeps_every_candidate():
    say("filter, first step")
    w = I.make_workload(1)
    p = U.Pair(w.spec, w.data, DEV, filter_margin=1.25)
    T.run_steps(p, w.schedule, 1, tag="filter first")
    lo, hi = p.ref.cand_range(0, 0)
    c = counts(p)[(0, 0)]
    assert c["kept"] == hi - lo and c["fallbacks"] == 0
    pos, _ = p.gpu.kept_rows(0, 0)
    assert np.array_equal(pos.cpu().numpy(), np.arange(lo, hi))
    p.close()


@pytest.mark.parametrize("how", ["all_heads_flat", "one_head_flat", "sharper"])
def test_filter_falls_back_when_the_query_changes_abruptly(how):
    """After a few ordinary steps the query is rescaled: flatter attention (every head, or one head of every
    group: the check's bound takes the worst head) makes the previous step's cut too high, so too few rows are
    kept or the check fails, and the dense passes must take over for that step; a sharper query only keeps
    more rows.  The results stay exact either way, and filtering resumes at the next step."""
    say("filter, abrupt change:", how)
    w = I.make_workload(2, N=16384, scale=0.5)
    p = U.Pair(w.spec, w.data, DEV, filter_margin=1.25)
    sched = w.schedule
    T.run_steps(p, sched, 3, side=torch.cuda.Stream(), tag="before")
    before = counts(p)
    assert all(c["fallbacks"] == 0 for c in before.values())
    if how == "all_heads_flat":
        sched.q *= 0.5
    elif how == "one_head_flat":
        sched.q[:, ::4] *= 0.4
    else:
        sched.q *= 1.5
    T.run_steps(p, sched, 1, side=torch.cuda.Stream(), tag="change")
    at = counts(p)
    say("  counters at the change", at)
    if how == "sharper":
        assert all(c["fallbacks"] == 0 for c in at.values())
    else:
        assert sum(c["fallbacks"] for c in at.values()) >= 1 and all((c["kept"] is None) == (c["fallbacks"] == 1) for c in at.values())
    T.run_steps(p, sched, 3, side=torch.cuda.Stream(), tag="after")
    after = counts(p)
    say("  counters after", after)
    assert all(after[k]["fallbacks"] == at[k]["fallbacks"] and after[k]["kept"] is not None for k in after)
    assert all(c["tests"] == 7 for c in after.values())
    p.close()


@pytest.mark.parametrize("G", [1, 2, 8])
def test_filter_other_group_sizes(G):
    say("filter, group size", G)
    heads = [I.HeadSpec(I.ROLE_FULL), I.HeadSpec(I.ROLE_SATELLITE, rep=0, sink=8, recent=40, budget=8 + 40 + 300),
             I.HeadSpec(I.ROLE_FULL), I.HeadSpec(I.ROLE_SATELLITE, rep=2, sink=8, recent=40, budget=8 + 40 + 77),
             I.HeadSpec(I.ROLE_SATELLITE, rep=2, sink=8, recent=40, budget=8 + 40 + 513)]
    spec = I.LayerSpec(B=2, Hq=5 * G, Hkv=5, D=128, ctx=[9001, 5003], heads=[heads, heads])
    q0 = I.draw_q(spec, 300 + G)
    data = I.draw_layer(spec, q0, 400 + G, heavy_count=30)
    sched = I.QuerySchedule(q0, 500 + G, step_deg=6.0)
    p = U.Pair(spec, data, DEV, filter_margin=1.25)
    resyncs, triggers = T.run_steps(p, sched, 8, side=torch.cuda.Stream(), tag=f"filter G={G}")
    c = counts(p)
    say("  counters", c)
    assert all(v["tests"] == 8 for v in c.values()) and triggers >= 4
    assert sum(v["fallbacks"] for v in c.values()) <= 2
    assert resyncs <= 1, (resyncs, U.NEAR_TIES[-4:])
    p.close()


@pytest.mark.parametrize("mode,W", [(0, 3), (1, 2)])
def test_filter_with_a_window(mode, W):
    say("filter, window", W, "tumbling" if mode else "sliding")
    w = I.make_workload(1)
    w.spec.window, w.spec.window_mode = W, mode
    p = U.Pair(w.spec, w.data, DEV, filter_margin=1.25)
    resyncs, triggers = T.run_steps(p, w.schedule, 12, tag=f"filter W{W}")
    assert triggers >= 1 and resyncs <= 1, (resyncs, U.NEAR_TIES[-4:])
    assert counts(p)[(0, 0)]["tests"] == p.ref.n_tests
    p.close()


def test_filter_with_a_growing_context():
    """70 appended tokens (the recent ring wraps, the plan is rebalanced once, the candidate range grows, planted
    tokens are retrieved after they have left the window), filter on."""
    say("filter, growing context, 70 steps")
    spec = I.spec_tiny(4096, budget=512, sink=16, recent=32)
    q0 = I.draw_q(spec, 71)
    data = I.draw_layer(spec, q0, 72, heavy_count=40)
    sched = I.QuerySchedule(q0, 73, step_deg=5.0)
    p = U.Pair(spec, data, DEV, growth=96, filter_margin=1.25)
    resyncs, triggers = T.run_steps(p, sched, 70, side=torch.cuda.Stream(), tag="filter grow", append_seed=7000,
                                    token_gain=lambda t: 40.0 if t % 9 == 4 else 0.0)
    c = counts(p)[(0, 0)]
    say("  counters", c, "resyncs", resyncs)
    assert p.gpu.context(0) == 4096 + 70 == p.ref.ctx[0]
    assert triggers >= 3 and resyncs <= 2, (resyncs, U.NEAR_TIES[-4:])
    planted = [4096 + t for t in range(70) if t % 9 == 4 and t < 70 - 34]
    assert all(pos in set(p.ref.retrieved[(0, 1)].tolist()) for pos in planted)
    p.close()


@pytest.mark.parametrize("n_layers,group,side_lds", [(5, 2, 0), (10, 8, 0), (5, 2, 81 * 1024), (10, 4, 100 * 1024)])
def test_filter_through_the_decode_step(n_layers, group, side_lds):
    """A stack of layers through hc_decode_step with the filter on: the filtered and the stand-by dense chains are
    batched over the layers of a group.  Also with the side stream's workgroups reserving most of a compute unit's LDS
    (hc_set_side_lds), which changes where and when they run, never what they compute."""
    say(f"filter, hc_decode_step, {n_layers} layers, groups of {group}, side LDS {side_lds}")
    ws = [I.make_workload(2, layer=l, N=8192, scale=0.25) for l in range(n_layers)]
    ctx = R.Context(R.make_config(ws[0].spec), DEV, filter_margin=1.25)
    hc.hc_set_side_lds(ctx.handle, side_lds)
    pairs = [U.Pair(w.spec, w.data, DEV, ctx=ctx) for w in ws]
    for p in pairs:
        p.gpu.rep_logits = torch.zeros_like(p.gpu.rep_logits)
        p.gpu.scores = torch.zeros_like(p.gpu.scores)
    q_cur = torch.zeros((n_layers, 1, 32, 128), dtype=torch.bfloat16, device=DEV)
    io = R.make_step_io([p.gpu for p in pairs], q_cur)
    side = torch.cuda.Stream()
    triggers = 0
    for t in range(6):
        qs = [w.schedule.next() for w in ws]
        if t == 4:
            qs[1] = (qs[1].float() * 0.5).to(torch.bfloat16)          # layer 1 alone has to fall back at this step
        q_cur.copy_(torch.stack(qs).to(DEV))
        hc.hc_decode_step(ctx.handle, io, n_layers, None, side, group)
        torch.cuda.synchronize()
        for l, (p, w) in enumerate(zip(pairs, ws)):
            rec = p.ref.step(qs[l])
            U.check_attention(p.gpu.out, p.gpu.lse, rec, f"step {t} layer {l}")
            topk = p.gpu.topk_idx.cpu().numpy()
            for (b, pv), s_ref in rec["scores"].items():
                lo, hi = p.ref.cand_range(b, pv)
                dabs, _ = U.check_gpu_scores(p.gpu, b, pv, s_ref, lo, hi, f"step {t} layer {l}")
                for h in [pv] + w.spec.satellites(b, pv):
                    Tl = rec["topk"][(b, h)]
                    assert U.check_set_valid(topk[b * 8 + h, :Tl.size], Tl, s_ref, U.band_of(dabs), f"step {t} layer {l} head {h}") == 0
                assert int(p.gpu.flag[pv]) == rec["flag"][(b, pv)] and int(p.gpu.inter[pv]) == rec["inter"][(b, pv)]
                triggers += rec["flag"][(b, pv)]
            assert p.slots_equal_oracle(), f"slots differ at step {t} layer {l}"
    fb = [sum(c["fallbacks"] for c in counts(p).values()) for p in pairs]
    say("  triggers", triggers, "fallbacks per layer", fb)
    assert fb[1] >= 2 and sum(fb) == fb[1]
    for p in pairs:
        p.close()
    ctx.close()


def test_side_lds_argument_range():
    ctx = R.Context(R.make_config(I.make_workload(1).spec), DEV)
    for ok in (0, 80 * 1024 + 1, 81 * 1024, 100 * 1024):
        hc.hc_set_side_lds(ctx.handle, ok)
    for bad in (-1, 1024, 80 * 1024, 100 * 1024 + 1):
        with pytest.raises(hc.HcError):
            hc.hc_set_side_lds(ctx.handle, bad)
    ctx.close()
