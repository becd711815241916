"""Pins of the oracle's score aggregation (App. C.1), TopIndices_k (Algorithm 1), overlap
(Eq. 1 / Eq. 9), windowed-median trigger (Eq. 10) and of the per-step state machine
(Algorithm 1, stage 3).  CPU only."""
import math
import os

import numpy as np
import pytest
import torch
from scipy.stats import multivariate_normal, norm

from oracle import ref
from paper_2601_13684_amd import inputs as I

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- A5 scores
def test_scores_are_group_mean_of_softmax_weights():
    rng = np.random.default_rng(0)
    logits = rng.normal(size=(4, 300))
    lse = np.log(np.exp(logits).sum(1))
    s = ref.scores(logits, lse, agg=0)
    want = torch.softmax(torch.from_numpy(logits), dim=1).mean(0).numpy()     # library softmax
    np.testing.assert_allclose(s, want, rtol=1e-12, atol=1e-16)
    assert abs(s.sum() - 1) < 1e-12


def test_single_head_group_ranks_like_its_logits():
    rng = np.random.default_rng(1)
    logits = rng.normal(size=(1, 500))
    lse = np.log(np.exp(logits).sum(1))
    s = ref.scores(logits, lse, agg=0)
    np.testing.assert_array_equal(np.argsort(-s, kind="stable"), np.argsort(-logits[0], kind="stable"))
    s1 = ref.scores(logits, lse, agg=1)
    np.testing.assert_allclose(s1, logits[0], rtol=0, atol=0)


# ---------------------------------------------------------------- A6 top-k
@pytest.mark.parametrize("seed,N,lo,hi,k", [(0, 1000, 0, 1000, 100), (1, 1000, 64, 872, 320), (2, 50, 3, 47, 44),
                                            (3, 4096, 64, 3968, 1), (4, 777, 10, 700, 690)])
def test_topk_equals_stable_argsort(seed, N, lo, hi, k):
    rng = np.random.default_rng(seed)
    s = rng.random(N).astype(np.float32)
    s[rng.integers(0, N, N // 3)] = s[rng.integers(0, N, N // 3)]        # plant exact ties
    got = ref.topk(s, lo, hi, k)
    order = np.argsort(-s[lo:hi], kind="stable")[:k] + lo                  # ties -> lowest index
    np.testing.assert_array_equal(got, np.sort(order).astype(np.int32))


def test_topk_k_equals_candidates_returns_all():
    s = np.random.default_rng(5).random(300).astype(np.float32)
    np.testing.assert_array_equal(ref.topk(s, 20, 280, 260), np.arange(20, 280, dtype=np.int32))


def test_topk_k1_is_argmax_lowest_index_on_ties():
    s = np.zeros(100, np.float32)
    s[[40, 17, 93]] = 2.5
    assert ref.topk(s, 0, 100, 1).tolist() == [17]
    assert ref.topk(s, 18, 100, 1).tolist() == [40]


def test_topk_all_equal_takes_lowest_indices_and_signed_zero_ties():
    s = np.full(64, 0.25, np.float32)
    assert ref.topk(s, 5, 60, 7).tolist() == list(range(5, 12))
    z = np.zeros(10, np.float32)
    z[::2] = -0.0                                            # -0 and +0 are the same score
    assert ref.topk(z, 0, 10, 4).tolist() == [0, 1, 2, 3]


def test_topk_sets_are_nested():
    s = np.random.default_rng(6).random(2000).astype(np.float32)
    s[::7] = 0.5
    prev = set()
    for k in (1, 10, 192, 704, 1728):
        cur = set(ref.topk(s, 64, 1900, k).tolist())
        assert prev <= cur and len(cur) == k
        prev = cur


def test_topk_rejects_nan_and_bad_k():
    s = np.ones(10, np.float32)
    with pytest.raises(ValueError):
        ref.topk(s, 0, 10, 11)
    s[3] = np.nan
    with pytest.raises(ValueError):
        ref.topk(s, 0, 10, 2)


# ---------------------------------------------------------------- A7 overlap + trigger
def test_intersection_matches_python_sets():
    rng = np.random.default_rng(7)
    for _ in range(20):
        a = rng.choice(500, 120, replace=False).astype(np.int32)
        b = rng.choice(500, 120, replace=False).astype(np.int32)
        assert ref.intersect(a, b) == len(set(a.tolist()) & set(b.tolist()))
    assert ref.intersect(a, a) == 120
    assert ref.intersect(np.arange(10, dtype=np.int32), np.arange(10, 20, dtype=np.int32)) == 0
    assert ref.intersect(np.full(5, -1, np.int32), np.full(5, -1, np.int32)) == 0     # empty baseline


def test_hand_derived_integer_thresholds():
    rows = [tuple(int(x) for x in l.split()) for l in open(os.path.join(GOLD, "drift_thresholds.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 10
    for k, num, den, metric, max_trig in rows:
        assert ref.trigger([max_trig], k, metric, num, den) == 1
        assert ref.trigger([max_trig + 1], k, metric, num, den) == 0
        assert ref.trigger([0], k, metric, num, den) == 1
        assert ref.trigger([k], k, metric, num, den) == 0           # identical sets never trigger


def test_trigger_agrees_with_real_valued_definitions():
    for k in (7, 64, 320):
        for inter in range(k + 1):
            o = inter / k
            j = inter / (2 * k - inter)
            assert j == pytest.approx(o / (2 - o))
            for num, den in ((4, 5), (1, 2), (2, 3)):
                # exact rational comparison through fractions, not floats
                from fractions import Fraction
                assert ref.trigger([inter], k, 0, num, den) == int(Fraction(inter, k) < Fraction(num, den))
                assert ref.trigger([inter], k, 1, num, den) == int(Fraction(inter, 2 * k - inter) < Fraction(num, den))


@pytest.mark.parametrize("W", [1, 2, 3, 4, 5, 8])
def test_window_median_is_lower_median(W):
    rng = np.random.default_rng(W)
    for _ in range(30):
        w = rng.integers(0, 101, W).astype(np.int32)
        med = int(torch.median(torch.from_numpy(w)).item())      # library: lower middle
        assert ref.trigger(w, 100, 0, 1, 2) == int(med * 2 < 100)


# ---------------------------------------------------------------- state machine (Algorithm 1, stage 3)
def small_workload(seed=0, N=1024, budget=160, sink=16, recent=32, anchors=False):
    heads = [I.HeadSpec(I.ROLE_FULL), I.HeadSpec(I.ROLE_SATELLITE, rep=0, sink=sink, recent=recent, budget=budget)]
    if anchors:
        heads.append(I.HeadSpec(I.ROLE_ANCHOR, sink=sink, recent=recent, budget=budget))
        heads.append(I.HeadSpec(I.ROLE_SATELLITE, rep=0, sink=sink, recent=recent, budget=budget // 2 + sink + recent))
    spec = I.LayerSpec(B=1, Hq=4 * len(heads), Hkv=len(heads), D=128, ctx=[N], heads=[heads])
    q0 = I.draw_q(spec, seed)
    data = I.draw_layer(spec, q0, seed + 1, heavy_count=10)
    return spec, q0, data


def test_step_equals_dense_when_budgets_cover_context():
    N = 256
    heads = [I.HeadSpec(I.ROLE_FULL), I.HeadSpec(I.ROLE_ANCHOR, sink=0, recent=0, budget=N)]
    spec = I.LayerSpec(B=1, Hq=8, Hkv=2, D=128, ctx=[N], heads=[heads])
    q0 = I.draw_q(spec, 3)
    data = I.draw_layer(spec, q0, 4)
    layer = ref.RefLayer(spec, data, {(0, 1): torch.arange(N, dtype=torch.int32)}, {})
    q = q0.to(torch.bfloat16)
    rec = layer.step(q)
    import torch.nn.functional as F
    for h in range(2):
        o = F.scaled_dot_product_attention(q[0, 4 * h:4 * h + 4].double()[None, :, None, :],
                                           data.K[(0, h)].double()[None, None].expand(1, 4, -1, -1),
                                           data.V[(0, h)].double()[None, None].expand(1, 4, -1, -1))[0, :, 0]
        np.testing.assert_allclose(rec["out"][0, 4 * h:4 * h + 4], o.numpy(), rtol=1e-12, atol=1e-13)


def test_first_step_refills_then_unchanged_query_keeps_full_overlap():
    spec, q0, data = small_workload(anchors=True)
    retrieved, base = I.initial_lists(spec)
    anchor_before = retrieved[(0, 2)].clone()
    layer = ref.RefLayer(spec, data, retrieved, base)
    q = q0.to(torch.bfloat16)
    r0 = layer.step(q)
    k = spec.k_mon(0, 0)
    assert k == 112 and spec.cand_range(0, 0) == (16, 992)
    # positional baseline vs. real top-k: small overlap -> trigger, refill, baseline update
    assert r0["flag"][(0, 0)] == 1 and r0["inter"][(0, 0)] < k * 4 // 9
    np.testing.assert_array_equal(layer.retrieved[(0, 1)], r0["topk"][(0, 1)])
    np.testing.assert_array_equal(layer.retrieved[(0, 3)], r0["topk"][(0, 3)])
    np.testing.assert_array_equal(layer.base[(0, 0)], r0["topk"][(0, 0)])
    assert set(r0["topk"][(0, 3)].tolist()) <= set(r0["topk"][(0, 1)].tolist())       # nested budgets
    # anchors are never refilled (Sec. 4.3, last sentence)
    np.testing.assert_array_equal(layer.retrieved[(0, 2)], anchor_before.numpy())
    r1 = layer.step(q)
    assert r1["inter"][(0, 0)] == k and r1["flag"][(0, 0)] == 0
    np.testing.assert_array_equal(layer.retrieved[(0, 2)], anchor_before.numpy())
    # the satellite now attends over sink + recent + retrieved, in slot order
    idx = layer.resident(0, 1)
    assert idx.size == 160 and idx[:16].tolist() == list(range(16)) and idx[16:48].tolist() == list(range(992, 1024))
    want = ref.attn(ref._bits(q[0, 4:8]), layer.Kb[(0, 1)], layer.Vb[(0, 1)], idx)
    np.testing.assert_array_equal(r1["out"][0, 4:8], want[0])


def test_refill_decided_at_step_t_is_used_from_step_t_plus_1():
    spec, q0, data = small_workload(seed=5)
    retrieved, base = I.initial_lists(spec)
    layer = ref.RefLayer(spec, data, retrieved, base)
    q = q0.to(torch.bfloat16)
    before = layer.resident(0, 1).copy()
    r0 = layer.step(q)
    want0 = ref.attn(ref._bits(q[0, 4:8]), layer.Kb[(0, 1)], layer.Vb[(0, 1)], before)
    np.testing.assert_array_equal(r0["out"][0, 4:8], want0[0])      # step 0 still saw the old slots
    assert not np.array_equal(layer.resident(0, 1), before)


def test_window_debounces_and_ring_clears_on_trigger():
    spec, q0, data = small_workload(seed=6)
    spec.window = 3
    retrieved, base = I.initial_lists(spec)
    layer = ref.RefLayer(spec, data, retrieved, base)
    q = q0.to(torch.bfloat16)
    flags = [layer.step(q)["flag"][(0, 0)] for _ in range(7)]
    # the window fills at the third step, triggers (low overlap), is cleared; after the baseline
    # update the overlap is k, so the next full window (steps 4-6) does not trigger
    assert flags == [0, 0, 1, 0, 0, 0, 0]
    assert layer.n_tests == 3 and layer.n_triggers == 1


def test_tumbling_window_tests_only_every_w_steps():
    """Algorithm 1's loop: with W = 3 the signal is evaluated at steps 3, 6, 9, ... over the three steps
    since the last evaluation.  Worked by hand for an unchanged query: the window of steps 1-3 (overlap
    low: positional baseline) triggers and the baseline becomes the true top-k; steps 4-6 then see full
    overlap and do not trigger; the sliding window of Eq. 10 evaluates at 3 (trigger), then at every step
    from 6 on."""
    spec, q0, data = small_workload(seed=6)
    spec.window = 3
    q = q0.to(torch.bfloat16)
    tests = {}
    for mode in (0, 1):
        spec.window_mode = mode
        retrieved, base = I.initial_lists(spec)
        layer = ref.RefLayer(spec, data, retrieved, base)
        flags = [layer.step(q)["flag"][(0, 0)] for _ in range(9)]
        assert flags == [0, 0, 1, 0, 0, 0, 0, 0, 0]
        tests[mode] = layer.n_tests
    assert tests == {0: 1 + 4, 1: 3}          # sliding: steps 3, 6, 7, 8, 9; tumbling: steps 3, 6, 9


def test_tumbling_window_misses_what_a_sliding_window_sees():
    """Overlap sequence by construction (the baseline is swapped by hand): high at steps 1-2, low at steps
    3-5, high afterwards; W = 3, lower median.  Sliding: {1,2,3} = h,h,l -> high; {2,3,4} = h,l,l -> low:
    fires at step 4.  Tumbling: {1,2,3} -> high; {4,5,6} = l,l,h -> low: fires at step 6."""
    spec, q0, data = small_workload(seed=7)
    spec.window = 3
    q = q0.to(torch.bfloat16)
    fired = {}
    for mode in (0, 1):
        spec.window_mode = mode
        retrieved, base = I.initial_lists(spec)
        layer = ref.RefLayer(spec, data, retrieved, base)
        true_top = ref.topk(layer.step(q, monitor=True)["scores"][(0, 0)].astype(np.float32),
                            *spec.cand_range(0, 0), spec.k_mon(0, 0))
        layer = ref.RefLayer(spec, data, retrieved, base)
        good, bad = true_top.copy(), base[(0, 0)].numpy().copy()
        flags = []
        for t in range(1, 8):
            layer.base[(0, 0)] = bad if t in (3, 4, 5) else good
            before = layer.n_triggers
            f = layer.step(q)["flag"][(0, 0)]
            flags.append(f)
            if layer.n_triggers > before:
                break
        fired[mode] = len(flags)
    assert fired == {0: 4, 1: 6}


def test_overlap_after_rotation_matches_bivariate_normal_expectation():
    """G = 1, keys ~ N(0,1): the logits of q and of q rotated by theta are jointly normal with
    correlation cos(theta), so E[overlap of the two top-k sets] = P(z>c, z'>c)/f, f = k/#candidates.
    Pins score -> top-k -> intersection as a chain against a closed form."""
    N, sink, recent, r = 16384, 64, 256, 1400
    heads = [I.HeadSpec(I.ROLE_FULL), I.HeadSpec(I.ROLE_SATELLITE, rep=0, sink=sink, recent=recent, budget=sink + recent + r)]
    spec = I.LayerSpec(B=1, Hq=2, Hkv=2, D=128, ctx=[N], heads=[heads], tau_num=0, tau_den=1)   # never trigger after init
    q0 = I.draw_q(spec, 21)
    data = I.draw_layer(spec, q0, 22)
    f = r / (N - sink - recent)
    c = norm.isf(f)
    for theta in (5.0, 10.0, 15.0, 30.0):
        rho = math.cos(math.radians(theta))
        joint = multivariate_normal(mean=[0, 0], cov=[[1, rho], [rho, 1]])
        expect = joint.cdf([-c, -c]) / f                      # P(z>c,z'>c) by symmetry
        sched = I.QuerySchedule(q0, 23, step_deg=theta)
        retrieved, base = I.initial_lists(spec)
        layer = ref.RefLayer(spec, data, retrieved, base)
        T0 = layer.step(sched.next())["topk"][(0, 0)]
        layer.base[(0, 0)] = T0.copy()
        o = layer.step(sched.next())["inter"][(0, 0)] / r
        sigma = math.sqrt(expect * (1 - expect) / r)
        assert abs(o - expect) < 5 * sigma + 0.01, (theta, o, expect)
