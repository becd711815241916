"""Pins of the oracle's re-scored window (RefLayer with window_mode 2; Algorithm 1, the loop over the
buffered queries at t mod W = 0): every query of the window is scored again against the pivot's cache as it
is at the test step, and the median of those overlaps decides."""
import numpy as np
import torch

from oracle import ref
from paper_2601_13684_amd import inputs as I


def layer_spec(N, sink, recent, r, W, mode, **kw):
    heads = [I.HeadSpec(I.ROLE_FULL), I.HeadSpec(I.ROLE_SATELLITE, rep=0, sink=sink, recent=recent, budget=sink + recent + r)]
    spec = I.LayerSpec(B=1, Hq=8, Hkv=2, D=128, ctx=[N], heads=[heads], **kw)
    spec.window, spec.window_mode = W, mode
    return spec


def test_with_an_unchanged_cache_rescoring_changes_nothing():
    """Same query, same cache: the overlap computed again equals the stored one, so modes 1 and 2 agree in
    every value over a run with rotating and jumping queries (several windows, with and without triggers)."""
    runs = {}
    for mode in (1, 2):
        spec = layer_spec(700, 8, 16, 48, 3, mode, tau_num=7, tau_den=10)
        q0 = I.draw_q(spec, 11)
        data = I.draw_layer(spec, q0, 12, heavy_count=30)
        sched = I.QuerySchedule(q0, 13, step_deg=4.0, jump_every=4, jump_deg=50.0)
        retrieved, base = I.initial_lists(spec)
        layer = ref.RefLayer(spec, data, retrieved, base)
        log = []
        for t in range(13):
            rec = layer.step(sched.next())
            log.append((rec["inter"][(0, 0)], rec["flag"][(0, 0)], list(layer.ring[(0, 0)]), layer.retrieved[(0, 1)].tolist(),
                        layer.base[(0, 0)].tolist()))
            if mode == 2 and (t + 1) % 3 == 0:
                assert len(rec["rescored"][(0, 0)]) == 2
        runs[mode] = log
        assert 0 < layer.n_triggers < layer.n_tests == 4
    assert runs[1] == runs[2]


def test_hand_worked_window_over_a_growing_cache():
    """k = 2, W = 3, one recent slot, scores = mean of the logits (so the order of the old tokens cannot
    change), the same query at every step, baseline = the two best old tokens.  Before each step a token is
    appended whose key dominates everything before it.  The token appended before step s is a candidate
    from step s + 1 on.  Overlaps as first computed: step 1 sees no new candidate (2 of 2), step 2 sees the
    first token (1 of 2), step 3 the first two (0 of 2): stored window 2, 1, 0, lower median 1, overlap 1/2,
    not below tau = 1/2.  Scored again at step 3, every query of the window sees both new candidates:
    0, 0, 0, median 0 < 1/2.  So the tumbling window with stored overlaps does not fire and the re-scored
    one does."""
    N = 400
    got = {}
    for mode in (1, 2):
        spec = layer_spec(N, 4, 1, 2, 3, mode, tau_num=1, tau_den=2, metric=I.METRIC_OVERLAP, agg=I.AGG_LOGIT)
        q0 = I.draw_q(spec, 21)
        data = I.draw_layer(spec, q0, 22)
        q = q0.to(torch.bfloat16)
        retrieved, base = I.initial_lists(spec)
        probe = ref.RefLayer(spec, data, retrieved, base)
        best2 = probe.step(q)["topk"][(0, 0)].copy()
        layer = ref.RefLayer(spec, data, retrieved, base)
        layer.base[(0, 0)] = best2
        inters, flags = [], []
        for t in range(3):
            kn, vn = I.draw_token(spec, 30 + t, toward=q, gain=20.0 + 5 * t)
            layer.append(kn, vn)
            rec = layer.step(q)
            inters.append(rec["inter"][(0, 0)])
            flags.append(rec["flag"][(0, 0)])
        assert inters == [2, 1, 0]                       # as first computed, in both modes
        got[mode] = flags
        if mode == 2:
            assert [x[2] for x in rec["rescored"][(0, 0)]] == [0, 0]
            assert sorted(rec["rescored"][(0, 0)][0][1].tolist()) == [N, N + 1]
            assert layer.base[(0, 0)].tolist() == [N, N + 1] and layer.retrieved[(0, 1)].tolist() == [N, N + 1]
    assert got == {1: [0, 0, 0], 2: [0, 0, 1]}


def test_rescored_weights_are_a_softmax_over_the_whole_grown_cache():
    """Mean of post-softmax weights: the re-computed scores of a buffered query sum to one over ALL positions
    of the cache at the test step, appended tokens included, and have that length."""
    N, W = 300, 4
    spec = layer_spec(N, 4, 8, 24, W, 2)
    q0 = I.draw_q(spec, 31)
    data = I.draw_layer(spec, q0, 32, heavy_count=12)
    sched = I.QuerySchedule(q0, 33, step_deg=10.0)
    retrieved, base = I.initial_lists(spec)
    layer = ref.RefLayer(spec, data, retrieved, base)
    for t in range(W):
        kn, vn = I.draw_token(spec, 40 + t)
        layer.append(kn, vn)
        rec = layer.step(sched.next())
    again = rec["rescored"][(0, 0)]
    assert len(again) == W - 1
    for s_k, T_k, inter in again:
        assert s_k.shape == (N + W,)
        assert abs(s_k.sum() - 1.0) < 1e-12
        assert T_k.min() >= 4 and T_k.max() < N + W - 8


def bf16_to_f64(t):
    return t.to(torch.float32).double().numpy()


def test_brute_force_on_a_tiny_growing_layer():
    """Everything the test step decides, recomputed here with numpy from the definitions (softmax over the
    current cache, mean over the group, fp32 scores, k best by (score descending, index ascending), overlap
    count, lower median, exact rational comparison with tau)."""
    N, W, sink, recent, r = 60, 3, 2, 3, 7
    for seed in range(6):
        spec = layer_spec(N, sink, recent, r, W, 2, tau_num=3, tau_den=5, metric=I.METRIC_JACCARD if seed % 2 else I.METRIC_OVERLAP)
        q0 = I.draw_q(spec, 50 + seed)
        data = I.draw_layer(spec, q0, 60 + seed, heavy_count=6)
        sched = I.QuerySchedule(q0, 70 + seed, step_deg=25.0)
        retrieved, base = I.initial_lists(spec)
        layer = ref.RefLayer(spec, data, retrieved, base)
        K = bf16_to_f64(data.K[(0, 0)])
        qs = []
        for t in range(2 * W):
            kn, vn = I.draw_token(spec, 80 + 10 * seed + t, toward=q0, gain=6.0 * (t % 2))
            layer.append(kn, vn)
            K = np.concatenate([K, bf16_to_f64(kn[0, 0])[None]])
            q = sched.next()
            qs.append(bf16_to_f64(q[0, 0:4]))
            base_before = set(layer.base[(0, 0)].tolist())
            rec = layer.step(q)
            if (t + 1) % W:
                assert rec["flag"][(0, 0)] == 0 and not rec["rescored"]
                continue
            n = N + t + 1
            lo, hi = sink, n - recent
            overlaps = []
            for qk in qs[-W:]:
                lg = qk @ K.T / np.sqrt(128.0)
                p = np.exp(lg - lg.max(1, keepdims=True))
                p /= p.sum(1, keepdims=True)
                s32 = p.mean(0).astype(np.float32)
                order = sorted(range(lo, hi), key=lambda j: (-s32[j], j))[:r]
                overlaps.append(len(set(order) & base_before))
            med = sorted(overlaps)[(W - 1) // 2]
            if spec.metric == I.METRIC_OVERLAP:
                want = int(med * 5 < 3 * r)
            else:
                want = int(med * 5 < 3 * (2 * r - med))
            assert [x[2] for x in rec["rescored"][(0, 0)]] == overlaps[:-1], (seed, t)
            assert rec["inter"][(0, 0)] == overlaps[-1]
            assert rec["flag"][(0, 0)] == want, (seed, t, overlaps)
