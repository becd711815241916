"""Pins of the oracle's context growth (RefLayer.append): the decode token's K/V enters every head's
master cache, compressed heads see it through their window of recent positions, and the position
that leaves the window becomes a candidate of the pivot's top-k (Algorithm 1: ModelForward returns the
updated cache; the reading of how is stated in RefLayer's docstring)."""
import numpy as np
import torch
import torch.nn.functional as F

from oracle import ref
from paper_2601_13684_amd import inputs as I


def dense(q, K, V):
    """Library attention of 4 query heads over K, V (fp64)."""
    return F.scaled_dot_product_attention(q.double()[None, :, None, :], K.double()[None, None].expand(1, q.shape[0], -1, -1),
                                          V.double()[None, None].expand(1, q.shape[0], -1, -1))[0, :, 0].numpy()


def test_appended_tokens_are_attended_by_full_heads_like_dense_attention_over_the_grown_cache():
    N = 200
    heads = [I.HeadSpec(I.ROLE_FULL), I.HeadSpec(I.ROLE_FULL)]
    spec = I.LayerSpec(B=2, Hq=8, Hkv=2, D=128, ctx=[N, N - 50], heads=[heads, heads])
    q0 = I.draw_q(spec, 1)
    data = I.draw_layer(spec, q0, 2)
    layer = ref.RefLayer(spec, data, {}, {})
    K = {k: v.clone() for k, v in data.K.items()}
    V = {k: v.clone() for k, v in data.V.items()}
    q = q0.to(torch.bfloat16)
    for t in range(5):
        kn, vn = I.draw_token(spec, 100 + t)
        layer.append(kn, vn)
        for b in range(2):
            for h in range(2):
                K[(b, h)] = torch.cat([K[(b, h)], kn[b, h][None]])
                V[(b, h)] = torch.cat([V[(b, h)], vn[b, h][None]])
        rec = layer.step(q, monitor=False)
        for b in range(2):
            for h in range(2):
                np.testing.assert_allclose(rec["out"][b, 4 * h:4 * h + 4], dense(q[b, 4 * h:4 * h + 4], K[(b, h)], V[(b, h)]),
                                           rtol=1e-12, atol=1e-13)
    assert layer.ctx == [N + 5, N - 50 + 5]


def test_compressed_head_sees_sink_the_sliding_recent_window_and_its_retrieved_positions():
    N, sink, recent, r = 300, 4, 8, 20
    heads = [I.HeadSpec(I.ROLE_FULL), I.HeadSpec(I.ROLE_SATELLITE, rep=0, sink=sink, recent=recent, budget=sink + recent + r)]
    spec = I.LayerSpec(B=1, Hq=8, Hkv=2, D=128, ctx=[N], heads=[heads], tau_num=0, tau_den=1)      # never refill
    q0 = I.draw_q(spec, 5)
    data = I.draw_layer(spec, q0, 6)
    retrieved, base = I.initial_lists(spec)
    layer = ref.RefLayer(spec, data, retrieved, base)
    K, V = data.K[(0, 1)].clone(), data.V[(0, 1)].clone()
    q = q0.to(torch.bfloat16)
    for t in range(recent + 3):                 # the window turns over completely
        kn, vn = I.draw_token(spec, 200 + t)
        layer.append(kn, vn)
        K, V = torch.cat([K, kn[0, 1][None]]), torch.cat([V, vn[0, 1][None]])
        n = N + t + 1
        want_set = list(range(sink)) + list(range(n - recent, n)) + retrieved[(0, 1)].tolist()
        assert layer.resident(0, 1).tolist() == want_set
        rec = layer.step(q)
        idx = torch.tensor(want_set)
        np.testing.assert_allclose(rec["out"][0, 4:8], dense(q[0, 4:8], K[idx], V[idx]), rtol=1e-12, atol=1e-13)
        assert layer.cand_range(0, 0) == (sink, n - recent)


def test_a_token_that_left_the_recent_window_can_be_retrieved():
    """A generated token with a dominant key: while it is in the window it is resident anyway and is not a
    candidate; the step it leaves the window it enters the candidate range, the pivot's top-k picks it up,
    and a refill makes it resident again (its row comes from the grown master cache, i.e. the host tier)."""
    N, sink, recent, r = 400, 4, 6, 16
    heads = [I.HeadSpec(I.ROLE_FULL), I.HeadSpec(I.ROLE_SATELLITE, rep=0, sink=sink, recent=recent, budget=sink + recent + r)]
    spec = I.LayerSpec(B=1, Hq=8, Hkv=2, D=128, ctx=[N], heads=[heads], tau_num=1, tau_den=1, metric=I.METRIC_OVERLAP)
    q0 = I.draw_q(spec, 7)
    data = I.draw_layer(spec, q0, 8)
    retrieved, base = I.initial_lists(spec)
    layer = ref.RefLayer(spec, data, retrieved, base)
    q = q0.to(torch.bfloat16)
    kn, vn = I.draw_token(spec, 300, toward=q, gain=60.0)       # position N: dominant for every head
    layer.append(kn, vn)
    seen_as_candidate = []
    for t in range(recent + 2):
        rec = layer.step(q)
        lo, hi = layer.cand_range(0, 0)
        seen_as_candidate.append(N in rec["topk"][(0, 0)].tolist())
        assert (N < hi) == seen_as_candidate[-1], "the dominant token is selected exactly when it is a candidate"
        if not seen_as_candidate[-1]:
            assert N in layer.resident(0, 1).tolist()            # still inside the recent window
        kf, vf = I.draw_token(spec, 301 + t)
        layer.append(kf, vf)
    # position N is inside the window while ctx - recent <= N, i.e. for the first `recent` steps after it
    assert seen_as_candidate == [False] * recent + [True] * 2
    # once selected, with tau = 1 (any change of the set triggers) it was refilled
    assert N in layer.retrieved[(0, 1)].tolist()
