"""Pins of the oracle's attention (Algorithm 1, ModelForward over the resident cache of
Sec. 4.3) to things other than itself: a library routine in fp64, closed forms, a hand-derived
fixture, and structural invariants.  CPU only."""
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import ref

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def bf16_bits(x: torch.Tensor) -> np.ndarray:
    return ref._bits(x.to(torch.bfloat16))


def rand_case(seed, G, N, D):
    g = torch.Generator().manual_seed(seed)
    q = torch.randn(G, D, generator=g).to(torch.bfloat16)
    K = torch.randn(N, D, generator=g).to(torch.bfloat16)
    V = torch.randn(N, D, generator=g).to(torch.bfloat16)
    return q, K, V


def sdpa64(q, K, V):
    """Library dense attention in float64: q [G,D], K,V [n,D] -> [G,D]."""
    o = F.scaled_dot_product_attention(q.double()[None, :, None, :],       # [1,G,1,D]
                                       K.double()[None, None, :, :].expand(1, q.shape[0], -1, -1),
                                       V.double()[None, None, :, :].expand(1, q.shape[0], -1, -1))
    return o[0, :, 0, :].numpy()


@pytest.mark.parametrize("seed,G,N,D", [(0, 4, 257, 128), (1, 1, 64, 128), (2, 8, 1000, 64), (3, 4, 1, 128)])
def test_dense_matches_library_sdpa(seed, G, N, D):
    q, K, V = rand_case(seed, G, N, D)
    out, lse, logits = ref.attn(bf16_bits(q), bf16_bits(K), bf16_bits(V), None, want_logits=True)
    np.testing.assert_allclose(out, sdpa64(q, K, V), rtol=1e-12, atol=1e-13)
    want_lse = torch.logsumexp(q.double() @ K.double().T / math.sqrt(D), dim=-1).numpy()
    np.testing.assert_allclose(lse, want_lse, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(logits, (q.double() @ K.double().T / math.sqrt(D)).numpy(), rtol=1e-13, atol=1e-13)


def test_budget_equal_context_reproduces_dense():
    q, K, V = rand_case(5, 4, 300, 128)
    dense = ref.attn(bf16_bits(q), bf16_bits(K), bf16_bits(V), None)
    full_idx = np.arange(300, dtype=np.int32)
    comp = ref.attn(bf16_bits(q), bf16_bits(K), bf16_bits(V), full_idx)
    np.testing.assert_array_equal(dense[0], comp[0])
    np.testing.assert_array_equal(dense[1], comp[1])


def test_compressed_equals_library_on_selected_rows():
    q, K, V = rand_case(6, 4, 500, 128)
    g = torch.Generator().manual_seed(60)
    idx = torch.randperm(500, generator=g)[:77]
    out, lse, _ = ref.attn(bf16_bits(q), bf16_bits(K), bf16_bits(V), idx.numpy().astype(np.int32))
    np.testing.assert_allclose(out, sdpa64(q, K[idx], V[idx]), rtol=1e-12, atol=1e-13)


def test_hand_derived_two_token_fixture():
    vals = {}
    for line in open(os.path.join(GOLD, "two_token_softmax.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        vals[k] = [float(x) for x in v]
    q = torch.tensor([[2.0, 0, 0, 0]])
    K = torch.tensor([[0.0, 0, 0, 0], [1.0, 0, 0, 0]])
    V = torch.tensor([[1.0, 0, 2, -4], [0.0, 1, -2, 4]])
    out, lse, logits = ref.attn(bf16_bits(q), bf16_bits(K), bf16_bits(V), None, want_logits=True)
    np.testing.assert_allclose(logits[0], [0.0, 1.0], atol=0)
    np.testing.assert_allclose(out[0], vals["out"], rtol=1e-15, atol=1e-15)
    np.testing.assert_allclose(lse[0], vals["lse"][0], rtol=1e-15)
    w = np.exp(logits[0] - lse[0])
    np.testing.assert_allclose(w, [vals["w_a"][0], vals["w_b"][0]], rtol=1e-15)


def test_identical_keys_give_mean_of_values():
    g = torch.Generator().manual_seed(7)
    q = torch.randn(4, 128, generator=g).to(torch.bfloat16)
    k = torch.randn(1, 128, generator=g).to(torch.bfloat16)
    K = k.expand(50, 128).contiguous()
    V = torch.randn(50, 128, generator=g).to(torch.bfloat16)
    out, lse, _ = ref.attn(bf16_bits(q), bf16_bits(K), bf16_bits(V), None)
    np.testing.assert_allclose(out, V.double().mean(0)[None, :].expand(4, -1).numpy(), rtol=1e-12, atol=1e-14)
    logit = (q.double() @ k.double().T / math.sqrt(128))[:, 0].numpy()
    np.testing.assert_allclose(lse, logit + math.log(50), rtol=1e-13)


def test_dominant_key_selects_its_value_row():
    g = torch.Generator().manual_seed(8)
    q = torch.zeros(1, 128)
    q[0, 0] = 64.0
    K = (0.01 * torch.randn(40, 128, generator=g))
    K[:, 0] = 0.0
    K[17, 0] = 16.0            # logit 64*16/sqrt(128) = 90.5, all others 0
    V = torch.randn(40, 128, generator=g).to(torch.bfloat16)
    out, _, _ = ref.attn(bf16_bits(q), bf16_bits(K), bf16_bits(V), None)
    np.testing.assert_allclose(out[0], V[17].double().numpy(), rtol=0, atol=1e-30)


def test_permuting_slots_leaves_output_unchanged():
    q, K, V = rand_case(9, 4, 200, 128)
    idx = np.arange(10, 150, dtype=np.int32)
    a = ref.attn(bf16_bits(q), bf16_bits(K), bf16_bits(V), idx)
    perm = np.random.default_rng(9).permutation(idx).astype(np.int32)
    b = ref.attn(bf16_bits(q), bf16_bits(K), bf16_bits(V), perm)
    np.testing.assert_allclose(a[0], b[0], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(a[1], b[1], rtol=1e-13)


@pytest.mark.parametrize("cuts", [[100], [1, 2, 3], [64, 128, 192, 255]])
def test_lse_merge_of_any_partition_equals_unsplit(cuts):
    """Split-K identity every flash-decode relies on: partial (out, lse) of disjoint chunks,
    merged with weights exp(lse_c - lse), give the unsplit result."""
    q, K, V = rand_case(10, 4, 256, 128)
    whole = ref.attn(bf16_bits(q), bf16_bits(K), bf16_bits(V), None)
    edges = [0] + cuts + [256]
    parts = [ref.attn(bf16_bits(q), bf16_bits(K), bf16_bits(V), np.arange(a, b, dtype=np.int32))
             for a, b in zip(edges[:-1], edges[1:])]
    lses = np.stack([p[1] for p in parts])                    # [C,G]
    lse = np.log(np.exp(lses - lses.max(0)).sum(0)) + lses.max(0)
    out = sum(np.exp(p[1] - lse)[:, None] * p[0] for p in parts)
    np.testing.assert_allclose(out, whole[0], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(lse, whole[1], rtol=1e-13)


def test_identical_query_heads_give_identical_outputs():
    q, K, V = rand_case(11, 4, 120, 128)
    q[:] = q[0]
    out, lse, _ = ref.attn(bf16_bits(q), bf16_bits(K), bf16_bits(V), None)
    for g in range(1, 4):
        np.testing.assert_array_equal(out[g], out[0])
        assert lse[g] == lse[0]


def test_brute_force_tiny_python_loops():
    """Independent third opinion on tiny inputs: exact rationals are not needed, plain Python
    floats with math.fsum are."""
    q, K, V = rand_case(12, 2, 9, 8)
    out, lse, _ = ref.attn(bf16_bits(q), bf16_bits(K), bf16_bits(V), None)
    qf, Kf, Vf = q.double().tolist(), K.double().tolist(), V.double().tolist()
    for g in range(2):
        l = [math.fsum(qf[g][d] * Kf[j][d] for d in range(8)) / math.sqrt(8) for j in range(9)]
        w = [math.exp(x) for x in l]
        Z = math.fsum(w)
        for d in range(8):
            assert out[g][d] == pytest.approx(math.fsum(w[j] * Vf[j][d] for j in range(9)) / Z, rel=1e-13, abs=1e-15)
        assert lse[g] == pytest.approx(math.log(Z), rel=1e-13)


def test_softmax_weights_sum_to_one_and_scores_sum_to_one():
    q, K, V = rand_case(13, 4, 700, 128)
    ones = torch.ones_like(V)
    out, lse, logits = ref.attn(bf16_bits(q), bf16_bits(K), bf16_bits(ones), None, want_logits=True)
    np.testing.assert_allclose(out, 1.0, rtol=1e-13)          # sum_j w_j * 1 = 1
    s = ref.scores(logits, lse, agg=0)
    assert abs(s.sum() - 1.0) < 1e-12
    assert (s >= 0).all()


def test_non_finite_input_is_an_error():
    q, K, V = rand_case(14, 4, 10, 128)
    K[3, 5] = float("inf")
    with pytest.raises(ValueError):
        ref.attn(bf16_bits(q), bf16_bits(K), bf16_bits(V), None)
