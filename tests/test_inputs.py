"""The seeded generators: shapes, determinism, and the byte counts the configs quote."""
import numpy as np
import torch

from paper_2601_13684_amd import inputs as I


def test_config4_spec_byte_count_matches_the_quoted_figure():
    spec = I.spec_llama(I.CONFIG_CTX[4], I.CONFIG_BUDGETS[4])
    assert spec.kv_bytes() == 2 * 229376 * 512 + 21504 * 512 == 245_891_072
    assert I.spec_dense(229376).kv_bytes() == 8 * 229376 * 512
    assert [spec.r(0, h) for h in range(2, 8)] == [7872, 3776, 3776, 1728, 1728, 704]
    assert spec.reps(0) == [0, 1] and spec.satellites(0, 0) == [2, 4, 6] and spec.satellites(0, 1) == [3, 5, 7]
    assert spec.k_mon(0, 0) == 7872 and spec.k_mon(0, 1) == 3776
    assert spec.cand_range(0, 0) == (64, 229376 - 256)


def test_tiny_workload_is_deterministic_and_shaped():
    a = I.make_workload(1, N=1024)
    b = I.make_workload(1, N=1024)
    assert a.spec.kv_bytes() == (1024 + 512) * 512
    for key in a.data.K:
        assert a.data.K[key].dtype == torch.bfloat16 and a.data.K[key].shape == (1024, 128)
        assert torch.equal(a.data.K[key], b.data.K[key]) and torch.equal(a.data.V[key], b.data.V[key])
        assert a.data.heavy[key].numel() == 40
    qa = [a.schedule.next() for _ in range(3)]
    qb = [b.schedule.next() for _ in range(3)]
    assert all(torch.equal(x, y) for x, y in zip(qa, qb))
    # 5 degrees per step, norm preserved (up to bf16 rounding)
    c = torch.nn.functional.cosine_similarity(qa[0].double(), qa[1].double(), dim=-1)
    assert torch.allclose(c, torch.full_like(c, np.cos(np.radians(5.0))), atol=2e-3)


def test_segmented_heavy_tokens_and_jump_schedule():
    w = I.make_workload(4, N=8192, scale=1 / 16)
    pos = w.data.heavy[(0, 0)]
    assert pos.numel() == round(0.005 * 8192)
    runs = 1 + int((pos[1:] - pos[:-1] != 1).sum())
    assert runs == 16
    qs = [w.schedule.next() for _ in range(18)]
    assert torch.equal(qs[1], qs[15]) and not torch.equal(qs[15], qs[16]) and torch.equal(qs[16], qs[17])


def test_ragged_spec():
    spec = I.spec_ragged(5000, B=16)
    assert len(spec.ctx) == 16 and min(spec.ctx) >= 8192 and max(spec.ctx) <= 131072
    for b in range(16):
        roles = [h.role for h in spec.heads[b]]
        assert roles.count(I.ROLE_FULL) == 2
        for h in spec.heads[b]:
            if h.role == I.ROLE_SATELLITE:
                assert spec.heads[b][h.rep].role == I.ROLE_FULL and h.budget in (512, 1024, 2048, 4096)
