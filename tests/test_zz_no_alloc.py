"""hc_decode_attn_static, the entry point for callers that cannot allocate: same results as hc_decode_attn,
bit for bit (the same kernels over the same plan; only the place of the split-K partial results differs), on
two calls in a row that share the library's fixed scratch array, the second with a smaller input; a plan
larger than the array is refused before anything is launched.  Collected last on purpose."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2601_13684_amd import binding as hc
from paper_2601_13684_amd import inputs as I
from paper_2601_13684_amd import runtime as R

import gpu_util as U

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(*a):
    print(*a, flush=True)


def both_ways(w, tag):
    """One layer, one query: hc_decode_attn, then hc_decode_attn_static into separate outputs."""
    spec = w.spec
    retrieved, base = I.initial_lists(spec)
    ctx = R.Context(R.make_config(spec), DEV)
    gpu = R.LayerRuntime(ctx, spec, w.data, retrieved, base, host_tier=False)
    q = w.schedule.next()
    qd = q.to(DEV)
    say(f"  {tag}: partials {hc.hc_layer_num_partials(gpu.handle)}, workgroups {hc.hc_layer_num_workgroups(gpu.handle)}")
    assert hc.hc_layer_num_partials(gpu.handle) <= hc.HC_STATIC_MAX_PARTIALS
    gpu.attn(qd)                                             # existing entry point: out, lse, rep_logits
    torch.cuda.synchronize()
    want = (gpu.out.clone(), gpu.lse.clone(), gpu.rep_logits.clone())
    out2, lse2, rl2 = torch.full_like(gpu.out, 7.0), torch.full_like(gpu.lse, 7.0), torch.full_like(gpu.rep_logits, 7.0)
    hc.hc_decode_attn_static(ctx.handle, gpu.handle, gpu.arena, qd, out2, lse2, rl2)
    torch.cuda.synchronize()
    assert torch.equal(out2, want[0]) and torch.equal(lse2, want[1]), tag
    for b in range(spec.B):
        for p in spec.reps(b):
            slot, n = gpu.rep_slot(b, p), spec.ctx[b]
            assert torch.equal(rl2[slot, :n], want[2][slot, :n]), (tag, "pivot logits")
    # and against the oracle, to the attention tolerance
    cpu = I.LayerData({k: v.cpu() for k, v in w.data.K.items()}, {k: v.cpu() for k, v in w.data.V.items()}, {})
    rec = ref.RefLayer(spec, cpu, retrieved, base).step(q.cpu(), monitor=False)
    worst, lerr = U.check_attention(out2, lse2, rec, tag)
    say(f"  {tag}: identical to hc_decode_attn; against the oracle err/rms {worst:.2e}, lse {lerr:.1e}")
    gpu.close()
    ctx.close()


def test_static_scratch_entry_point_matches_on_two_calls_in_a_row():
    say("hc_decode_attn_static: 32K layer, then the 4K layer (the same scratch array, a smaller plan)")
    both_ways(I.make_workload(2, device=DEV), "32K, 8 KV heads")
    both_ways(I.make_workload(1, device=DEV), "4K, 2 KV heads")


def test_static_scratch_entry_point_refuses_a_plan_that_does_not_fit():
    """B = 72 sequences of 8 KV heads: 512 workgroups plus up to one extra partial per head boundary > 1024."""
    say("hc_decode_attn_static: oversize plan")
    B = 80
    spec = I.spec_dense(4096, B=B)
    ctx = R.Context(R.make_config(spec), DEV)
    q0 = I.draw_q(spec, 5)
    data = I.LayerData()
    g = torch.Generator(device=DEV)
    g.manual_seed(3)
    for b in range(B):
        for h in range(8):
            data.K[(b, h)] = torch.randn((4096, 128), generator=g, device=DEV).to(torch.bfloat16)
            data.V[(b, h)] = torch.randn((4096, 128), generator=g, device=DEV).to(torch.bfloat16)
    gpu = R.LayerRuntime(ctx, spec, data, {}, {}, host_tier=False)
    n = hc.hc_layer_num_partials(gpu.handle)
    say("  partials", n)
    assert n > hc.HC_STATIC_MAX_PARTIALS
    qd = q0.to(torch.bfloat16).to(DEV)
    before = gpu.out.clone()
    with pytest.raises(hc.HcError) as e:
        hc.hc_decode_attn_static(ctx.handle, gpu.handle, gpu.arena, qd, gpu.out, gpu.lse, None)
    assert e.value.status == hc.HC_ESHAPE and "fixed scratch" in str(e.value)
    torch.cuda.synchronize()
    assert torch.equal(gpu.out, before)
    gpu.attn(qd, monitor=False)                      # the ordinary entry point takes the same layer
    torch.cuda.synchronize()
    assert np.isfinite(gpu.out.cpu().numpy()).all()
    gpu.close()
    ctx.close()
