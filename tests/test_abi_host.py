"""The C-ABI library on a machine without a GPU: it loads, exports every symbol the header
declares, rejects bad arguments on the host, and builds a sound split-K plan."""
import ctypes as C
import os
import re

import pytest

from paper_2601_13684_amd import binding as hc
from paper_2601_13684_amd import inputs as I
from paper_2601_13684_amd import runtime as R

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    src = open(os.path.join(ROOT, "include", "hc.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(hc_[a-z_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    names = header_functions()
    assert {"hc_decode_attn", "hc_rep_topk_drift", "hc_gather_retrieve", "hc_create", "hc_layer_create"} <= set(names)
    L = hc.lib()
    for n in names:
        assert getattr(L, n) is not None
    assert sorted(hc.EXPORTS) == names


def test_struct_sizes_match_the_header_layout():
    assert C.sizeof(hc.hc_config) == 12 * 4
    assert C.sizeof(hc.hc_head_desc) == 3 * 8 + 8 * 4
    assert C.sizeof(hc.hc_plan_info) == 8 * 4 + 2 * 8


def test_strerror():
    assert hc.lib().hc_strerror(0) == b"ok"
    assert b"invalid" in hc.lib().hc_strerror(1)


def cfg_for(spec, **kw):
    c = R.make_config(spec)
    for k, v in kw.items():
        setattr(c, k, v)
    return c


@pytest.mark.parametrize("field,value,status", [
    ("D", 64, hc.HC_ESHAPE), ("Hq", 7, hc.HC_EINVAL), ("Hq", 32, hc.HC_ESHAPE),   # G = 16
    ("max_ctx", 100, hc.HC_ESHAPE), ("window", 0, hc.HC_EINVAL), ("window", 65, hc.HC_EINVAL),
    ("metric", 2, hc.HC_EINVAL), ("tau_den", 0, hc.HC_EINVAL), ("agg", 3, hc.HC_EINVAL), ("max_k", 0, hc.HC_EINVAL),
    ("window_mode", 3, hc.HC_EINVAL),
])
def test_bad_config_is_rejected_before_any_gpu_call(field, value, status):
    spec = I.spec_tiny(1024, budget=160, sink=16, recent=32)
    cfg = cfg_for(spec, **{field: value})
    descs, _, _ = R.make_descs(spec)
    with pytest.raises(hc.HcError) as e:
        hc.hc_plan_describe(cfg, descs)
    assert e.value.status == status
    h = C.c_void_p()
    assert hc.lib().hc_create(C.byref(cfg), C.byref(h)) == status and not h.value


def test_null_arguments():
    assert hc.lib().hc_create(None, None) == hc.HC_EINVAL
    assert hc.lib().hc_destroy(None) == hc.HC_ESTATE
    assert hc.lib().hc_layer_destroy(None) == hc.HC_ESTATE
    assert hc.lib().hc_decode_attn(None, None, None, None, None, None, None, None) == hc.HC_ESTATE
    assert hc.lib().hc_rep_topk_drift(None, None, None, None, None, 0, None, None, None, None, None, None) == hc.HC_ESTATE
    assert hc.lib().hc_gather_retrieve(None, None, None, None, None, None, None, None, None, None) == hc.HC_ESTATE
    assert hc.lib().hc_rescore_window(None, None, None, None, None, None, None, None, 0, None) == hc.HC_ESTATE
    assert hc.lib().hc_rescore_work_bytes(None, None) == 0 and hc.lib().hc_prefill_work_bytes(None, None) == 0
    assert hc.lib().hc_prefill_init(*([None] * 6 + [1] + [None] * 7 + [0, None])) == hc.HC_ESTATE
    assert hc.lib().hc_layer_window_slot(None) == -1 and hc.lib().hc_layer_set_window_slot(None, 0) == hc.HC_ESTATE
    assert hc.lib().hc_layer_num_reps(None) == -1


def mutate(descs, i, **kw):
    for k, v in kw.items():
        setattr(descs[i], k, v)
    return descs


@pytest.mark.parametrize("i,change,needle", [
    (1, dict(rep=1), "not a full head"),
    (1, dict(rep=5), "not a full head"),
    (0, dict(len=100), "len == ctx"),
    (1, dict(len=0), "len"),
    (1, dict(sink=600), "sink + recent"),
    (1, dict(k_off=3), "multiples of 8"),
    (1, dict(role=7), "bad role"),
    (1, dict(cap=5), "cap"),
    (1, dict(ctx=2048), "ctx"),
    (1, dict(k_off=0), "overlap"),
    (0, dict(k_mon=5000), "k_mon"),
])
def test_bad_head_tables_are_rejected(i, change, needle):
    spec = I.spec_tiny(4096)
    descs, _, _ = R.make_descs(spec)
    with pytest.raises(hc.HcError) as e:
        hc.hc_plan_describe(R.make_config(spec), mutate(descs, i, **change))
    assert needle in str(e.value)


def test_satellites_of_one_pivot_must_share_sink_and_recent():
    heads = [I.HeadSpec(I.ROLE_FULL), I.HeadSpec(I.ROLE_SATELLITE, rep=0, sink=64, recent=128, budget=512),
             I.HeadSpec(I.ROLE_SATELLITE, rep=0, sink=32, recent=128, budget=512)]
    spec = I.LayerSpec(B=1, Hq=12, Hkv=3, D=128, ctx=[4096], heads=[heads])
    descs, _, _ = R.make_descs(spec)
    with pytest.raises(hc.HcError) as e:
        hc.hc_plan_describe(R.make_config(spec), descs)
    assert "share sink and recent" in str(e.value)


def test_plan_of_the_224k_layer_is_balanced_and_covers_every_row():
    spec = I.spec_llama(I.CONFIG_CTX[4], I.CONFIG_BUDGETS[4])
    descs, arena, tier = R.make_descs(spec)
    assert arena * 2 == spec.kv_bytes() and tier * 2 == 6 * 229376 * 512
    info = hc.hc_plan_describe(R.make_config(spec), descs, compute_units=256, workgroups_per_cu=2)
    assert info.n_workgroups == 512
    assert info.total_rows == 2 * 229376 + 21504 == info.rows_covered
    assert info.n_reps == 2 and info.n_satellites == 6 and info.n_lists == 8
    assert info.n_partials <= 512 + 8
    # the shares are equal up to the built-in die / dispatch-slot weights (0.92 .. 1.08 of the mean), one
    # 32-row granule (+ the ragged tails of the heads a share crosses), and 96 rows less for every head
    # boundary inside a share (at most two here)
    mean = 480256 / 512
    assert 0.92 * mean - 64 - 2 * 96 <= info.min_rows_per_workgroup <= info.max_rows_per_workgroup <= 1.08 * mean + 64


@pytest.mark.parametrize("cus,wg", [(1, 1), (8, 2), (256, 2), (256, 8), (304, 4)])
def test_plan_covers_ragged_batch(cus, wg):
    spec = I.spec_ragged(77, B=5, lo=300, hi=9000)
    # make some lengths awkward: 1 row, 31, 33
    spec.ctx[0] = 1000
    descs, _, _ = R.make_descs(spec)
    info = hc.hc_plan_describe(R.make_config(spec), descs, compute_units=cus, workgroups_per_cu=wg)
    assert info.rows_covered == info.total_rows == sum(d.len for d in descs)
    assert 1 <= info.n_workgroups <= cus * wg
    assert info.n_partials >= 5 * 8


def test_single_row_heads():
    heads = [I.HeadSpec(I.ROLE_FULL), I.HeadSpec(I.ROLE_ANCHOR, sink=1, recent=0, budget=1)]
    spec = I.LayerSpec(B=1, Hq=8, Hkv=2, D=128, ctx=[1], heads=[heads])
    descs, _, _ = R.make_descs(spec)
    info = hc.hc_plan_describe(R.make_config(spec, max_ctx=64), descs)
    assert info.n_workgroups == 1 and info.n_partials == 2 and info.rows_covered == 2


def test_benchmark_refuses_more_than_one_gpu():
    """The build runs on one GPU; asking the benchmark for more ends with a message, before anything touches a GPU."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
