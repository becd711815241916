"""ctypes binding of the C ABI in include/hc.h: same names, argument marshalling only.

Every function takes torch tensors (or raw integer addresses) where the C call takes pointers
and raises ``HcError`` on a non-zero status.  Nothing is computed here and there is no fallback:
if the HIP library has not been built, loading fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence, Union

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhc.so")

HC_OK, HC_EINVAL, HC_ESHAPE, HC_ENOMEM, HC_EHIP, HC_ESTATE = range(6)
HC_MAX_WINDOW, HC_MAX_K_PER_REP, HC_MAX_GROUP = 64, 8, 8
HC_STATIC_MAX_PARTIALS = 1024

EXPORTS = ["hc_create", "hc_destroy", "hc_strerror", "hc_last_error", "hc_layer_create", "hc_layer_destroy",
           "hc_layer_num_reps", "hc_layer_rep_slot", "hc_layer_num_workgroups", "hc_layer_num_partials",
           "hc_set_split", "hc_set_gather_shape", "hc_set_side_lds", "hc_set_logit_filter", "hc_layer_monitor_counts", "hc_layer_filter_view", "hc_set_share_weights", "hc_get_share_weights", "hc_layer_tune", "hc_set_monitor_span",
           "hc_set_timing_events", "hc_plan_describe", "hc_decode_attn", "hc_decode_attn_static", "hc_rep_topk_drift", "hc_gather_retrieve",
           "hc_append_kv", "hc_rescore_work_bytes", "hc_rescore_work_layout", "hc_rescore_window", "hc_prefill_work_bytes", "hc_prefill_work_layout", "hc_prefill_init",
           "hc_layer_window_slot",
           "hc_layer_set_window_slot", "hc_layer_context",
           "hc_decode_step", "hc_taxonomy", "hc_budgets", "hc_probe_stream_read", "hc_probe_host_copy"]


HC_WINDOW_SLIDING, HC_WINDOW_TUMBLING, HC_WINDOW_RESCORED = 0, 1, 2


class hc_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("B", "Hq", "Hkv", "D", "max_ctx", "max_k", "window", "metric",
                                         "tau_num", "tau_den", "agg", "window_mode")]


class hc_head_desc(C.Structure):
    _fields_ = [("k_off", C.c_int64), ("v_off", C.c_int64), ("tier_off", C.c_int64),
                ("ctx", C.c_int32), ("len", C.c_int32), ("role", C.c_int32), ("rep", C.c_int32),
                ("sink", C.c_int32), ("recent", C.c_int32), ("k_mon", C.c_int32), ("cap", C.c_int32)]


class hc_plan_info(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_workgroups", "n_partials", "n_reps", "n_lists", "n_satellites",
                                         "max_rows_per_workgroup", "min_rows_per_workgroup", "reserved")] + \
               [("total_rows", C.c_int64), ("rows_covered", C.c_int64)]


class hc_layer_io(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("layer", "kv_arena", "host_tier", "q", "out", "lse", "rep_logits", "scores",
                                          "topk_idx", "base_idx", "ring", "inter", "flag", "slot_pos", "k_new", "v_new",
                                          "q_window", "rescore_work")] + [("rescore_work_bytes", C.c_size_t)]


class HcError(RuntimeError):
    def __init__(self, status: int, where: str, detail: str = ""):
        self.status = status
        super().__init__(f"{where}: status {status} ({_strerror(status)}){': ' + detail if detail else ''}")


_lib = None


def lib():
    """The loaded HIP library.  Raises if it has not been built (no CPU fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2601_13684_amd.build` "
                               "(hipcc, gfx950); this package has no other execution path")
        L = C.CDLL(LIB_PATH)
        vp, i32 = C.c_void_p, C.c_int32
        L.hc_create.argtypes = [C.POINTER(hc_config), C.POINTER(vp)]
        L.hc_destroy.argtypes = [vp]
        L.hc_strerror.argtypes = [C.c_int]
        L.hc_strerror.restype = C.c_char_p
        L.hc_last_error.argtypes = [vp]
        L.hc_last_error.restype = C.c_char_p
        L.hc_layer_create.argtypes = [vp, C.POINTER(hc_head_desc), C.POINTER(vp)]
        L.hc_layer_destroy.argtypes = [vp]
        for n in ("hc_layer_num_reps", "hc_layer_num_workgroups", "hc_layer_num_partials"):
            getattr(L, n).argtypes = [vp]
            getattr(L, n).restype = i32
        L.hc_layer_rep_slot.argtypes = [vp, i32, i32]
        L.hc_layer_rep_slot.restype = i32
        L.hc_set_split.argtypes = [vp, i32, i32]
        L.hc_set_logit_filter.argtypes = [vp, C.c_float, i32]
        L.hc_set_gather_shape.argtypes = [vp, i32, i32]
        L.hc_set_side_lds.argtypes = [vp, i32]
        L.hc_layer_monitor_counts.argtypes = [vp, i32, i32, C.POINTER(C.c_uint32)]
        L.hc_layer_filter_view.argtypes = [vp, C.POINTER(vp), C.POINTER(vp)]
        L.hc_set_share_weights.argtypes = [vp, C.POINTER(C.c_float)]
        L.hc_set_monitor_span.argtypes = [vp, i32]
        L.hc_get_share_weights.argtypes = [vp, C.POINTER(C.c_float)]
        L.hc_rescore_work_bytes.argtypes = [vp, vp]
        L.hc_rescore_work_bytes.restype = C.c_size_t
        L.hc_rescore_work_layout.argtypes = [vp, vp, C.POINTER(i32)] + [C.POINTER(C.c_size_t)] * 4
        L.hc_rescore_window.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
        L.hc_prefill_work_bytes.argtypes = [vp, vp]
        L.hc_prefill_work_bytes.restype = C.c_size_t
        L.hc_prefill_work_layout.argtypes = [vp, vp, C.POINTER(i32), C.POINTER(i32)] + [C.POINTER(C.c_size_t)] * 3
        L.hc_prefill_init.argtypes = [vp, vp, vp, C.POINTER(C.c_int64), C.POINTER(C.c_int64), vp, i32, vp, vp, vp, vp, vp, vp, vp,
                                      C.c_size_t, vp]
        L.hc_layer_window_slot.argtypes = [vp]
        L.hc_layer_window_slot.restype = i32
        L.hc_layer_set_window_slot.argtypes = [vp, i32]
        L.hc_layer_tune.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, vp]
        L.hc_set_timing_events.argtypes = [vp, vp, vp, i32]
        L.hc_plan_describe.argtypes = [C.POINTER(hc_config), C.POINTER(hc_head_desc), i32, i32,
                                       C.POINTER(hc_plan_info), C.c_char_p, i32]
        L.hc_decode_attn.argtypes = [vp] * 8
        L.hc_decode_attn_static.argtypes = [vp] * 8
        L.hc_rep_topk_drift.argtypes = [vp, vp, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp]
        L.hc_gather_retrieve.argtypes = [vp] * 10
        L.hc_append_kv.argtypes = [vp] * 7
        L.hc_taxonomy.argtypes = [i32, vp, vp, C.c_double, vp, vp, vp]
        L.hc_budgets.argtypes = [i32, vp, vp, i32, i32, i32, vp]
        L.hc_probe_stream_read.argtypes = [vp, C.c_size_t, vp, i32, i32, vp]
        L.hc_probe_host_copy.argtypes = [vp, vp, C.c_size_t, i32, vp]
        L.hc_layer_context.argtypes = [vp, i32]
        L.hc_layer_context.restype = i32
        L.hc_decode_step.argtypes = [vp, C.POINTER(hc_layer_io), i32, i32, vp, vp]
        for n in EXPORTS:
            if n not in ("hc_strerror", "hc_last_error", "hc_layer_num_reps", "hc_layer_rep_slot",
                         "hc_layer_num_workgroups", "hc_layer_num_partials", "hc_rescore_work_bytes", "hc_prefill_work_bytes",
                         "hc_layer_window_slot"):
                getattr(L, n).restype = C.c_int
        _lib = L
    return _lib


def _strerror(st: int) -> str:
    try:
        return lib().hc_strerror(st).decode()
    except Exception:
        return "?"


Ptr = Union[torch.Tensor, int, None]


def _p(x: Ptr) -> Optional[int]:
    if x is None:
        return None
    if isinstance(x, torch.Tensor):
        assert x.is_contiguous(), "tensors handed to the C ABI must be contiguous"
        return x.data_ptr()
    return int(x)


def _stream(s) -> Optional[int]:
    if s is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(s, torch.cuda.Stream):
        return s.cuda_stream
    return int(s)


def _event(e) -> Optional[int]:
    if e is None:
        return None
    if isinstance(e, torch.cuda.Event):
        h = e.cuda_event
        if not h:
            raise ValueError("torch.cuda.Event has no HIP event yet: record it once before handing it to the C ABI")
        return h
    return int(e)


def _check(st: int, where: str, ctx=None):
    if st != HC_OK:
        detail = lib().hc_last_error(ctx).decode() if ctx else ""
        raise HcError(st, where, detail)


def hc_create(cfg: hc_config) -> int:
    h = C.c_void_p()
    _check(lib().hc_create(C.byref(cfg), C.byref(h)), "hc_create")
    return h.value


def hc_destroy(ctx: int) -> None:
    _check(lib().hc_destroy(ctx), "hc_destroy")


def hc_set_split(ctx: int, workgroups_per_cu: int = 2, compute_units: int = 0) -> None:
    _check(lib().hc_set_split(ctx, workgroups_per_cu, compute_units), "hc_set_split", ctx)


def hc_set_logit_filter(ctx: int, margin: float, min_candidates: int = 0) -> None:
    _check(lib().hc_set_logit_filter(ctx, float(margin), int(min_candidates)), "hc_set_logit_filter", ctx)


def hc_set_gather_shape(ctx: int, workgroups: int = 96, threads: int = 256) -> None:
    _check(lib().hc_set_gather_shape(ctx, workgroups, threads), "hc_set_gather_shape", ctx)


def hc_set_side_lds(ctx: int, nbytes: int) -> None:
    _check(lib().hc_set_side_lds(ctx, int(nbytes)), "hc_set_side_lds", ctx)


def hc_layer_monitor_counts(layer: int, b: int, h: int) -> dict:
    out = (C.c_uint32 * 4)()
    _check(lib().hc_layer_monitor_counts(layer, b, h, out), "hc_layer_monitor_counts")
    return dict(tests=int(out[0]), triggers=int(out[1]), fallbacks=int(out[2]), kept=None if out[3] == 0xffffffff else int(out[3]))


def hc_layer_filter_view(layer: int):
    """(device address of kept_pos [num_reps][max_ctx] int32, of fell_back [num_reps] int32); (None, None): no filter."""
    a, b = C.c_void_p(), C.c_void_p()
    _check(lib().hc_layer_filter_view(layer, C.byref(a), C.byref(b)), "hc_layer_filter_view")
    return a.value, b.value


def hc_set_share_weights(ctx: int, weights=None) -> None:
    """weights: 16 floats [die * 2 + slot], or None for the built-in defaults."""
    arr = None
    if weights is not None:
        if len(weights) != 16:
            raise ValueError("hc_set_share_weights: 16 weights")
        arr = (C.c_float * 16)(*[float(w) for w in weights])
    _check(lib().hc_set_share_weights(ctx, arr), "hc_set_share_weights", ctx)


def hc_get_share_weights(ctx: int) -> list:
    w = (C.c_float * 16)()
    _check(lib().hc_get_share_weights(ctx, w), "hc_get_share_weights", ctx)
    return [float(x) for x in w]


def hc_layer_tune(ctx: int, layer: int, kv_arena: Ptr, q: Ptr, out: Ptr, lse: Ptr, rep_logits: Ptr = None, rounds: int = 4,
                  stream=None) -> None:
    _check(lib().hc_layer_tune(ctx, layer, _p(kv_arena), _p(q), _p(out), _p(lse), _p(rep_logits), rounds, _stream(stream)),
           "hc_layer_tune", ctx)


def hc_set_monitor_span(ctx: int, span: int = 0) -> None:
    _check(lib().hc_set_monitor_span(ctx, span), "hc_set_monitor_span", ctx)


def hc_set_timing_events(ctx: int, ev_begin=(), ev_end=()) -> None:
    """ev_begin / ev_end: equally long sequences of torch.cuda.Event (timing enabled, recorded once)."""
    n = len(ev_begin)
    if len(ev_end) != n:
        raise ValueError("hc_set_timing_events: sequences of equal length")
    arr_b = (C.c_void_p * max(n, 1))(*[_event(e) for e in ev_begin])
    arr_e = (C.c_void_p * max(n, 1))(*[_event(e) for e in ev_end])
    _check(lib().hc_set_timing_events(ctx, arr_b if n else None, arr_e if n else None, n), "hc_set_timing_events", ctx)


def hc_plan_describe(cfg: hc_config, heads: Sequence[hc_head_desc], compute_units: int = 256,
                     workgroups_per_cu: int = 2) -> hc_plan_info:
    arr = (hc_head_desc * len(heads))(*heads)
    info = hc_plan_info()
    err = C.create_string_buffer(512)
    st = lib().hc_plan_describe(C.byref(cfg), arr, compute_units, workgroups_per_cu, C.byref(info), err, 512)
    if st != HC_OK:
        raise HcError(st, "hc_plan_describe", err.value.decode())
    return info


def hc_layer_create(ctx: int, heads: Sequence[hc_head_desc]) -> int:
    arr = (hc_head_desc * len(heads))(*heads)
    h = C.c_void_p()
    _check(lib().hc_layer_create(ctx, arr, C.byref(h)), "hc_layer_create", ctx)
    return h.value


def hc_layer_destroy(layer: int) -> None:
    _check(lib().hc_layer_destroy(layer), "hc_layer_destroy")


def hc_layer_num_reps(layer: int) -> int:
    return lib().hc_layer_num_reps(layer)


def hc_layer_rep_slot(layer: int, b: int, h: int) -> int:
    return lib().hc_layer_rep_slot(layer, b, h)


def hc_layer_num_workgroups(layer: int) -> int:
    return lib().hc_layer_num_workgroups(layer)


def hc_layer_num_partials(layer: int) -> int:
    return lib().hc_layer_num_partials(layer)


def hc_decode_attn(ctx: int, layer: int, kv_arena: Ptr, q: Ptr, out: Ptr, lse: Ptr, rep_logits: Ptr = None,
                   stream=None) -> None:
    _check(lib().hc_decode_attn(ctx, layer, _p(kv_arena), _p(q), _p(out), _p(lse), _p(rep_logits), _stream(stream)),
           "hc_decode_attn", ctx)


def hc_decode_attn_static(ctx: int, layer: int, kv_arena: Ptr, q: Ptr, out: Ptr, lse: Ptr, rep_logits: Ptr = None,
                          stream=None) -> None:
    _check(lib().hc_decode_attn_static(ctx, layer, _p(kv_arena), _p(q), _p(out), _p(lse), _p(rep_logits), _stream(stream)),
           "hc_decode_attn_static", ctx)


def hc_rep_topk_drift(ctx: int, layer: int, rep_logits: Ptr, lse: Ptr, scores: Ptr, scores_given: bool,
                      topk_idx: Ptr, base_idx: Ptr, ring: Ptr, inter: Ptr, flag: Ptr, stream=None) -> None:
    _check(lib().hc_rep_topk_drift(ctx, layer, _p(rep_logits), _p(lse), _p(scores), int(bool(scores_given)),
                                   _p(topk_idx), _p(base_idx), _p(ring), _p(inter), _p(flag), _stream(stream)),
           "hc_rep_topk_drift", ctx)


def hc_gather_retrieve(ctx: int, layer: int, host_tier: Ptr, topk_idx: Ptr, flag: Ptr, kv_arena: Ptr,
                       slot_pos: Ptr = None, stream=None, wait_event=None, done_event=None) -> None:
    _check(lib().hc_gather_retrieve(ctx, layer, _p(host_tier), _p(topk_idx), _p(flag), _p(kv_arena), _p(slot_pos),
                                    _stream(stream), _event(wait_event), _event(done_event)),
           "hc_gather_retrieve", ctx)


def hc_append_kv(ctx: int, layer: int, k_new: Ptr, v_new: Ptr, kv_arena: Ptr, host_tier: Ptr = None, stream=None) -> None:
    _check(lib().hc_append_kv(ctx, layer, _p(k_new), _p(v_new), _p(kv_arena), _p(host_tier), _stream(stream)),
           "hc_append_kv", ctx)


def hc_rescore_work_bytes(ctx: int, layer: int) -> int:
    return int(lib().hc_rescore_work_bytes(ctx, layer))


def hc_rescore_work_layout(ctx: int, layer: int) -> dict:
    """Where the first pass's results lie inside the work buffer (byte offsets) and how many queries a pass holds."""
    n = C.c_int32(0)
    off = [C.c_size_t(0) for _ in range(4)]
    _check(lib().hc_rescore_work_layout(ctx, layer, C.byref(n), *[C.byref(o) for o in off]), "hc_rescore_work_layout", ctx)
    return dict(items_per_pass=n.value, logits=off[0].value, scores=off[1].value, lse=off[2].value, topk=off[3].value)


def hc_rescore_window(ctx: int, layer: int, kv_arena: Ptr, q: Ptr, q_window: Ptr, base_idx: Ptr, ring: Ptr,
                      work: Ptr, work_bytes: int, stream=None) -> None:
    _check(lib().hc_rescore_window(ctx, layer, _p(kv_arena), _p(q), _p(q_window), _p(base_idx), _p(ring), _p(work),
                                   work_bytes, _stream(stream)), "hc_rescore_window", ctx)


def hc_prefill_work_bytes(ctx: int, layer: int) -> int:
    return int(lib().hc_prefill_work_bytes(ctx, layer))


def hc_prefill_work_layout(ctx: int, layer: int, n_heads: int) -> dict:
    n = C.c_int32(0)
    head_of = (C.c_int32 * n_heads)()
    off = [C.c_size_t(0) for _ in range(3)]
    _check(lib().hc_prefill_work_layout(ctx, layer, C.byref(n), head_of, *[C.byref(o) for o in off]), "hc_prefill_work_layout", ctx)
    return dict(heads=[int(head_of[i]) for i in range(n.value)], logits=off[0].value, scores=off[1].value, lse=off[2].value)


def hc_prefill_init(ctx: int, layer: int, kv_prefill: Ptr, k_src_off, v_src_off, q_last: Ptr, pool: int, kv_arena: Ptr,
                    host_tier: Ptr, topk_idx: Ptr, base_idx: Ptr, slot_pos: Ptr, ring: Ptr, work: Ptr, work_bytes: int,
                    stream=None) -> None:
    n = len(k_src_off)
    ko = (C.c_int64 * n)(*[int(x) for x in k_src_off])
    vo = (C.c_int64 * n)(*[int(x) for x in v_src_off])
    _check(lib().hc_prefill_init(ctx, layer, _p(kv_prefill), ko, vo, _p(q_last), pool, _p(kv_arena), _p(host_tier), _p(topk_idx),
                                 _p(base_idx), _p(slot_pos), _p(ring), _p(work), work_bytes, _stream(stream)), "hc_prefill_init", ctx)


def hc_layer_window_slot(layer: int) -> int:
    return lib().hc_layer_window_slot(layer)


def hc_layer_set_window_slot(layer: int, slot: int) -> None:
    _check(lib().hc_layer_set_window_slot(layer, slot), "hc_layer_set_window_slot")


def hc_layer_context(layer: int, b: int) -> int:
    return lib().hc_layer_context(layer, b)


def hc_probe_stream_read(dev_buf: Ptr, nbytes: int, dev_sink: Ptr = None, workgroups: int = 2048, streaming: bool = True,
                         stream=None) -> None:
    _check(lib().hc_probe_stream_read(_p(dev_buf), nbytes, _p(dev_sink), workgroups, int(bool(streaming)), _stream(stream)),
           "hc_probe_stream_read")


def hc_probe_host_copy(pinned_src: Ptr, dev_dst: Ptr, nbytes: int, workgroups: int = 96, stream=None) -> None:
    _check(lib().hc_probe_host_copy(_p(pinned_src), _p(dev_dst), nbytes, workgroups, _stream(stream)), "hc_probe_host_copy")


def hc_decode_step(ctx: int, io, n_layers: int, main_stream=None, side_stream=None, layers_per_group: int = 4) -> None:
    """io: a ctypes array of hc_layer_io (build it once and reuse it: the q pointers may stay fixed)."""
    _check(lib().hc_decode_step(ctx, io, n_layers, layers_per_group, _stream(main_stream),
                                None if side_stream is None else _stream(side_stream)), "hc_decode_step", ctx)
