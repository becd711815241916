#!/usr/bin/env python3
"""Benchmark of the HeteroCache decode hot path on one MI355X.

A "step" is one decode step of the whole stack: for every layer, attention over the heterogeneous
cache (hc_decode_attn), the pivot drift monitor (hc_rep_topk_drift) and the device-predicated
host-tier gather (hc_gather_retrieve, on a side stream).  The default workload is synthetic config 4:
32 layers, batch 1, 32 query / 8 KV heads, head_dim 128, 224K context; per layer 2 full KV heads and
6 compressed heads with budgets {8192, 4096, 4096, 2048, 2048, 1024}; bf16 K/V resident in HBM, the
satellites' full K/V in pinned host memory; the query jumps every 16 steps so that every pivot
triggers a refill then.

Prints ONE JSON line.  `value` = microseconds per decode step per layer (wall clock over the timed
steps / steps / layers).  `roofline` times the split-pass attention kernel alone with HIP events
recorded by the library around that kernel, on the stream it is launched on.  `cpu_baseline` times
the CPU oracle on a small sample of the same workload (a reported baseline, not a target).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "µs per decode step per layer + achieved HBM GB/s at 224K context, 1 GPU"
HBM_PEAK_GBPS = 8000.0
# HBM traffic of one launch of the split kernel (bytes), from the hardware counters FETCH_SIZE and
# WRITE_SIZE of profiler runs of this script, scaled by what the same counters read for the streaming
# kernel of --calibrate-copy; keyed by (config, dense, pivot-logit filter on).  The runs and factors are in profiles/.
MEASURED_TRAFFIC = {(4, False, True): 249581207, (4, False, False): 254641233}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=48)
    ap.add_argument("--warmup", type=int, default=4)
    ap.add_argument("--config", type=int, default=4, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--layers", type=int, default=0, help="0 = the config's own layer count")
    ap.add_argument("--ctx", type=int, default=0, help="override the context length (testing)")
    ap.add_argument("--mode", default="step", choices=["step", "graph", "eager"],
                    help="step: hc_decode_step (native launch loop, two streams); graph: captured HIP graph; eager: Python loop")
    ap.add_argument("--dense", action="store_true", help="uncompressed comparison: all 8 KV heads full")
    ap.add_argument("--no-tier", action="store_true", help="no host tier / gather (attention + monitor only)")
    ap.add_argument("--append", action="store_true", help="every step appends the generated token's K/V first (growing context)")
    ap.add_argument("--full-gather", action="store_true", help="refills fetch whole lists (no slot map: nothing is kept)")
    ap.add_argument("--wg-per-cu", type=int, default=0)
    ap.add_argument("--dump-kernel-times", default="", help="write the split kernel's per-launch durations (us, launch order) to this file")
    ap.add_argument("--prefill-init", type=int, default=0, help="odd P >= 1: every layer's initial state is built by the library from "
                    "the full K/V and the last prompt token's queries (hc_prefill_init, pooling width P) instead of the positional "
                    "fill, and the call is timed (prefill_init_ms_per_layer)")
    ap.add_argument("--window", type=int, default=0, help="W of the drift test (0: the config's, which is 1)")
    ap.add_argument("--window-mode", type=int, default=-1, help="0 sliding (Eq. 10), 1 tumbling, 2 tumbling with the window's "
                    "queries scored again at the test step (Algorithm 1); -1: the config's (sliding)")
    ap.add_argument("--monitor-span", type=int, default=0, help="1024-candidate chunks per workgroup of the selection passes (0: chosen per launch)")
    ap.add_argument("--tune-rounds", type=int, default=0, help="rounds of on-device measurement of the share weights on the first layer (0: built-in weights, as the parity tests use)")
    ap.add_argument("--share-weights", default="", help="16 comma-separated share weights [die*2+slot] (tuning)")
    ap.add_argument("--filter-margin", type=float, default=-1.0, help="pivot-logit filter (hc_set_logit_filter): 0 = off, every "
                    "logit of a pivot is stored and scored; >= 1: only the rows that can reach a list, checked on the device; "
                    "-1 (default): 1.25")
    ap.add_argument("--filter-min-candidates", type=int, default=65536, help="layers whose pivots all have fewer candidate positions "
                    "than this do not filter (the filtered monitor costs more launches, which a short context does not earn back)")
    ap.add_argument("--side-lds", type=int, default=-1, help="KB of LDS every side-stream workgroup reserves (hc_set_side_lds; tuning; "
                    "-1: the library's default of 81, 0: none)")
    ap.add_argument("--gather-shape", default="", help="workgroups,threads of the gather kernel (tuning; default 96,256)")
    ap.add_argument("--group", type=int, default=0, help="layers per cross-stream sync group in step mode (0: half of the "
                    "stack, at most 8, so that the side work of all but the last group overlaps later groups' attention)")
    ap.add_argument("--serial", action="store_true", help="monitor and gather on the main stream (no overlap)")
    ap.add_argument("--attn-only", action="store_true", help="time hc_decode_attn alone (no monitor, no gather)")
    ap.add_argument("--oracle-seconds", type=float, default=12.0)
    ap.add_argument("--no-oracle", action="store_true")
    ap.add_argument("--no-probes", action="store_true", help="skip the streaming-read / host-link probes and the gather-alone pass")
    ap.add_argument("--no-kernel-timing", action="store_true", help="skip the pass that times the split kernel")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MiB",
                    help="first run 8 plain streaming kernels (out = in + 1 over MiB of fp32 in, MiB out) so that a "
                         "counter run can scale FETCH_SIZE / WRITE_SIZE by a kernel of known traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2601_13684_amd import binding as hc
    from paper_2601_13684_amd import inputs as I
    from paper_2601_13684_amd import runtime as R

    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        n = args.calibrate_copy * (1 << 20) // 4
        src = torch.ones((n,), dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(8):
            torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst
    L = args.layers or I.CONFIG_LAYERS[args.config]
    if args.group == 0:
        args.group = max(1, min(8, L // 2))
    K, W = args.steps, args.warmup
    T_total = W + 2 * K + 9           # warm-up, timed pass, kernel-timing pass, comparison pass
    t_setup = time.time()

    # ---- build the stack, layer by layer (masters are dropped once packed) ----
    layers, scheds, keep = [], [], {}
    prefill_ms = []
    ctx = None
    for l in range(L):
        extra = {}
        if args.config == 5 and layers:
            extra["ctx"] = layers[0].spec.ctx        # one batch: every layer sees the same sequences; roles are drawn per layer
        w = I.make_workload(args.config, layer=l, device=dev, N=args.ctx or None, **extra)
        spec = w.spec
        if args.dense:
            spec = I.spec_dense(spec.ctx[0])
        if args.window:
            spec.window = args.window
        if args.window_mode >= 0:
            spec.window_mode = args.window_mode
        if ctx is None:
            if args.filter_margin < 0:
                args.filter_margin = 1.25
            cfg = R.make_config(spec, growth=T_total if args.append else 0)
            if args.config == 5:
                cfg.max_k = 4096 - 64 - 256          # the largest list any layer of this config can draw
            ctx = R.Context(cfg, dev, workgroups_per_cu=args.wg_per_cu or None, filter_margin=args.filter_margin,
                            filter_min_candidates=args.filter_min_candidates)
            if args.share_weights:
                hc.hc_set_share_weights(ctx.handle, [float(x) for x in args.share_weights.split(",")])
            if args.monitor_span:
                hc.hc_set_monitor_span(ctx.handle, args.monitor_span)
            if args.gather_shape:
                hc.hc_set_gather_shape(ctx.handle, *[int(x) for x in args.gather_shape.split(",")])
            if args.side_lds < 0:
                args.side_lds = 81
            hc.hc_set_side_lds(ctx.handle, args.side_lds * 1024)
        retrieved, base = I.initial_lists(spec)
        pre = None
        if args.prefill_init:
            pre = (w.schedule.q.to(torch.bfloat16).to(dev), args.prefill_init)
        layers.append(R.LayerRuntime(ctx, spec, w.data, retrieved, base, host_tier=not args.no_tier, own_scratch=True,
                                     delta_gather=not args.full_gather, growth=T_total if args.append else 0, prefill=pre))
        if pre is not None:
            # timed a second time (the first call paid the first-touch costs); the state comes out the same
            ev = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
            torch.cuda.synchronize()
            ev[0].record()
            layers[-1].prefill_init(None, pre[0], pre[1])
            ev[1].record()
            torch.cuda.synchronize()
            prefill_ms.append(ev[0].elapsed_time(ev[1]))
            del layers[-1].kv_prefill, layers[-1].prefill_work
            if l < 2 and not args.no_oracle:
                from oracle import prefill as oracle_prefill
                cpu_data = I.LayerData({k: v.cpu() for k, v in w.data.K.items()}, {k: v.cpu() for k, v in w.data.V.items()}, {})
                r_np, b_np, _ = oracle_prefill.prefill_init(spec, cpu_data, pre[0].cpu(), pre[1])
                retrieved = {k: torch.from_numpy(v) for k, v in r_np.items()}
                base = {k: torch.from_numpy(v) for k, v in b_np.items()}
        if l == 0 and args.tune_rounds and not args.share_weights:
            layers[0].tune(w.schedule.q.to(torch.bfloat16).to(dev), args.tune_rounds)       # untimed set-up
            print("[bench] share weights " + " ".join(f"{x:.3f}" for x in hc.hc_get_share_weights(ctx.handle)), file=sys.stderr, flush=True)
        scheds.append(w.schedule)
        if l < 2 and not args.no_oracle:
            keep[l] = (spec, I.LayerData({k: v.cpu() for k, v in w.data.K.items()},
                                         {k: v.cpu() for k, v in w.data.V.items()}, {}), retrieved, base)
        del w
        print(f"[bench] layer {l + 1}/{L} packed ({time.time() - t_setup:.0f}s)", file=sys.stderr, flush=True)
    spec0 = layers[0].spec
    kv_bytes = int(sum(lay.spec.kv_bytes() for lay in layers) // len(layers))      # (config 5 draws the roles per layer)
    Q_all = torch.stack([torch.stack([s.next() for s in scheds]) for _ in range(T_total)]).contiguous()   # [T,L,B,Hq,D]
    q_cur = Q_all[0].clone()
    KV_new = None
    if args.append:       # the generated tokens' K/V rows: [T, 2, L, B, Hkv, D]
        gk = torch.Generator(device=dev)
        gk.manual_seed(4242)
        KV_new = torch.randn((T_total, 2, L, spec0.B, spec0.Hkv, 128), generator=gk, device=dev).to(torch.bfloat16)
        kv_cur = KV_new[0].clone()
    t_dev = torch.zeros((1,), dtype=torch.long, device=dev)
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    setup_s = time.time() - t_setup

    # Every step's queries (and generated tokens) are resident in HBM before the timed region.  A captured graph has
    # to pick the step's rows on the device (a gather into fixed buffers, part of the replayed work); the other modes
    # simply hand the library the step's rows.
    dev_index = args.mode == "graph"
    t_pos = [0]

    def load_q():
        q_cur.copy_(Q_all.index_select(0, t_dev)[0])
        if KV_new is not None:
            kv_cur.copy_(KV_new.index_select(0, t_dev)[0])
        t_dev.add_(1)

    def step_eager():
        if dev_index:
            load_q()
            q_t, kv_t = q_cur, (kv_cur if KV_new is not None else None)
        else:
            q_t, kv_t = Q_all[t_pos[0]], (KV_new[t_pos[0]] if KV_new is not None else None)
        t_pos[0] += 1
        for l, lay in enumerate(layers):
            if kv_t is not None:
                if lay._side_pending:
                    torch.cuda.current_stream().wait_event(lay.ev_done)
                lay.append(kv_t[0, l], kv_t[1, l])
            if args.attn_only:
                lay.attn(q_t[l], monitor=False)
            else:
                lay.step(q_t[l], side=None if args.serial else side)

    def step_for_capture():
        # the same calls; every layer's side-stream work (monitor, gather) is joined back before the step
        # ends, so that the captured graph is closed and a refill decided in this step is complete before
        # the next replay starts
        load_q()
        main = torch.cuda.current_stream()
        for l, lay in enumerate(layers):
            lay.attn(q_cur[l], monitor=not args.attn_only)
            if lay.n_reps and not args.attn_only:
                if args.serial:
                    lay.monitor()
                    if lay.tier is not None:
                        lay.gather()
                else:
                    lay.ev_topk.record(main)
                    side.wait_event(lay.ev_topk)
                    lay.monitor(stream=side)
                    if lay.tier is not None:
                        lay.gather(stream=side)
        if not args.attn_only and not args.serial:
            main.wait_stream(side)

    # ---- warm-up (eager) + optional parity spot check against the oracle on layer 0 ----
    flags_hist = []
    snap = {}
    for t in range(W):
        step_eager()
        torch.cuda.synchronize()
        flags_hist.append(int(sum(int(lay.flag.sum()) for lay in layers)))
        if t < 4 and 0 in keep:
            snap[t] = (layers[0].out.cpu().double().numpy(), layers[0].lse.cpu().double().numpy())

    # ---- timed region ----
    graph = None
    if args.mode == "step":
        io = R.make_step_io(layers, q_cur, monitor=not args.attn_only)
        main_s = torch.cuda.current_stream()
        q_base, q_step, q_layer = Q_all.data_ptr(), Q_all.stride(0) * 2, Q_all.stride(1) * 2
        if KV_new is not None:
            kv_base, kv_step, kv_which, kv_layer = KV_new.data_ptr(), KV_new.stride(0) * 2, KV_new.stride(1) * 2, KV_new.stride(2) * 2

        def run():
            t = t_pos[0]
            t_pos[0] += 1
            for l in range(L):
                io[l].q = q_base + t * q_step + l * q_layer
                if KV_new is not None:
                    io[l].k_new = kv_base + t * kv_step + l * kv_layer
                    io[l].v_new = kv_base + t * kv_step + kv_which + l * kv_layer
            hc.hc_decode_step(ctx.handle, io, L, main_s, None if (args.serial or args.attn_only) else side, args.group)
    elif args.mode == "graph":
        cap = torch.cuda.Stream()
        cap.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        t_keep = t_dev.clone()
        with torch.cuda.stream(cap):
            with torch.cuda.graph(graph, stream=cap):
                step_for_capture()
        t_dev.copy_(t_keep)               # capture does not execute; keep the schedule position
        torch.cuda.synchronize()
        run = graph.replay
    else:
        run = step_eager
    # one event between consecutive steps on the main stream: the distribution of the step time (GPU side)
    step_ev = [torch.cuda.Event(enable_timing=True) for _ in range(K + 1)]
    first_timed_t = t_pos[0] if args.mode != "graph" else W
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    step_ev[0].record()
    host_t = [t0]
    for i in range(K):
        run()
        step_ev[i + 1].record()
        host_t.append(time.perf_counter())
    t_host = host_t[-1]
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    step_ms = np.array([step_ev[i].elapsed_time(step_ev[i + 1]) for i in range(K)])
    host_enqueue_ms = (t_host - t0) * 1e3 / K
    # the first steps after the synchronisation are enqueued into empty queues: what a step costs the host when
    # nothing holds it back (later steps may wait for room in the queues, which then reads as host time)
    host_first_ms = float(np.median(np.diff(host_t[:min(K, 4) + 1])) * 1e3)
    ms_per_step = (t1 - t0) * 1e3 / K
    us_per_layer = ms_per_step * 1e3 / L

    # ---- kernel-timing pass: the same steps launched the same way, with one event pair attached to every
    # split-pass dispatch by the library (a captured graph cannot carry them: that mode is timed eagerly) ----
    n_pairs = 0 if args.no_kernel_timing else K * L
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_pairs)]
    for a, b in evs:
        a.record()
        b.record()
    torch.cuda.synchronize()
    if n_pairs:
        hc.hc_set_timing_events(ctx.handle, [a for a, _ in evs], [b for _, b in evs])
        timed_run = step_eager if args.mode == "graph" else run
        for _ in range(K):
            timed_run()
        hc.hc_set_timing_events(ctx.handle)
    torch.cuda.synchronize()
    kern_ms = np.array([a.elapsed_time(b) for a, b in evs]) if n_pairs else np.array([float("nan")])
    kern_us = float(kern_ms.mean() * 1e3)
    if args.dump_kernel_times and n_pairs:
        np.savetxt(args.dump_kernel_times, kern_ms.reshape(K, L) * 1e3, fmt="%.2f")
    achieved = kv_bytes / (kern_us * 1e-6) / 1e9

    # ---- for comparison: the same kernel with nothing else on the GPU (monitor and gather on the same stream,
    # so that no other kernel shares HBM with it), a few steps ----
    iso_us = None
    if n_pairs and args.mode == "step" and not (args.serial or args.attn_only):
        n_iso = min(K, 8)
        hc.hc_set_timing_events(ctx.handle, [a for a, _ in evs[:n_iso * L]], [b for _, b in evs[:n_iso * L]])
        for _ in range(n_iso):
            t = t_pos[0]
            t_pos[0] += 1
            for l in range(L):
                io[l].q = q_base + t * q_step + l * q_layer
                if KV_new is not None:
                    io[l].k_new = kv_base + t * kv_step + l * kv_layer
                    io[l].v_new = kv_base + t * kv_step + kv_which + l * kv_layer
            hc.hc_decode_step(ctx.handle, io, L, main_s, None, args.group)
        hc.hc_set_timing_events(ctx.handle)
        torch.cuda.synchronize()
        iso_us = float(np.mean([a.elapsed_time(b) for a, b in evs[:n_iso * L]]) * 1e3)

    # ---- step-time distribution (GPU side, events between steps of the timed region) ----
    def dist(a):
        a = np.asarray(a, dtype=np.float64)
        return {"n": int(a.size), "median": float(np.median(a)), "p95": float(np.percentile(a, 95)), "max": float(a.max())} if a.size else None
    jump_every = getattr(scheds[0], "jump_every", 0)
    kinds = []
    for i in range(K):
        t = first_timed_t + i                                    # index of the step's query in the schedule
        if jump_every and t > 0 and t % jump_every == 0:
            kinds.append("jump")                                 # every pivot of every layer fires and refills
        elif jump_every and t > 1 and (t - 1) % jump_every == 0:
            kinds.append("after_jump")                           # its attention waits for the refills of the jump step
        elif args.append and (t + 1) % 64 == 0:
            kinds.append("replan")                               # the split-K plans are rebalanced on the host
        else:
            kinds.append("plain")
    step_stats = {"unit": "ms per decode step (all layers)", "all": dist(step_ms)}
    for kind in ("plain", "jump", "after_jump", "replan"):
        sel = [step_ms[i] for i in range(K) if kinds[i] == kind]
        if sel:
            step_stats[kind] = dist(sel)
    if "after_jump" in step_stats and "plain" in step_stats:
        # what the step after a refill loses against an ordinary step: waiting for the refill (lag 1) shows here
        step_stats["stall_ms_after_jump"] = max(0.0, step_stats["after_jump"]["median"] - step_stats["plain"]["median"])

    # ---- what the machine gives: streaming-read rate of HBM, rates of the host link ----
    probes = {}
    if not args.no_probes:
        ev_a, ev_b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        sink = torch.zeros((4,), dtype=torch.int32, device=dev)
        # HBM: one streaming read of every layer's arena in turn (the stack is far larger than the last-level cache),
        # for a few launch shapes and both kinds of load; the best is what a kernel can get out of this machine
        arenas = [lay.arena for lay in layers]
        reps = max(1, 32 // len(arenas))
        nbytes = reps * sum(a.numel() * 2 for a in arenas)
        sweep = {}
        for nt in (True, False):
            for wg in (1024, 2048, 8192):
                for a in arenas[:2]:
                    hc.hc_probe_stream_read(a, a.numel() * 2, sink, wg, nt)
                torch.cuda.synchronize()
                ev_a.record()
                for _ in range(reps):
                    for a in arenas:
                        hc.hc_probe_stream_read(a, a.numel() * 2, sink, wg, nt)
                ev_b.record()
                torch.cuda.synchronize()
                sweep[f"{'streaming' if nt else 'plain'}_loads_{wg}wg"] = nbytes / (ev_a.elapsed_time(ev_b) * 1e-3) / 1e9
        probes["stream_read_sweep_GBps"] = sweep
        probes["stream_read_GBps"] = max(sweep.values())
        probes["stream_read_bytes_per_launch"] = int(arenas[0].numel() * 2)
        probes["stream_read_us_per_launch"] = probes["stream_read_bytes_per_launch"] / probes["stream_read_GBps"] * 1e-3
        tier0 = next((lay.tier for lay in layers if lay.tier is not None), None)
        if tier0 is not None:
            # host link: plain pinned host-to-device copies of growing size, and a kernel that reads pinned memory
            n_max = min(tier0.numel(), 128 << 20)                # up to 256 MB of bf16
            dst = torch.empty((n_max,), dtype=torch.bfloat16, device=dev)
            sweep = {}
            for mib in (1, 4, 16, 64, 256):
                n = min(n_max, mib << 19)
                dst[:n].copy_(tier0[:n], non_blocking=True)
                torch.cuda.synchronize()
                r = 4 if mib < 64 else 2
                ev_a.record()
                for _ in range(r):
                    dst[:n].copy_(tier0[:n], non_blocking=True)
                ev_b.record()
                torch.cuda.synchronize()
                sweep[f"{n * 2 >> 20}MiB"] = r * n * 2 / (ev_a.elapsed_time(ev_b) * 1e-3) / 1e9
            probes["host_to_device_copy_GBps"] = sweep
            ksweep = {}
            for wg in (48, 96, 192, 512):
                hc.hc_probe_host_copy(tier0, dst, n_max * 2, wg)
                torch.cuda.synchronize()
                ev_a.record()
                hc.hc_probe_host_copy(tier0, dst, n_max * 2, wg)
                ev_b.record()
                torch.cuda.synchronize()
                ksweep[f"{wg}wg"] = n_max * 2 / (ev_a.elapsed_time(ev_b) * 1e-3) / 1e9
            probes["kernel_read_of_pinned_GBps"] = ksweep
            probes["link_peak_GBps"] = max(max(sweep.values()), max(ksweep.values()))
            del dst

    # ---- the gather alone: a whole-list refill and a difference-only refill of known size, per layer ----
    gather = None
    sat_layers = [lay for lay in layers[:8] if lay.tier is not None and lay.n_reps]
    if sat_layers and not args.no_probes and not args.attn_only:
        ev_a, ev_b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        Hkv = spec0.Hkv

        def sat_rows(lay):
            return [(b * Hkv + h, lay.spec.r(b, h), lay.spec.ctx[b], lay.spec.heads[b][h]) for b in range(lay.spec.B)
                    for h in range(Hkv) if lay.spec.heads[b][h].role == I.ROLE_SATELLITE and lay.spec.r(b, h) > 0]
        torch.cuda.synchronize()
        for lay in sat_layers:
            lay.flag.fill_(1)
        # (a) whole lists: every retrieved slot of every satellite is fetched again (no slot map)
        rows_full = sum(r for lay in sat_layers for _, r, _, _ in sat_rows(lay))
        torch.cuda.synchronize()
        ev_a.record()
        for lay in sat_layers:
            hc.hc_gather_retrieve(ctx.handle, lay.handle, lay.tier, lay.topk_idx, lay.flag, lay.arena, None)
        ev_b.record()
        torch.cuda.synchronize()
        us_full = ev_a.elapsed_time(ev_b) * 1e3
        rows_delta = 0
        us_delta = None
        if all(lay.slot_pos is not None for lay in sat_layers):
            # the slots now hold the lists in list order; (b) new lists that keep 75 % of every list and replace
            # the rest by positions that are not resident: only those rows may cross the link
            gd = torch.Generator(device=dev)
            gd.manual_seed(99)
            for lay in sat_layers:
                for row, r, n_ctx, hs in sat_rows(lay):
                    cur = lay.topk_idx[row, :r].long()
                    lay.slot_pos[row, :r] = cur.int()
                    n_new = r // 4
                    resident = torch.zeros((n_ctx,), dtype=torch.bool, device=dev)
                    resident[cur] = True
                    resident[:hs.sink] = True
                    resident[n_ctx - hs.recent:] = True
                    free = (~resident).nonzero().flatten()
                    fresh = free[torch.randperm(free.numel(), generator=gd, device=dev)[:n_new]]
                    keep_ix = torch.randperm(r, generator=gd, device=dev)[:r - n_new]
                    lay.topk_idx[row, :r] = torch.cat([cur[keep_ix], fresh]).sort().values.int()
                    rows_delta += n_new
            torch.cuda.synchronize()
            ev_a.record()
            for lay in sat_layers:
                hc.hc_gather_retrieve(ctx.handle, lay.handle, lay.tier, lay.topk_idx, lay.flag, lay.arena, lay.slot_pos)
            ev_b.record()
            torch.cuda.synchronize()
            us_delta = ev_a.elapsed_time(ev_b) * 1e3
        for lay in sat_layers:
            lay.flag.zero_()
        gather = {"layers": len(sat_layers), "alone_on_the_gpu": True,
                  "whole_lists": {"rows": rows_full, "bytes": rows_full * 512, "us": us_full, "GBps": rows_full * 512 / (us_full * 1e-6) / 1e9},
                  "difference_only": None if us_delta is None else
                  {"rows": rows_delta, "bytes": rows_delta * 512, "us": us_delta, "GBps": rows_delta * 512 / (us_delta * 1e-6) / 1e9,
                   "rows_kept_resident": rows_full - rows_delta}}
        if probes.get("link_peak_GBps"):
            gather["link_peak_GBps"] = probes["link_peak_GBps"]
            gather["frac_of_link_peak"] = gather["whole_lists"]["GBps"] / probes["link_peak_GBps"]

    # ---- the monitor's own counters (per pivot, since the layers were created) ----
    mon = None
    if not args.attn_only and any(lay.n_reps for lay in layers):
        cs = [lay.monitor_counts(b, p) for lay in layers for b in range(lay.spec.B) for p in lay.spec.reps(b)]
        kept = [c["kept"] for c in cs if c["kept"] is not None]
        mon = {"pivots": len(cs), "decisions": sum(c["tests"] for c in cs), "retrievals": sum(c["triggers"] for c in cs),
               "filter_margin": args.filter_margin, "filter_fallbacks": sum(c["fallbacks"] for c in cs),
               "rows_kept_last_step_mean": float(np.mean(kept)) if kept else None}

    # ---- CPU oracle on a bounded sample: layers 0..1, first steps (the same inputs as warm-up) ----
    cpu = None
    parity = None
    if keep and not args.no_oracle:
        from oracle import ref
        sample_t, n_ls, oracles = [], 0, {}
        worst = 0.0
        t_or = time.perf_counter()
        n_steps_or = 0
        while time.perf_counter() - t_or < args.oracle_seconds and n_steps_or < T_total:
            for l, (sp, data, retrieved, base) in keep.items():
                if n_steps_or == 0:
                    oracles[l] = ref.RefLayer(sp, data, retrieved, base)
                ts = time.perf_counter()
                if KV_new is not None:
                    oracles[l].append(KV_new[n_steps_or, 0, l].cpu(), KV_new[n_steps_or, 1, l].cpu())
                rec = oracles[l].step(Q_all[n_steps_or, l].cpu())
                sample_t.append(time.perf_counter() - ts)
                n_ls += 1
                if l == 0 and n_steps_or in snap:
                    t = n_steps_or
                    err = np.abs(snap[t][0] - rec["out"]).max(-1) / np.sqrt((rec["out"] ** 2).mean(-1))
                    worst = max(worst, float(err.max()))
                    assert err.max() < 1e-2 and np.abs(snap[t][1] - rec["lse"]).max() < 1e-4, "GPU/oracle mismatch in bench"
            n_steps_or += 1
        cpu = {"value": float(np.mean(sample_t) * 1e6), "unit": "us per decode step per layer",
               "cores": ref.threads(), "kind": "oracle",
               "sample": f"{n_ls} layer-steps (layers 0..{len(keep) - 1}, first {n_steps_or} decode steps) of the same workload, "
                         f"{sum(sample_t):.1f}s of CPU time"}
        parity = worst

    out = {
        "metric": METRIC, "value": us_per_layer, "unit": "us per decode step per layer",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": ms_per_step, "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"config{args.config}{' dense' if args.dense else ''}: "
                               f"{spec0.ctx[0] if spec0.B == 1 else '%d..%d (sum %d)' % (min(spec0.ctx), max(spec0.ctx), sum(spec0.ctx))} ctx, {L} layers, "
                               f"B={spec0.B}, {spec0.Hq}q/{spec0.Hkv}kv heads, D=128",
                   "layers": L, "context": spec0.ctx[0], "mode": args.mode, "host_tier": not args.no_tier, "gather": "none" if args.no_tier else ("whole lists" if args.full_gather else "difference only"), "overlap_monitor": not args.serial, "logit_filter_margin": args.filter_margin, "side_lds_kb": args.side_lds, "layers_per_group": args.group, "growing_context": args.append,
                   "kv_bytes_per_layer_step": kv_bytes,
                   "split_workgroups": hc.hc_layer_num_workgroups(layers[0].handle),
                   "split_partials": hc.hc_layer_num_partials(layers[0].handle)},
        "host_enqueue_ms_per_step": host_enqueue_ms,
        "host_enqueue_ms_first_steps": host_first_ms,
        "prefill_init_ms_per_layer": float(np.mean(prefill_ms)) if prefill_ms else None,
        "tokens_per_s": spec0.B / (ms_per_step * 1e-3),
        "step_GBps": kv_bytes * L / (ms_per_step * 1e-3) / 1e9,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": MEASURED_TRAFFIC.get((args.config, args.dense, args.filter_margin > 0)) if not args.ctx else None,
                     "kernel": "attn_split_kernel", "kernel_us_mean": kern_us,
                     "kernel_us_median": float(np.median(kern_ms) * 1e3), "kernel_us_p95": float(np.percentile(kern_ms, 95) * 1e3),
                     "launches_timed": n_pairs,
                     "kernel_us_mean_without_overlap": iso_us,
                     "frac_without_overlap": (kv_bytes / (iso_us * 1e-6) / 1e9 / HBM_PEAK_GBPS) if iso_us else None,
                     "measured_stream_read_GBps": probes.get("stream_read_GBps"),
                     "frac_of_measured_peak": (achieved / probes["stream_read_GBps"]) if probes.get("stream_read_GBps") else None},
        "step_time": step_stats,
        "monitor": mon,
        "gather_GBps": gather["whole_lists"]["GBps"] if gather else None,
        "link_peak_GBps": probes.get("link_peak_GBps"),
        "gather": gather,
        "probes": probes,
        "cpu_baseline": cpu,
        "parity_max_err_over_rms": parity,
        "warmup_flags": flags_hist,
        "setup_s": setup_s,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
