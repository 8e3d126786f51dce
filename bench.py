#!/usr/bin/env python3
"""Benchmark of the dynamic-batching hot path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic input:
  * program-tree engine, config 2 (256 IEP-shaped programs, 40 functions, C=128 @ 14x14, bf16):
    dynbatch_plan (host) + dynbatch_plan_upload + dynbatch_execute;
  * mixture-of-experts layer, config 4 (16384 tokens, d=1024, 1024 experts, h=2048, top-4,
    Zipf(1.2) load, 5 % empty experts, bf16): moe_forward.
Inputs are resident in HBM before the timed region.

Headline (`value`, `ms_per_step`, `roofline`): module evaluations per second with ONE minibatch at a
time on one stream, the protocol of the paper's Results / IEP.  K steps are timed between two
device synchronisations; that window is repeated (`windows`) and the median window is reported,
with the minimum and every window beside it.  `roofline` describes the dominant kernel of exactly
that configuration: useful flops of its launches / their duration, measured with HIP events on the
stream the kernels run on.

Extras: `in_flight` (several different batches in flight on their own streams: chip throughput),
`moe` (tokens per second of the MoE layer, per-stage times, its rooflines in `rooflines_other`),
`measured_peak` (what this card sustains in a register-only MFMA loop and a plain copy),
`naive_gpu` (the paper's unbatched comparison rows), `cpu_baseline` (the CPU oracle on the host cores).

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

FLOP_UNARY = 2 * 2 * 196 * 128 * 1152            # two conv3x3, 196 pixels, 128 out, K = 9*128
FLOP_BINARY = FLOP_UNARY + 2 * 196 * 128 * 256   # plus the conv1x1 over 2C channels
PEAK_BF16_TFLOPS = 2500.0
PEAK_HBM_GBS = 8000.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--windows", type=int, default=5, help="repetitions of the timed K-step window (median and min are reported)")
    ap.add_argument("--iep-config", choices=["config1", "config2"], default="config2")
    ap.add_argument("--no-balance", action="store_true", help="plain improved sort, no pull-forward of nodes")
    ap.add_argument("--persistent", action="store_true",
                    help="headline with one dependency-driven launch per batch (DYNB_PLAN_PERSISTENT) instead of one launch per label")
    ap.add_argument("--streams", type=int, default=4,
                    help="program-tree batches in flight for the in_flight figure: step i runs on HIP stream i %% streams")
    ap.add_argument("--moe-streams", type=int, default=3,
                    help="MoE layers in flight: call i runs on HIP stream i %% moe-streams with its own workspace")
    ap.add_argument("--skip-moe", action="store_true")
    ap.add_argument("--skip-naive", action="store_true")
    ap.add_argument("--no-prepare", action="store_true", help="repack the module weights inside every dynbatch_execute")
    ap.add_argument("--skip-schedules", action="store_true", help="skip the side-by-side timing of the schedules")
    ap.add_argument("--skip-cpu", action="store_true")
    ap.add_argument("--skip-peak", action="store_true")
    ap.add_argument("--skip-extras", action="store_true", help="skip the classifier head and the backward pass")
    ap.add_argument("--wide-nodes", type=int, default=4096, help="nodes of the single wide launch group (0 = skip)")
    ap.add_argument("--moe-config", choices=["config3", "config4"], default="config4")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU; run with --gpus 1 (no multi-GPU path exists in it)",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import __graft_entry__
    __graft_entry__.ensure_built()          # loads the built library; compiles only if there is none
    import paper_1707_02402_amd as dyn
    from workloads import device as U
    from workloads import iep, moe

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    K, Wm, NW = args.steps, args.warmup, max(1, args.windows)
    log = lambda *a: print(*a, file=sys.stderr, flush=True)

    def gpu_ms(fn, reps, warm_ms=0.0):
        """Mean GPU time of fn() over reps calls, from one HIP event pair on the current stream.  warm_ms: keep the
        GPU busy with fn() for about that long first (after an idle spell the card takes some 20 ms of load to reach
        the clock it then holds; a single warm-up call measures the ramp)."""
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        fn()
        torch.cuda.synchronize()
        t_w = time.perf_counter()
        while (time.perf_counter() - t_w) * 1e3 < warm_ms:
            for _ in range(4):
                fn()
            torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    # ------------------------------------------------------------------ what the card sustains
    # (the plain 1 GiB copy is also the known-size reference for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE)
    peak = None
    cal_src = torch.ones(1 << 28, dtype=torch.int32, device="cuda")
    cal_dst = torch.empty_like(cal_src)
    copy_ms = gpu_ms(lambda: dyn.dynb_probe_copy(cal_dst, cal_src), 1 if args.skip_peak else 10)
    if not args.skip_peak:
        sink = torch.zeros(1, dtype=torch.float32, device="cuda")
        fl = [0.0]

        def mfma_probe():
            fl[0] = dyn.dynb_probe_mfma_bf16(4000, 256 * 2 * 4, sink)      # 8 waves per SIMD-set keep the pipes full

        mfma_ms = gpu_ms(mfma_probe, 5)
        rsink = torch.zeros(4, dtype=torch.int32, device="cuda")
        read_ms = gpu_ms(lambda: dyn.dynb_probe_read(cal_src, rsink), 10, warm_ms=10.0)
        peak = {"mfma_bf16_tflops": round(fl[0] / mfma_ms / 1e9, 1),
                "mfma_bf16_frac_of_published": round(fl[0] / mfma_ms / 1e9 / PEAK_BF16_TFLOPS, 4),
                "mfma_kind": "register-only loop of independent v_mfma_f32_32x32x16_bf16, 2048 workgroups x 4 waves (dynb_probe_mfma_bf16)",
                "copy_gbs": round(2 * cal_src.numel() * 4 / copy_ms / 1e6, 1),
                "copy_frac_of_published": round(2 * cal_src.numel() * 4 / copy_ms / 1e6 / PEAK_HBM_GBS, 4),
                "copy_kind": "1 GiB read + 1 GiB written by a plain 16-byte copy kernel (dynb_probe_copy)",
                "read_gbs": round(cal_src.numel() * 4 / read_ms / 1e6, 1),
                "read_frac_of_published": round(cal_src.numel() * 4 / read_ms / 1e6 / PEAK_HBM_GBS, 4),
                "read_kind": "1 GiB read, nothing written, 16-byte loads, 8 in flight per lane, a contiguous share per workgroup (dynb_probe_read)"}
    del cal_src, cal_dst

    # ------------------------------------------------------------------ program-tree engine
    w = getattr(iep, args.iep_config)()
    weights = U.iep_weights_dev(w)
    # constant weights are put into the kernels' fragment order once, outside the timed steps
    if not args.no_prepare:
        weights["packed"] = dyn.dynbatch_pack_weights(weights, w.C, w.H, w.W, dyn.DYNB_BF16)
    base_flags = dyn.DYNB_SCHED_IMPROVED | (0 if args.no_balance else dyn.DYNB_PLAN_BALANCE)
    SCHEDULES = {"improved": dyn.DYNB_SCHED_IMPROVED, "improved+balance": dyn.DYNB_SCHED_IMPROVED | dyn.DYNB_PLAN_BALANCE,
                 "standard": dyn.DYNB_SCHED_STANDARD, "dependency_depth": dyn.DYNB_SCHED_DEPTH}
    SCHEDULES["improved, one dependency-driven launch per batch"] = dyn.DYNB_SCHED_IMPROVED | dyn.DYNB_PLAN_PERSISTENT
    one_flags = (dyn.DYNB_SCHED_IMPROVED | dyn.DYNB_PLAN_PERSISTENT) if args.persistent else base_flags

    def batch_of(lane):
        """Lane 0 runs the configuration itself, the others further batches of the same recipe (own programs and
        feature maps, the same modules)."""
        if lane == 0 or args.iep_config != "config2":      # other recipes draw their modules from the seed
            return w
        seed0 = iep.config2.__defaults__[0]
        return iep.config2(seed=seed0 + 1000 * lane, weight_seed=seed0)

    S = max(1, args.streams)
    batches = [batch_of(i) for i in range(S)]
    all_flags = [dyn.DYNB_SCHED_NAIVE, *SCHEDULES.values(), one_flags, base_flags | dyn.DYNB_PLAN_THROUGHPUT]
    lanes = []
    for i, wl in enumerate(batches):
        plans = [dyn.dynbatch_plan(wl.prog, wl.prog_off, wl.arity, f) for f in (all_flags if i == 0 else all_flags[-2:])]
        ws_bytes = max(dyn.dynbatch_workspace_bytes(p, w.C, w.H, w.W, dyn.DYNB_BF16) for p in plans)
        db_bytes = max(dyn.dynbatch_plan_device_bytes(p) for p in plans) + 4096
        feats = U.to_dev(wl.feats, w.dtype)
        lanes.append(dict(stream=None if i == 0 else torch.cuda.Stream(), w=wl, feats=feats, out=torch.empty_like(feats),
                          ws=torch.empty(ws_bytes, dtype=torch.uint8, device="cuda"),
                          devbuf=torch.empty(db_bytes, dtype=torch.uint8, device="cuda")))
        del plans
    torch.cuda.synchronize()                           # side streams must not meet memory the default stream still uses
    L0 = lanes[0]
    plan0 = dyn.dynbatch_plan(w.prog, w.prog_off, w.arity, one_flags)
    view = dyn.dynbatch_plan_view(plan0)
    n_evals = view.n_compute_nodes
    n_binary = int((w.arity[w.prog] == 2).sum())
    flops_step = (n_evals - n_binary) * FLOP_UNARY + n_binary * FLOP_BINARY
    log(f"[bench] {w.name}: B={w.B} nodes={view.n_nodes} evals={n_evals} levels={view.n_levels} "
        f"launches={view.n_launches} buckets={view.n_buckets}")

    keep = []

    def iep_step(flags, lane, host_ms=None):
        wl = lane["w"]
        t0 = time.perf_counter()
        plan = dyn.dynbatch_plan(wl.prog, wl.prog_off, wl.arity, flags)
        t1 = time.perf_counter()
        dyn.dynbatch_plan_upload(plan, lane["devbuf"], stream=lane["stream"])
        dyn.dynbatch_execute(plan, weights, lane["feats"], lane["out"], lane["ws"], stream=lane["stream"])
        if host_ms is not None:
            host_ms.append((t1 - t0) * 1e3)
        keep.append(plan)                              # a plan lives until its upload has run

    def timed_windows(n_lanes, flags):
        """NW windows of exactly K steps each, every window between two device synchronisations."""
        for i in range(n_lanes):                      # every lane's buffers and stream are touched once,
            iep_step(flags, lanes[i])                 # whatever --warmup says
        torch.cuda.synchronize()
        keep.clear()
        for i in range(Wm):
            iep_step(flags, lanes[i % n_lanes])
        torch.cuda.synchronize()
        keep.clear()
        wins, host = [], []
        for _ in range(NW):
            t0 = time.perf_counter()
            for i in range(K):
                iep_step(flags, lanes[i % n_lanes], host_ms=host)
            torch.cuda.synchronize()
            wins.append((time.perf_counter() - t0) * 1e3 / K)
            keep.clear()
        return wins, host

    one_wins, plan_ms = timed_windows(1, one_flags)   # one batch at a time: the headline
    one_ms = float(np.median(one_wins))
    ref_out = L0["out"].clone()
    fly = None
    if S > 1:                                         # S different batches in flight: chip throughput
        fly_flags = base_flags | dyn.DYNB_PLAN_THROUGHPUT
        fly_wins, _ = timed_windows(S, fly_flags)
        if K >= S or Wm >= S:
            assert torch.equal(L0["out"], ref_out)    # lane 0 ran the same batch in another kernel layout: same bits
        fl_lane, ev_lane = [], []
        for ln in lanes:
            nb = int((ln["w"].arity[ln["w"].prog] == 2).sum())
            ev_lane.append(int(ln["w"].n_module_evals))
            fl_lane.append((ln["w"].n_module_evals - nb) * FLOP_UNARY + nb * FLOP_BINARY)
        evals_fly = float(np.mean([ev_lane[i % S] for i in range(K)]))
        flops_fly = float(np.mean([fl_lane[i % S] for i in range(K)]))
        fms = float(np.median(fly_wins))
        fly = {"batches_in_flight": S,
               "batches": "config 2 and %d further batches of the same recipe (own programs and feature maps, same modules)" % (S - 1),
               "kernel_layout": "throughput (DYNB_PLAN_THROUGHPUT), one launch per label",
               "ms_per_step": round(fms, 4), "ms_per_step_min": round(min(fly_wins), 4),
               "module_evals_per_sec": round(evals_fly / fms * 1e3, 1),
               "chip_mfma_frac_of_step": round(flops_fly / (fms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
               "windows_ms": [round(v, 4) for v in fly_wins]}

    # execute only (plan reused), and the GPU time of the module kernels from HIP events on the same stream
    dyn.dynbatch_plan_upload(plan0, L0["devbuf"])
    run0 = lambda: dyn.dynbatch_execute(plan0, weights, L0["feats"], L0["out"], L0["ws"])
    run0()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(K):
        run0()
    torch.cuda.synchronize()
    exec_ms = (time.perf_counter() - t0) * 1e3 / K
    # the same launches replayed from a HIP graph (the call enqueues kernels only, so it can be captured)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run0()
    graph.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(K):
        graph.replay()
    torch.cuda.synchronize()
    graph_ms = (time.perf_counter() - t0) * 1e3 / K
    del graph
    # one event pair around all module-kernel launches of a step (set-up work is a stage of its own)
    dyn.dynb_timing_enable(2)
    launch_ms, launch_n = [], int(view.n_launches)
    for _ in range(K):
        run0()
        launch_ms.append(sum(ms for tag, _, ms in dyn.dynb_timing_read() if tag >= 0))
    dyn.dynb_timing_enable(0)
    kern_ms_step = float(np.median(launch_ms))        # all module-kernel launches of one step
    avg_launch_us = kern_ms_step * 1e3 / launch_n
    achieved_tflops = flops_step / (kern_ms_step * 1e-3) / 1e12

    # the paper's schedules side by side (execute only, plan reused): launch groups, widest group, time
    sched_cmp = {}
    for name, fl_ in ([] if args.skip_schedules else SCHEDULES.items()):
        pl = dyn.dynbatch_plan(w.prog, w.prog_off, w.arity, fl_)
        dyn.dynbatch_plan_upload(pl, L0["devbuf"])
        v_ = dyn.dynbatch_plan_view(pl)
        for _ in range(3):
            dyn.dynbatch_execute(pl, weights, L0["feats"], L0["out"], L0["ws"])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(K):
            dyn.dynbatch_execute(pl, weights, L0["feats"], L0["out"], L0["ws"])
        torch.cuda.synchronize()
        sched_ms = (time.perf_counter() - t0) * 1e3 / K
        assert torch.equal(L0["out"], ref_out)         # every schedule: the same root maps, bit for bit
        sched_cmp[name] = {"launch_groups": int(v_.n_launches), "max_group": int(v_.max_launch_nodes),
                           "pools": int((w.arity[v_.bucket_type] > 0).sum()), "execute_ms": round(sched_ms, 4)}

    naive = None
    if not args.skip_naive:
        iep_step(dyn.DYNB_SCHED_NAIVE, L0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        iep_step(dyn.DYNB_SCHED_NAIVE, L0)
        torch.cuda.synchronize()
        naive_ms = (time.perf_counter() - t0) * 1e3
        keep.clear()
        naive = {"kind": "same kernels, one launch per node, example by example", "ms_per_step": round(naive_ms, 3),
                 "module_evals_per_sec": round(n_evals / naive_ms * 1e3, 1), "speedup_batched": round(naive_ms / one_ms, 2),
                 "speedup_note": "against one batched step at a time on one stream"}

    # ------------------------------------------------------------------ one wide launch group (the module kernel at full width)
    wide = None
    if args.wide_nodes > 0:
        nw = args.wide_nodes
        n_un = int((w.arity == 1).sum())
        wprog = np.empty(2 * nw, np.int32)
        wprog[0::2] = 1 + np.arange(nw) % n_un                    # one one-argument module per program, functions in turn
        wprog[1::2] = 0
        woff = (2 * np.arange(nw + 1)).astype(np.int32)
        wfeats = L0["feats"].repeat((nw + w.B - 1) // w.B, 1, 1, 1)[:nw].contiguous()
        wout = torch.empty_like(wfeats)
        wide = {"nodes": nw, "programs": "one one-argument module per program, the %d one-argument functions in turn" % n_un}
        # (a launch group wider than the chip runs the two-workgroups-per-CU layout whatever the plan's flags)
        wplan = dyn.dynbatch_plan(wprog, woff, w.arity, 0)
        dyn.dynbatch_plan_upload(wplan)
        wws = torch.empty(dyn.dynbatch_workspace_bytes(wplan, w.C, w.H, w.W, dyn.DYNB_BF16), dtype=torch.uint8, device="cuda")
        ms_ = gpu_ms(lambda: dyn.dynbatch_execute(wplan, weights, wfeats, wout, wws), K, warm_ms=40.0)
        tf = nw * FLOP_UNARY / ms_ / 1e9
        wide.update({"kernel": "k_module_mfma<4> (two workgroups per CU)", "ms": round(ms_, 4), "tflops": round(tf, 1),
                     "frac": round(tf / PEAK_BF16_TFLOPS, 4),
                     "frac_of_measured_peak": None if peak is None else round(tf / peak["mfma_bf16_tflops"], 4),
                     "warm_up": "40 ms of the same launches before the timed ones"})
        del wws, wplan
        del wfeats, wout

    # ------------------------------------------------------------------ classifier head and backward pass (config 2)
    extras = {}
    if not args.skip_extras:
        head = iep.make_head(iep.config2.__defaults__[0], w.C, w.H, w.W, 32, 256, 28, w.dtype)
        hd = U.head_dev(head, w.dtype)
        hws = torch.empty(dyn.dynbatch_classify_workspace_bytes(w.C, w.H, w.W, dyn.DYNB_BF16, 32, 256, 28, w.B), dtype=torch.uint8, device="cuda")
        probs = torch.empty((w.B, 28), dtype=torch.float32, device="cuda")
        head_ms = gpu_ms(lambda: dyn.dynbatch_classify(ref_out, hd, probs=probs, workspace=hws), K)
        head_flops = 2.0 * w.B * (w.H * w.W * w.C * 32 + w.H * w.W * 32 * 256 + 256 * 28)
        extras["classifier_head"] = {"shape": "conv1x1 128->32, fc 6272->256, fc 256->28, softmax, on the %d root maps" % w.B,
                                     "ms": round(head_ms, 4), "tflops": round(head_flops / head_ms / 1e9, 2),
                                     "share_of_a_step": round(head_ms / one_ms, 4)}
        kplan = dyn.dynbatch_plan(w.prog, w.prog_off, w.arity, base_flags | dyn.DYNB_PLAN_KEEP)
        dyn.dynbatch_plan_upload(kplan)
        kws = torch.empty(dyn.dynbatch_workspace_bytes(kplan, w.C, w.H, w.W, dyn.DYNB_BF16), dtype=torch.uint8, device="cuda")
        kout = dyn.dynbatch_execute(kplan, weights, L0["feats"], workspace=kws)
        assert torch.equal(kout, ref_out)
        dout = torch.randn(kout.shape, dtype=torch.float32, device="cuda", generator=torch.Generator(device="cuda").manual_seed(1))
        bws = torch.empty(dyn.dynbatch_backward_workspace_bytes(kplan, w.C, w.H, w.W, dyn.DYNB_BF16), dtype=torch.uint8, device="cuda")
        grads = dyn.dynbatch_backward(kplan, weights, L0["feats"], kout, kws, dout, workspace=bws)
        bwd_ms = gpu_ms(lambda: dyn.dynbatch_backward(kplan, weights, L0["feats"], kout, kws, dout, workspace=bws, grads=grads), max(K // 5, 3), warm_ms=20.0)
        kfwd_ms = gpu_ms(lambda: dyn.dynbatch_execute(kplan, weights, L0["feats"], out=kout, workspace=kws), K)
        # two transposed convolutions and two weight-gradient contractions per module: twice the forward pass's flops
        # (the recomputation of u and mid, half a forward pass, is not counted as useful work)
        extras["backward"] = {"ms_per_step": round(bwd_ms, 3), "forward_ms_per_step": round(kfwd_ms, 4),
                              "ratio_to_forward": round(bwd_ms / kfwd_ms, 2),
                              "flops": 2.0 * flops_step, "tflops": round(2.0 * flops_step / bwd_ms / 1e9, 1),
                              "frac_of_mfma_peak": round(2.0 * flops_step / bwd_ms / 1e9 / PEAK_BF16_TFLOPS, 4),
                              "workspace_mb": round(bws.numel() / 1e6, 1),
                              "kind": "MFMA kernels: one fused launch per label in reverse order (both transposed convolutions, "
                                      "fp32 gradient maps), then one launch for the parameter gradients of all functions and one that "
                                      "sums their partial results; forward = the same plan (DYNB_PLAN_KEEP: a slot per node, u and mid "
                                      "of every node saved)"}
        del bws, grads
        del kws, kout, dout, kplan

    # ------------------------------------------------------------------ mixture of experts
    moe_res, moe_roof = None, []
    if not args.skip_moe:
        t0 = time.perf_counter()
        m = getattr(moe, args.moe_config)()
        W1b = np.empty((m.E, m.h, m.d), np.uint16)
        W2b = np.empty((m.E, m.d, m.h), np.uint16)
        m.all_expert_weights_bits(W1b, W2b, threads=16)
        dev = U.moe_inputs_dev(m, np.zeros((1, 1, 1), np.float32), np.zeros((1, 1, 1), np.float32))
        dev["W1"] = torch.from_numpy(W1b.view(np.int16)).cuda().view(torch.bfloat16)
        dev["W2"] = torch.from_numpy(W2b.view(np.int16)).cuda().view(torch.bfloat16)
        del W1b, W2b
        log(f"[bench] {m.name}: inputs generated and uploaded in {time.perf_counter() - t0:.1f} s")
        mws = torch.empty(dyn.moe_workspace_bytes(m.T, m.d, m.h, m.E, m.k), dtype=torch.uint8, device="cuda")
        mout = torch.empty_like(dev["x"])

        def moe_step():
            dyn.moe_forward(dev["x"], dev["Wg"], dev["Wn"], dev["noise"], dev["W1"], dev["W2"], m.k, out=mout, workspace=mws)

        for _ in range(Wm):
            moe_step()
        torch.cuda.synchronize()
        moe_wins = []
        for _ in range(NW):
            t0 = time.perf_counter()
            for _ in range(K):
                moe_step()
            torch.cuda.synchronize()
            moe_wins.append((time.perf_counter() - t0) * 1e3 / K)
        moe_one_ms = float(np.median(moe_wins))
        # several layers (batches) in flight: the gate and grouping kernels of one run under the weight
        # streaming of another.  Lane buffers are allocated before, and the device drained, so that no
        # side stream touches memory the default stream may still be using.
        MS = max(1, args.moe_streams)
        moe_fly_ms = None
        if MS > 1:
            mlanes = [dict(stream=torch.cuda.Stream(), ws=torch.empty_like(mws), out=torch.empty_like(mout)) for _ in range(MS)]
            torch.cuda.synchronize()

            def moe_lane_step(i):
                ln = mlanes[i % MS]
                dyn.moe_forward(dev["x"], dev["Wg"], dev["Wn"], dev["noise"], dev["W1"], dev["W2"], m.k, out=ln["out"],
                                workspace=ln["ws"], stream=ln["stream"])

            for i in range(MS + Wm):                  # every lane once, then the warm-up steps
                moe_lane_step(i)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(K):
                moe_lane_step(i)
            torch.cuda.synchronize()
            moe_fly_ms = (time.perf_counter() - t0) * 1e3 / K
            for ln in mlanes:
                assert torch.equal(ln["out"], mout)
            del mlanes
        dyn.dynb_timing_enable(True)
        stages = {n: [] for n in dyn.MOE_STAGES}
        for _ in range(K):
            moe_step()
            for tag, _, ms in dyn.dynb_timing_read():
                stages[dyn.MOE_STAGES[tag]].append(ms)
        dyn.dynb_timing_enable(False)
        stage_ms = {n: float(np.median(v)) for n, v in stages.items() if v}
        # the stacking as a kernel of its own (MOE_SEPARATE_PERMUTE): the HBM-bound scatter, timed alone
        dyn.dynb_timing_enable(True)
        perm_alone = []
        for _ in range(K):
            dyn.moe_forward(dev["x"], dev["Wg"], dev["Wn"], dev["noise"], dev["W1"], dev["W2"], m.k, out=mout, workspace=mws,
                            flags=dyn.MOE_SEPARATE_PERMUTE)
            perm_alone += [ms for tag, _, ms in dyn.dynb_timing_read() if dyn.MOE_STAGES[tag] == "permute"]
        dyn.dynb_timing_enable(False)
        permute_ms = float(np.median(perm_alone))
        _, aux = dyn.moe_forward(dev["x"], dev["Wg"], dev["Wn"], dev["noise"], dev["W1"], dev["W2"], m.k, want_aux=True,
                                 workspace=mws)
        counts = aux.counts.cpu().numpy()
        n_active = int((counts > 0).sum())
        A = m.A
        by_perm = m.T * m.d * 2 + A * m.d * 2 + A * 4
        by_comb = A * m.d * 2 + m.T * m.d * 2 + A * 8
        by_w = 2 * m.d * m.h * 2 * n_active                      # both layers' weights of every non-empty expert
        by_ffn = by_w + A * (m.d + 2 * m.h + m.d) * 2             # + xs read, hid written and read, y written
        fl_ffn = 4.0 * m.d * m.h * A
        ffn_ms = stage_ms.get("ffn1", 0.0) + stage_ms.get("ffn2", 0.0)
        # per expert max(compute at the published MFMA peak, weight bytes at the published HBM peak), summed
        bound_ms = float(sum(max(4.0 * m.d * m.h * c / (PEAK_BF16_TFLOPS * 1e12), 4.0 * m.d * m.h / (PEAK_HBM_GBS * 1e9))
                             for c in counts if c > 0) * 1e3)
        moe_naive = None
        if not args.skip_naive:
            stride = 16
            dyn.moe_forward(dev["x"], dev["Wg"], dev["Wn"], dev["noise"], dev["W1"], dev["W2"], m.k, out=mout, workspace=mws,
                            naive_stride=stride * 8)                      # warm-up of the host loop path
            torch.cuda.synchronize()
            dyn.dynb_timing_enable(True)
            dyn.moe_forward(dev["x"], dev["Wg"], dev["Wn"], dev["noise"], dev["W1"], dev["W2"], m.k, out=mout, workspace=mws,
                            naive_stride=stride)
            nst = {dyn.MOE_STAGES[tag]: ms for tag, _, ms in dyn.dynb_timing_read()}
            dyn.dynb_timing_enable(False)
            sampled = nst["ffn1"] + nst["ffn2"]
            moe_naive = {"kind": "same kernels, one expert call (2 launches) per (token, expert) use from a host loop",
                         "sample": f"every {stride}th of {A} uses executed, time scaled by {stride}",
                         "expert_stage_ms_sampled": round(sampled, 3), "expert_stage_ms_est": round(sampled * stride, 2),
                         "speedup_batched_expert_stage": round(sampled * stride / ffn_ms, 1)}
        moe_res = {"workload": m.name, "tokens_per_sec": round(m.T / moe_one_ms * 1e3, 1), "ms_per_step": round(moe_one_ms, 4),
                   "ms_per_step_min": round(min(moe_wins), 4), "windows_ms": [round(v, 4) for v in moe_wins],
                   "protocol": "one layer at a time on one stream",
                   "in_flight": None if moe_fly_ms is None else {"layers_in_flight": MS, "ms_per_step": round(moe_fly_ms, 4),
                                                                 "tokens_per_sec": round(m.T / moe_fly_ms * 1e3, 1)},
                   "stage_ms": {k_: round(v, 4) for k_, v in stage_ms.items()}, "permute_kernel_alone_ms": round(permute_ms, 4),
                   "active_experts": n_active,
                   "max_expert_rows": int(counts.max()),
                   "expert_layers_bound_ms": round(bound_ms, 4), "expert_layers_frac_of_bound": round(bound_ms / ffn_ms, 4),
                   "naive_gpu": moe_naive}

        def roof(kernel, nbytes, ms, **extra):
            return dict(kernel=kernel, bound="hbm", achieved=round(nbytes / ms / 1e6, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                        frac=round(nbytes / ms / 1e6 / PEAK_HBM_GBS, 4), traffic=None, **extra)

        moe_roof.append(roof("k_permute", by_perm, permute_ms, note="as a kernel of its own (MOE_SEPARATE_PERMUTE); by default the "
                             "first expert layer gathers the token rows itself and this kernel does not run"))
        moe_roof.append(roof("k_combine", by_comb, stage_ms["combine"]))
        moe_roof.append(roof("k_grouped_gemm (both expert layers)", by_ffn, ffn_ms, mfma_tflops=round(fl_ffn / ffn_ms / 1e9, 1)))
        if "gate" in stage_ms and "topk" in stage_ms:
            fl_gate = 4.0 * m.T * m.d * m.E                       # both gate matrices
            moe_roof.append(dict(kernel="k_gate_big / k_gate (gate stage)", bound="mfma",
                                 achieved=round(fl_gate / stage_ms["gate"] / 1e9, 1), peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                                 frac=round(fl_gate / stage_ms["gate"] / 1e9 / PEAK_BF16_TFLOPS, 4), traffic=None,
                                 note="also reads x and the noise values and writes the logits: %.0f MB" %
                                      ((m.T * m.d * 2 + 2 * m.E * m.d * 2 + 2 * m.T * m.E * 4) / 1e6)))
            moe_roof.append(roof("k_topk_small / k_topk (top-k stage)", m.T * m.E * 4 + m.T * m.k * 8, stage_ms["topk"]))
            moe_res["gate_plus_topk_ms"] = round(stage_ms["gate"] + stage_ms["topk"], 4)

    # ------------------------------------------------------------------ CPU oracle baseline (bounded samples)
    cpu = None
    if not args.skip_cpu:
        import oracle
        cores = oracle.num_threads()

        def iep_oracle(n_s, threads):
            sub = w.subset(list(range(0, w.B, max(1, w.B // n_s)))[:n_s])
            oracle.set_threads(threads)
            t0 = time.perf_counter()
            oracle.iep_forward_workload(sub)
            dt = time.perf_counter() - t0
            oracle.set_threads(cores)
            return sub, dt

        sub, dt = iep_oracle(min(96, w.B), cores)
        cpu = {"value": round(sub.n_module_evals / dt, 2), "unit": "module_evals/s", "cores": cores,
               "kind": "oracle", "sample": f"{sub.B} of {w.B} examples of {w.name} ({sub.n_module_evals} module evaluations, "
               f"{dt:.1f} s wall, fp64 per-example tree recursion, one example per thread)"}
        sub1, dt1 = iep_oracle(min(6, w.B), 1)
        cpu["one_thread"] = {"value": round(sub1.n_module_evals / dt1, 2), "unit": "module_evals/s", "cores": 1,
                             "sample": f"{sub1.B} of {w.B} examples ({sub1.n_module_evals} module evaluations, {dt1:.1f} s wall)"}
        if moe_res is not None:
            from concurrent.futures import ThreadPoolExecutor
            rows = np.random.default_rng(0).choice(m.T, 192, replace=False)
            idx = aux.topk_idx.cpu().numpy()
            wts = aux.topk_w.cpu().numpy().astype(np.float64)
            used = np.unique(idx[rows])
            with ThreadPoolExecutor(cores) as ex:
                packs = dict(zip(used.tolist(), ex.map(lambda e: m.expert_weights(int(e)), used)))

            def tok(t):
                return oracle.moe_token(m.x[t], wts[t], [packs[int(e)][0] for e in idx[t]], [packs[int(e)][1] for e in idx[t]])

            t0 = time.perf_counter()
            for t in rows[:32]:
                tok(t)
            dt1 = time.perf_counter() - t0
            t0 = time.perf_counter()
            with ThreadPoolExecutor(cores) as ex:
                list(ex.map(tok, rows))
            dtn = time.perf_counter() - t0
            cpu["moe"] = {"value": round(len(rows) / dtn, 2), "unit": "tokens/s", "cores": cores, "kind": "oracle",
                          "sample": f"expert+combine stage of {len(rows)} of {m.T} tokens of {m.name}, one token per thread, {dtn:.1f} s wall",
                          "one_thread": {"value": round(32 / dt1, 2), "unit": "tokens/s", "cores": 1,
                                         "sample": f"32 of those tokens, {dt1:.1f} s wall"}}

    # HBM-side bytes per launch as measured by rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE: counters cannot be read
    # from inside this process, so the committed measurement of the same command is quoted, with its source
    persistent = one_flags != base_flags
    traffic, traffic_src = None, None
    moe_traffic = {}
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        tj = json.load(open(tpath))
        dom = tj.get("dominant", {})
        if args.iep_config == "config2" and "bytes_per_launch" in dom and bool(dom.get("persistent", False)) == persistent:
            traffic = round(dom["bytes_per_launch"])
            traffic_src = "profiles/hbm_traffic.json (rocprofv3 --pmc FETCH_SIZE, then WRITE_SIZE, of this command; not measured in this run)"
        if args.moe_config == "config4":
            moe_traffic = {k_: round(v["fetch_bytes"] + v["write_bytes"]) for k_, v in tj.get("moe", {}).items()}
    for r_ in moe_roof:
        key = r_["kernel"].split(" ")[0]
        key = "k_gate" if key.startswith("k_gate") else "k_topk" if key.startswith("k_topk") else key
        if key == "k_grouped_gemm":
            parts = [v for k_, v in moe_traffic.items() if k_.startswith("k_grouped_gemm")]
            if parts:
                r_["traffic"] = sum(parts)
        elif key in moe_traffic:
            r_["traffic"] = moe_traffic[key]
        if r_["traffic"] is not None:
            r_["traffic_source"] = "profiles/hbm_traffic.json"

    res = {
        "metric": "module_evals_per_sec", "value": round(n_evals / one_ms * 1e3, 1), "unit": "module_evals/s",
        "n_gpus": 1, "steps": K, "warmup": Wm, "ms_per_step": round(one_ms, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "windows": NW, "ms_per_step_min": round(min(one_wins), 4), "windows_ms": [round(v, 4) for v in one_wins],
        "config": {"workload": w.name, "batch": w.B, "nodes": int(view.n_nodes), "module_evals": int(n_evals),
                   "levels": int(view.n_levels), "launch_groups": int(view.n_launches), "C": w.C, "H": w.H, "W": w.W,
                   "step": "dynbatch_plan + dynbatch_plan_upload + dynbatch_execute",
                   "protocol": "one minibatch at a time on one stream (Results / IEP)",
                   "weights": "repacked per call" if args.no_prepare else "fragment order prepared once (dynbatch_pack_weights)",
                   "schedule": "improved topological sort" + (", one dependency-driven launch per batch" if persistent
                                                              else ("" if args.no_balance else " + balanced launch groups"))},
        "plan_host_ms": round(float(np.mean(plan_ms)), 4), "execute_only_ms": round(exec_ms, 4),
        "execute_only_graph_replay_ms": round(graph_ms, 4),
        "execute_only_module_evals_per_sec": round(n_evals / exec_ms * 1e3, 1),
        "roofline": {"kernel": "k_module_persist" if persistent else "k_module_mfma", "bound": "mfma",
                     "achieved": round(achieved_tflops, 2),
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved_tflops / PEAK_BF16_TFLOPS, 4),
                     "traffic": traffic, "traffic_source": traffic_src,
                     "launches_per_step": launch_n, "avg_launch_us": round(avg_launch_us, 2),
                     "flops_per_step": flops_step,
                     "frac_of_measured_peak": None if peak is None else round(achieved_tflops / peak["mfma_bf16_tflops"], 4),
                     "configuration": "the headline's: one batch at a time on one stream; useful flops of a step / duration of its "
                                      "module-kernel launches (one HIP event pair around them on that stream)"},
        "measured_peak": peak, "in_flight": fly, "wide_launch": wide, "classifier_head": extras.get("classifier_head"), "backward": extras.get("backward"),
        "rooflines_other": moe_roof, "schedules": sched_cmp, "moe": moe_res, "naive_gpu": naive, "cpu_baseline": cpu,
        "paper_context": "paper reports ratios only: >14x cell execution (IEP, GTX 1080 Ti), up to 1000x (MoE, 11 GB card)",
    }
    print(json.dumps(res))


if __name__ == "__main__":
    main()
