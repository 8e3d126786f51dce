#!/usr/bin/env python3
"""Benchmark of the dynamic-batching hot path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic input:
  * program-tree engine, config 2 (256 IEP-shaped programs, 40 functions, C=128 @ 14x14, bf16):
    dynbatch_plan (host) + dynbatch_plan_upload + dynbatch_execute;
  * mixture-of-experts layer, config 4 (16384 tokens, d=1024, 1024 experts, h=2048, top-4,
    Zipf(1.2) load, 5 % empty experts, bf16): moe_forward.
Inputs are resident in HBM before the timed region.  `value` is module evaluations per second of
the program-tree part (the metric's first half); the MoE half is in the "moe" object.

By default several independent batches are in flight: step i runs on HIP stream i % --streams (4) with
its own plan buffer, workspace and output, MoE call i on stream i % --moe-streams (3); every timed step
still plans, uploads and executes one whole batch, and all K steps end inside the timed region.
"single_stream" holds the same measurement with one batch at a time; "roofline" describes that
one-at-a-time configuration (per-launch durations are only meaningful without overlap).

Prints ONE JSON line (see the keys at the bottom of main()).
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
    ap.add_argument("--iep-config", choices=["config1", "config2"], default="config2")
    ap.add_argument("--no-balance", action="store_true", help="plain improved sort, no pull-forward of nodes")
    ap.add_argument("--streams", type=int, default=4,
                    help="program-tree batches in flight: step i runs on HIP stream i %% streams with its own workspace")
    ap.add_argument("--moe-streams", type=int, default=3,
                    help="MoE layers in flight: call i runs on HIP stream i %% moe-streams with its own workspace")
    ap.add_argument("--skip-moe", action="store_true")
    ap.add_argument("--skip-naive", action="store_true")
    ap.add_argument("--no-prepare", action="store_true", help="repack the module weights inside every dynbatch_execute")
    ap.add_argument("--skip-schedules", action="store_true", help="skip the side-by-side timing of the four schedules")
    ap.add_argument("--skip-cpu", action="store_true")
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
    K, Wm = args.steps, args.warmup
    log = lambda *a: print(*a, file=sys.stderr, flush=True)

    # one plain 1 GiB device-to-device copy: the reference for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE
    cal_src = torch.ones(1 << 28, dtype=torch.int32, device="cuda")
    cal_dst = torch.empty_like(cal_src)
    cal_dst.copy_(cal_src)
    torch.cuda.synchronize()
    del cal_src, cal_dst

    # ------------------------------------------------------------------ program-tree engine
    w = getattr(iep, args.iep_config)()
    weights = U.iep_weights_dev(w)
    # constant weights are put into the kernels' fragment order once, outside the timed steps
    if not args.no_prepare:
        weights["packed"] = dyn.dynbatch_pack_weights(weights, w.C, w.H, w.W, dyn.DYNB_BF16)
    feats = U.to_dev(w.feats, w.dtype)
    out = torch.empty_like(feats)
    plan_flags = dyn.DYNB_SCHED_IMPROVED | (0 if args.no_balance else dyn.DYNB_PLAN_BALANCE)
    plan0 = dyn.dynbatch_plan(w.prog, w.prog_off, w.arity, plan_flags)
    view = dyn.dynbatch_plan_view(plan0)
    SCHEDULES = {"improved": dyn.DYNB_SCHED_IMPROVED, "improved+balance": dyn.DYNB_SCHED_IMPROVED | dyn.DYNB_PLAN_BALANCE,
                 "standard": dyn.DYNB_SCHED_STANDARD, "dependency_depth": dyn.DYNB_SCHED_DEPTH}
    ws_bytes = max(dyn.dynbatch_workspace_bytes(dyn.dynbatch_plan(w.prog, w.prog_off, w.arity, f), w.C, w.H, w.W,
                                                dyn.DYNB_BF16) for f in [dyn.DYNB_SCHED_NAIVE, *SCHEDULES.values()])
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    devbuf = torch.empty(dyn.dynbatch_plan_device_bytes(plan0) + 4096, dtype=torch.uint8, device="cuda")
    n_evals = view.n_compute_nodes
    n_binary = int((w.arity[w.prog] == 2).sum())
    flops_step = (n_evals - n_binary) * FLOP_UNARY + n_binary * FLOP_BINARY
    log(f"[bench] {w.name}: B={w.B} nodes={view.n_nodes} evals={n_evals} levels={view.n_levels} "
        f"launches={view.n_launches} buckets={view.n_buckets}")

    keep = []
    # Independent batches may be in flight together: every lane is a HIP stream (default priority) with its
    # own plan buffer, workspace and output, all resident in HBM.  Lane 0 is the current stream.
    S = max(1, args.streams)
    lanes = [dict(stream=None, devbuf=devbuf, ws=ws, out=out)]
    for _ in range(S - 1):
        lanes.append(dict(stream=torch.cuda.Stream(), devbuf=torch.empty_like(devbuf), ws=torch.empty_like(ws),
                          out=torch.empty_like(out)))

    def iep_step(flags=plan_flags, host_ms=None, lane=None):
        ln = lane if lane is not None else lanes[0]
        t0 = time.perf_counter()
        plan = dyn.dynbatch_plan(w.prog, w.prog_off, w.arity, flags)
        t1 = time.perf_counter()
        dyn.dynbatch_plan_upload(plan, ln["devbuf"], stream=ln["stream"])
        dyn.dynbatch_execute(plan, weights, feats, ln["out"], ln["ws"], stream=ln["stream"])
        if host_ms is not None:
            host_ms.append((t1 - t0) * 1e3)
        keep.append(plan)

    def timed_steps(n_lanes, flags):
        for i in range(n_lanes):                      # every lane's buffers and stream are touched once,
            iep_step(flags, lane=lanes[i])            # whatever --warmup says
        torch.cuda.synchronize()
        keep.clear()
        for i in range(Wm):
            iep_step(flags, lane=lanes[i % n_lanes])
        torch.cuda.synchronize()
        keep.clear()
        host = []
        t0 = time.perf_counter()
        for i in range(K):
            iep_step(flags, host_ms=host, lane=lanes[i % n_lanes])
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / K
        keep.clear()
        return ms, host

    one_ms, plan_ms = timed_steps(1, plan_flags)      # one batch at a time: the latency of a step
    iep_ms = one_ms
    if S > 1:                                         # S batches in flight: the throughput figure
        iep_ms, plan_ms = timed_steps(S, plan_flags | dyn.DYNB_PLAN_THROUGHPUT)
        for ln in lanes[1:min(S, K)]:                 # every lane that ran a step holds the same root maps
            assert torch.equal(ln["out"], lanes[0]["out"])

    # execute only (plan reused), and per-launch-group GPU times from HIP events on the same stream
    dyn.dynbatch_plan_upload(plan0, devbuf)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(K):
        dyn.dynbatch_execute(plan0, weights, feats, out, ws)
    torch.cuda.synchronize()
    exec_ms = (time.perf_counter() - t0) * 1e3 / K
    # the same launches replayed from a HIP graph (the call enqueues kernels only, so it can be captured)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        dyn.dynbatch_execute(plan0, weights, feats, out, ws)
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
        dyn.dynbatch_execute(plan0, weights, feats, out, ws)
        launch_ms.append(sum(ms for tag, _, ms in dyn.dynb_timing_read() if tag >= 0))
    dyn.dynb_timing_enable(0)
    kern_ms_step = float(np.mean(launch_ms))          # all module-kernel launches of one step
    avg_launch_us = kern_ms_step * 1e3 / launch_n
    achieved_tflops = flops_step / (kern_ms_step * 1e-3) / 1e12

    # the paper's schedules side by side (execute only, plan reused): launch groups, widest group, time
    sched_cmp = {}
    for name, fl in ([] if args.skip_schedules else SCHEDULES.items()):
        pl = dyn.dynbatch_plan(w.prog, w.prog_off, w.arity, fl)
        dyn.dynbatch_plan_upload(pl, devbuf)
        v_ = dyn.dynbatch_plan_view(pl)
        for _ in range(3):
            dyn.dynbatch_execute(pl, weights, feats, out, ws)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(K):
            dyn.dynbatch_execute(pl, weights, feats, out, ws)
        torch.cuda.synchronize()
        sched_cmp[name] = {"launch_groups": int(v_.n_launches), "max_group": int(v_.max_launch_nodes),
                           "pools": int((w.arity[v_.bucket_type] > 0).sum()),
                           "execute_ms": round((time.perf_counter() - t0) * 1e3 / K, 4)}

    naive = None
    if not args.skip_naive:
        iep_step(dyn.DYNB_SCHED_NAIVE)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        iep_step(dyn.DYNB_SCHED_NAIVE)
        torch.cuda.synchronize()
        naive_ms = (time.perf_counter() - t0) * 1e3
        keep.clear()
        naive = {"kind": "same kernels, one launch per node, example by example", "ms_per_step": round(naive_ms, 3),
                 "module_evals_per_sec": round(n_evals / naive_ms * 1e3, 1), "speedup_batched": round(naive_ms / one_ms, 2), "speedup_note": "against one batched step at a time on one stream"}

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
        t0 = time.perf_counter()
        for _ in range(K):
            moe_step()
        torch.cuda.synchronize()
        moe_ms = (time.perf_counter() - t0) * 1e3 / K
        # several layers (batches) in flight: the gate and grouping kernels of one run under the weight
        # streaming of another.  Lane buffers are allocated before, and the device drained, so that no
        # side stream touches memory the default stream may still be using.
        MS = max(1, args.moe_streams)
        moe_one_ms = moe_ms
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
            moe_ms = (time.perf_counter() - t0) * 1e3 / K
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
        stage_ms = {n: float(np.mean(v)) for n, v in stages.items()}
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
        ffn_ms = stage_ms["ffn1"] + stage_ms["ffn2"]
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
        moe_res = {"workload": m.name, "tokens_per_sec": round(m.T / moe_ms * 1e3, 1), "ms_per_step": round(moe_ms, 4),
                   "layers_in_flight": MS,
                   "single_stream": {"ms_per_step": round(moe_one_ms, 4), "tokens_per_sec": round(m.T / moe_one_ms * 1e3, 1)},
                   "stage_ms": {k_: round(v, 4) for k_, v in stage_ms.items()}, "active_experts": n_active,
                   "max_expert_rows": int(counts.max()), "naive_gpu": moe_naive}
        moe_roof = [
            {"kernel": "k_permute", "bound": "hbm", "achieved": round(by_perm / stage_ms["permute"] / 1e6, 1),
             "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(by_perm / stage_ms["permute"] / 1e6 / PEAK_HBM_GBS, 4),
             "traffic": None},
            {"kernel": "k_combine", "bound": "hbm", "achieved": round(by_comb / stage_ms["combine"] / 1e6, 1),
             "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(by_comb / stage_ms["combine"] / 1e6 / PEAK_HBM_GBS, 4),
             "traffic": None},
            {"kernel": "k_grouped_gemm (both expert layers)", "bound": "hbm", "achieved": round(by_ffn / ffn_ms / 1e6, 1),
             "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(by_ffn / ffn_ms / 1e6 / PEAK_HBM_GBS, 4),
             "mfma_tflops": round(fl_ffn / ffn_ms / 1e9, 1), "traffic": None},
        ]

    # ------------------------------------------------------------------ CPU oracle baseline (bounded sample)
    cpu = None
    if not args.skip_cpu:
        import oracle
        n_s = min(32, w.B)
        sub = w.subset(range(0, w.B, w.B // n_s)[:n_s])
        t0 = time.perf_counter()
        oracle.iep_forward_workload(sub)
        dt = time.perf_counter() - t0
        cpu = {"value": round(sub.n_module_evals / dt, 2), "unit": "module_evals/s", "cores": oracle.num_threads(),
               "kind": "oracle", "sample": f"{sub.B} of {w.B} examples of {w.name} ({sub.n_module_evals} module evaluations, "
               f"{dt:.1f} s wall, fp64 per-example tree recursion)"}
        if moe_res is not None:
            rows = np.random.default_rng(0).choice(m.T, 48, replace=False)
            idx = aux.topk_idx.cpu().numpy()
            wts = aux.topk_w.cpu().numpy().astype(np.float64)
            packs = {int(e): m.expert_weights(int(e)) for e in np.unique(idx[rows])}
            t0 = time.perf_counter()
            for t in rows:
                oracle.moe_token(m.x[t], wts[t], [packs[int(e)][0] for e in idx[t]], [packs[int(e)][1] for e in idx[t]])
            dt = time.perf_counter() - t0
            cpu["moe"] = {"value": round(len(rows) / dt, 2), "unit": "tokens/s", "cores": 1,
                          "sample": f"expert+combine stage of 48 of {m.T} tokens, one thread, {dt:.1f} s"}

    # HBM-side bytes per launch as measured by rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (see profiles/): counters
    # cannot be read from inside this process, so the committed measurement is quoted
    traffic = None
    moe_traffic = {}
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath) and args.iep_config == "config2":
        tj = json.load(open(tpath))
        traffic = round(tj["k_module_mfma"]["bytes_per_launch"])
        if args.moe_config == "config4":
            moe_traffic = {k_: round(v["fetch_bytes"] + v["write_bytes"]) for k_, v in tj["moe"].items()}
    for r_ in moe_roof:
        key = r_["kernel"].split(" ")[0]
        if key == "k_grouped_gemm" and "k_grouped_gemm<true>" in moe_traffic:
            r_["traffic"] = moe_traffic["k_grouped_gemm<true>"] + moe_traffic["k_grouped_gemm<false>"]
        elif key in moe_traffic:
            r_["traffic"] = moe_traffic[key]

    res = {
        "metric": "module_evals_per_sec", "value": round(n_evals / iep_ms * 1e3, 1), "unit": "module_evals/s",
        "n_gpus": 1, "steps": K, "warmup": Wm, "ms_per_step": round(iep_ms, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "batch": w.B, "nodes": int(view.n_nodes), "module_evals": int(n_evals),
                   "levels": int(view.n_levels), "launch_groups": int(view.n_launches), "C": w.C, "H": w.H, "W": w.W,
                   "step": "dynbatch_plan + dynbatch_plan_upload + dynbatch_execute",
                   "batches_in_flight": S, "kernel_layout": "throughput (DYNB_PLAN_THROUGHPUT)" if S > 1 else "latency",
                   "weights": "repacked per call" if args.no_prepare else "fragment order prepared once (dynbatch_pack_weights)",
                   "schedule": "improved topological sort" + ("" if args.no_balance else " + balanced launch groups")},
        "single_stream": {"ms_per_step": round(one_ms, 4), "module_evals_per_sec": round(n_evals / one_ms * 1e3, 1)},
        "chip_mfma_frac_of_step": round(flops_step / (iep_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
        "plan_host_ms": round(float(np.mean(plan_ms)), 4), "execute_only_ms": round(exec_ms, 4), "execute_only_graph_replay_ms": round(graph_ms, 4),
        "execute_only_module_evals_per_sec": round(n_evals / exec_ms * 1e3, 1),
        "roofline": {"kernel": "k_module_mfma", "bound": "mfma", "achieved": round(achieved_tflops, 2),
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved_tflops / PEAK_BF16_TFLOPS, 4),
                     "traffic": traffic, "launches_per_step": launch_n, "avg_launch_us": round(avg_launch_us, 2),
                     "flops_per_step": flops_step,
                     "configuration": "one batch at a time on one stream (layouts k_module_mfma<2>/<3>); with batches in "
                                      "flight kernels of different batches overlap on the chip, so a per-launch duration "
                                      "does not describe that mode: chip_mfma_frac_of_step = flops of a step / ms_per_step / peak",
                     "frac_of_step_with_batches_in_flight": round(flops_step / (iep_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)},
        "rooflines_other": moe_roof, "schedules": sched_cmp, "moe": moe_res, "naive_gpu": naive, "cpu_baseline": cpu,
        "paper_context": "paper reports ratios only: >14x cell execution (IEP, GTX 1080 Ti), up to 1000x (MoE, 11 GB card)",
    }
    print(json.dumps(res))


if __name__ == "__main__":
    main()
