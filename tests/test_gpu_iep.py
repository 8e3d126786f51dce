"""Parity of dynbatch_execute (HIP) against the CPU oracle, through the C ABI.

Tolerances (max |got - ref| / max |ref| per output tensor): 1e-4 for fp32 storage, 2e-2 for bf16
storage with fp32 accumulation.
"""
import numpy as np
import pytest

from workloads import iep

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


@pytest.fixture(scope="module")
def dyn():
    import torch
    assert torch.cuda.is_available()
    import paper_1707_02402_amd as d
    return d


@pytest.fixture(scope="module")
def util():
    from tests import gpu_util
    return gpu_util


@pytest.mark.parametrize("flags", [0, 1, 2, 3])
def test_config0_fp32_all_schedules(dyn, util, oracle, flags):
    w = iep.config0()
    ref = oracle.iep_forward_workload(w)
    got = util.iep_run(dyn, w, flags)
    for i in range(w.B):
        assert util.normwise(got[i], ref[i]) < TOL["f32"], i


@pytest.mark.parametrize("dtype,C,H,W", [("f32", 5, 3, 7), ("bf16", 16, 6, 5), ("f32", 33, 9, 9), ("bf16", 128, 7, 7)])
def test_generic_kernels_on_ragged_shapes(dyn, util, oracle, dtype, C, H, W):
    w = iep.small_mixed(seed=C + H, B=9, C=C, H=H, W=W, dtype=dtype, min_len=1, max_len=9)
    ref = oracle.iep_forward_workload(w)
    got = util.iep_run(dyn, w)
    for i in range(w.B):
        assert util.normwise(got[i], ref[i]) < TOL[dtype], i
        if len(w.program(i)) == 1:
            assert (got[i] == w.feats[i]).all()


@pytest.mark.parametrize("flags", [0, 1, 2, 3])
def test_mfma_path_small_batch_every_element(dyn, util, oracle, flags):
    """bf16, C=128, 14x14: 13 pixel tiles with a ragged last tile, unary and binary functions,
    single-SCENE programs, odd batch so the two-node workgroups get a lone node."""
    w = iep.small_mixed(seed=21, B=11, C=128, H=14, W=14, dtype="bf16", min_len=1, max_len=8)
    assert (w.arity[w.prog] == 2).any() and (w.arity[w.prog] == 1).any()
    ref = oracle.iep_forward_workload(w)
    got = util.iep_run(dyn, w, flags)
    for i in range(w.B):
        assert util.normwise(got[i], ref[i]) < TOL["bf16"], (i, util.normwise(got[i], ref[i]))


def test_mfma_path_launch_group_wider_than_the_chip(dyn, util, oracle):
    """More than 256 nodes in one launch group selects the layout with two workgroups per CU; sampled examples vs oracle."""
    w = iep.small_mixed(seed=5, B=701, C=128, H=14, W=14, dtype="bf16", min_len=2, max_len=4)
    v = dyn.dynbatch_plan_view(dyn.dynbatch_plan(w.prog, w.prog_off, w.arity))
    assert v.max_launch_nodes > 512 and v.max_launch_nodes % 2 == 1
    got = util.iep_run(dyn, w)
    sample = [0, 1, 350, 699, 700]
    ref = oracle.iep_forward_workload(w.subset(sample))
    for j, i in enumerate(sample):
        assert util.normwise(got[i], ref[j]) < TOL["bf16"], i
    naive = util.iep_run(dyn, w.subset(sample), dyn.DYNB_SCHED_NAIVE)
    assert (naive == got[sample]).all()          # batched == per-example, bit for bit


def test_identity_kernels_are_exact_on_the_mfma_path(dyn, util):
    """Unary module = 2x, binary module = 2(x0+x1) for identity kernels: exact powers of two in bf16."""
    C = 128
    g = np.random.default_rng(0)
    arity = np.array([0, 1, 2], np.uint8)
    progs = [np.array([1] * n + [0], np.int32) for n in (1, 4, 9)] + [iep.balanced_program(g, D, [2]) for D in (2, 4)]
    off = np.zeros(len(progs) + 1, np.int32)
    off[1:] = np.cumsum([len(p) for p in progs])
    f = np.abs(iep.make_feats(1, len(progs), 14, 14, C, "bf16"))
    w3 = np.zeros((3, C, 3, 3, C), np.float32)
    w1 = np.zeros((3, C, 2 * C), np.float32)
    for t in (1, 2):
        w3[t, np.arange(C), 1, 1, np.arange(C)] = 1
        w1[t, np.arange(C), np.arange(C)] = 1
        w1[t, np.arange(C), C + np.arange(C)] = 1
    w = iep.IepWorkload("closed-form", "bf16", arity, np.concatenate(progs), off, C, 14, 14, f, w1,
                        np.zeros((3, C), np.float32), w3, np.zeros((3, C), np.float32), w3.copy(),
                        np.zeros((3, C), np.float32))
    got = util.iep_run(dyn, w)
    for i, scale in enumerate([2.0, 16.0, 512.0, 4.0, 64.0]):
        assert (got[i] == scale * f[i]).all(), i


def lane_batch(lane: int):
    """Batch of lane `lane` of the benchmark: config 2 itself for lane 0, further batches of the same recipe
    (own programs and feature maps, the same 40 modules) for the others."""
    base = iep.config2.__defaults__[0]
    return iep.config2() if lane == 0 else iep.config2(seed=base + 1000 * lane, weight_seed=base)


def assert_every_example(util, got, ref, tol, what=""):
    errs = np.array([util.normwise(got[i], ref[i]) for i in range(len(ref))])
    assert errs.max() < tol, (what, int(errs.argmax()), float(errs.max()))
    return errs


def test_config1_balanced_trees_every_example(dyn, util, full_refs):
    w, ref = full_refs.get("config1", iep.config1)
    v = dyn.dynbatch_plan_view(dyn.dynbatch_plan(w.prog, w.prog_off, w.arity))
    assert v.n_levels == 5 and v.n_launches == 4 and v.n_compute_nodes == 960
    got = util.iep_run(dyn, w)
    assert_every_example(util, got, ref, TOL["bf16"], "config1")                # all 64 examples
    again = util.iep_run(dyn, w)
    assert (again == got).all()                  # deterministic
    assert np.isfinite(got).all() and (got >= 0).all()
    assert (util.iep_run(dyn, w, dyn.DYNB_PLAN_THROUGHPUT) == got).all()        # the other kernel layout: same bits


def test_config2_iep_shaped_every_example(dyn, util, full_refs):
    w, ref = full_refs.get("config2", iep.config2)
    got = util.iep_run(dyn, w)
    errs = assert_every_example(util, got, ref, TOL["bf16"], "config2")         # all 256 examples
    print(f"config 2: per-example error max {errs.max():.2e} median {np.median(errs):.2e}")
    # batched (improved sort) == standard sort == per-example loop, bit for bit, on a subset
    sub = w.subset(range(0, 256, 16))
    a = util.iep_run(dyn, sub, 0)
    assert (a == got[::16]).all()
    assert (util.iep_run(dyn, sub, 1) == a).all()
    assert (util.iep_run(dyn, sub, 2) == a).all()
    assert (util.iep_run(dyn, w, dyn.DYNB_PLAN_BALANCE) == got).all()      # balanced launch groups: same bits
    assert np.isfinite(got).all() and (got >= 0).all()


def test_config2_in_the_benchmarks_launch_configurations(dyn, util, full_refs):
    """Full config 2 as bench.py times it, every example of every batch against the oracle:
    (a) one batch at a time: balanced plan, prepared weights, latency layouts;
    (b) four different batches in flight on four streams: balanced + throughput plan, own workspaces."""
    import torch
    w, ref = full_refs.get("config2", iep.config2)
    weights = util.iep_weights_dev(w)
    weights["packed"] = dyn.dynbatch_pack_weights(weights, w.C, w.H, w.W, dyn.DYNB_BF16)
    got = util.iep_run(dyn, w, dyn.DYNB_SCHED_IMPROVED | dyn.DYNB_PLAN_BALANCE, weights=weights)
    assert_every_example(util, got, ref, TOL["bf16"], "config2, one batch at a time")
    flags = dyn.DYNB_SCHED_IMPROVED | dyn.DYNB_PLAN_BALANCE | dyn.DYNB_PLAN_THROUGHPUT
    batches = [full_refs.get("config2" if i == 0 else f"config2-lane{i}", lambda i=i: lane_batch(i)) for i in range(4)]
    for i in range(1, 4):
        assert (batches[i][0].w3a == w.w3a).all() and not (batches[i][0].feats == w.feats).all()
    torch.cuda.synchronize()
    lanes = []
    for wl, _ in batches:
        plan = dyn.dynbatch_plan(wl.prog, wl.prog_off, wl.arity, flags)
        feats = util.to_dev(wl.feats, "bf16")
        lanes.append(dict(stream=torch.cuda.Stream(), plan=plan, feats=feats, out=torch.empty_like(feats),
                          ws=torch.empty(dyn.dynbatch_workspace_bytes(plan, w.C, w.H, w.W, dyn.DYNB_BF16),
                                         dtype=torch.uint8, device="cuda")))
    torch.cuda.synchronize()
    for step in range(8):
        ln = lanes[step % 4]
        if step < 4:
            dyn.dynbatch_plan_upload(ln["plan"], stream=ln["stream"])
        dyn.dynbatch_execute(ln["plan"], weights, ln["feats"], ln["out"], ln["ws"], stream=ln["stream"])
    torch.cuda.synchronize()
    for i, (ln, (wl, r)) in enumerate(zip(lanes, batches)):
        assert_every_example(util, util.to_host(ln["out"]), r, TOL["bf16"], f"lane {i}")
    assert torch.equal(lanes[0]["out"], util.to_dev(got, "bf16"))               # lane 0 ran config 2 itself


def test_execute_error_paths(dyn, util):
    import torch
    w = iep.config0()
    plan = dyn.dynbatch_plan(w.prog, w.prog_off, w.arity)
    weights = util.iep_weights_dev(w)
    feats = util.to_dev(w.feats, "f32")
    with pytest.raises(dyn.DynbError) as e:
        dyn.dynbatch_execute(plan, weights, feats)
    assert e.value.name == "DYNB_E_WORKSPACE"            # not uploaded
    dyn.dynbatch_plan_upload(plan)
    with pytest.raises(dyn.DynbError) as e:
        dyn.dynbatch_execute(plan, weights, feats, workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert e.value.name == "DYNB_E_WORKSPACE"
    with pytest.raises(dyn.DynbError) as e:
        dyn.dynbatch_execute(plan, dict(weights, w1=None), feats)
    assert e.value.name == "DYNB_E_UNSUPPORTED"
    with pytest.raises(dyn.DynbError) as e:
        dyn.dynbatch_plan_upload(plan, torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert e.value.name == "DYNB_E_WORKSPACE"


def test_stage_timing_modes(dyn, util):
    """Mode 1: set-up stage, then one stage per launch group; mode 2: set-up stage, then one stage for all groups."""
    import torch
    w = iep.small_mixed(seed=77, B=9, C=128, H=14, W=14, dtype="bf16", min_len=3, max_len=9)
    plan = dyn.dynbatch_plan(w.prog, w.prog_off, w.arity)
    view = dyn.dynbatch_plan_view(plan)
    dyn.dynbatch_plan_upload(plan)
    weights = util.iep_weights_dev(w)
    feats = util.to_dev(w.feats, "bf16")
    out = torch.empty_like(feats)
    ws = torch.empty(dyn.dynbatch_workspace_bytes(plan, w.C, w.H, w.W, 1), dtype=torch.uint8, device="cuda")
    try:
        dyn.dynb_timing_enable(1)
        dyn.dynbatch_execute(plan, weights, feats, out, ws)
        st = dyn.dynb_timing_read()
        assert [t for t, _, _ in st] == [-2] + list(range(view.n_launches))
        assert sum(u for t, u, _ in st if t >= 0) == view.n_compute_nodes
        assert all(ms >= 0 for _, _, ms in st)
        dyn.dynb_timing_enable(2)
        dyn.dynbatch_execute(plan, weights, feats, out, ws)
        st2 = dyn.dynb_timing_read()
        assert [(t, u) for t, u, _ in st2] == [(-2, 0), (0, view.n_compute_nodes)]
        with pytest.raises(dyn.DynbError):
            dyn.dynb_timing_enable(3)
    finally:
        dyn.dynb_timing_enable(0)
    dyn.dynbatch_execute(plan, weights, feats, out, ws)      # untimed again: the marks of the last timed call stay readable
    assert [(t, u) for t, u, _ in dyn.dynb_timing_read()] == [(-2, 0), (0, view.n_compute_nodes)]


def test_dependency_depth_schedule_on_config2_equals_improved_bitwise(dyn, util):
    """Discussion / batching by dependency depth: another valid order of the same module calls, so the same bits;
    its slot recycling (results live until their consumer's label) is exercised at full size."""
    w = iep.config2()
    a = util.iep_run(dyn, w, dyn.DYNB_SCHED_IMPROVED)
    b = util.iep_run(dyn, w, dyn.DYNB_SCHED_DEPTH)
    assert (a == b).all()


def test_prepared_weights_give_the_same_bits(dyn, util):
    """dynbatch_pack_weights once, then execute with weights.packed: same kernels on the same fragments."""
    import torch
    w = iep.small_mixed(seed=31, B=13, C=128, H=14, W=14, dtype="bf16", min_len=2, max_len=9)
    plan = dyn.dynbatch_plan(w.prog, w.prog_off, w.arity)
    dyn.dynbatch_plan_upload(plan)
    weights = util.iep_weights_dev(w)
    feats = util.to_dev(w.feats, "bf16")
    a = dyn.dynbatch_execute(plan, weights, feats)
    nbytes = dyn.dynbatch_packed_weights_bytes(w.C, w.H, w.W, dyn.DYNB_BF16, w.n_types)
    assert nbytes == w.n_types * 20 * 128 * 128 * 2
    packed = dyn.dynbatch_pack_weights(weights, w.C, w.H, w.W, dyn.DYNB_BF16)
    assert packed.numel() == nbytes
    prepared = dict(weights, packed=packed)
    b = dyn.dynbatch_execute(plan, prepared, feats)
    c = dyn.dynbatch_execute(plan, prepared, feats)
    torch.cuda.synchronize()
    assert torch.equal(a, b) and torch.equal(b, c)
    # shapes without a fast path have no packed layout
    assert dyn.dynbatch_packed_weights_bytes(16, 8, 8, dyn.DYNB_F32, 5) == 0
    with pytest.raises(dyn.DynbError) as e:
        dyn.dynbatch_pack_weights(weights, 16, 8, 8, dyn.DYNB_F32)
    assert e.value.name == "DYNB_E_UNSUPPORTED"
    with pytest.raises(dyn.DynbError) as e:
        dyn.dynbatch_pack_weights(weights, w.C, w.H, w.W, dyn.DYNB_BF16, packed=packed[:4096])
    assert e.value.name == "DYNB_E_WORKSPACE"


@pytest.mark.parametrize("dtype,C,H,W", [("bf16", 128, 14, 14), ("f32", 4, 3, 3)])
def test_batches_without_any_module_call(dyn, util, dtype, C, H, W):
    """Every program is a lone SCENE token: no launch group, the output is the input, bit for bit."""
    w = iep.small_mixed(seed=2, B=5, C=C, H=H, W=W, dtype=dtype, min_len=1, max_len=1)
    v = dyn.dynbatch_plan_view(dyn.dynbatch_plan(w.prog, w.prog_off, w.arity))
    assert v.n_compute_nodes == 0 and v.n_launches == 0 and v.n_levels == 1
    got = util.iep_run(dyn, w)
    assert (got == w.feats).all()


@pytest.mark.parametrize("dtype,C,H,W", [("bf16", 128, 14, 14), ("f32", 3, 2, 5)])
def test_single_example_single_module(dyn, util, oracle, dtype, C, H, W):
    w = iep.small_mixed(seed=4, B=1, C=C, H=H, W=W, dtype=dtype, min_len=2, max_len=2)
    assert w.n_module_evals == 1
    got = util.iep_run(dyn, w)
    assert util.normwise(got, oracle.iep_forward_workload(w)) < TOL[dtype]


def test_generic_path_launch_group_wider_than_one_grid(dyn, util, oracle):
    """33000 one-module programs: the generic kernels split a launch group at 32768 nodes (grid.y limit)."""
    w = iep.small_mixed(seed=6, B=33000, C=2, H=2, W=3, dtype="f32", min_len=2, max_len=2)
    v = dyn.dynbatch_plan_view(dyn.dynbatch_plan(w.prog, w.prog_off, w.arity))
    assert v.max_launch_nodes == 33000
    got = util.iep_run(dyn, w)
    ref = oracle.iep_forward_workload(w)
    assert util.normwise(got, ref) < TOL["f32"]
    assert util.normwise(got[32760:32780], ref[32760:32780]) < TOL["f32"]      # around the split


def test_throughput_mode_and_batches_in_flight_on_three_streams(dyn, util):
    """DYNB_PLAN_THROUGHPUT only changes the kernel layout; batches that run concurrently on their own
    streams and workspaces must not disturb each other: every output equals the latency-mode result bit for bit."""
    import torch
    w = iep.config2(B=96)
    ref = util.iep_run(dyn, w, dyn.DYNB_PLAN_BALANCE, return_dev=True)
    weights = util.iep_weights_dev(w)
    weights["packed"] = dyn.dynbatch_pack_weights(weights, w.C, w.H, w.W, dyn.DYNB_BF16)
    feats = util.to_dev(w.feats, "bf16")
    flags = dyn.DYNB_PLAN_BALANCE | dyn.DYNB_PLAN_THROUGHPUT
    torch.cuda.synchronize()
    lanes = []
    for _ in range(3):
        plan = dyn.dynbatch_plan(w.prog, w.prog_off, w.arity, flags)
        lanes.append(dict(stream=torch.cuda.Stream(), plan=plan, out=torch.empty_like(feats),
                          ws=torch.empty(dyn.dynbatch_workspace_bytes(plan, w.C, w.H, w.W, dyn.DYNB_BF16),
                                         dtype=torch.uint8, device="cuda")))
    for rep in range(4):
        for ln in lanes:
            if rep == 0:
                dyn.dynbatch_plan_upload(ln["plan"], stream=ln["stream"])
            dyn.dynbatch_execute(ln["plan"], weights, feats, ln["out"], ln["ws"], stream=ln["stream"])
    torch.cuda.synchronize()
    for ln in lanes:
        assert torch.equal(ln["out"], ref)


def test_random_shapes_and_schedules(dyn, util, oracle):
    """Seeded sweep: generic shapes in both dtypes and the fast shape, every schedule and flag combination."""
    g = np.random.default_rng(7)
    flag_sets = [0, 1, 2, 3, dyn.DYNB_PLAN_BALANCE, dyn.DYNB_PLAN_THROUGHPUT, 3 | dyn.DYNB_PLAN_THROUGHPUT,
                 dyn.DYNB_PLAN_BALANCE | dyn.DYNB_PLAN_THROUGHPUT]
    for case in range(10):
        fast = case % 3 == 0
        dtype = "bf16" if fast else str(g.choice(["f32", "bf16"]))
        C, H, W = (128, 14, 14) if fast else (int(g.integers(1, 40)), int(g.integers(1, 9)), int(g.integers(1, 9)))
        if dtype == "bf16" and (C * H * W) % 2:
            C += 1                                     # bf16 maps are copied in 4-byte words
        w = iep.small_mixed(seed=300 + case, B=int(g.integers(1, 14)), C=C, H=H, W=W, dtype=dtype, min_len=1,
                            max_len=int(g.integers(1, 12)))
        ref = oracle.iep_forward_workload(w)
        base = None
        for flags in flag_sets:
            got = util.iep_run(dyn, w, flags)
            assert util.normwise(got, ref) < TOL[dtype] or np.abs(ref).max() == 0, (case, flags, C, H, W, dtype)
            if base is None:
                base = got
            assert (got == base).all(), (case, flags)   # every schedule gives the same bits


# ------------------------------------------------------------------------------------------------
# DYNB_PLAN_PERSISTENT: one dependency-driven launch per batch
# ------------------------------------------------------------------------------------------------
def run_persistent(dyn, util, w, flags, weights=None, feats=None):
    """plan -> upload -> execute -> check; returns the root maps (device tensor)."""
    import torch
    plan = dyn.dynbatch_plan(w.prog, w.prog_off, w.arity, flags | dyn.DYNB_PLAN_PERSISTENT)
    assert dyn.dynbatch_plan_view(plan).n_tickets >= dyn.dynbatch_plan_view(plan).n_compute_nodes
    dyn.dynbatch_plan_upload(plan)
    weights = weights if weights is not None else util.iep_weights_dev(w)
    feats = feats if feats is not None else util.to_dev(w.feats, w.dtype)
    ws = torch.empty(dyn.dynbatch_workspace_bytes(plan, w.C, w.H, w.W, dyn.DYNB_BF16 if w.dtype == "bf16" else dyn.DYNB_F32),
                     dtype=torch.uint8, device="cuda")
    out = dyn.dynbatch_execute(plan, weights, feats, workspace=ws)
    dyn.dynbatch_execute_check(plan, feats, ws)              # synchronises; raises if a bounded wait expired
    return out


@pytest.mark.parametrize("mode", [0, 1, 3])
def test_one_launch_per_batch_small_batches_every_element(dyn, util, oracle, mode):
    """Halves and whole nodes, unary and binary functions, single-SCENE programs; against the oracle and, bit for
    bit, against one launch per label."""
    w = iep.small_mixed(seed=21, B=11, C=128, H=14, W=14, dtype="bf16", min_len=1, max_len=8)
    ref = oracle.iep_forward_workload(w)
    got = util.to_host(run_persistent(dyn, util, w, mode))
    for i in range(w.B):
        assert util.normwise(got[i], ref[i]) < TOL["bf16"], (i, util.normwise(got[i], ref[i]))
    assert (got == util.iep_run(dyn, w, mode)).all()
    wide = iep.small_mixed(seed=5, B=301, C=128, H=14, W=14, dtype="bf16", min_len=2, max_len=5)   # whole-node units
    assert (util.to_host(run_persistent(dyn, util, wide, mode)) == util.iep_run(dyn, wide, mode)).all()


def test_one_launch_per_batch_full_configurations(dyn, util, full_refs):
    """Configs 1 and 2 in one dependency-driven launch each: every example against the oracle, and the same bits
    as one launch per label; twice in a row on the same workspace (flags and counters are cleared by the call)."""
    import torch
    for key, make in (("config1", iep.config1), ("config2", iep.config2)):
        w, ref = full_refs.get(key, make)
        weights = util.iep_weights_dev(w)
        weights["packed"] = dyn.dynbatch_pack_weights(weights, w.C, w.H, w.W, dyn.DYNB_BF16)
        feats = util.to_dev(w.feats, "bf16")
        plan = dyn.dynbatch_plan(w.prog, w.prog_off, w.arity, dyn.DYNB_SCHED_IMPROVED | dyn.DYNB_PLAN_PERSISTENT)
        dyn.dynbatch_plan_upload(plan)
        ws = torch.empty(dyn.dynbatch_workspace_bytes(plan, w.C, w.H, w.W, dyn.DYNB_BF16), dtype=torch.uint8, device="cuda")
        out = torch.empty_like(feats)
        for rep in range(2):
            out.fill_(float("nan"))
            dyn.dynbatch_execute(plan, weights, feats, out, ws)
            dyn.dynbatch_execute_check(plan, feats, ws)
            got = util.to_host(out)
            assert_every_example(util, got, ref, TOL["bf16"], f"{key}, one launch per batch, run {rep}")
        assert (got == util.iep_run(dyn, w, dyn.DYNB_PLAN_BALANCE, weights=weights)).all()


def test_one_launch_per_batch_dependency_graphs(dyn, util):
    d = iep.dag_batch(seed=8, B=150, C=128, H=14, W=14, dtype="bf16", max_nodes=10)
    import torch
    ref = util.dag_run(dyn, d, 0)
    plan = dyn.dynbatch_plan_dag(d.node_type, d.arg0, d.arg1, d.node_off, d.root, d.arity, dyn.DYNB_PLAN_PERSISTENT)
    dyn.dynbatch_plan_upload(plan)
    feats = util.to_dev(d.feats, "bf16")
    ws = torch.empty(dyn.dynbatch_workspace_bytes(plan, d.C, d.H, d.W, dyn.DYNB_BF16), dtype=torch.uint8, device="cuda")
    out = dyn.dynbatch_execute(plan, util.iep_weights_dev(d), feats, workspace=ws)
    dyn.dynbatch_execute_check(plan, feats, ws)
    assert (util.to_host(out) == ref).all()


def test_one_launch_per_batch_generic_shapes_fall_back_to_labels(dyn, util, oracle):
    w = iep.small_mixed(seed=9, B=7, C=6, H=3, W=4, dtype="f32", min_len=1, max_len=7)
    got = util.to_host(run_persistent(dyn, util, w, 0))
    assert util.normwise(got, oracle.iep_forward_workload(w)) < TOL["f32"]


def test_a_wait_that_expires_is_reported_and_every_workgroup_still_exits(dyn, util):
    """Error path forced from the host: with a spin limit of 0 a workgroup gives up as soon as an argument is not
    ready.  A chain of 6 nodes claimed by 6 resident workgroups at once cannot have its arguments ready (a node
    takes tens of microseconds), so the status word is raised, the kernel drains and the check reports it."""
    import torch
    w = iep.small_mixed(seed=4, B=1, C=128, H=14, W=14, dtype="bf16", min_len=7, max_len=7)
    w.prog, w.prog_off = np.array([1, 2, 3, 1, 2, 3, 0], np.int32), np.array([0, 7], np.int32)     # a chain of 6 unary modules
    assert w.n_module_evals == 6
    plan = dyn.dynbatch_plan(w.prog, w.prog_off, w.arity, dyn.DYNB_PLAN_PERSISTENT)
    dyn.dynbatch_plan_upload(plan)
    feats = util.to_dev(w.feats, "bf16")
    weights = util.iep_weights_dev(w)
    ws = torch.empty(dyn.dynbatch_workspace_bytes(plan, w.C, w.H, w.W, dyn.DYNB_BF16), dtype=torch.uint8, device="cuda")
    old = dyn.dynb_set_spin_limit(0)
    try:
        dyn.dynbatch_execute(plan, weights, feats, workspace=ws)
        with pytest.raises(dyn.DynbError) as e:
            dyn.dynbatch_execute_check(plan, feats, ws)
        assert e.value.name == "DYNB_E_HIP"
    finally:
        dyn.dynb_set_spin_limit(old)
    good = dyn.dynbatch_execute(plan, weights, feats, workspace=ws)          # the next call clears the status word
    dyn.dynbatch_execute_check(plan, feats, ws)
    assert (util.to_host(good) == util.iep_run(dyn, w)).all()
