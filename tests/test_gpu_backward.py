"""Parity of dynbatch_backward (HIP) against the CPU oracle's backward pass, through the C ABI.

fp32 storage: every gradient tensor within 1e-4 (max |got - ref| / max |ref|).
bf16 storage: the ReLU decisions [y > 0], [mid > 0], [u > 0] of the backward pass are taken on the stored activations,
which are bfloat16 on the GPU.  Both sides take them in that precision: the oracle runs its bf16-storage mode (it
rounds u, mid and y to bfloat16 where the kernels store them and keeps everything else in fp64).  Bar: 2e-2 in the
max norm wherever the two sides hold the same stored activations: single modules at the full size, and programs of
any depth at a small channel count (there every fp32 sum rounds to the same bfloat16 as the fp64 sum).  At C = 128 a
3x3 convolution sums 1152 products; fp32 and fp64 sums then differ by ~5e-5 of the result, which moves 1-2 % of the
stored activations of every module to the neighbouring bfloat16.  Such a difference cannot be removed by any choice of
rounding points, and the gradient of a ReLU network is not continuous in its activations (the oracle's own gradients
with and without bf16 storage differ by 8 % in the Frobenius norm on this workload): deep programs at C = 128 are
therefore compared in the relative Frobenius norm of every gradient tensor with a bar of 5e-2 (observed 2-4e-2).
At the shape of the fused kernels (bf16, C = 128, 14 x 14) the backward pass runs on MFMAs, whose operands are bf16:
the gradient maps g, dmid and dc are rounded to bfloat16 (relative error up to 2^-9, independent from element to
element) before they are multiplied.  A sum of n such products then deviates by about 2^-9 / sqrt(3) of its own
typical size whatever n is, i.e. ~1e-3; with two or three such stages in a row a single module is off by 2-3e-3
of the tensor maximum (observed), against a bar of 1e-2.
"""
import numpy as np
import pytest

from workloads import iep

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dyn():
    import torch
    assert torch.cuda.is_available()
    import paper_1707_02402_amd as d
    return d


@pytest.fixture(scope="module")
def util():
    from workloads import device
    return device


def run_backward(dyn, util, w, dout, flags=0):
    import torch
    dt = dyn.DYNB_BF16 if w.dtype == "bf16" else dyn.DYNB_F32
    plan = dyn.dynbatch_plan(w.prog, w.prog_off, w.arity, flags | dyn.DYNB_PLAN_KEEP)
    dyn.dynbatch_plan_upload(plan)
    weights = util.iep_weights_dev(w)
    if weights["w1"] is None:
        weights["w1"] = util.to_dev(w.w1, w.dtype)
    feats = util.to_dev(w.feats, w.dtype)
    ws = torch.empty(dyn.dynbatch_workspace_bytes(plan, w.C, w.H, w.W, dt), dtype=torch.uint8, device="cuda")
    out = dyn.dynbatch_execute(plan, weights, feats, workspace=ws)
    g = dyn.dynbatch_backward(plan, weights, feats, out, ws, torch.from_numpy(dout).cuda())
    torch.cuda.synchronize()
    return {k: v.cpu().numpy() for k, v in g.items()}, util.to_host(out)


def maxnorm(got, ref):
    den = np.abs(ref).max()
    return float(np.abs(got - ref).max() / (den if den > 0 else 1.0))


def frob(got, ref):
    den = np.sqrt((ref.astype(np.float64) ** 2).sum())
    return float(np.sqrt(((got - ref) ** 2).sum()) / (den if den > 0 else 1.0))


NAMES = ("dfeats", "dw1", "db1", "dw3a", "db3a", "dw3b", "db3b")


@pytest.mark.parametrize("flags", [0, 1, 3, 4])
def test_config0_fp32_every_gradient(dyn, util, oracle, flags):
    w = iep.config0()
    dout = np.random.default_rng(0).standard_normal(w.feats.shape).astype(np.float32)
    ref = oracle.iep_backward_workload(w, dout)
    got, _ = run_backward(dyn, util, w, dout, flags)
    for name in NAMES:
        assert maxnorm(got[name], getattr(ref, name)) < 1e-4, (name, maxnorm(got[name], getattr(ref, name)))


@pytest.mark.parametrize("C,H,W,B", [(5, 3, 7, 9), (33, 4, 4, 6), (3, 1, 1, 4)])
def test_ragged_shapes_fp32_with_single_scene_programs(dyn, util, oracle, C, H, W, B):
    w = iep.small_mixed(seed=C + B, B=B, C=C, H=H, W=W, dtype="f32", min_len=1, max_len=9)
    dout = np.random.default_rng(C).standard_normal(w.feats.shape).astype(np.float32)
    ref = oracle.iep_backward_workload(w, dout)
    got, _ = run_backward(dyn, util, w, dout)
    for name in NAMES:
        assert maxnorm(got[name], getattr(ref, name)) < 1e-4, (name, maxnorm(got[name], getattr(ref, name)))
    for i in range(w.B):
        if len(w.program(i)) == 1:
            assert (got["dfeats"][i] == dout[i]).all()
    again, _ = run_backward(dyn, util, w, dout)
    for name in NAMES:
        assert (again[name] == got[name]).all(), name                     # fixed summation order: same bits


def test_bf16_fast_shape_after_the_fused_forward(dyn, util, oracle):
    """bf16, C = 128, 14 x 14: the forward pass runs the fused MFMA kernels and leaves every node's result in the
    workspace; the backward pass reads them from there."""
    w = iep.small_mixed(seed=23, B=5, C=128, H=14, W=14, dtype="bf16", min_len=1, max_len=6)
    assert (w.arity[w.prog] == 2).any()
    dout = np.random.default_rng(1).standard_normal(w.feats.shape).astype(np.float32)
    ref = oracle.iep_backward_workload(w, dout, round_bf16=True)
    got, out = run_backward(dyn, util, w, dout, dyn.DYNB_PLAN_BALANCE)
    assert util.normwise(out, oracle.iep_forward_workload(w)) < 2e-2
    assert util.normwise(out, ref.roots) < 2e-2
    errs = {name: frob(got[name], getattr(ref, name)) for name in NAMES}
    print("relative Frobenius errors", errs)
    for name in NAMES:
        assert errs[name] < 5e-2, (name, errs[name])
    plain = oracle.iep_backward_workload(w, dout)
    assert frob(plain.dfeats, ref.dfeats) > errs["dfeats"]           # closer to the bf16-storage oracle than that is to fp64


def test_bf16_deep_programs_at_a_small_channel_count(dyn, util, oracle):
    """Programs of any depth, two-argument functions with computed arguments, bf16 storage, 144 products per sum: the
    stored activations of both sides are the same bfloat16 values, so the gradients agree tightly."""
    w = iep.small_mixed(seed=23, B=7, C=16, H=6, W=5, dtype="bf16", min_len=1, max_len=9)
    assert (w.arity[w.prog] == 2).any()
    dout = np.random.default_rng(1).standard_normal(w.feats.shape).astype(np.float32)
    ref = oracle.iep_backward_workload(w, dout, round_bf16=True)
    got, out = run_backward(dyn, util, w, dout)
    assert (out != ref.roots).mean() < 0.01
    for name in NAMES:
        assert maxnorm(got[name], getattr(ref, name)) < 2e-2, (name, maxnorm(got[name], getattr(ref, name)))


def test_bf16_single_modules(dyn, util, oracle):
    """One module per program (a one-argument or a two-argument function on SCENE leaves): no upstream activation
    can differ, so only the bf16 rounding of the gradient operands separates the two sides."""
    arity = np.array([0, 1, 1, 2, 2], np.uint8)
    progs = [np.array(p, np.int32) for p in ([1, 0], [3, 0, 0], [2, 0], [4, 0, 0], [1, 0], [3, 0, 0])]
    off = np.concatenate([[0], np.cumsum([len(p) for p in progs])]).astype(np.int32)
    C, H, W = 128, 14, 14
    wts = iep.make_weights(77, arity, C, "bf16")
    w = iep.IepWorkload("single-modules", "bf16", arity, np.concatenate(progs), off, C, H, W,
                        iep.make_feats(77, len(progs), H, W, C, "bf16"), *wts)
    dout = np.random.default_rng(3).standard_normal(w.feats.shape).astype(np.float32)
    ref = oracle.iep_backward_workload(w, dout, round_bf16=True)
    got, out = run_backward(dyn, util, w, dout)
    for name in NAMES:
        assert maxnorm(got[name], getattr(ref, name)) < 1e-2, (name, maxnorm(got[name], getattr(ref, name)))
        assert frob(got[name], getattr(ref, name)) < 5e-3, (name, frob(got[name], getattr(ref, name)))
    again, _ = run_backward(dyn, util, w, dout)
    for name in NAMES:
        assert (again[name] == got[name]).all(), name                     # no atomics: same bits


def _sampled(w, seed):
    """dout that is zero outside a sample of the examples, and the sample as a workload of its own.  The backward
    pass is linear in dout and examples are independent, so every parameter gradient of the full batch equals that
    of the sample alone, which the oracle computes program by program."""
    sample = np.arange(3, w.B, 11)                                          # 23 of 256 programs
    sub = w.subset(sample)
    dsub = np.random.default_rng(seed).standard_normal(sub.feats.shape).astype(np.float32)
    dout = np.zeros(w.feats.shape, np.float32)
    dout[sample] = dsub
    return sample, sub, dsub, dout


def test_config2_full_batch_with_every_unit_active(dyn, util, oracle):
    """The benchmark's programs, shapes and launch configuration (256 programs, 27 labels, balanced launch groups,
    MFMA kernels) with non-negative weights, biases and feature maps: every ReLU is active, the network is linear,
    and nothing but rounding separates the two sides at any depth.  This pins the routing of the gradients through
    4066 nodes, the sums over all nodes of a function and every launch shape; the masks are pinned by the tests above."""
    import dataclasses
    from workloads.rng import round_bf16, stream
    w = iep.config2()
    g = stream(4242, 1)
    C = w.C
    pos = lambda shape, mean: round_bf16((g.random(shape, dtype=np.float32) * 2 * mean).astype(np.float32))
    binary = (w.arity == 2)[:, None, None]
    w = dataclasses.replace(
        w, feats=pos(w.feats.shape, 0.5),
        w1=pos(w.w1.shape, 0.5 / (2 * C)) * binary, b1=pos(w.b1.shape, 0.05) * binary[:, :, 0],
        w3a=pos(w.w3a.shape, 0.3 / (9 * C)), b3a=pos(w.b3a.shape, 0.05),
        w3b=pos(w.w3b.shape, 0.3 / (9 * C)), b3b=pos(w.b3b.shape, 0.05))
    sample, sub, dsub, dout = _sampled(w, 6)
    ref = oracle.iep_backward_workload(sub, dsub, round_bf16=True)
    got, out = run_backward(dyn, util, w, dout, dyn.DYNB_PLAN_BALANCE)
    assert (out > 0).all()
    assert util.normwise(out[sample], ref.roots) < 2e-2
    errs = {name: maxnorm(got[name][sample] if name == "dfeats" else got[name], getattr(ref, name)) for name in NAMES}
    print("max-norm errors, all units active", errs)
    for name in NAMES:
        assert errs[name] < 1e-2, (name, errs[name])                        # observed 1e-4 (dfeats) .. 2e-3
    rest = np.setdiff1d(np.arange(w.B), sample)
    assert (got["dfeats"][rest] == 0).all()


def test_config2_full_batch_against_the_oracle_on_sampled_examples(dyn, util, oracle):
    """The benchmark's configuration as bench.py runs it.  Programs of up to 30 modules amplify what the module
    docstring describes: a stored activation that rounds to the neighbouring bfloat16 flips a ReLU decision somewhere
    downstream, and the oracle's own gradients with fp64 and with bf16 storage differ by 15-30 % in the Frobenius norm
    on these programs (the forward results by 1 %).  The kernels are held to that spread: no gradient tensor may be
    further from the bf16-storage oracle than 1.25 times the distance between the oracle's two modes (+ 0.02), and short
    programs must be close."""
    w = iep.config2()
    sample, sub, dsub, dout = _sampled(w, 5)
    ref = oracle.iep_backward_workload(sub, dsub, round_bf16=True)
    plain = oracle.iep_backward_workload(sub, dsub)
    got, out = run_backward(dyn, util, w, dout, dyn.DYNB_PLAN_BALANCE)
    assert util.normwise(out[sample], ref.roots) < 2e-2
    for name in NAMES:
        err = frob(got[name][sample] if name == "dfeats" else got[name], getattr(ref, name))
        spread = frob(getattr(plain, name), getattr(ref, name))
        print(name, "kernels vs bf16-storage oracle", round(err, 4), "fp64 oracle vs bf16-storage oracle", round(spread, 4))
        assert err < 1.25 * spread + 0.02, (name, err, spread)
    rest = np.setdiff1d(np.arange(w.B), sample)
    assert (got["dfeats"][rest] == 0).all()


def test_keep_plans_with_the_persistent_flag(dyn, util):
    """A plan that keeps u and mid for the backward pass runs one launch per label even if one dependency-driven
    launch was asked for; its status word reads "no wait expired" and its backward pass gives the same bits."""
    import torch
    w = iep.small_mixed(seed=23, B=5, C=128, H=14, W=14, dtype="bf16", min_len=1, max_len=6)
    dout = np.random.default_rng(1).standard_normal(w.feats.shape).astype(np.float32)
    ref, out0 = run_backward(dyn, util, w, dout, dyn.DYNB_PLAN_BALANCE)
    got, out1 = run_backward(dyn, util, w, dout, dyn.DYNB_PLAN_PERSISTENT)
    assert (out0 == out1).all()
    for name in NAMES:
        assert (got[name] == ref[name]).all(), name
    plan = dyn.dynbatch_plan(w.prog, w.prog_off, w.arity, dyn.DYNB_PLAN_PERSISTENT | dyn.DYNB_PLAN_KEEP)
    dyn.dynbatch_plan_upload(plan)
    feats = util.to_dev(w.feats, w.dtype)
    ws = torch.empty(dyn.dynbatch_workspace_bytes(plan, w.C, w.H, w.W, dyn.DYNB_BF16), dtype=torch.uint8, device="cuda")
    ws.fill_(0xff)
    dyn.dynbatch_execute(plan, util.iep_weights_dev(w), feats, workspace=ws)
    dyn.dynbatch_execute_check(plan, feats, ws)


def test_closed_form_identity_kernels(dyn, util):
    """Chains of n doubling modules on positive maps: dL/dx = 2^n dout, exactly."""
    C, H, W = 8, 4, 4
    arity = np.array([0, 1], np.uint8)
    progs = [np.array([1] * n + [0], np.int32) for n in (1, 3, 6)]
    off = np.concatenate([[0], np.cumsum([len(p) for p in progs])]).astype(np.int32)
    w3 = np.zeros((2, C, 3, 3, C), np.float32)
    w3[1, np.arange(C), 1, 1, np.arange(C)] = 1
    z = np.zeros((2, C), np.float32)
    feats = np.abs(iep.make_feats(2, 3, H, W, C, "f32")) + 0.5
    w = iep.IepWorkload("chains", "f32", arity, np.concatenate(progs), off, C, H, W, feats, np.zeros((2, C, 2 * C), np.float32),
                        z, w3, z, w3.copy(), z)
    dout = np.random.default_rng(2).standard_normal(feats.shape).astype(np.float32)
    got, out = run_backward(dyn, util, w, dout)
    for i, n in enumerate((1, 3, 6)):
        assert (out[i] == 2.0 ** n * feats[i]).all()
        assert (got["dfeats"][i] == np.float32(2.0 ** n) * dout[i]).all()


def test_backward_error_paths(dyn, util):
    import torch
    w = iep.config0()
    weights = util.iep_weights_dev(w)
    feats = util.to_dev(w.feats, "f32")
    dout = torch.zeros_like(feats)
    plan = dyn.dynbatch_plan(w.prog, w.prog_off, w.arity)              # no DYNB_PLAN_KEEP
    dyn.dynbatch_plan_upload(plan)
    ws = torch.empty(dyn.dynbatch_workspace_bytes(plan, w.C, w.H, w.W, dyn.DYNB_F32), dtype=torch.uint8, device="cuda")
    out = dyn.dynbatch_execute(plan, weights, feats, workspace=ws)
    with pytest.raises(dyn.DynbError) as e:
        dyn.dynbatch_backward(plan, weights, feats, out, ws, dout)
    assert e.value.name == "DYNB_E_UNSUPPORTED"
    keep = dyn.dynbatch_plan(w.prog, w.prog_off, w.arity, dyn.DYNB_PLAN_KEEP)
    with pytest.raises(dyn.DynbError) as e:
        dyn.dynbatch_backward(keep, weights, feats, out, ws, dout, workspace=torch.empty(1 << 20, dtype=torch.uint8, device="cuda"))
    assert e.value.name == "DYNB_E_WORKSPACE"                          # not uploaded
    dyn.dynbatch_plan_upload(keep)
    with pytest.raises(dyn.DynbError) as e:
        dyn.dynbatch_backward(keep, weights, feats, out, ws, dout, workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert e.value.name == "DYNB_E_WORKSPACE"
    d = iep.dag_batch(seed=1, B=3, C=4, H=2, W=2, dtype="f32")
    dplan = dyn.dynbatch_plan_dag(d.node_type, d.arg0, d.arg1, d.node_off, d.root, d.arity, dyn.DYNB_PLAN_KEEP)
    dyn.dynbatch_plan_upload(dplan)
    with pytest.raises(dyn.DynbError) as e:
        dyn.dynbatch_backward(dplan, weights, feats, out, ws, dout)
    assert e.value.name == "DYNB_E_UNSUPPORTED"
