"""dynbatch_execute and moe_forward enqueue only kernels (no memset nodes, no host synchronisation), so a
caller may capture them into a HIP graph.  Every replay is checked against the eager result, with eager work
and synchronisations between the replays."""
import numpy as np
import pytest

from workloads import iep, moe

pytestmark = pytest.mark.gpu


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


def test_program_tree_execute_replays_from_a_graph(dyn, util):
    import torch
    w = iep.config2(B=48)
    plan = dyn.dynbatch_plan(w.prog, w.prog_off, w.arity, dyn.DYNB_PLAN_BALANCE)
    dyn.dynbatch_plan_upload(plan)
    weights = util.iep_weights_dev(w)
    weights["packed"] = dyn.dynbatch_pack_weights(weights, w.C, w.H, w.W, dyn.DYNB_BF16)
    feats = util.to_dev(w.feats, "bf16")
    ws = torch.empty(dyn.dynbatch_workspace_bytes(plan, w.C, w.H, w.W, dyn.DYNB_BF16), dtype=torch.uint8, device="cuda")
    eager = dyn.dynbatch_execute(plan, weights, feats, workspace=ws).clone()      # also sets kernel attributes
    out = torch.empty_like(feats)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        dyn.dynbatch_execute(plan, weights, feats, out, ws)
    for rep in range(3):
        out.zero_()
        ws.random_(0, 255)                                  # scratch contents must not matter
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), rep
        other = dyn.dynbatch_execute(plan, weights, feats)  # eager work between the replays
        torch.cuda.synchronize()
        assert torch.equal(other, eager)


def test_moe_forward_replays_from_a_graph(dyn, util):
    import torch
    m = moe.small(seed=8, T=700, d=128, h=192, E=24, k=3, empty_frac=0.1)
    W1 = np.stack([m.expert_weights(e)[0] for e in range(m.E)])
    W2 = np.stack([m.expert_weights(e)[1] for e in range(m.E)])
    dev = util.moe_inputs_dev(m, W1, W2)
    args = (dev["x"], dev["Wg"], dev["Wn"], dev["noise"], dev["W1"], dev["W2"], m.k)
    ws = torch.empty(dyn.moe_workspace_bytes(m.T, m.d, m.h, m.E, m.k), dtype=torch.uint8, device="cuda")
    eager = dyn.moe_forward(*args, workspace=ws).clone()
    out = torch.empty_like(dev["x"])
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        dyn.moe_forward(*args, out=out, workspace=ws)
    for rep in range(3):
        out.zero_()
        ws.random_(0, 255)
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), rep
        other = dyn.moe_forward(*args)
        torch.cuda.synchronize()
        assert torch.equal(other, eager)
