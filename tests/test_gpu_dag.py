"""Dependency graphs with shared nodes on the GPU (dynbatch_plan_dag + dynbatch_execute) against the CPU
oracle, and against the same computation written out as trees (every shared sub-graph once per use), which the
deterministic kernels must reproduce bit for bit while evaluating fewer modules."""
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


def oracle_out(oracle, d):
    return oracle.iep_forward_dag(d.node_type, d.arg0, d.arg1, d.node_off, d.root, d.arity, d.feats,
                                  d.w1, d.b1, d.w3a, d.b3a, d.w3b, d.b3b)


@pytest.mark.parametrize("flags", [0, 3])
@pytest.mark.parametrize("dtype,C,H,W", [("f32", 6, 5, 4), ("bf16", 128, 14, 14)])
def test_small_graph_batches_every_element(dyn, util, oracle, dtype, C, H, W, flags):
    d = iep.dag_batch(seed=C + flags, B=10, C=C, H=H, W=W, dtype=dtype, max_nodes=10)
    got = util.dag_run(dyn, d, flags)
    ref = oracle_out(oracle, d)
    for i in range(d.B):
        assert util.normwise(got[i], ref[i]) < TOL[dtype], i
    tree = util.iep_run(dyn, d.expanded(), flags)
    assert (tree == got).all()


def test_fast_path_wide_graph_batch_with_throughput_layout(dyn, util, oracle):
    d = iep.dag_batch(seed=77, B=300, C=128, H=14, W=14, dtype="bf16", min_nodes=6, max_nodes=24, window=6)
    x = d.expanded()
    assert x.n_module_evals > 1.3 * d.n_module_evals        # sharing is substantial
    v = dyn.dynbatch_plan_view(dyn.dynbatch_plan_dag(d.node_type, d.arg0, d.arg1, d.node_off, d.root, d.arity))
    assert v.n_compute_nodes == d.n_module_evals and v.n_slots < v.n_compute_nodes
    got = util.dag_run(dyn, d)
    assert (util.dag_run(dyn, d, dyn.DYNB_PLAN_THROUGHPUT) == got).all()
    assert (util.dag_run(dyn, d, dyn.DYNB_SCHED_DEPTH) == got).all()
    assert (util.iep_run(dyn, x, dyn.DYNB_PLAN_BALANCE) == got).all()
    sample = [0, 1, 150, 299]
    import dataclasses
    for i in sample:
        b, e = int(d.node_off[i]), int(d.node_off[i + 1])
        one = dataclasses.replace(d, node_type=d.node_type[b:e], arg0=d.arg0[b:e], arg1=d.arg1[b:e],
                                  node_off=np.array([0, e - b], np.int32), root=d.root[i:i + 1], feats=d.feats[i:i + 1])
        assert util.normwise(got[i], oracle_out(oracle, one)[0]) < TOL["bf16"], i
