"""Parity of dynbatch_classify (HIP) against the CPU oracle's classifier head, through the C ABI.

Tolerances: probabilities and logits, max |got - ref| / max |ref| per tensor: 1e-4 for fp32 storage; 2e-2 for bf16
storage (the kernels round z and h1 to bf16, the oracle keeps fp64).
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
    from workloads import device
    return device


def run_head(dyn, util, roots, head, dtype):
    import torch
    probs, logits = dyn.dynbatch_classify(util.to_dev(roots, dtype), util.head_dev(head, dtype), want_logits=True)
    torch.cuda.synchronize()
    return probs.cpu().numpy(), logits.cpu().numpy()


@pytest.mark.parametrize("dtype,B,C,H,W,Cc,F,A", [
    ("f32", 5, 7, 3, 4, 5, 9, 4),             # nothing a multiple of anything
    ("bf16", 9, 16, 6, 5, 8, 24, 10),         # MFMA path, ragged tiles everywhere
    ("bf16", 3, 12, 3, 3, 5, 7, 3),           # bf16 with inner extents that are not multiples of 8: FMA path
    ("bf16", 70, 128, 14, 14, 32, 256, 28),   # the fast shape: several row tiles, fc 1 cut along k
    ("f32", 130, 16, 8, 8, 16, 64, 28),
    ("bf16", 1, 128, 14, 14, 8, 8, 2),
])
def test_every_probability_against_the_oracle(dyn, util, oracle, dtype, B, C, H, W, Cc, F, A):
    roots = np.abs(iep.make_feats(B + C, B, H, W, C, dtype))          # root maps are outputs of a ReLU: non-negative
    head = iep.make_head(B * 7 + A, C, H, W, Cc, F, A, dtype)
    ref_p, ref_l = oracle.classify(roots, head["wc"], head["bc"], head["wf1"], head["bf1"], head["wf2"], head["bf2"],
                                   want_logits=True)
    got_p, got_l = run_head(dyn, util, roots, head, dtype)
    assert util.normwise(got_l, ref_l) < TOL[dtype], util.normwise(got_l, ref_l)
    for i in range(B):
        assert util.normwise(got_p[i], ref_p[i]) < TOL[dtype], (i, util.normwise(got_p[i], ref_p[i]))
    assert np.abs(got_p.sum(1) - 1).max() < 1e-5
    again_p, _ = run_head(dyn, util, roots, head, dtype)
    assert (again_p == got_p).all()                                    # k slices are summed in a fixed order


def test_without_biases_and_closed_forms(dyn, util, oracle):
    B, C, H, W, Cc, F, A = 6, 8, 2, 4, 8, 8, 8
    roots = np.abs(iep.make_feats(3, B, H, W, C, "bf16"))
    head = iep.make_head(11, C, H, W, Cc, F, A, "bf16")
    nb = dict(head, bc=None, bf1=None, bf2=None)
    got_p, got_l = run_head(dyn, util, roots, nb, "bf16")
    ref_p = oracle.classify(roots, nb["wc"], None, nb["wf1"], None, nb["wf2"], None)
    assert util.normwise(got_p, ref_p) < TOL["bf16"]
    zero = dict(nb, wf2=np.zeros_like(head["wf2"]))
    got_p, _ = run_head(dyn, util, roots, zero, "bf16")
    assert (got_p == np.float32(1.0 / A)).all()                       # zero last layer: exactly uniform
    # identity convolution, fc 1 picks flattened entries, fc 2 the identity: the logits are input values, exactly
    pick = [0, 9, 17, C * H * W - 1, 30, 2, 5, 40]
    wf1 = np.zeros((F, H * W * C), np.float32)
    for f, j in enumerate(pick):
        wf1[f, j] = 1.0
    ident = dict(wc=np.eye(C, dtype=np.float32), bc=None, wf1=wf1, bf1=None, wf2=np.eye(F, dtype=np.float32), bf2=None)
    _, got_l = run_head(dyn, util, roots, ident, "bf16")
    assert (got_l == roots.reshape(B, -1)[:, pick]).all()


def test_head_on_the_roots_of_an_executed_batch(dyn, util, oracle):
    """Programs -> dynbatch_execute -> dynbatch_classify, against the oracle's tree recursion followed by its head."""
    import torch
    w = iep.small_mixed(seed=17, B=12, C=128, H=14, W=14, dtype="bf16", min_len=1, max_len=7)
    head = iep.make_head(5, w.C, w.H, w.W, 16, 64, 28, "bf16")
    roots = util.iep_run(dyn, w, return_dev=True)
    probs = dyn.dynbatch_classify(roots, util.head_dev(head, "bf16"))
    torch.cuda.synchronize()
    ref = oracle.classify(oracle.iep_forward_workload(w).astype(np.float32), head["wc"], head["bc"], head["wf1"], head["bf1"],
                          head["wf2"], head["bf2"])
    got = probs.cpu().numpy()
    for i in range(w.B):
        assert util.normwise(got[i], ref[i]) < TOL["bf16"], (i, util.normwise(got[i], ref[i]))


def test_head_error_paths_and_empty_batch(dyn, util):
    import torch
    head = util.head_dev(iep.make_head(1, 8, 2, 2, 4, 4, 3, "f32"), "f32")
    roots = torch.zeros((2, 2, 2, 8), dtype=torch.float32, device="cuda")
    with pytest.raises(dyn.DynbError) as e:
        dyn.dynbatch_classify(roots, head, workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
    assert e.value.name == "DYNB_E_WORKSPACE"
    assert dyn.dynbatch_classify_workspace_bytes(8, 2, 2, dyn.DYNB_F32, 4, 4, 0, 2) == 0
    assert dyn.dynbatch_classify_workspace_bytes(8, 2, 2, 7, 4, 4, 3, 2) == 0
    out = dyn.dynbatch_classify(roots[:0], head)
    assert out.shape == (0, 3)
