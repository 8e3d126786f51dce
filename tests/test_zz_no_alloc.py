"""moe_forward_static (the entry point that allocates nothing) against moe_forward, through the C ABI.

Both run the same kernels, one on the caller's workspace, the other on the library's built-in device
array, so every routing table must agree bit for bit and the output must agree within the layer's
tolerance (it is in fact bit-identical).  Two calls in a row, the second on a smaller layer, show that
what a call leaves behind in the shared array does not leak into the next one.
"""
import numpy as np
import pytest

from workloads import moe

pytestmark = pytest.mark.gpu

OUT_TOL = 2e-2


def _run_both(dyn, util, m):
    import torch
    W1 = np.stack([m.expert_weights(e)[0] for e in range(m.E)])
    W2 = np.stack([m.expert_weights(e)[1] for e in range(m.E)])
    dev = util.moe_inputs_dev(m, W1, W2)
    args = (dev["x"], dev["Wg"], dev["Wn"], dev["noise"], dev["W1"], dev["W2"], m.k)
    ref_out, ref_aux = dyn.moe_forward(*args, want_aux=True)
    # the caller's memory: output and (optional) routing tables; poisoned so that a skipped write shows
    out = torch.full_like(ref_out, float("nan"))
    aux = type(ref_aux)(**{n: torch.full_like(t, -7) for n, t in vars(ref_aux).items()})
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    dyn.moe_forward_static(*args, out=out, aux=aux)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before          # the binding itself allocated no tensor either
    for name in ("topk_idx", "counts", "offsets", "perm", "inv"):
        assert torch.equal(getattr(aux, name), getattr(ref_aux, name)), name      # integers: bit-exact
    assert torch.equal(aux.logits, ref_aux.logits) and torch.equal(aux.topk_w, ref_aux.topk_w)
    got, ref = util.to_host(out), util.to_host(ref_out)
    assert np.isfinite(got).all()
    assert util.normwise(got, ref) < OUT_TOL
    assert (got == ref).all()                               # same kernels, same order of operations
    return got


def test_two_calls_in_a_row_the_second_smaller():
    import torch
    assert torch.cuda.is_available()
    import paper_1707_02402_amd as dyn
    from tests import gpu_util as util
    big = moe.small(seed=77, T=1500, d=128, h=160, E=48, k=4, empty_frac=0.1)
    small = moe.small(seed=78, T=130, d=64, h=96, E=10, k=2)
    assert dyn.moe_workspace_bytes(big.T, big.d, big.h, big.E, big.k) <= dyn.MOE_STATIC_SCRATCH_BYTES
    _run_both(dyn, util, big)
    _run_both(dyn, util, small)
    # without aux pointers as well
    W1 = np.stack([small.expert_weights(e)[0] for e in range(small.E)])
    W2 = np.stack([small.expert_weights(e)[1] for e in range(small.E)])
    dev = util.moe_inputs_dev(small, W1, W2)
    args = (dev["x"], dev["Wg"], dev["Wn"], dev["noise"], dev["W1"], dev["W2"], small.k)
    ref = dyn.moe_forward(*args)
    out = torch.empty_like(ref)
    dyn.moe_forward_static(*args, out=out)
    torch.cuda.synchronize()
    assert torch.equal(out, ref)


def test_a_layer_beyond_the_built_in_array_is_rejected():
    import torch
    import paper_1707_02402_amd as dyn
    T, d, h, E, k = 16384, 1024, 2048, 1024, 4              # needs ~600 MB
    assert dyn.moe_workspace_bytes(T, d, h, E, k) > dyn.MOE_STATIC_SCRATCH_BYTES
    z = lambda *shape, dt=torch.bfloat16: torch.zeros(shape, dtype=dt, device="cuda")
    with pytest.raises(dyn.DynbError) as e:
        dyn.moe_forward_static(z(T, d), z(E, d), None, None, z(1, h, d).expand(E, h, d), z(1, d, h).expand(E, d, h), k,
                               out=z(T, d))
    assert e.value.name == "DYNB_E_WORKSPACE" and "built-in" in str(e.value)
