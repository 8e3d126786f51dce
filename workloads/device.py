"""Moves a synthetic workload to the device and calls the library through its binding: shared by the GPU
tests, the smoke check and the benchmark.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np
import torch

from .rng import bf16_bits, bf16_to_f32


def to_dev(a: np.ndarray, dtype: str) -> torch.Tensor:
    """float32 host array -> device tensor of `dtype` ("f32" or "bf16"; bf16 inputs are already representable)."""
    if a is None:
        return None
    if dtype == "bf16":
        bits = torch.from_numpy(bf16_bits(a).view(np.int16).reshape(a.shape))
        return bits.cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def to_host(t: torch.Tensor) -> np.ndarray:
    """device tensor -> float32 host array (exact for bf16)."""
    if t.dtype == torch.bfloat16:
        bits = t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        return bf16_to_f32(bits).reshape(t.shape)
    return t.cpu().numpy()


def normwise(got, ref) -> float:
    """max |got - ref| / max |ref| over the whole tensor."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    den = np.abs(ref).max()
    return float(np.abs(got - ref).max() / (den if den > 0 else 1.0))


def iep_weights_dev(w):
    return dict(w1=to_dev(w.w1, w.dtype) if (w.arity == 2).any() else None, b1=to_dev(w.b1, "f32"),
                w3a=to_dev(w.w3a, w.dtype), b3a=to_dev(w.b3a, "f32"),
                w3b=to_dev(w.w3b, w.dtype), b3b=to_dev(w.b3b, "f32"))


def iep_run(dyn, w, flags: int = 0, weights=None, feats=None, return_dev: bool = False):
    """plan -> upload -> execute; returns root maps as float32 host array [B,H,W,C]."""
    plan = dyn.dynbatch_plan(w.prog, w.prog_off, w.arity, flags)
    dyn.dynbatch_plan_upload(plan)
    weights = weights if weights is not None else iep_weights_dev(w)
    feats = feats if feats is not None else to_dev(w.feats, w.dtype)
    out = dyn.dynbatch_execute(plan, weights, feats)
    torch.cuda.synchronize()
    return out if return_dev else to_host(out)


def dag_run(dyn, d, flags: int = 0, weights=None, feats=None):
    """dependency graphs: plan -> upload -> execute; returns root maps as float32 host array [B,H,W,C]."""
    plan = dyn.dynbatch_plan_dag(d.node_type, d.arg0, d.arg1, d.node_off, d.root, d.arity, flags)
    dyn.dynbatch_plan_upload(plan)
    weights = weights if weights is not None else iep_weights_dev(d)
    feats = feats if feats is not None else to_dev(d.feats, d.dtype)
    out = dyn.dynbatch_execute(plan, weights, feats)
    torch.cuda.synchronize()
    return to_host(out)


def moe_inputs_dev(m, W1: np.ndarray, W2: np.ndarray):
    """Device tensors in the library's layouts (gate matrices transposed to [E,d])."""
    return dict(x=to_dev(m.x, "bf16"), Wg=to_dev(np.ascontiguousarray(m.Wg.T), "bf16"),
                Wn=to_dev(np.ascontiguousarray(m.Wn.T), "bf16"), noise=to_dev(m.noise, "f32"),
                W1=to_dev(W1, "bf16"), W2=to_dev(W2, "bf16"))


def moe_run(dyn, m, W1=None, W2=None, dev=None, noise: bool = True):
    """Whole layer; returns (out float32 [T,d], dict of host aux arrays)."""
    dev = dev if dev is not None else moe_inputs_dev(m, W1, W2)
    out, aux = dyn.moe_forward(dev["x"], dev["Wg"], dev["Wn"] if noise else None, dev["noise"] if noise else None,
                               dev["W1"], dev["W2"], m.k, want_aux=True)
    torch.cuda.synchronize()
    return to_host(out), {k: v.cpu().numpy() for k, v in vars(aux).items()}


def head_dev(head: dict, dtype: str) -> dict:
    """Classifier-head weights on the device (weights in `dtype`, biases float32)."""
    return {k: (to_dev(v, dtype) if k in ("wc", "wf1", "wf2") else to_dev(v, "f32")) for k, v in head.items()}
