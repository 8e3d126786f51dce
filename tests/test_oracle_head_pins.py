"""Pins of the oracle's classifier head (CPU only): what it computes is fixed by library routines, closed forms
and a brute-force sum, none of which share code with it."""
import numpy as np
import pytest


def _rand_head(g, B, C, H, W, Cc, F, A, bias=True):
    x = g.standard_normal((B, H, W, C)).astype(np.float32)
    wc = (g.standard_normal((Cc, C)) / np.sqrt(C)).astype(np.float32)
    wf1 = (g.standard_normal((F, H * W * Cc)) / np.sqrt(H * W * Cc)).astype(np.float32)
    wf2 = (g.standard_normal((A, F)) / np.sqrt(F)).astype(np.float32)
    bc = g.standard_normal(Cc).astype(np.float32) * 0.1 if bias else None
    bf1 = g.standard_normal(F).astype(np.float32) * 0.1 if bias else None
    bf2 = g.standard_normal(A).astype(np.float32) * 0.1 if bias else None
    return x, wc, bc, wf1, bf1, wf2, bf2


@pytest.mark.parametrize("B,C,H,W,Cc,F,A,bias", [(3, 5, 4, 3, 6, 7, 4, True), (2, 16, 8, 8, 8, 12, 10, False), (1, 3, 1, 1, 2, 2, 2, True)])
def test_against_torch_conv2d_linear_softmax(oracle, B, C, H, W, Cc, F, A, bias):
    """The same network from library layers in their own layout (NCHW, flatten in [C][H][W] order, so the first
    fully connected layer's columns are permuted here): a wrong flatten order, transposed weight or missing ReLU shows."""
    import torch
    import torch.nn.functional as Fn
    g = np.random.default_rng(B * 100 + C)
    x, wc, bc, wf1, bf1, wf2, bf2 = _rand_head(g, B, C, H, W, Cc, F, A, bias)
    probs, logits = oracle.classify(x, wc, bc, wf1, bf1, wf2, bf2, want_logits=True)
    t = lambda a: None if a is None else torch.from_numpy(a).double()
    z = Fn.relu(Fn.conv2d(t(x).permute(0, 3, 1, 2), t(wc)[:, :, None, None], t(bc)))           # [B,Cc,H,W]
    wf1_chw = t(wf1).reshape(F, H, W, Cc).permute(0, 3, 1, 2).reshape(F, Cc * H * W)         # columns in [Cc][H][W] order
    h1 = Fn.relu(Fn.linear(z.reshape(B, -1), wf1_chw, t(bf1)))
    lg = Fn.linear(h1, t(wf2), t(bf2))
    assert np.abs(logits - lg.numpy()).max() < 1e-12 * max(1.0, np.abs(lg.numpy()).max())
    assert np.abs(probs - torch.softmax(lg, 1).numpy()).max() < 1e-13
    assert np.abs(probs.sum(1) - 1).max() < 1e-14


def test_brute_force_sums_on_a_tiny_head(oracle):
    g = np.random.default_rng(7)
    B, C, H, W, Cc, F, A = 2, 2, 2, 2, 3, 2, 3
    x, wc, bc, wf1, bf1, wf2, bf2 = _rand_head(g, B, C, H, W, Cc, F, A)
    probs = oracle.classify(x, wc, bc, wf1, bf1, wf2, bf2)
    for i in range(B):
        z = []
        for y in range(H):
            for xx in range(W):
                for cc in range(Cc):
                    z.append(max(0.0, sum(float(x[i, y, xx, c]) * float(wc[cc, c]) for c in range(C)) + float(bc[cc])))
        h1 = [max(0.0, sum(z[j] * float(wf1[f, j]) for j in range(len(z))) + float(bf1[f])) for f in range(F)]
        lg = [sum(h1[f] * float(wf2[a, f]) for f in range(F)) + float(bf2[a]) for a in range(A)]
        e = [np.exp(v - max(lg)) for v in lg]
        assert np.allclose(probs[i], np.array(e) / sum(e), rtol=1e-13, atol=0)


def test_closed_forms(oracle):
    g = np.random.default_rng(1)
    B, C, H, W, Cc, F, A = 4, 3, 2, 3, 3, 5, 6
    x, wc, bc, wf1, bf1, wf2, bf2 = _rand_head(g, B, C, H, W, Cc, F, A)
    # all-zero last layer: uniform distribution whatever comes before
    p = oracle.classify(x, wc, bc, wf1, bf1, np.zeros_like(wf2), None)
    assert np.abs(p - 1.0 / A).max() < 1e-15
    # only the last bias: softmax of the bias, the same for every example
    p = oracle.classify(x, wc, bc, wf1, bf1, np.zeros_like(wf2), bf2)
    e = np.exp(bf2.astype(np.float64) - bf2.max())
    assert np.abs(p - e / e.sum()).max() < 1e-15
    # identity convolution on non-negative maps, first FC picks single flattened entries, second FC the identity:
    # logits are chosen input values, in [H][W][C] flatten order
    xpos = np.abs(x)
    pick = [0, 4, 7, C * H * W - 1, 9]
    wf1p = np.zeros((F, H * W * C), np.float32)
    for f, j in enumerate(pick):
        wf1p[f, j] = 1.0
    _, lg = oracle.classify(xpos, np.eye(C, dtype=np.float32), None, wf1p, None, np.eye(F, dtype=np.float32), None, want_logits=True)
    assert (lg == xpos.reshape(B, -1)[:, pick].astype(np.float64)).all()
    # a negative pre-activation is cut by the first ReLU: with -identity the map vanishes and only biases remain
    _, lg = oracle.classify(xpos, -np.eye(C, dtype=np.float32), None, wf1p, bf1, np.eye(F, dtype=np.float32), None, want_logits=True)
    assert np.allclose(lg, np.maximum(bf1, 0).astype(np.float64)[None, :].repeat(B, 0), rtol=0, atol=1e-15)
