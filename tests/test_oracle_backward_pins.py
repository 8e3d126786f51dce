"""Pins of the oracle's backward pass (CPU only): torch's reverse-mode differentiation of an independent
library-layer implementation of the same programs, central finite differences of the oracle's own (separately
pinned) forward pass, and closed forms."""
import numpy as np
import pytest

from workloads import iep


def torch_tree_grads(w, dout, round_bf16=False):
    """The programs of w from torch layers (conv2d on NCHW, cat, relu), differentiated by autograd in fp64.
    round_bf16: stored activations pass through torch's own bfloat16 conversion (identity in the backward pass)."""
    import torch
    import torch.nn.functional as F

    def st(x):
        return x + (x.detach().to(torch.float32).to(torch.bfloat16).to(torch.float64) - x.detach()) if round_bf16 else x

    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).double().requires_grad_(True)
    feats = t(w.feats)
    P = dict(w1=t(w.w1), b1=t(w.b1), w3a=t(w.w3a), b3a=t(w.b3a), w3b=t(w.w3b), b3b=t(w.b3b))

    def conv3(x, wt, b):                      # x [1,C,H,W]; wt [Cout,3,3,Cin] -> OIHW
        return F.conv2d(x, wt.permute(0, 3, 1, 2), b, padding=1)

    def ev(i, pos):
        ty = int(w.prog[pos]); pos += 1
        if w.arity[ty] == 0:
            return feats[i].permute(2, 0, 1)[None], pos
        a, pos = ev(i, pos)
        if w.arity[ty] == 2:
            b, pos = ev(i, pos)
            u = st(F.relu(F.conv2d(torch.cat([a, b], 1), P["w1"][ty][:, :, None, None], P["b1"][ty])))
        else:
            u = a
        m = st(F.relu(conv3(u, P["w3a"][ty], P["b3a"][ty])))
        return st(F.relu(u + conv3(m, P["w3b"][ty], P["b3b"][ty]))), pos

    loss = 0
    for i in range(w.B):
        y, end = ev(i, int(w.prog_off[i]))
        assert end == w.prog_off[i + 1]
        loss = loss + (y[0].permute(1, 2, 0) * torch.from_numpy(dout[i]).double()).sum()
    loss.backward()
    out = {k: v.grad.numpy() if v.grad is not None else np.zeros(v.shape) for k, v in P.items()}
    out["feats"] = feats.grad.numpy()
    return out


@pytest.mark.parametrize("seed,B,C,H,W", [(1, 5, 3, 4, 5), (2, 4, 6, 3, 3), (3, 3, 2, 1, 1), (4, 6, 4, 6, 2)])
def test_against_torch_autograd(oracle, seed, B, C, H, W):
    w = iep.small_mixed(seed=seed, B=B, C=C, H=H, W=W, dtype="f32", min_len=1, max_len=9)
    assert (w.arity[w.prog] == 2).any() or seed == 3
    dout = np.random.default_rng(seed).standard_normal(w.feats.shape).astype(np.float32)
    g = oracle.iep_backward_workload(w, dout)
    ref = torch_tree_grads(w, dout)
    for mine, theirs in ((g.dfeats, ref["feats"]), (g.dw1, ref["w1"]), (g.db1, ref["b1"]), (g.dw3a, ref["w3a"]),
                         (g.db3a, ref["b3a"]), (g.dw3b, ref["w3b"]), (g.db3b, ref["b3b"])):
        scale = max(1.0, np.abs(theirs).max())
        assert np.abs(mine - theirs).max() < 1e-11 * scale


@pytest.mark.parametrize("seed,B,C,H,W", [(11, 4, 5, 3, 4), (12, 5, 8, 2, 2)])
def test_bf16_storage_mode_against_torch_with_its_own_bfloat16_conversion(oracle, seed, B, C, H, W):
    """round_bf16: the forward evaluation rounds u, mid and y to bfloat16 (checked against torch's conversion, so a
    wrong rounding rule or a missed rounding point shows in the root maps), the gradients follow the rounded values."""
    w = iep.small_mixed(seed=seed, B=B, C=C, H=H, W=W, dtype="bf16", min_len=1, max_len=8)
    dout = np.random.default_rng(seed).standard_normal(w.feats.shape).astype(np.float32)
    g = oracle.iep_backward_workload(w, dout, round_bf16=True)
    plain = oracle.iep_backward_workload(w, dout)
    assert np.abs(plain.roots - oracle.iep_forward_workload(w)).max() == 0          # the unrounded mode is the forward oracle
    from workloads.rng import round_bf16
    assert (g.roots == round_bf16(g.roots.astype(np.float32))).all()                  # root maps are bfloat16 values
    assert 0 < np.abs(g.roots - plain.roots).max() < 2e-2 * np.abs(plain.roots).max()
    ref = torch_tree_grads(w, dout, round_bf16=True)
    for mine, theirs in ((g.dfeats, ref["feats"]), (g.dw1, ref["w1"]), (g.db1, ref["b1"]), (g.dw3a, ref["w3a"]),
                         (g.db3a, ref["b3a"]), (g.dw3b, ref["w3b"]), (g.db3b, ref["b3b"])):
        scale = max(1.0, np.abs(theirs).max())
        assert np.abs(mine - theirs).max() < 1e-11 * scale


def test_central_differences_of_the_forward_oracle(oracle):
    """dL/dtheta from (L(theta + e) - L(theta - e)) / 2e with the oracle's own forward pass, on entries of every
    parameter tensor and of the feature maps (ReLU kinks are far enough for e = 1e-4 on these seeds: checked by
    comparing two step sizes)."""
    w = iep.small_mixed(seed=9, B=3, C=3, H=3, W=4, dtype="f32", min_len=2, max_len=7)
    g_rng = np.random.default_rng(0)
    dout = g_rng.standard_normal(w.feats.shape).astype(np.float32)
    g = oracle.iep_backward_workload(w, dout)

    def loss():
        return float((oracle.iep_forward_workload(w) * dout.astype(np.float64)).sum())

    used = set(int(t) for t in w.prog)
    checked = 0
    for name, arr, grad in (("feats", w.feats, g.dfeats), ("w1", w.w1, g.dw1), ("b1", w.b1, g.db1), ("w3a", w.w3a, g.dw3a),
                            ("b3a", w.b3a, g.db3a), ("w3b", w.w3b, g.dw3b), ("b3b", w.b3b, g.db3b)):
        flat, gflat = arr.reshape(-1), grad.reshape(-1)
        for j in g_rng.choice(flat.size, 12, replace=False):
            old = flat[j]
            est = []
            for e in (1e-2, 5e-3):              # float32 storage: steps well above its rounding
                flat[j] = old + e; lp = loss()
                flat[j] = old - e; lm = loss()
                est.append((lp - lm) / (float(np.float32(old + e)) - float(np.float32(old - e))))
            flat[j] = old
            if abs(est[0] - est[1]) > 1e-6 * max(1.0, abs(est[0])):
                continue                        # a ReLU kink inside the step: the loss is not smooth there
            assert abs(est[1] - gflat[j]) < 1e-6 * max(1.0, abs(gflat[j])), (name, j, est, gflat[j])
            checked += 1
    assert checked > 60
    # parameters of functions that no program uses get no gradient
    for t in range(len(w.arity)):
        if t not in used:
            assert not g.dw3a[t].any() and not g.dw3b[t].any() and not g.dw1[t].any()


def test_closed_forms(oracle):
    """Identity kernels on positive maps: a chain of n unary modules is y = 2^n x, so dL/dx = 2^n dout exactly; a lone
    SCENE program passes the gradient through; gradients of two examples add up in the shared parameters."""
    C, H, W = 2, 3, 3
    arity = np.array([0, 1, 2], np.uint8)
    w3 = np.zeros((3, C, 3, 3, C), np.float32)
    w1 = np.zeros((3, C, 2 * C), np.float32)
    for t in (1, 2):
        w3[t, np.arange(C), 1, 1, np.arange(C)] = 1
        w1[t, np.arange(C), np.arange(C)] = 1
        w1[t, np.arange(C), C + np.arange(C)] = 1
    zb = np.zeros((3, C), np.float32)
    progs = [np.array([1, 1, 1, 0], np.int32), np.array([0], np.int32), np.array([2, 0, 1, 0], np.int32)]
    off = np.concatenate([[0], np.cumsum([len(p) for p in progs])]).astype(np.int32)
    g_rng = np.random.default_rng(5)
    feats = np.abs(g_rng.standard_normal((3, H, W, C))).astype(np.float32) + 0.5
    dout = g_rng.standard_normal((3, H, W, C)).astype(np.float32)
    g = oracle.iep_backward(np.concatenate(progs), off, arity, feats, w1, zb, w3, zb, w3.copy(), zb, dout)
    assert (g.dfeats[0] == 8.0 * dout[0]).all()            # three doublings
    assert (g.dfeats[1] == dout[1]).all()                  # SCENE alone
    assert (g.dfeats[2] == 6.0 * dout[2].astype(np.float64)).all()    # binary: 2 (x + 2x): both leaves are the same map
    # bias gradients: db3b of the unary function = sum over its nodes of the gradient arriving at them
    # (example 0: 1 + 2 + 4 times dout summed over pixels; example 2's unary node receives 2 dout)
    want = (1 + 2 + 4) * dout[0].astype(np.float64).sum((0, 1)) + 2 * dout[2].astype(np.float64).sum((0, 1))
    assert np.allclose(g.db3b[1], want, rtol=1e-12)
    one = oracle.iep_backward(progs[0], np.array([0, 4], np.int32), arity, feats[:1], w1, zb, w3, zb, w3.copy(), zb, dout[:1])
    two = oracle.iep_backward(progs[2], np.array([0, 4], np.int32), arity, feats[2:], w1, zb, w3, zb, w3.copy(), zb, dout[2:])
    assert np.allclose(one.dw3a + two.dw3a, g.dw3a, rtol=1e-12, atol=1e-12)
