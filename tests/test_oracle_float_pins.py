"""Pins of the float oracle (module execution and MoE layer) against library routines, closed
forms and brute force.  None of the expected values below comes from the oracle itself or
from the HIP path.

What is pinned follows Results / IEP (batched and per-example execution build the same
network), Background / Visual Reasoning Programs (SCENE outputs the example's features, every
other function is a network applied to its arguments) and Results / Sparsely Gated Mixture
of Experts (k of n bias-free one-hidden-layer experts per example).
"""
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F
from scipy.signal import correlate2d

from workloads import iep, moe
from workloads.rng import round_bf16

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ convolution
def test_conv3x3_equals_library_cross_correlation(oracle):
    g = np.random.default_rng(0)
    C, H, W = 5, 6, 7
    x = g.standard_normal((H, W, C)).astype(np.float32)
    w = g.standard_normal((C, 3, 3, C)).astype(np.float32)     # [Cout][kh][kw][Cin], deliberately asymmetric
    b = g.standard_normal(C).astype(np.float32)
    got = oracle.conv3x3(x, w, b)
    # torch: NCHW input, weight [Cout][Cin][kh][kw]
    ref = F.conv2d(torch.from_numpy(x).double().permute(2, 0, 1)[None],
                   torch.from_numpy(w).double().permute(0, 3, 1, 2), torch.from_numpy(b).double(), padding=1)
    assert np.allclose(got, ref[0].permute(1, 2, 0).numpy(), rtol=0, atol=1e-12)
    # scipy: one 2-D correlation per (cout, cin) pair, summed over cin
    ref2 = np.zeros((H, W, C))
    for co in range(C):
        for ci in range(C):
            ref2[:, :, co] += correlate2d(x[:, :, ci].astype(np.float64), w[co, :, :, ci].astype(np.float64),
                                          mode="same", boundary="fill")
        ref2[:, :, co] += b[co]
    assert np.allclose(got, ref2, rtol=0, atol=1e-12)
    assert np.allclose(oracle.conv3x3(x, w, None), ref2 - b[None, None, :], rtol=0, atol=1e-12)


# ------------------------------------------------------------------ independent whole-tree reference
def torch_tree_reference(w, example):
    """Per-example recursion with torch.nn.functional.conv2d in float64 (NCHW)."""
    prog = w.program(example)
    pos = [0]
    T = lambda a: torch.from_numpy(np.asarray(a)).double()

    def ev():
        t = int(prog[pos[0]])
        pos[0] += 1
        ar = int(w.arity[t])
        if ar == 0:
            return T(w.feats[example]).permute(2, 0, 1)[None]
        if ar == 1:
            u = ev()
        else:
            a = ev()
            b = ev()
            u = F.relu(F.conv2d(torch.cat([a, b], 1), T(w.w1[t])[:, :, None, None], T(w.b1[t])))
        mid = F.relu(F.conv2d(u, T(w.w3a[t]).permute(0, 3, 1, 2), T(w.b3a[t]), padding=1))
        return F.relu(u + F.conv2d(mid, T(w.w3b[t]).permute(0, 3, 1, 2), T(w.b3b[t]), padding=1))

    return ev()[0].permute(1, 2, 0).numpy()


def test_config0_whole_trees_equal_library_recursion(oracle):
    w = iep.config0()
    got = oracle.iep_forward_workload(w)
    assert got.shape == (8, 8, 8, 16)
    for i in range(w.B):
        ref = torch_tree_reference(w, i)
        assert np.abs(got[i] - ref).max() <= 1e-10 * max(1.0, np.abs(ref).max())


def test_mixed_trees_with_single_scene_programs(oracle):
    w = iep.small_mixed(seed=11, B=12, C=3, H=4, W=5, dtype="f32", min_len=1, max_len=8)
    assert any(len(w.program(i)) == 1 for i in range(w.B))
    got = oracle.iep_forward_workload(w)
    for i in range(w.B):
        assert np.allclose(got[i], torch_tree_reference(w, i), rtol=0, atol=1e-10)
        if len(w.program(i)) == 1:
            assert (got[i] == w.feats[i]).all()        # SCENE alone: the features themselves


def numpy_module_bruteforce(w, t, xs):
    """Direct-sum module on a tiny map: padded array + explicit index arithmetic (no conv routine)."""
    C, H, W = w.C, w.H, w.W

    def conv(u, k, b):
        pad = np.zeros((H + 2, W + 2, C))
        pad[1:-1, 1:-1] = u
        o = np.zeros((H, W, C))
        for y in range(H):
            for x in range(W):
                patch = pad[y:y + 3, x:x + 3, :]                 # [kh][kw][ci]
                o[y, x, :] = np.einsum("hwc,ohwc->o", patch, k.astype(np.float64)) + b
        return o

    if len(xs) == 2:
        cat = np.concatenate(xs, axis=-1)
        u = np.maximum(cat @ w.w1[t].astype(np.float64).T + w.b1[t], 0)
    else:
        u = xs[0]
    mid = np.maximum(conv(u, w.w3a[t], w.b3a[t]), 0)
    return np.maximum(u + conv(mid, w.w3b[t], w.b3b[t]), 0)


def test_tiny_modules_equal_direct_sum(oracle):
    w = iep.small_mixed(seed=5, B=2, C=2, H=3, W=3, dtype="f32")
    f = w.feats.astype(np.float64)
    for t in range(1, w.n_types):
        if w.arity[t] == 1:
            prog, exp = [t, 0], numpy_module_bruteforce(w, t, [f[0]])
        else:
            prog, exp = [t, 0, 0], numpy_module_bruteforce(w, t, [f[0], f[0]])
        got = oracle.iep_forward(np.array(prog, np.int32), np.array([0, len(prog)], np.int32), w.arity,
                                 w.feats[:1], w.w1, w.b1, w.w3a, w.b3a, w.w3b, w.b3b)[0]
        assert np.allclose(got, exp, rtol=0, atol=1e-12)
    # two levels, binary over (unary(scene), scene): checks argument order of the concatenation
    tb = int(np.nonzero(w.arity == 2)[0][0])
    tu = int(np.nonzero(w.arity == 1)[0][0])
    prog = [tb, tu, 0, 0]
    exp = numpy_module_bruteforce(w, tb, [numpy_module_bruteforce(w, tu, [f[1]]), f[1]])
    got = oracle.iep_forward(np.array(prog, np.int32), np.array([0, 4], np.int32), w.arity, w.feats[1:2],
                             w.w1, w.b1, w.w3a, w.b3a, w.w3b, w.b3b)[0]
    assert np.allclose(got, exp, rtol=0, atol=1e-12)
    swapped = numpy_module_bruteforce(w, tb, [f[1], numpy_module_bruteforce(w, tu, [f[1]])])
    assert not np.allclose(got, swapped, atol=1e-6)


def _closed_form_weights(n_types, C, arity, identity):
    w1 = np.zeros((n_types, C, 2 * C), np.float32)
    w3 = np.zeros((n_types, C, 3, 3, C), np.float32)
    if identity:
        for t in range(n_types):
            w3[t, np.arange(C), 1, 1, np.arange(C)] = 1.0
            w1[t, np.arange(C), np.arange(C)] = 1.0
            w1[t, np.arange(C), C + np.arange(C)] = 1.0
    z = np.zeros((n_types, C), np.float32)
    return w1, z, w3, z, w3.copy(), z


def test_zero_weights_give_relu_of_features(oracle):
    w = iep.small_mixed(seed=7, B=6, C=4, H=5, W=5, dtype="f32", min_len=1)
    ws = _closed_form_weights(w.n_types, w.C, w.arity, identity=False)
    got = oracle.iep_forward(w.prog, w.prog_off, w.arity, w.feats, *ws)
    for i in range(w.B):
        # a lone SCENE is passed through untouched; binary nodes with zero 1x1 weights output ReLU(0) = 0
        if len(w.program(i)) == 1:
            assert (got[i] == w.feats[i]).all()
        elif (w.arity[w.program(i)] == 2).any():
            pass
        else:
            assert (got[i] == np.maximum(w.feats[i], 0)).all()


def test_identity_kernels_give_powers_of_two(oracle):
    """Centre-tap identity 3x3 and [I | I] 1x1 on non-negative features: a unary module doubles its
    input, a binary module gives 2 (x0 + x1); chain of n modules -> 2^n f, full binary tree with
    D levels -> 4^(D-1) f.  Exact in floating point."""
    C, H, W = 4, 5, 6
    f = np.abs(np.random.default_rng(2).standard_normal((1, H, W, C))).astype(np.float32)
    arity = np.array([0, 1, 2], np.uint8)
    ws = _closed_form_weights(3, C, arity, identity=True)
    for n in (1, 3, 9):
        prog = np.array([1] * n + [0], np.int32)
        got = oracle.iep_forward(prog, np.array([0, n + 1], np.int32), arity, f, *ws)
        assert (got[0] == (2.0 ** n) * f[0].astype(np.float64)).all()
    g = np.random.default_rng(0)
    for D in (2, 3, 5):
        prog = iep.balanced_program(g, D, [2])
        got = oracle.iep_forward(prog, np.array([0, len(prog)], np.int32), arity, f, *ws)
        assert (got[0] == (4.0 ** (D - 1)) * f[0].astype(np.float64)).all()


def test_batched_call_equals_per_example_calls(oracle):
    """Results / IEP: grouping examples into one call must not change any example's output."""
    w = iep.config0()
    whole = oracle.iep_forward_workload(w)
    for i in range(w.B):
        one = oracle.iep_forward_workload(w.subset([i]))
        assert (one[0] == whole[i]).all()
    oracle.set_threads(1)
    assert (oracle.iep_forward_workload(w) == whole).all()     # thread count must not matter
    oracle.set_threads(0)


# ------------------------------------------------------------------ MoE
def test_gate_logits_equal_fp64_matmul(oracle):
    m = moe.small(seed=1, T=33, d=24, h=8, E=10, k=2)
    got = oracle.moe_logits(m.x, m.Wg, m.Wn, m.noise)
    x = m.x.astype(np.float64)
    ref = x @ m.Wg.astype(np.float64) + m.noise * np.logaddexp(0.0, x @ m.Wn.astype(np.float64))
    assert np.allclose(got, ref, rtol=0, atol=1e-12)
    assert np.allclose(oracle.moe_logits(m.x, m.Wg, None, None), x @ m.Wg.astype(np.float64), rtol=0, atol=1e-12)
    # large-magnitude softplus arguments stay finite and accurate
    big = oracle.moe_logits(np.array([[40.0], [-40.0]], np.float32), np.zeros((1, 1), np.float32),
                            np.ones((1, 1), np.float32), np.ones((2, 1), np.float32))
    assert np.allclose(big[:, 0], [40.0, np.exp(-40.0)], rtol=1e-12)


def test_topk_equals_stable_argsort_and_tie_rule(oracle):
    g = np.random.default_rng(4)
    logits = g.standard_normal((50, 17)).astype(np.float32)
    logits[3, :] = 0.5                         # all equal: lowest ids win, in order
    logits[4, [2, 9, 11]] = 7.0                # three-way tie at the top
    logits[5, 16] = logits[5, 0] = 9.0
    for k in (1, 2, 4, 17):
        r = oracle.moe_route(logits, k)
        ref = np.argsort(-logits, axis=1, kind="stable")[:, :k]
        assert (r.topk_idx == ref).all()
        sel = np.take_along_axis(logits.astype(np.float64), ref, 1)
        sm = np.exp(sel - sel.max(1, keepdims=True))
        sm /= sm.sum(1, keepdims=True)
        assert np.allclose(r.topk_w, sm, rtol=1e-13, atol=0)
        assert np.allclose(r.topk_w.sum(1), 1.0, atol=1e-14)
    assert list(oracle.moe_route(logits, 3).topk_idx[3]) == [0, 1, 2]
    assert list(oracle.moe_route(logits, 3).topk_idx[4]) == [2, 9, 11]
    assert (oracle.moe_route(logits, 1).topk_w == 1.0).all()
    full = oracle.moe_route(logits, 17)            # k = E: the textbook softmax over all experts
    ref = torch.softmax(torch.from_numpy(logits).double(), 1).numpy()
    assert np.allclose(np.take_along_axis(ref, full.topk_idx, 1), full.topk_w, rtol=1e-12)
    with pytest.raises(ValueError):
        oracle.moe_route(logits, 18)


def test_grouping_equals_stable_sort_by_expert(oracle):
    m = moe.small(seed=2, T=257, d=16, h=8, E=12, k=3, empty_frac=0.2)
    lg = oracle.moe_logits(m.x, m.Wg, m.Wn, m.noise).astype(np.float32)
    r = oracle.moe_route(lg, m.k)
    flat = r.topk_idx.ravel()
    assert (r.perm == np.argsort(flat, kind="stable")).all()
    assert (r.inv[r.perm] == np.arange(m.A)).all()
    assert (r.counts == np.bincount(flat, minlength=m.E)).all()
    assert (r.offsets == np.concatenate([[0], np.cumsum(r.counts)])).all() and r.offsets[-1] == m.A
    assert (r.counts[m.empty] == 0).all() and len(m.empty) == 2
    # the paper's call counts: at most n expert calls instead of k*b
    assert (r.counts > 0).sum() <= m.E and r.counts.sum() == m.k * m.T


def _expert_stack(m):
    W1 = np.stack([m.expert_weights(e)[0] for e in range(m.E)])
    W2 = np.stack([m.expert_weights(e)[1] for e in range(m.E)])
    return W1, W2


def test_single_expert_is_a_dense_two_layer_mlp(oracle):
    m = moe.small(seed=3, T=19, d=12, h=20, E=1, k=1)
    W1, W2 = _expert_stack(m)
    r = oracle.moe_forward(m.x, m.Wg, m.Wn, m.noise, W1, W2, 1)
    x = torch.from_numpy(m.x).double()
    ref = F.linear(F.relu(F.linear(x, torch.from_numpy(W1[0]).double())), torch.from_numpy(W2[0]).double())
    assert np.allclose(r.out, ref.numpy(), rtol=0, atol=1e-12)


def test_moe_bruteforce_tiny(oracle):
    m = moe.small(seed=4, T=4, d=3, h=2, E=3, k=2)
    W1, W2 = _expert_stack(m)
    r = oracle.moe_forward(m.x, m.Wg, m.Wn, m.noise, W1, W2, 2)
    x = m.x.astype(np.float64)
    lg = (x @ m.Wg + m.noise * np.logaddexp(0, x @ m.Wn)).astype(np.float32).astype(np.float64)
    for t in range(4):
        order = sorted(range(3), key=lambda e: (-lg[t, e], e))[:2]
        ws = np.exp(lg[t, order] - lg[t, order].max())
        ws /= ws.sum()
        exp = np.zeros(3)
        for wgt, e in zip(ws, order):
            hid = np.maximum(W1[e].astype(np.float64) @ x[t], 0)
            exp += wgt * (W2[e].astype(np.float64) @ hid)
        assert list(r.topk_idx[t]) == order
        assert np.allclose(r.out[t], exp, rtol=0, atol=1e-13)


def test_identical_experts_make_routing_irrelevant_and_zero_w2_gives_zero(oracle):
    m = moe.small(seed=6, T=40, d=8, h=6, E=5, k=3)
    w1, w2 = m.expert_weights(0)
    W1 = np.repeat(w1[None], m.E, 0)
    W2 = np.repeat(w2[None], m.E, 0)
    r = oracle.moe_forward(m.x, m.Wg, m.Wn, m.noise, W1, W2, m.k)
    x = m.x.astype(np.float64)
    ref = np.maximum(x @ w1.astype(np.float64).T, 0) @ w2.astype(np.float64).T
    assert np.allclose(r.out, ref, rtol=0, atol=1e-12)          # gate weights sum to one
    r0 = oracle.moe_forward(m.x, m.Wg, m.Wn, m.noise, W1, np.zeros_like(W2), m.k)
    assert (r0.out == 0).all()


def test_token_entry_point_equals_stacked_entry_point(oracle):
    m = moe.small(seed=8, T=9, d=8, h=6, E=7, k=2)
    W1, W2 = _expert_stack(m)
    r = oracle.moe_forward(m.x, m.Wg, m.Wn, m.noise, W1, W2, m.k)
    for t in range(m.T):
        one = oracle.moe_token(m.x[t], r.topk_w[t], [W1[e] for e in r.topk_idx[t]], [W2[e] for e in r.topk_idx[t]])
        assert (one == r.out[t]).all()


def test_memory_ratio_printed_in_the_paper():
    v = {}
    for line in open(os.path.join(GOLD, "memory_ratio.txt")):
        line = line.split("#")[0].split()
        if line:
            v[line[0]] = float(line[1])
    ratio = v["m"] * (2 * v["d"] + v["h"]) / (2 * v["k"] * v["h"] * v["d"])
    assert round(ratio, 1) == v["ratio_printed"]


# ------------------------------------------------------------------ workloads
def test_workloads_are_reproducible_and_bf16_clean():
    a, b = iep.config1(B=4), iep.config1(B=4)
    assert (a.prog == b.prog).all() and (a.feats == b.feats).all() and (a.w3a == b.w3a).all()
    assert (round_bf16(a.feats) == a.feats).all() and (round_bf16(a.w3b) == a.w3b).all()
    w2 = iep.config2()
    lens = np.diff(w2.prog_off)
    assert lens.min() >= 10 and lens.max() <= 30 and w2.n_types == 41
    internal = w2.arity[w2.prog] > 0
    frac_bin = (w2.arity[w2.prog] == 2).sum() / internal.sum()
    assert 0.08 < frac_bin < 0.2


def test_moe_workload_load_shape():
    m = moe.config3()
    x = m.x.astype(np.float64)
    lg = x @ m.Wg + m.noise * np.logaddexp(0, x @ m.Wn)
    idx = np.argsort(-lg, axis=1, kind="stable")[:, :m.k]
    load = np.sort(np.bincount(idx.ravel(), minlength=m.E))[::-1].astype(np.float64)
    ranks = np.arange(1, m.E + 1)
    ok = load >= 8
    slope = np.polyfit(np.log(ranks[ok]), np.log(load[ok]), 1)[0]
    assert abs(slope + 1.1) < 0.1
    assert (round_bf16(m.x) == m.x).all() and (round_bf16(m.Wg) == m.Wg).all()
