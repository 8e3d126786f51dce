"""ctypes front end of the CPU oracle (`dynb_oracle.c`).

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke check and by the
benchmark's CPU-baseline leg, never by the product package.  This file only
marshals numpy arrays; every computation is in the C file.
"""
from __future__ import annotations

import ctypes as ct
import os
import subprocess
from types import SimpleNamespace

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dynb_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, no fast-math, OpenMP across examples/tokens)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        _lib = ct.CDLL(build())
        _lib.oracle_num_threads.restype = ct.c_int
    return _lib


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def set_threads(n: int) -> None:
    lib().oracle_set_threads(ct.c_int(n))


def _p(a, typ):
    return None if a is None else a.ctypes.data_as(ct.POINTER(typ))


def _f32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


class MalformedProgram(ValueError):
    def __init__(self, example):
        super().__init__(f"malformed program in example {example}")
        self.example = example


def plan(prog, prog_off, arity, mode: int = 0) -> SimpleNamespace:
    """Plan of a batch of prefix programs. mode 0: root-distance labels, 1: post-order position labels,
    2: dependency-depth labels (0 for leaves, pools run in ascending order)."""
    prog, prog_off = _i32(prog), _i32(prog_off)
    arity = np.ascontiguousarray(arity, dtype=np.uint8)
    B = len(prog_off) - 1
    N = int(prog_off[-1])
    n = max(N, 1)
    a = {k: np.full(n, -7, np.int32) for k in
         ("level", "type", "child0", "child1", "bucket_level", "bucket_type", "bucket_start",
          "bucket_count", "members", "in0", "in1", "out")}
    root = np.full(max(B, 1), -7, np.int32)
    n_levels, n_buckets, bad = ct.c_int32(0), ct.c_int32(0), ct.c_int32(-1)
    I = ct.c_int32
    rc = lib().oracle_plan(_p(prog, I), _p(prog_off, I), I(B), _p(arity, ct.c_uint8), I(len(arity)), I(mode),
                           _p(a["level"], I), _p(a["type"], I), _p(a["child0"], I), _p(a["child1"], I),
                           _p(root, I), ct.byref(n_levels), ct.byref(n_buckets), _p(a["bucket_level"], I),
                           _p(a["bucket_type"], I), _p(a["bucket_start"], I), _p(a["bucket_count"], I),
                           _p(a["members"], I), _p(a["in0"], I), _p(a["in1"], I), _p(a["out"], I),
                           ct.byref(bad))
    if rc == -2:
        raise MalformedProgram(bad.value)
    if rc != 0:
        raise ValueError(f"oracle_plan: invalid arguments (rc={rc})")
    nb = n_buckets.value
    return SimpleNamespace(
        n_nodes=N, n_levels=n_levels.value, n_buckets=nb,
        node_level=a["level"][:N], node_type=a["type"][:N], child0=a["child0"][:N], child1=a["child1"][:N],
        root=root[:B], bucket_level=a["bucket_level"][:nb], bucket_type=a["bucket_type"][:nb],
        bucket_start=a["bucket_start"][:nb], bucket_count=a["bucket_count"][:nb],
        members=a["members"][:N], in0=a["in0"][:N], in1=a["in1"][:N], out=a["out"][:N])


def plan_dag(node_type, arg0, arg1, node_off, root, arity, mode: int = 0) -> SimpleNamespace:
    """Plan of a batch of dependency graphs (explicit argument indices, local to each example).
    mode 0: maximum-root-distance labels (deepest first), 2: dependency-depth labels (ascending)."""
    node_type, arg0, arg1, node_off, root = map(_i32, (node_type, arg0, arg1, node_off, root))
    arity = np.ascontiguousarray(arity, dtype=np.uint8)
    B = len(node_off) - 1
    N = int(node_off[-1])
    n = max(N, 1)
    a = {k: np.full(n, -7, np.int32) for k in
         ("level", "type", "child0", "child1", "bucket_level", "bucket_type", "bucket_start",
          "bucket_count", "members", "in0", "in1", "out")}
    groot = np.full(max(B, 1), -7, np.int32)
    n_levels, n_buckets, bad = ct.c_int32(0), ct.c_int32(0), ct.c_int32(-1)
    I = ct.c_int32
    rc = lib().oracle_plan_dag(_p(node_type, I), _p(arg0, I), _p(arg1, I), _p(node_off, I), _p(root, I), I(B),
                               _p(arity, ct.c_uint8), I(len(arity)), I(mode),
                               _p(a["level"], I), _p(a["type"], I), _p(a["child0"], I), _p(a["child1"], I),
                               _p(groot, I), ct.byref(n_levels), ct.byref(n_buckets), _p(a["bucket_level"], I),
                               _p(a["bucket_type"], I), _p(a["bucket_start"], I), _p(a["bucket_count"], I),
                               _p(a["members"], I), _p(a["in0"], I), _p(a["in1"], I), _p(a["out"], I),
                               ct.byref(bad))
    if rc == -2:
        raise MalformedProgram(bad.value)
    if rc != 0:
        raise ValueError(f"oracle_plan_dag: invalid arguments (rc={rc})")
    nb = n_buckets.value
    return SimpleNamespace(
        n_nodes=N, n_levels=n_levels.value, n_buckets=nb,
        node_level=a["level"][:N], node_type=a["type"][:N], child0=a["child0"][:N], child1=a["child1"][:N],
        root=groot[:B], bucket_level=a["bucket_level"][:nb], bucket_type=a["bucket_type"][:nb],
        bucket_start=a["bucket_start"][:nb], bucket_count=a["bucket_count"][:nb],
        members=a["members"][:N], in0=a["in0"][:N], in1=a["in1"][:N], out=a["out"][:N])


def iep_forward_dag(node_type, arg0, arg1, node_off, root, arity, feats, w1, b1, w3a, b3a, w3b, b3b) -> np.ndarray:
    """Root output of every example, float64 [B,H,W,C]; every node of a graph is evaluated once."""
    node_type, arg0, arg1, node_off, root = map(_i32, (node_type, arg0, arg1, node_off, root))
    arity = np.ascontiguousarray(arity, dtype=np.uint8)
    plan_dag(node_type, arg0, arg1, node_off, root, arity)      # raises on malformed graphs
    feats = _f32(feats)
    B, H, W, C = feats.shape
    assert B == len(node_off) - 1
    w1, b1, w3a, b3a, w3b, b3b = map(_f32, (w1, b1, w3a, b3a, w3b, b3b))
    out = np.empty((B, H, W, C), np.float64)
    I, F = ct.c_int32, ct.c_float
    rc = lib().oracle_iep_forward_dag(_p(node_type, I), _p(arg0, I), _p(arg1, I), _p(node_off, I), _p(root, I), I(B),
                                      _p(arity, ct.c_uint8), I(len(arity)), I(C), I(H), I(W), _p(feats, F),
                                      _p(w1, F), _p(b1, F), _p(w3a, F), _p(b3a, F), _p(w3b, F), _p(b3b, F),
                                      _p(out, ct.c_double))
    assert rc == 0, rc
    return out


def iep_forward(prog, prog_off, arity, feats, w1, b1, w3a, b3a, w3b, b3b) -> np.ndarray:
    """Root output of every example, float64 [B,H,W,C]; per-example tree recursion."""
    prog, prog_off = _i32(prog), _i32(prog_off)
    arity = np.ascontiguousarray(arity, dtype=np.uint8)
    plan(prog, prog_off, arity)                       # raises on malformed programs
    feats = _f32(feats)
    B, H, W, C = feats.shape
    assert B == len(prog_off) - 1
    w1, b1, w3a, b3a, w3b, b3b = map(_f32, (w1, b1, w3a, b3a, w3b, b3b))
    n_types = len(arity)
    assert w3a.shape == (n_types, C, 3, 3, C) and w3b.shape == (n_types, C, 3, 3, C)
    assert w1 is None or w1.shape == (n_types, C, 2 * C)
    if w1 is None:
        assert not (arity == 2).any()
    out = np.empty((B, H, W, C), np.float64)
    I, F = ct.c_int32, ct.c_float
    rc = lib().oracle_iep_forward(_p(prog, I), _p(prog_off, I), I(B), _p(arity, ct.c_uint8), I(n_types),
                                  I(C), I(H), I(W), _p(feats, F), _p(w1, F), _p(b1, F), _p(w3a, F),
                                  _p(b3a, F), _p(w3b, F), _p(b3b, F), _p(out, ct.c_double))
    assert rc == 0, rc
    return out


def iep_forward_workload(w) -> np.ndarray:
    return iep_forward(w.prog, w.prog_off, w.arity, w.feats, w.w1, w.b1, w.w3a, w.b3a, w.w3b, w.b3b)


def conv3x3(x, w, b=None) -> np.ndarray:
    """x [H,W,C] float32, w [C,3,3,C], b [C] or None -> float64 [H,W,C]."""
    x, w, b = _f32(x), _f32(w), _f32(b)
    H, W, C = x.shape
    out = np.empty((H, W, C), np.float64)
    lib().oracle_conv3x3(_p(x, ct.c_float), _p(w, ct.c_float), _p(b, ct.c_float), _p(out, ct.c_double),
                         ct.c_int(C), ct.c_int(H), ct.c_int(W))
    return out


def moe_logits(x, Wg, Wn, noise) -> np.ndarray:
    x, Wg, Wn, noise = _f32(x), _f32(Wg), _f32(Wn), _f32(noise)
    T, d = x.shape
    E = Wg.shape[1]
    assert Wg.shape == (d, E) and (Wn is None or Wn.shape == (d, E))
    assert noise is None or noise.shape == (T, E)
    out = np.empty((T, E), np.float64)
    F, I = ct.c_float, ct.c_int32
    lib().oracle_moe_logits(_p(x, F), _p(Wg, F), _p(Wn, F), _p(noise, F), I(T), I(d), I(E), _p(out, ct.c_double))
    return out


def moe_route(logits_f32, k: int) -> SimpleNamespace:
    """Routing tables from float32 logits [T,E]."""
    logits = np.ascontiguousarray(logits_f32, dtype=np.float32)
    T, E = logits.shape
    A = T * k
    idx = np.full((T, k), -7, np.int32)
    w = np.zeros((T, k), np.float64)
    counts = np.full(E, -7, np.int32)
    offsets = np.full(E + 1, -7, np.int32)
    perm = np.full(A, -7, np.int32)
    inv = np.full(A, -7, np.int32)
    I = ct.c_int32
    rc = lib().oracle_moe_route(_p(logits, ct.c_float), I(T), I(E), I(k), _p(idx, I), _p(w, ct.c_double),
                                _p(counts, I), _p(offsets, I), _p(perm, I), _p(inv, I))
    if rc != 0:
        raise ValueError("oracle_moe_route: need 0 < k <= E")
    return SimpleNamespace(topk_idx=idx, topk_w=w, counts=counts, offsets=offsets, perm=perm, inv=inv)


def moe_experts(x, topk_idx, topk_w, W1, W2) -> np.ndarray:
    """x [T,d], W1 [E,h,d], W2 [E,d,h] -> float64 [T,d], token by token."""
    x, W1, W2 = _f32(x), _f32(W1), _f32(W2)
    idx = _i32(topk_idx)
    w = np.ascontiguousarray(topk_w, dtype=np.float64)
    T, d = x.shape
    E, h, d2 = W1.shape
    k = idx.shape[1]
    assert d2 == d and W2.shape == (E, d, h) and idx.shape == (T, k) and w.shape == (T, k) and k <= 64
    assert idx.min() >= 0 and idx.max() < E
    out = np.empty((T, d), np.float64)
    F, I = ct.c_float, ct.c_int32
    lib().oracle_moe_experts(_p(x, F), _p(idx, I), _p(w, ct.c_double), _p(W1, F), _p(W2, F),
                             I(T), I(d), I(h), I(k), _p(out, ct.c_double))
    return out


def moe_token(x_t, w, W1_list, W2_list) -> np.ndarray:
    """One token: x_t [d], weights w [k], per chosen expert W1 [h,d] and W2 [d,h] -> float64 [d]."""
    x_t = _f32(x_t)
    w = np.ascontiguousarray(w, dtype=np.float64)
    W1_list = [_f32(a) for a in W1_list]
    W2_list = [_f32(a) for a in W2_list]
    k = len(w)
    h, d = W1_list[0].shape
    assert all(a.shape == (h, d) for a in W1_list) and all(a.shape == (d, h) for a in W2_list)
    FP = ct.POINTER(ct.c_float)
    p1 = (FP * k)(*[_p(a, ct.c_float) for a in W1_list])
    p2 = (FP * k)(*[_p(a, ct.c_float) for a in W2_list])
    out = np.empty(d, np.float64)
    lib().oracle_moe_token(_p(x_t, ct.c_float), ct.c_int32(d), ct.c_int32(h), ct.c_int32(k),
                           _p(w, ct.c_double), p1, p2, _p(out, ct.c_double))
    return out


def moe_forward(x, Wg, Wn, noise, W1, W2, k: int) -> SimpleNamespace:
    """The whole layer from raw inputs: logits (fp64, rounded once to fp32 for routing), routing, experts."""
    lg = moe_logits(x, Wg, Wn, noise)
    r = moe_route(lg.astype(np.float32), k)
    out = moe_experts(x, r.topk_idx, r.topk_w, W1, W2)
    return SimpleNamespace(logits=lg, out=out, **vars(r))


def classify(x, wc, bc, wf1, bf1, wf2, bf2, want_logits: bool = False):
    """Classifier head on root maps x [B,H,W,C]: conv1x1 (wc [Cc,C]) + ReLU, flatten [H,W,Cc], FC (wf1 [F,H*W*Cc]) +
    ReLU, FC (wf2 [A,F]), softmax.  Returns probs float64 [B,A] (and the logits if wanted)."""
    x, wc, bc, wf1, bf1, wf2, bf2 = map(_f32, (x, wc, bc, wf1, bf1, wf2, bf2))
    B, H, W, C = x.shape
    Cc, F, A = wc.shape[0], wf1.shape[0], wf2.shape[0]
    assert wc.shape == (Cc, C) and wf1.shape == (F, H * W * Cc) and wf2.shape == (A, F)
    probs = np.empty((B, A), np.float64)
    logits = np.empty((B, A), np.float64)
    Fp, I = ct.c_float, ct.c_int32
    rc = lib().oracle_classify(_p(x, Fp), I(B), I(C), I(H), I(W), I(Cc), I(F), I(A), _p(wc, Fp), _p(bc, Fp), _p(wf1, Fp),
                               _p(bf1, Fp), _p(wf2, Fp), _p(bf2, Fp), _p(probs, ct.c_double), _p(logits, ct.c_double))
    assert rc == 0, rc
    return (probs, logits) if want_logits else probs


def iep_backward(prog, prog_off, arity, feats, w1, b1, w3a, b3a, w3b, b3b, dout, round_bf16: bool = False) -> SimpleNamespace:
    """Gradients of L = sum_i <dout[i], root_i> with respect to the feature maps and every module parameter
    (float64 arrays in the shapes of the inputs): dfeats, dw1, db1, dw3a, db3a, dw3b, db3b; roots = the root maps
    of the forward evaluation they belong to.  round_bf16: every stored activation (u of two-argument functions,
    mid, y) is rounded to bfloat16 in that forward evaluation, as an implementation with bf16 storage holds them."""
    prog, prog_off = _i32(prog), _i32(prog_off)
    arity = np.ascontiguousarray(arity, dtype=np.uint8)
    plan(prog, prog_off, arity)                       # raises on malformed programs
    feats, dout = _f32(feats), _f32(dout)
    B, H, W, C = feats.shape
    assert dout.shape == feats.shape and B == len(prog_off) - 1
    w1, b1, w3a, b3a, w3b, b3b = map(_f32, (w1, b1, w3a, b3a, w3b, b3b))
    n_types = len(arity)
    if w1 is None:
        assert not (arity == 2).any()
    D = np.float64
    g = SimpleNamespace(dfeats=np.empty((B, H, W, C), D), dw1=np.empty((n_types, C, 2 * C), D), db1=np.empty((n_types, C), D),
                        dw3a=np.empty((n_types, C, 3, 3, C), D), db3a=np.empty((n_types, C), D),
                        dw3b=np.empty((n_types, C, 3, 3, C), D), db3b=np.empty((n_types, C), D),
                        roots=np.empty((B, H, W, C), D))
    I, F, Dp = ct.c_int32, ct.c_float, ct.c_double
    rc = lib().oracle_iep_backward(_p(prog, I), _p(prog_off, I), I(B), _p(arity, ct.c_uint8), I(n_types), I(C), I(H), I(W),
                                   _p(feats, F), _p(w1, F), _p(b1, F), _p(w3a, F), _p(b3a, F), _p(w3b, F), _p(b3b, F),
                                   _p(dout, F), I(int(round_bf16)), _p(g.dfeats, Dp), _p(g.dw1, Dp), _p(g.db1, Dp), _p(g.dw3a, Dp),
                                   _p(g.db3a, Dp), _p(g.dw3b, Dp), _p(g.db3b, Dp), _p(g.roots, Dp))
    assert rc == 0, rc
    return g


def iep_backward_workload(w, dout, round_bf16: bool = False) -> SimpleNamespace:
    return iep_backward(w.prog, w.prog_off, w.arity, w.feats, w.w1, w.b1, w.w3a, w.b3a, w.w3b, w.b3b, dout, round_bf16)
