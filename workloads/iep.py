"""Seeded synthetic inputs for the program-tree execution engine (configs 0-2).

Stand-ins for CLEVR programs and trained IEP module weights, which are not
available: the trees take the *shape* the paper describes (function vocabulary of
40, fixed arities, a SCENE leaf, strongly imbalanced chain-like programs; or the
predetermined balanced binary tree of the paper's stronger bound), the features
and weights take the sizes the benchmark configurations fix.

This module only draws random numbers and assembles arrays.  It performs none of
the method's arithmetic (no tree labelling, no convolution).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

from .rng import BASE_SEED, round_bf16, stream

SCENE = 0

# sub-stream ids
_S_TREE, _S_FEAT, _S_W = 1, 2, 3


@dataclass
class IepWorkload:
    name: str
    dtype: str                  # "f32" or "bf16" (bf16: all values are bf16-representable float32)
    arity: np.ndarray           # uint8 [n_types]; type 0 = SCENE (arity 0)
    prog: np.ndarray            # int32 [N] concatenated prefix sequences of type ids
    prog_off: np.ndarray        # int32 [B+1]
    C: int
    H: int
    W: int
    feats: np.ndarray           # float32 [B,H,W,C]
    w1: np.ndarray              # float32 [n_types, C, 2C]      conv1x1 of binary types (zeros elsewhere)
    b1: np.ndarray              # float32 [n_types, C]
    w3a: np.ndarray             # float32 [n_types, C, 3, 3, C] first conv3x3  [Cout][kh][kw][Cin]
    b3a: np.ndarray             # float32 [n_types, C]
    w3b: np.ndarray             # float32 [n_types, C, 3, 3, C] second conv3x3
    b3b: np.ndarray             # float32 [n_types, C]
    meta: dict = field(default_factory=dict)

    @property
    def B(self) -> int:
        return len(self.prog_off) - 1

    @property
    def n_types(self) -> int:
        return len(self.arity)

    def program(self, i: int) -> np.ndarray:
        return self.prog[self.prog_off[i]:self.prog_off[i + 1]]

    @property
    def n_module_evals(self) -> int:
        return int((self.arity[self.prog] > 0).sum())

    def subset(self, examples) -> "IepWorkload":
        """The same workload restricted to some examples (weights shared)."""
        examples = list(examples)
        progs = [self.program(i) for i in examples]
        off = np.zeros(len(progs) + 1, np.int32)
        off[1:] = np.cumsum([len(p) for p in progs])
        return IepWorkload(self.name + "-subset", self.dtype, self.arity,
                           np.concatenate(progs).astype(np.int32), off, self.C, self.H, self.W,
                           np.ascontiguousarray(self.feats[examples]), self.w1, self.b1, self.w3a,
                           self.b3a, self.w3b, self.b3b, dict(self.meta, examples=examples))


def _pack(progs):
    off = np.zeros(len(progs) + 1, np.int32)
    off[1:] = np.cumsum([len(p) for p in progs])
    return np.concatenate(progs).astype(np.int32), off


def make_weights(seed: int, arity: np.ndarray, C: int, dtype: str, bias_std: float = 0.01):
    """He-normal conv weights (std = sqrt(2 / fan_in)) and small N(0, bias_std^2) biases per type."""
    n_types = len(arity)
    w1 = np.zeros((n_types, C, 2 * C), np.float32)
    b1 = np.zeros((n_types, C), np.float32)
    w3a = np.zeros((n_types, C, 3, 3, C), np.float32)
    b3a = np.zeros((n_types, C), np.float32)
    w3b = np.zeros((n_types, C, 3, 3, C), np.float32)
    b3b = np.zeros((n_types, C), np.float32)
    for t in range(n_types):
        if arity[t] == 0:
            continue
        g = stream(seed, _S_W, t)
        s3 = np.sqrt(2.0 / (9 * C))
        w3a[t] = g.standard_normal((C, 3, 3, C), dtype=np.float32) * s3
        w3b[t] = g.standard_normal((C, 3, 3, C), dtype=np.float32) * s3
        b3a[t] = g.standard_normal(C, dtype=np.float32) * bias_std
        b3b[t] = g.standard_normal(C, dtype=np.float32) * bias_std
        if arity[t] == 2:
            w1[t] = g.standard_normal((C, 2 * C), dtype=np.float32) * np.sqrt(2.0 / (2 * C))
            b1[t] = g.standard_normal(C, dtype=np.float32) * bias_std
    if dtype == "bf16":
        w1, w3a, w3b = round_bf16(w1), round_bf16(w3a), round_bf16(w3b)
    return w1, b1, w3a, b3a, w3b, b3b


def make_feats(seed: int, B: int, H: int, W: int, C: int, dtype: str) -> np.ndarray:
    f = np.empty((B, H, W, C), np.float32)
    for i in range(B):
        f[i] = stream(seed, _S_FEAT, i).standard_normal((H, W, C), dtype=np.float32)
    return round_bf16(f) if dtype == "bf16" else f


def _assemble(name, seed, dtype, arity, progs, C, H, W, meta=None, weight_seed=None) -> IepWorkload:
    prog, off = _pack(progs)
    feats = make_feats(seed, len(progs), H, W, C, dtype)
    w = make_weights(seed if weight_seed is None else weight_seed, arity, C, dtype)
    return IepWorkload(name, dtype, arity, prog, off, C, H, W, feats, *w, meta=meta or {})


_S_HEAD = 4


def make_head(seed: int, C: int, H: int, W: int, Cc: int, F: int, n_answers: int, dtype: str, bias_std: float = 0.01) -> dict:
    """He-normal weights of the classifier head (1x1 convolution C -> Cc, fully connected H*W*Cc -> F -> n_answers)
    and small biases: wc [Cc,C], wf1 [F,H*W*Cc], wf2 [n_answers,F], bc, bf1, bf2 (float32; weights bf16-representable
    if dtype is "bf16")."""
    g = stream(seed, _S_HEAD)
    J = H * W * Cc
    head = dict(wc=g.standard_normal((Cc, C), dtype=np.float32) * np.float32(np.sqrt(2.0 / C)),
                wf1=g.standard_normal((F, J), dtype=np.float32) * np.float32(np.sqrt(2.0 / J)),
                wf2=g.standard_normal((n_answers, F), dtype=np.float32) * np.float32(np.sqrt(2.0 / F)),
                bc=g.standard_normal(Cc, dtype=np.float32) * np.float32(bias_std),
                bf1=g.standard_normal(F, dtype=np.float32) * np.float32(bias_std),
                bf2=g.standard_normal(n_answers, dtype=np.float32) * np.float32(bias_std))
    if dtype == "bf16":
        for k in ("wc", "wf1", "wf2"):
            head[k] = round_bf16(head[k])
    return head


# --------------------------------------------------------------------------- config 0
def random_small_tree(g: np.random.Generator, unary, binary, max_levels=4, max_nodes=12):
    """Random prefix program: root never SCENE, at most max_levels levels, at most max_nodes nodes."""
    unary, binary = list(unary), list(binary)
    while True:
        seq = []

        def gen(lvl):
            if lvl == max_levels - 1 or len(seq) >= max_nodes:
                seq.append(SCENE)
                return
            u = g.random()
            if lvl > 0 and u < 0.2:
                seq.append(SCENE)
            elif u < 0.6 or not binary:
                seq.append(int(g.choice(unary)))
                gen(lvl + 1)
            else:
                seq.append(int(g.choice(binary)))
                gen(lvl + 1)
                gen(lvl + 1)

        gen(0)
        if len(seq) <= max_nodes:
            return np.array(seq, np.int32)


def config0(seed: int = BASE_SEED * 10 + 0, B: int = 8, C: int = 16, H: int = 8, W: int = 8) -> IepWorkload:
    """Tiny fp32 engine: 8 random trees, 2 unary + 2 binary types, <=4 levels, <=12 nodes."""
    arity = np.array([0, 1, 1, 2, 2], np.uint8)
    g = stream(seed, _S_TREE)
    progs = [random_small_tree(g, [1, 2], [3, 4]) for _ in range(B)]
    return _assemble("cfg0-tiny-fp32", seed, "f32", arity, progs, C, H, W)


# --------------------------------------------------------------------------- config 1
def balanced_program(g: np.random.Generator, n_levels: int, binary_types) -> np.ndarray:
    """Prefix sequence of a full binary tree with n_levels levels, internal types drawn uniformly."""
    seq = []

    def gen(lvl):
        if lvl == n_levels - 1:
            seq.append(SCENE)
        else:
            seq.append(int(g.choice(binary_types)))
            gen(lvl + 1)
            gen(lvl + 1)

    gen(0)
    return np.array(seq, np.int32)


def config1(seed: int = BASE_SEED * 10 + 1, B: int = 64, C: int = 128, H: int = 14, W: int = 14,
            n_levels: int = 5, n_binary: int = 8, dtype: str = "bf16") -> IepWorkload:
    """Predetermined balanced binary trees: 16 leaves, 31 nodes, 8 binary types."""
    arity = np.array([0] + [2] * n_binary, np.uint8)
    g = stream(seed, _S_TREE)
    progs = [balanced_program(g, n_levels, list(range(1, n_binary + 1))) for _ in range(B)]
    return _assemble("cfg1-balanced-bf16", seed, dtype, arity, progs, C, H, W)


# --------------------------------------------------------------------------- config 2
def chain_like_program(g: np.random.Generator, length: int, unary, binary,
                       p_binary: float = 0.15, p_early_leaf: float = 0.10) -> np.ndarray:
    """Prefix program of exactly `length` tokens, mostly a chain, binary nodes with p ~ p_binary."""
    seq = []
    open_slots, rem = 1, length
    while rem > 0:
        if rem == open_slots:
            tok, d_open = SCENE, -1
        elif open_slots >= 2 and g.random() < p_early_leaf:
            tok, d_open = SCENE, -1
        elif g.random() < p_binary and rem >= open_slots + 2:
            tok, d_open = int(g.choice(binary)), +1
        else:
            tok, d_open = int(g.choice(unary)), 0
        seq.append(tok)
        open_slots += d_open
        rem -= 1
    assert open_slots == 0
    return np.array(seq, np.int32)


def config2(seed: int = BASE_SEED * 10 + 2, B: int = 256, C: int = 128, H: int = 14, W: int = 14,
            n_unary: int = 30, n_binary: int = 10, min_len: int = 10, max_len: int = 30,
            dtype: str = "bf16", weight_seed=None) -> IepWorkload:
    """IEP-shaped engine: 40 module types, program length U{10..30}, mostly chains.
    weight_seed: draw the module weights from another seed's stream (several batches for one set of modules)."""
    arity = np.array([0] + [1] * n_unary + [2] * n_binary, np.uint8)
    unary = list(range(1, n_unary + 1))
    binary = list(range(n_unary + 1, n_unary + n_binary + 1))
    g = stream(seed, _S_TREE)
    progs = []
    for _ in range(B):
        length = int(g.integers(min_len, max_len + 1))
        progs.append(chain_like_program(g, length, unary, binary))
    return _assemble("cfg2-iep-bf16", seed, dtype, arity, progs, C, H, W, weight_seed=weight_seed)


def small_mixed(seed: int, B: int, C: int, H: int, W: int, dtype: str, n_unary: int = 3, n_binary: int = 2,
                min_len: int = 2, max_len: int = 9) -> IepWorkload:
    """Small parity workload of arbitrary shape (also emits single-SCENE programs when min_len = 1)."""
    arity = np.array([0] + [1] * n_unary + [2] * n_binary, np.uint8)
    unary = list(range(1, n_unary + 1))
    binary = list(range(n_unary + 1, n_unary + n_binary + 1))
    g = stream(seed, _S_TREE)
    progs = []
    for _ in range(B):
        length = int(g.integers(min_len, max_len + 1))
        progs.append(chain_like_program(g, length, unary, binary, p_binary=0.3))
    return _assemble(f"mixed-{dtype}-B{B}-C{C}-{H}x{W}", seed, dtype, arity, progs, C, H, W)


# --------------------------------------------------------------------------- dependency graphs
@dataclass
class DagWorkload:
    """A batch of dependency graphs: explicit argument indices (local to the example), nodes in arbitrary
    order, one root per example; a node may feed several consumers."""
    name: str
    dtype: str
    arity: np.ndarray
    node_type: np.ndarray       # int32 [N]
    arg0: np.ndarray            # int32 [N] local index of the first argument or -1
    arg1: np.ndarray            # int32 [N] local index of the second argument or -1
    node_off: np.ndarray        # int32 [B+1]
    root: np.ndarray            # int32 [B] local index of the output node
    C: int
    H: int
    W: int
    feats: np.ndarray
    w1: np.ndarray
    b1: np.ndarray
    w3a: np.ndarray
    b3a: np.ndarray
    w3b: np.ndarray
    b3b: np.ndarray

    @property
    def B(self) -> int:
        return len(self.node_off) - 1

    @property
    def n_types(self) -> int:
        return len(self.arity)

    @property
    def n_module_evals(self) -> int:
        return int((self.arity[self.node_type] > 0).sum())

    def expanded(self) -> IepWorkload:
        """The same computation as prefix programs: every shared sub-graph is written out once per use."""
        progs = []
        for i in range(self.B):
            b = int(self.node_off[i])
            seq = []

            def emit(j):
                seq.append(int(self.node_type[b + j]))
                for a in (self.arg0[b + j], self.arg1[b + j]):
                    if a >= 0:
                        emit(int(a))

            emit(int(self.root[i]))
            progs.append(np.array(seq, np.int32))
        prog, off = _pack(progs)
        return IepWorkload(self.name + "-expanded", self.dtype, self.arity, prog, off, self.C, self.H, self.W,
                           self.feats, self.w1, self.b1, self.w3a, self.b3a, self.w3b, self.b3b)


def random_dag(g: np.random.Generator, n_nodes: int, unary, binary, window: int = 4, p_binary: float = 0.4):
    """Random graph built bottom up (a node's arguments are earlier nodes, so no cycle can arise), cut down to
    what the last node depends on, then renumbered in random order.  Returns (type, arg0, arg1, root)."""
    types, a0, a1 = [SCENE], [-1], [-1]
    for i in range(1, n_nodes):
        lo = max(0, i - window)
        if i >= 2 and g.random() < p_binary:
            types.append(int(g.choice(binary)))
            a0.append(int(g.integers(lo, i)))
            a1.append(int(g.integers(lo, i)))
        elif g.random() < 0.1:
            types.append(SCENE)
            a0.append(-1)
            a1.append(-1)
        else:
            types.append(int(g.choice(unary)))
            a0.append(int(g.integers(lo, i)))
            a1.append(-1)
    keep, stack = set(), [n_nodes - 1]
    while stack:
        j = stack.pop()
        if j in keep:
            continue
        keep.add(j)
        stack += [a for a in (a0[j], a1[j]) if a >= 0]
    old = sorted(keep)
    order = g.permutation(len(old))                      # new index of old[k] is order[k]
    new_of = {o: int(order[k]) for k, o in enumerate(old)}
    n = len(old)
    t2, b0, b1 = np.zeros(n, np.int32), np.full(n, -1, np.int32), np.full(n, -1, np.int32)
    for o in old:
        q = new_of[o]
        t2[q] = types[o]
        b0[q] = new_of[a0[o]] if a0[o] >= 0 else -1
        b1[q] = new_of[a1[o]] if a1[o] >= 0 else -1
    return t2, b0, b1, new_of[n_nodes - 1]


def dag_batch(seed: int, B: int, C: int, H: int, W: int, dtype: str, n_unary: int = 3, n_binary: int = 2,
              min_nodes: int = 2, max_nodes: int = 12, window: int = 4) -> DagWorkload:
    arity = np.array([0] + [1] * n_unary + [2] * n_binary, np.uint8)
    unary = list(range(1, n_unary + 1))
    binary = list(range(n_unary + 1, n_unary + n_binary + 1))
    g = stream(seed, _S_TREE)
    parts = [random_dag(g, int(g.integers(min_nodes, max_nodes + 1)), unary, binary, window) for _ in range(B)]
    off = np.zeros(B + 1, np.int32)
    off[1:] = np.cumsum([len(p[0]) for p in parts])
    feats = make_feats(seed, B, H, W, C, dtype)
    w = make_weights(seed, arity, C, dtype)
    return DagWorkload(f"dag-{dtype}-B{B}-C{C}-{H}x{W}", dtype, arity,
                       np.concatenate([p[0] for p in parts]).astype(np.int32),
                       np.concatenate([p[1] for p in parts]).astype(np.int32),
                       np.concatenate([p[2] for p in parts]).astype(np.int32), off,
                       np.array([p[3] for p in parts], np.int32), C, H, W, feats, *w)
