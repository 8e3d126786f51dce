"""Pins of the dependency-graph oracle (plan and float) against things other than itself.

A graph whose nodes all have one consumer is a tree, so the graph oracle must reproduce the (separately
pinned) tree oracle there; a graph with shared nodes computes what its written-out tree computes; labels
are checked against an independent Kahn-order relaxation and a hand-labelled fixture.
"""
import itertools
import os

import numpy as np
import pytest

from workloads import iep

GOLD = os.path.join(os.path.dirname(__file__), "golden")
ARITY3 = np.array([0, 1, 2], np.uint8)


# ------------------------------------------------------------------ independent checker
def check_graph(types, a0, a1, root, arity):
    """None if malformed, else (max root distance, dependency depth) by Kahn's algorithm + relaxation."""
    n = len(types)
    if n == 0 or not (0 <= root < n):
        return None
    args = []
    for j in range(n):
        if not (0 <= types[j] < len(arity)):
            return None
        mine = [a for a in (a0[j], a1[j]) if a != -1]
        if any(not (0 <= a < n) for a in mine) or len(mine) != arity[types[j]] or (a1[j] != -1 and a0[j] == -1):
            return None
        args.append(mine)
    pending = [len(set(m)) for m in args]                 # distinct arguments still missing
    users = [[] for _ in range(n)]
    for j, m in enumerate(args):
        for a in set(m):
            users[a].append(j)
    ready = [j for j in range(n) if pending[j] == 0]
    order = []
    while ready:
        j = ready.pop()
        order.append(j)
        for u in users[j]:
            pending[u] -= 1
            if pending[u] == 0:
                ready.append(u)
    if len(order) != n:
        return None                                       # a cycle
    depth = [0] * n
    for j in order:                                       # arguments before consumers
        depth[j] = 1 + max(depth[a] for a in args[j]) if args[j] else 0
    dist = [-1] * n
    dist[root] = 0
    for j in reversed(order):                             # consumers before arguments
        if dist[j] >= 0:
            for a in args[j]:
                dist[a] = max(dist[a], dist[j] + 1)
    if min(dist) < 0:
        return None                                       # a node the root does not depend on
    return dist, depth


def as_graph(prog, arity):
    """Prefix program -> (type, arg0, arg1) with node index = position."""
    n = len(prog)
    a0, a1 = np.full(n, -1, np.int32), np.full(n, -1, np.int32)

    def build(pos):
        nxt = pos + 1
        for k in range(arity[prog[pos]]):
            (a0 if k == 0 else a1)[pos] = nxt
            nxt = build(nxt)
        return nxt

    assert build(0) == n
    return np.asarray(prog, np.int32), a0, a1


FIELDS = ("node_level", "node_type", "child0", "child1", "root", "bucket_level", "bucket_type", "bucket_start",
          "bucket_count", "members", "in0", "in1", "out")


# ------------------------------------------------------------------ tests
@pytest.mark.parametrize("mode", [0, 2])
def test_trees_written_as_graphs_give_the_tree_plan(oracle, mode):
    w = iep.config2(B=60)
    parts = [as_graph(w.program(i), w.arity) for i in range(w.B)]
    t, a0, a1 = (np.concatenate([p[k] for p in parts]) for k in range(3))
    g = oracle.plan_dag(t, a0, a1, w.prog_off, np.zeros(w.B, np.int32), w.arity, mode=mode)
    tr = oracle.plan(w.prog, w.prog_off, w.arity, mode=mode)
    assert (g.n_nodes, g.n_levels, g.n_buckets) == (tr.n_nodes, tr.n_levels, tr.n_buckets)
    for f in FIELDS:
        assert (getattr(g, f) == getattr(tr, f)).all(), f


def test_golden_hand_labelled_graph(oracle):
    rows, pools = {}, []
    for line in open(os.path.join(GOLD, "labelled_dag.txt")):
        line = line.split("#")[0].split()
        if not line:
            continue
        if line[0] == "pool":
            pools.append((int(line[1]), int(line[2]), [int(v) for v in line[3:]]))
        else:
            rows[line[0]] = [int(v) for v in line[1:]]
    arity = np.array([0, 1, 1, 2, 2], np.uint8)
    off = np.array([0, len(rows["type"])], np.int32)
    pl = oracle.plan_dag(rows["type"], rows["arg0"], rows["arg1"], off, rows["root"], arity, mode=0)
    assert list(pl.node_level) == rows["maxdist"]
    got = [(int(pl.bucket_level[b]), int(pl.bucket_type[b]),
            list(pl.members[pl.bucket_start[b]:pl.bucket_start[b] + pl.bucket_count[b]])) for b in range(pl.n_buckets)]
    assert got == pools
    dd = oracle.plan_dag(rows["type"], rows["arg0"], rows["arg1"], off, rows["root"], arity, mode=2)
    assert list(dd.node_level) == rows["depdepth"]
    assert check_graph(rows["type"], rows["arg0"], rows["arg1"], rows["root"][0], arity) == (rows["maxdist"], rows["depdepth"])


def test_brute_force_all_graphs_up_to_three_nodes(oracle):
    """Every assignment of {leaf, unary, binary} nodes with arbitrary argument indices (self loops and cycles
    included) and every root: accepted iff the independent checker accepts, with its labels."""
    good = bad = 0
    for n in (1, 2, 3):
        options = [(0, -1, -1)] + [(1, a, -1) for a in range(n)] + [(2, a, b) for a in range(n) for b in range(n)]
        for nodes in itertools.product(options, repeat=n):
            t, a0, a1 = ([x[k] for x in nodes] for k in range(3))
            for root in range(n):
                exp = check_graph(t, a0, a1, root, ARITY3)
                off = np.array([0, n], np.int32)
                if exp is None:
                    with pytest.raises(oracle.MalformedProgram):
                        oracle.plan_dag(t, a0, a1, off, [root], ARITY3)
                    bad += 1
                else:
                    assert list(oracle.plan_dag(t, a0, a1, off, [root], ARITY3, mode=0).node_level) == exp[0]
                    assert list(oracle.plan_dag(t, a0, a1, off, [root], ARITY3, mode=2).node_level) == exp[1]
                    good += 1
    assert good > 20 and bad > 1000


@pytest.mark.parametrize("mode", [0, 2])
def test_random_graphs_against_the_independent_checker_and_invariants(oracle, mode):
    d = iep.dag_batch(seed=11, B=200, C=1, H=1, W=1, dtype="f32", max_nodes=14)
    pl = oracle.plan_dag(d.node_type, d.arg0, d.arg1, d.node_off, d.root, d.arity, mode=mode)
    shared = 0
    for i in range(d.B):
        b, e = int(d.node_off[i]), int(d.node_off[i + 1])
        exp = check_graph(list(d.node_type[b:e]), list(d.arg0[b:e]), list(d.arg1[b:e]), int(d.root[i]), d.arity)
        assert exp is not None and list(pl.node_level[b:e]) == exp[0 if mode == 0 else 1], i
        uses = np.bincount(np.concatenate([d.arg0[b:e], d.arg1[b:e]])[np.concatenate([d.arg0[b:e], d.arg1[b:e]]) >= 0],
                           minlength=e - b)
        shared += int((uses > 1).sum())
    assert shared > 50                                     # the batch really has shared nodes
    assert sorted(pl.members.tolist()) == list(range(pl.n_nodes)) and int(pl.bucket_count.sum()) == pl.n_nodes
    when = np.empty(pl.n_nodes, np.int64)
    for bk in range(pl.n_buckets):
        when[pl.members[pl.bucket_start[bk]:pl.bucket_start[bk] + pl.bucket_count[bk]]] = bk
    for child in (pl.child0, pl.child1):
        has = child >= 0
        assert (when[child[has]] < when[np.nonzero(has)[0]]).all()      # arguments run strictly earlier
    if mode == 0:
        assert (pl.node_level[pl.root] == 0).all()


def test_a_graph_computes_what_its_written_out_tree_computes(oracle):
    """Float pin: the graph oracle against the tree oracle (pinned on its own) on the expanded programs."""
    d = iep.dag_batch(seed=5, B=12, C=3, H=4, W=3, dtype="f32", max_nodes=9)
    x = d.expanded()
    assert x.n_module_evals > d.n_module_evals             # sharing saves evaluations
    got = oracle.iep_forward_dag(d.node_type, d.arg0, d.arg1, d.node_off, d.root, d.arity, d.feats,
                                 d.w1, d.b1, d.w3a, d.b3a, d.w3b, d.b3b)
    ref = oracle.iep_forward_workload(x)
    assert np.abs(got).max() > 0 and (got == ref).all()    # same arithmetic in the same order


def test_malformed_graphs_name_the_example(oracle):
    ok = ([1, 0], [1, -1], [-1, -1], 0)                    # un(SCENE)
    cases = [([1, 1], [1, 0], [-1, -1], 0),                # two-node cycle
             ([1, 0], [0, -1], [-1, -1], 0),               # self loop
             ([1, 0, 0], [1, -1, -1], [-1, -1, -1], 0),    # node 2 feeds nothing
             ([2, 0], [1, -1], [-1, -1], 0),               # binary with one argument
             ([1, 0], [1, -1], [1, -1], 0),                # unary with two
             ([1, 0], [5, -1], [-1, -1], 0),               # argument out of range
             ([1, 0], [1, -1], [-1, -1], 2),               # root out of range
             ([7, 0], [1, -1], [-1, -1], 0)]               # unknown function
    for t, a0, a1, r in cases:
        types = ok[0] + t + ok[0]
        arg0 = ok[1] + a0 + ok[1]
        arg1 = ok[2] + a1 + ok[2]
        off = np.array([0, 2, 2 + len(t), 4 + len(t)], np.int32)
        with pytest.raises(oracle.MalformedProgram) as e:
            oracle.plan_dag(types, arg0, arg1, off, [0, r, 0], ARITY3)
        assert e.value.example == 1
