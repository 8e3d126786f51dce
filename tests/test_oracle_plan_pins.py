"""Pins of the plan oracle against things other than itself.

The planner rules are from the paper's Background / "Visual Reasoning Programs" (unique tree
from a prefix sequence with fixed arities) and Methods ("Improved" and "Standard"
topological sort).  The independent checker below builds an explicit pointer tree with an
iterative stack parse and labels it breadth first; it shares nothing with the C oracle.
"""
import itertools
import os

import numpy as np
import pytest

from workloads import iep

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ independent checker
def parse_iterative(seq, arity):
    """Pointer tree by an explicit stack of open argument slots. Returns children lists or None."""
    kids = [[] for _ in seq]
    stack = []            # (node, args still missing)
    for pos, t in enumerate(seq):
        if pos > 0:
            if not stack:
                return None           # tokens left after the tree closed
            par, miss = stack.pop()
            kids[par].append(pos)
            if miss > 1:
                stack.append((par, miss - 1))
        if arity[t] > 0:
            stack.append((pos, arity[t]))
    return kids if not stack and len(seq) > 0 else None


def bfs_levels(kids):
    lvl = [-1] * len(kids)
    lvl[0] = 0
    frontier = [0]
    while frontier:
        nxt = []
        for n in frontier:
            for c in kids[n]:
                lvl[c] = lvl[n] + 1
                nxt.append(c)
        frontier = nxt
    return lvl


def postorder_positions(kids):
    order = []

    def visit(n):
        for c in kids[n]:
            visit(c)
        order.append(n)

    visit(0)
    pos = [0] * len(kids)
    for j, n in enumerate(order):
        pos[n] = j
    return pos


def peel_heights(kids):
    """Dependency depth by peeling: round r removes the nodes whose arguments were all removed before round r."""
    h = [-1] * len(kids)
    left, r = len(kids), 0
    while left:
        now = [n for n in range(len(kids)) if h[n] < 0 and all(0 <= h[c] < r for c in kids[n])]
        assert now
        for n in now:
            h[n] = r
        left -= len(now)
        r += 1
    return h


def expected_buckets(labels, types, descending):
    keys = sorted(range(len(labels)), key=lambda i: ((-labels[i] if descending else labels[i]), types[i], i))
    buckets = []
    for key, grp in itertools.groupby(keys, key=lambda i: (labels[i], types[i])):
        buckets.append((key[0], key[1], list(grp)))
    return buckets


def check_against_independent(o, progs, arity, mode):
    off = np.zeros(len(progs) + 1, np.int32)
    off[1:] = np.cumsum([len(p) for p in progs])
    prog = np.concatenate(progs).astype(np.int32)
    pl = o.plan(prog, off, arity, mode=mode)
    labels, types, c0, c1 = [], [], [], []
    for i, p in enumerate(progs):
        kids = parse_iterative(list(p), arity)
        assert kids is not None
        lab = bfs_levels(kids) if mode == 0 else postorder_positions(kids) if mode == 1 else peel_heights(kids)
        labels += lab
        types += list(p)
        base = int(off[i])
        c0 += [base + k[0] if len(k) > 0 else -1 for k in kids]
        c1 += [base + k[1] if len(k) > 1 else -1 for k in kids]
    assert list(pl.node_level) == labels
    assert list(pl.node_type) == types
    assert list(pl.child0) == c0 and list(pl.child1) == c1
    assert list(pl.root) == list(off[:-1])
    assert pl.n_levels == max(labels) + 1
    exp = expected_buckets(labels, types, descending=(mode == 0))
    assert pl.n_buckets == len(exp)
    for b, (lv, t, mem) in enumerate(exp):
        s, c = pl.bucket_start[b], pl.bucket_count[b]
        assert (pl.bucket_level[b], pl.bucket_type[b]) == (lv, t)
        assert list(pl.members[s:s + c]) == mem
        assert list(pl.out[s:s + c]) == mem
        assert list(pl.in0[s:s + c]) == [c0[m] for m in mem]
        assert list(pl.in1[s:s + c]) == [c1[m] for m in mem]
    return pl


# ------------------------------------------------------------------ tests
ARITY3 = np.array([0, 1, 2], np.uint8)


def all_sequences(max_len):
    for n in range(1, max_len + 1):
        for seq in itertools.product(range(3), repeat=n):
            yield list(seq)


@pytest.mark.parametrize("mode", [0, 1, 2])
def test_brute_force_all_programs_up_to_length_7(oracle, mode):
    """Every sequence over {leaf, unary, binary} up to length 7: accepted iff well formed, labels as BFS."""
    good, bad = [], 0
    for seq in all_sequences(7):
        kids = parse_iterative(seq, ARITY3)
        off = np.array([0, len(seq)], np.int32)
        if kids is None:
            with pytest.raises(oracle.MalformedProgram):
                oracle.plan(np.array(seq, np.int32), off, ARITY3, mode=mode)
            bad += 1
        else:
            good.append(np.array(seq, np.int32))
    # well-formed sequences of length n over arities {0,1,2} are counted by the Motzkin numbers
    assert len(good) == 1 + 1 + 2 + 4 + 9 + 21 + 51
    assert bad > 0
    for p in good:                              # one at a time
        check_against_independent(oracle, [p], ARITY3, mode)
    check_against_independent(oracle, good, ARITY3, mode)   # and as one minibatch


def test_golden_hand_labelled_tree(oracle):
    rows = {}
    pools = []
    for line in open(os.path.join(GOLD, "labelled_tree.txt")):
        line = line.split("#")[0].split()
        if not line:
            continue
        if line[0] == "pool":
            pools.append((int(line[1]), int(line[2]), [int(v) for v in line[3:]]))
        else:
            rows[line[0]] = [int(v) for v in line[1:]]
    arity = np.array([0, 1, 1, 2, 2], np.uint8)
    prog = np.array(rows["prog"], np.int32)
    off = np.array([0, len(prog)], np.int32)
    pl = oracle.plan(prog, off, arity, mode=0)
    assert list(pl.node_level) == rows["rootdist"]
    assert list(pl.child0) == rows["child0"] and list(pl.child1) == rows["child1"]
    got = [(int(pl.bucket_level[b]), int(pl.bucket_type[b]),
            list(pl.members[pl.bucket_start[b]:pl.bucket_start[b] + pl.bucket_count[b]]))
           for b in range(pl.n_buckets)]
    assert got == pools
    assert list(oracle.plan(prog, off, arity, mode=1).node_level) == rows["postorder"]
    dd = oracle.plan(prog, off, arity, mode=2)
    assert list(dd.node_level) == rows["depdepth"]
    # ascending labels, then function id: SCENE leaves first, the root last and alone
    assert (int(dd.bucket_level[0]), int(dd.bucket_type[0])) == (0, 0)
    assert list(dd.members[:3]) == [3, 5, 8]
    assert (int(dd.bucket_level[-1]), int(dd.bucket_type[-1]), int(dd.bucket_count[-1])) == (4, 3, 1)


@pytest.mark.parametrize("n", [1, 2, 7, 30])
def test_chain_has_one_node_per_level(oracle, n):
    arity = np.array([0, 1], np.uint8)
    prog = np.array([1] * (n - 1) + [0], np.int32)
    pl = oracle.plan(prog, np.array([0, n], np.int32), arity)
    assert pl.n_levels == n
    assert list(pl.node_level) == list(range(n))
    assert pl.n_buckets == n                       # one pool per (level, type)
    assert int(pl.bucket_count.sum()) == n


@pytest.mark.parametrize("n", [1, 2, 7, 30])
def test_chain_dependency_depth_counts_up_from_the_leaf(oracle, n):
    arity = np.array([0, 1], np.uint8)
    prog = np.array([1] * (n - 1) + [0], np.int32)
    pl = oracle.plan(prog, np.array([0, n], np.int32), arity, mode=2)
    assert pl.n_levels == n
    assert list(pl.node_level) == list(range(n - 1, -1, -1))
    assert list(pl.members) == list(range(n - 1, -1, -1))          # the leaf runs first, the root last


@pytest.mark.parametrize("m", [0, 1, 3, 5])
def test_balanced_tree_dependency_depth_mirrors_root_distance(oracle, m):
    """In a full binary tree every leaf is equally deep, so depth-from-leaves = m - distance-from-root."""
    g = np.random.default_rng(100 + m)
    arity = np.array([0] + [2] * 8, np.uint8)
    progs = [iep.balanced_program(g, m + 1, list(range(1, 9))) for _ in range(3)]
    dd = check_against_independent(oracle, progs, arity, 2)
    rd = check_against_independent(oracle, progs, arity, 0)
    assert dd.n_levels == m + 1
    assert (dd.node_level == m - rd.node_level).all()
    for h in range(m + 1):
        assert int((dd.node_level == h).sum()) == 3 * 2 ** (m - h)


@pytest.mark.parametrize("m", [0, 1, 2, 4, 6])
def test_balanced_tree_levels_are_log2_leaves_plus_1(oracle, m):
    """Methods / Improved topological sort: balanced trees give O(p log2 s); 2^m leaves -> m+1 labels."""
    g = np.random.default_rng(m)
    arity = np.array([0] + [2] * 8, np.uint8)
    progs = [iep.balanced_program(g, m + 1, list(range(1, 9))) for _ in range(5)]
    pl = check_against_independent(oracle, progs, arity, 0)
    leaves = int((pl.node_type == 0).sum()) // 5
    assert leaves == 2 ** m
    assert pl.n_levels == int(np.log2(leaves)) + 1
    for lvl in range(m + 1):
        assert int((pl.node_level == lvl).sum()) == 5 * 2 ** lvl
    compute = pl.bucket_type != 0
    assert compute.sum() <= 8 * m                                    # p * (levels with network calls)


def test_config1_is_the_stated_balanced_case(oracle):
    w = iep.config1()
    pl = oracle.plan(w.prog, w.prog_off, w.arity)
    assert pl.n_nodes == 64 * 31 and pl.n_levels == 5 == int(np.log2(16)) + 1
    assert w.n_module_evals == 960
    assert (pl.bucket_type != 0).sum() <= 4 * 8


@pytest.mark.parametrize("mode", [0, 1, 2])
def test_invariants_on_iep_shaped_batch(oracle, mode):
    w = iep.config2()
    pl = oracle.plan(w.prog, w.prog_off, w.arity, mode=mode)
    N, p = pl.n_nodes, w.n_types - 1
    assert N == len(w.prog) and int(pl.bucket_count.sum()) == N
    assert sorted(pl.members.tolist()) == list(range(N))             # every node in exactly one pool
    assert (pl.bucket_start == np.concatenate([[0], np.cumsum(pl.bucket_count)[:-1]])).all()
    # children are labelled so that they run strictly before their consumer
    when = np.empty(N, np.int64)
    for b in range(pl.n_buckets):
        when[pl.members[pl.bucket_start[b]:pl.bucket_start[b] + pl.bucket_count[b]]] = b
    for child in (pl.child0, pl.child1):
        has = child >= 0
        assert (when[child[has]] < when[np.nonzero(has)[0]]).all()
        if mode == 0:
            assert (pl.node_level[child[has]] == pl.node_level[np.nonzero(has)[0]] + 1).all()
    # call-count bounds of the paper: O(p d) for the improved sort, O(p s) for the standard one
    compute = pl.bucket_type != 0
    s_max = int(np.diff(w.prog_off).max())
    assert compute.sum() <= p * (s_max if mode == 1 else pl.n_levels)
    assert pl.n_levels <= s_max
    # arity of a node = number of children
    ar = w.arity[pl.node_type]
    assert ((pl.child0 >= 0).astype(int) + (pl.child1 >= 0).astype(int) == ar).all()


def test_dependency_depth_is_the_earliest_and_root_distance_the_latest_step(oracle):
    """Both labellings are schedules with the same number of steps; a node can never be ready before its
    dependency depth, and its root-distance label is the last step that still lets its consumers run in time."""
    w = iep.config2()
    rd = oracle.plan(w.prog, w.prog_off, w.arity, mode=0)
    dd = oracle.plan(w.prog, w.prog_off, w.arity, mode=2)
    assert dd.n_levels == rd.n_levels
    D = rd.n_levels
    assert (dd.node_level <= D - 1 - rd.node_level).all()
    ar = w.arity[dd.node_type]
    assert (dd.node_level[ar == 0] == 0).all() and (dd.node_level[ar > 0] >= 1).all()
    # label = 1 + the larger of the arguments' labels
    l0 = np.where(dd.child0 >= 0, dd.node_level[np.maximum(dd.child0, 0)], -1)
    l1 = np.where(dd.child1 >= 0, dd.node_level[np.maximum(dd.child1, 0)], -1)
    assert (dd.node_level == np.maximum(l0, l1) + 1).all()
    # each example's root carries that example's depth; the deepest one defines D
    assert int(dd.node_level[dd.root].max()) == D - 1
    assert (dd.node_level[dd.root] == np.array(
        [rd.node_level[w.prog_off[i]:w.prog_off[i + 1]].max() for i in range(w.B)])).all()


def test_permuting_examples_keeps_pool_sizes(oracle):
    w = iep.config2(B=40)
    a = oracle.plan(w.prog, w.prog_off, w.arity)
    order = np.random.default_rng(3).permutation(w.B)
    ws = w.subset(order)
    b = oracle.plan(ws.prog, ws.prog_off, ws.arity)
    assert (a.bucket_level == b.bucket_level).all() and (a.bucket_type == b.bucket_type).all()
    assert (a.bucket_count == b.bucket_count).all()


def test_improved_sort_needs_no_more_calls_than_standard(oracle):
    """Methods: the improved sort has an equal or better constant than the standard one."""
    w = iep.config2()
    imp = oracle.plan(w.prog, w.prog_off, w.arity, mode=0)
    std = oracle.plan(w.prog, w.prog_off, w.arity, mode=1)
    assert (imp.bucket_type != 0).sum() <= (std.bucket_type != 0).sum()


def test_malformed_names_the_example(oracle):
    arity = np.array([0, 1, 2], np.uint8)
    good = [1, 0]
    for bad in ([2, 0], [0, 0], [1], [2, 0, 0, 0], [5, 0], []):
        prog = np.array(good + bad + good, np.int32)
        off = np.array([0, 2, 2 + len(bad), 4 + len(bad)], np.int32)
        with pytest.raises(oracle.MalformedProgram) as e:
            oracle.plan(prog, off, arity)
        assert e.value.example == 1
