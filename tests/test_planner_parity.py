"""The C++ planner against the plan oracle: every array of the plan view must be bit-identical.
Host code only (no GPU needed)."""
import ctypes as ct
import os
import re

import numpy as np
import pytest

from workloads import iep

FIELDS = ("node_level", "node_type", "child0", "child1", "root", "bucket_level", "bucket_type", "bucket_start",
          "bucket_count", "members", "in0", "in1", "out")


@pytest.fixture(scope="module")
def dyn():
    import paper_1707_02402_amd as d
    return d


def assert_same_plan(v, o):
    assert (v.n_nodes, v.n_levels, v.n_buckets) == (o.n_nodes, o.n_levels, o.n_buckets)
    for f in FIELDS:
        a, b = getattr(v, f), getattr(o, f)
        assert a.dtype == np.int32 and a.shape == b.shape and (a == b).all(), f


# (library scheduling mode, oracle labelling mode): improved, standard, dependency depth
MODES = [(0, 0), (1, 1), (3, 2)]


@pytest.mark.parametrize("mode,omode", MODES)
@pytest.mark.parametrize("cfg", ["config0", "config1", "config2"])
def test_plan_is_bit_exact_on_the_configs(dyn, oracle, cfg, mode, omode):
    w = getattr(iep, cfg)()
    plan = dyn.dynbatch_plan(w.prog, w.prog_off, w.arity, mode)
    v = dyn.dynbatch_plan_view(plan)
    assert_same_plan(v, oracle.plan(w.prog, w.prog_off, w.arity, mode=omode))
    assert v.n_compute_nodes == w.n_module_evals
    if mode == 0:
        assert v.n_launches == v.n_levels - 1          # deepest label of these configs holds only SCENE leaves
    if mode == 3:
        assert v.n_launches == v.n_levels - 1          # label 0 holds exactly the SCENE leaves
        compute = w.arity[v.node_type] > 0
        assert (v.node_launch[compute] == v.node_level[compute] - 1).all()
        assert v.n_slots <= v.n_compute_nodes


def test_plan_is_bit_exact_on_many_random_batches(dyn, oracle):
    for seed in range(40):
        w = iep.small_mixed(seed=seed, B=1 + seed % 9, C=1, H=1, W=1, dtype="f32", min_len=1, max_len=3 + seed)
        for mode, omode in MODES:
            v = dyn.dynbatch_plan_view(dyn.dynbatch_plan(w.prog, w.prog_off, w.arity, mode))
            assert_same_plan(v, oracle.plan(w.prog, w.prog_off, w.arity, mode=omode))


@pytest.mark.parametrize("mode,omode", [(0, 0), (3, 2)])
def test_graph_plan_is_bit_exact(dyn, oracle, mode, omode):
    for seed in range(12):
        d = iep.dag_batch(seed=seed, B=1 + 7 * seed, C=1, H=1, W=1, dtype="f32", max_nodes=4 + 2 * seed)
        v = dyn.dynbatch_plan_view(dyn.dynbatch_plan_dag(d.node_type, d.arg0, d.arg1, d.node_off, d.root, d.arity, mode))
        assert_same_plan(v, oracle.plan_dag(d.node_type, d.arg0, d.arg1, d.node_off, d.root, d.arity, mode=omode))
        assert v.n_compute_nodes == d.n_module_evals and v.n_slots <= max(v.n_compute_nodes, 1)


def test_graph_plan_of_a_tree_equals_the_tree_plan(dyn):
    w = iep.config2(B=50)
    n = len(w.prog)
    a0, a1 = np.full(n, -1, np.int32), np.full(n, -1, np.int32)
    tree = dyn.dynbatch_plan_view(dyn.dynbatch_plan(w.prog, w.prog_off, w.arity))
    for i in range(w.B):                               # arguments as indices inside the example
        b, e = w.prog_off[i], w.prog_off[i + 1]
        a0[b:e] = np.where(tree.child0[b:e] >= 0, tree.child0[b:e] - b, -1)
        a1[b:e] = np.where(tree.child1[b:e] >= 0, tree.child1[b:e] - b, -1)
    g = dyn.dynbatch_plan_view(dyn.dynbatch_plan_dag(w.prog, a0, a1, w.prog_off, np.zeros(w.B, np.int32), w.arity))
    for f in FIELDS + ("node_launch",):
        assert (getattr(g, f) == getattr(tree, f)).all(), f


def test_graph_plan_errors(dyn):
    ar = np.array([0, 1, 2], np.uint8)
    good = dict(node_type=[1, 0], arg0=[1, -1], arg1=[-1, -1])
    off = np.array([0, 2, 4], np.int32)
    for t, a0, a1, r in [([1, 1], [1, 0], [-1, -1], 0), ([1, 0, 0][:2], [0, -1], [-1, -1], 0), ([2, 0], [1, -1], [-1, -1], 0),
                         ([1, 0], [1, -1], [-1, -1], 2), ([1, 0], [3, -1], [-1, -1], 0)]:
        with pytest.raises(dyn.DynbError) as e:
            dyn.dynbatch_plan_dag(good["node_type"] + t, good["arg0"] + a0, good["arg1"] + a1, off, [0, r], ar)
        assert e.value.name == "DYNB_E_MALFORMED" and "example 1" in str(e.value)
    with pytest.raises(dyn.DynbError) as e:
        dyn.dynbatch_plan_dag(good["node_type"], good["arg0"], good["arg1"], off[:2], [0], ar, flags=dyn.DYNB_SCHED_STANDARD)
    assert e.value.name == "DYNB_E_UNSUPPORTED"
    with pytest.raises(dyn.DynbError) as e:                # a node that the root does not depend on
        dyn.dynbatch_plan_dag([1, 0, 0], [1, -1, -1], [-1, -1, -1], np.array([0, 3], np.int32), [0], ar)
    assert e.value.name == "DYNB_E_MALFORMED"


def test_threaded_parse_of_a_large_batch(dyn, oracle):
    w = iep.config2(B=2500)                          # > 32768 nodes: the planner uses several threads
    assert len(w.prog) > (1 << 15)
    v = dyn.dynbatch_plan_view(dyn.dynbatch_plan(w.prog, w.prog_off, w.arity, 0))
    o = oracle.plan(w.prog, w.prog_off, w.arity)
    assert_same_plan(v, o)


def test_balanced_launch_groups_are_a_valid_schedule(dyn, oracle):
    """DYNB_PLAN_BALANCE may only move nodes to earlier launch groups, never before their arguments,
    and leaves the logical plan (labels, pools) untouched."""
    w = iep.config2()
    plain = dyn.dynbatch_plan_view(dyn.dynbatch_plan(w.prog, w.prog_off, w.arity, 0))
    bal = dyn.dynbatch_plan_view(dyn.dynbatch_plan(w.prog, w.prog_off, w.arity, dyn.DYNB_PLAN_BALANCE))
    assert_same_plan(bal, oracle.plan(w.prog, w.prog_off, w.arity))
    compute = w.arity[bal.node_type] > 0
    assert (bal.node_launch[~compute] == -1).all() and (bal.node_launch[compute] >= 0).all()
    assert (bal.node_launch <= plain.node_launch).all()              # the label is the latest group
    for child in (bal.child0, bal.child1):
        has = (child >= 0) & compute
        kids = child[has]
        ck = w.arity[bal.node_type[kids]] > 0
        assert (bal.node_launch[kids[ck]] < bal.node_launch[np.nonzero(has)[0][ck]]).all()
    sizes_plain = np.bincount(plain.node_launch[compute])
    sizes_bal = np.bincount(bal.node_launch[compute])
    assert sizes_bal.sum() == sizes_plain.sum() == w.n_module_evals and len(sizes_bal) == len(sizes_plain)
    assert (sizes_plain > 256).sum() > 0 and (sizes_bal > 256).sum() < (sizes_plain > 256).sum()
    assert bal.n_launches == plain.n_launches and bal.n_slots <= plain.n_compute_nodes


def test_naive_schedule_is_one_valid_call_per_node(dyn):
    w = iep.config2(B=16)
    v = dyn.dynbatch_plan_view(dyn.dynbatch_plan(w.prog, w.prog_off, w.arity, dyn.DYNB_SCHED_NAIVE))
    assert v.n_buckets == v.n_nodes and (v.bucket_count == 1).all()
    assert v.n_launches == w.n_module_evals and v.max_launch_nodes == 1
    when = np.empty(v.n_nodes, np.int64)
    when[v.members] = np.arange(v.n_nodes)
    for child in (v.child0, v.child1):
        has = child >= 0
        assert (when[child[has]] < when[np.nonzero(has)[0]]).all()
    ex = np.searchsorted(w.prog_off, v.members, side="right") - 1
    assert (np.diff(ex) >= 0).all()                  # example by example


def test_error_codes(dyn):
    ar = np.array([0, 1, 2], np.uint8)
    ok = np.array([1, 0], np.int32)
    for bad in ([2, 0], [0, 0], [1], [7, 0], []):
        prog = np.concatenate([ok, np.array(bad, np.int32), ok]).astype(np.int32)
        off = np.array([0, 2, 2 + len(bad), 4 + len(bad)], np.int32)
        with pytest.raises(dyn.DynbError) as e:
            dyn.dynbatch_plan(prog, off, ar)
        assert e.value.name == "DYNB_E_MALFORMED" and "example 1" in str(e.value)
    with pytest.raises(dyn.DynbError) as e:
        dyn.dynbatch_plan(ok, np.array([0, 2], np.int32), np.array([0, 3], np.uint8))
    assert e.value.name == "DYNB_E_UNSUPPORTED"
    dyn.dynbatch_plan(ok, np.array([0, 2], np.int32), ar, flags=dyn.DYNB_PLAN_THROUGHPUT | dyn.DYNB_PLAN_BALANCE)
    with pytest.raises(dyn.DynbError) as e:
        dyn.dynbatch_plan(ok, np.array([0, 2], np.int32), ar, flags=64)
    assert e.value.name == "DYNB_E_UNSUPPORTED"
    with pytest.raises(dyn.DynbError) as e:
        dyn.dynbatch_plan(ok, np.array([1, 2], np.int32), ar)
    assert e.value.name == "DYNB_E_INVAL"
    from paper_1707_02402_amd.binding import lib
    assert lib.dynbatch_plan(None, None, 1, None, 1, 0, None) == -1
    assert lib.dynbatch_workspace_bytes(None, None) == 0
    assert lib.moe_workspace_bytes(None) == 0


def test_library_exports_every_declared_symbol():
    from paper_1707_02402_amd.binding import EXPORTS, LIB_PATH
    header = open(os.path.join(os.path.dirname(__file__), "..", "include", "dynbatch.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(dynb_\w+|dynbatch_\w+|moe_\w+)\s*\(", header))
    assert declared == set(EXPORTS)
    L = ct.CDLL(LIB_PATH)
    for name in declared:
        assert getattr(L, name) is not None


def test_moe_shape_checks_need_no_gpu(dyn):
    from paper_1707_02402_amd.binding import _MoeShape, lib
    assert dyn.moe_workspace_bytes(64, 64, 64, 8, 2) > 0
    for bad in ((64, 64, 64, 8, 9), (64, 64, 64, 4, 5), (64, 44, 64, 8, 2), (64, 64, 0, 8, 2)):
        assert dyn.moe_workspace_bytes(*bad) == 0
    # T = 0 succeeds without touching any pointer
    assert lib.moe_forward(ct.byref(_MoeShape(0, 64, 64, 8, 2, 1)), None, None, None, None, None, None, None, None,
                           None, 0, None) == 0


# ------------------------------------------------------------------------------------------------
# DYNB_PLAN_PERSISTENT: the claim order of the single dependency-driven launch, checked on the host
# ------------------------------------------------------------------------------------------------
def _persistent_cases(dyn):
    cases = []
    for mode in (dyn.DYNB_SCHED_IMPROVED, dyn.DYNB_SCHED_STANDARD, dyn.DYNB_SCHED_DEPTH):
        for w in (iep.config0(), iep.config1(), iep.config2(), iep.small_mixed(seed=11, B=40, C=4, H=2, W=2, dtype="f32", min_len=1)):
            plan = dyn.dynbatch_plan(w.prog, w.prog_off, w.arity, mode | dyn.DYNB_PLAN_PERSISTENT)
            cases.append((f"{w.name}/mode{mode}", w.arity, dyn.dynbatch_plan_view(plan)))
    for mode in (dyn.DYNB_SCHED_IMPROVED, dyn.DYNB_SCHED_DEPTH):
        d = iep.dag_batch(seed=5, B=60, C=4, H=2, W=2, dtype="f32", max_nodes=14)
        plan = dyn.dynbatch_plan_dag(d.node_type, d.arg0, d.arg1, d.node_off, d.root, d.arity, mode | dyn.DYNB_PLAN_PERSISTENT)
        cases.append((f"dag/mode{mode}", d.arity, dyn.dynbatch_plan_view(plan)))
    return cases


def test_persistent_tickets_cover_every_node_and_follow_their_arguments(dyn):
    """Every unit of work is claimed after every unit of its node's arguments: the condition under which the
    bounded waits of the dependency-driven kernel always end (the unit with the smallest unfinished ticket has
    all its arguments finished)."""
    for name, arity, v in _persistent_cases(dyn):
        assert v.n_tickets == len(v.tickets) and v.n_tickets >= v.n_compute_nodes, name
        item_of_node = {int(n): i for i, n in enumerate(v.item_node)}
        assert len(item_of_node) == v.n_compute_nodes
        parts = {}
        last_ticket_of_item = {}
        for tk, t in enumerate(v.tickets):
            item, part = int(t) >> 2, int(t) & 3
            parts.setdefault(item, []).append(part)
            last_ticket_of_item[item] = tk
            node = int(v.item_node[item])
            for c in (v.child0[node], v.child1[node]):
                if c >= 0 and arity[v.node_type[c]] > 0:
                    ci = item_of_node[int(c)]
                    assert sorted(parts.get(ci, [])) in ([0], [1, 2]), (name, "argument not fully claimed before", tk)
                    assert last_ticket_of_item[ci] < tk
        assert sorted(parts) == list(range(v.n_compute_nodes)), name
        assert all(sorted(p) in ([0], [1, 2]) for p in parts.values()), name      # a whole node, or both halves once


def test_persistent_schedule_simulated_with_few_and_many_workers(dyn):
    """Host simulation of the kernel's protocol: workers claim tickets in order from one counter, wait until
    both halves (or the whole) of every argument have been published, work for a while and publish.  With any
    number of workers, any durations and any interleaving every ticket completes."""
    import heapq
    g = np.random.default_rng(3)
    for name, arity, v in _persistent_cases(dyn):
        item_of_node = {int(n): i for i, n in enumerate(v.item_node)}
        deps = []
        for t in v.tickets:
            node = int(v.item_node[int(t) >> 2])
            deps.append([item_of_node[int(c)] for c in (v.child0[node], v.child1[node]) if c >= 0 and arity[v.node_type[c]] > 0])
        for workers in (1, 3, 256):
            ready = np.zeros(v.n_compute_nodes, np.int64)            # published halves per item
            free_at = [(0.0, i) for i in range(workers)]             # (time a worker becomes free, id)
            heapq.heapify(free_at)
            publish = []                                             # (time, item, amount), applied in time order
            next_ticket, now, done = 0, 0.0, 0
            while next_ticket < v.n_tickets:
                now, wid = heapq.heappop(free_at)
                while publish and publish[0][0] <= now:
                    _, it, amt = heapq.heappop(publish)
                    ready[it] += amt
                tk = next_ticket
                next_ticket += 1
                start = now
                for dpd in deps[tk]:
                    while ready[dpd] < 2:                            # the wait: advance time to the next publication
                        assert publish, (name, workers, "deadlock at ticket", tk)
                        tpub, it, amt = heapq.heappop(publish)
                        ready[it] += amt
                        start = max(start, tpub)
                end = start + float(g.uniform(0.5, 2.0))
                heapq.heappush(publish, (end, int(v.tickets[tk]) >> 2, 2 if int(v.tickets[tk]) & 3 == 0 else 1))
                heapq.heappush(free_at, (end, wid))
                done += 1
            assert done == v.n_tickets


def test_backward_tables_of_a_keep_plan(dyn):
    """DYNB_PLAN_KEEP: gradient routes, per-function item lists and the work units of the parameter-gradient kernel."""
    w = iep.config2()
    v = dyn.dynbatch_plan_view(dyn.dynbatch_plan(w.prog, w.prog_off, w.arity, dyn.DYNB_PLAN_BALANCE | dyn.DYNB_PLAN_KEEP))
    n_items, arity = v.n_compute_nodes, w.arity
    item_of = np.full(v.n_nodes, -1)
    item_of[v.item_node] = np.arange(n_items)
    assert v.n_slots == n_items - (item_of[v.root] >= 0).sum()           # every result but the roots (they go to `out`) keeps a slot of its own
    # routes: an argument that is a module goes to the item that evaluates it; SCENE leaves are numbered in node order
    leaf_no = np.cumsum(arity[v.node_type] == 0) - 1
    for dst, child in ((v.grad_dst0, v.child0), (v.grad_dst1, v.child1)):
        c = child[v.item_node]
        has = c >= 0
        is_leaf = has & (arity[v.node_type[np.maximum(c, 0)]] == 0)
        assert (dst[has & ~is_leaf] == item_of[c[has & ~is_leaf]]).all()
        assert (dst[is_leaf] == -1 - leaf_no[c[is_leaf]]).all()
    # every module result but the roots is routed to exactly once (a tree: one consumer per node)
    routed = np.concatenate([v.grad_dst0[v.grad_dst0 >= 0], v.grad_dst1[(v.grad_dst1 >= 0) & (arity[v.node_type[v.item_node]] == 2)]])
    assert len(np.unique(routed)) == len(routed) == n_items - (item_of[v.root] >= 0).sum()
    # items of a function, ascending
    types = v.node_type[v.item_node]
    for t in range(v.n_types):
        mine = v.fn_items[v.fn_first[t]:v.fn_first[t + 1]]
        assert (mine == np.flatnonzero(types == t)).all()
    # work units: per (mode, function, part) the chunks tile the function's item list, at most 16 items each
    assert sorted(v.wg_order) == list(range(v.n_wg_units))
    cover = {}
    for mode, t, part, b, e in v.wg_units[:, :5]:
        assert 0 < e - b <= 16 and v.fn_first[t] <= b and e <= v.fn_first[t + 1]
        assert arity[t] == 2 if mode == 2 else arity[t] >= 1
        assert 0 <= part < (2 if mode == 2 else 3)
        cover.setdefault((mode, t, part), []).append((b, e))
    for t in range(v.n_types):
        for mode in range(3):
            wanted = arity[t] >= 1 and (mode != 2 or arity[t] == 2) and v.fn_first[t + 1] > v.fn_first[t]
            for part in range(2 if mode == 2 else 3):
                chunks = cover.get((mode, t, part), [])
                assert bool(chunks) == bool(wanted)
                if chunks:
                    assert chunks[0][0] == v.fn_first[t] and chunks[-1][1] == v.fn_first[t + 1]
                    assert all(a[1] == b[0] for a, b in zip(chunks, chunks[1:]))
    # the parts of one chunk are taken by workgroups 8 apart (they run on one die at the same time)
    pos = np.empty(v.n_wg_units, np.int64)
    pos[v.wg_order] = np.arange(v.n_wg_units)
    key = {tuple(u[[0, 1, 3]]): {} for u in v.wg_units}
    for i, u in enumerate(v.wg_units):
        key[tuple(u[[0, 1, 3]])][u[2]] = pos[i]
    apart = [p[1] - p[0] for p in key.values()]
    assert np.mean(np.array(apart) == 8) > 0.95
    # without the flag there are no such tables
    v0 = dyn.dynbatch_plan_view(dyn.dynbatch_plan(w.prog, w.prog_off, w.arity, dyn.DYNB_PLAN_BALANCE))
    assert v0.n_wg_units == 0 and len(v0.fn_items) == 0 and len(v0.grad_dst0) == 0
