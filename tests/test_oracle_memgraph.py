"""Pins for the oracle's memgraph builder, checkers and simulator (CPU only).

The pins are the relations Section 4 states for its worked examples (tests/golden), the three
correctness requirements of Section 6 checked two independent ways (structurally and by running
every dependency-respecting order on an address-level memory model), degenerate memory sizes,
and planted mistakes that each check must catch.
"""
import os

import numpy as np
import pytest

from oracle import memgraph as M
from workloads import random_dag

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _parse_example(fname):
    names, preds, facts, slots = [], {}, [], None
    mode = None
    for line in open(os.path.join(GOLDEN, fname)):
        line = line.split("#")[0].strip()
        if not line:
            continue
        if line == "vertices":
            mode = "v"
            continue
        tok = line.split()
        if mode == "v" and tok[0].endswith(":"):
            names.append(tok[0][:-1])
            preds[tok[0][:-1]] = tok[1:]
        else:
            mode = None
            if tok[0] == "slots":
                slots = int(tok[1])
            else:
                facts.append(tok)
    idx = {n: i for i, n in enumerate(names)}
    return names, [[idx[p] for p in preds[n]] for n in names], slots, facts


def _resolve(mg, names, token):
    """Golden-file vertex name -> memgraph vertex id ("offload_A" = the offload of tensor A)."""
    idx = {n: i for i, n in enumerate(names)}
    for kind in ("offload", "reload"):
        if token.startswith(kind + "_"):
            t = idx[token[len(kind) + 1:]]
            (v,) = [v for v in range(len(mg)) if mg.kind[v] == kind and mg.src[v] == t]
            return v
    return idx[token]


def _full_check(preds, mg, V, exhaustive=True, n_random=0, seed=0):
    M.check_forward_edges(mg)
    M.check_data_deps(preds, mg)
    M.check_race_free(mg)
    expected = M.taskgraph_values(preds, V)
    ref = M.simulate(mg, mg.order, preds, expected)
    assert ref["hw_live"] <= mg.cap
    orders = M.all_topological_orders(mg) if exhaustive else (
        M.random_topological_order(mg, np.random.default_rng(seed + i)) for i in range(n_random))
    count = 0
    for order in orders:
        r = M.simulate(mg, order, preds, expected)
        assert r["hw_live"] <= mg.cap
        assert r["results"] == ref["results"]
        count += 1
    return count


@pytest.mark.parametrize("fname", ["section4_five_slots.txt", "section4_four_slots.txt"])
def test_section4_worked_examples(fname):
    names, preds, slots, facts = _parse_example(fname)
    V = list(range(len(names)))
    mg = M.build_memgraph_uniform(preds, V, slots)
    eset = set(mg.edges)
    for tok in facts:
        if tok[0] == "share":
            a, b = (_resolve(mg, names, t) for t in tok[1:3])
            assert mg.loc[a] == mg.loc[b]
        elif tok[0] in ("mem", "data"):
            a, b = (_resolve(mg, names, t) for t in tok[1:3])
            assert (a, b, tok[0]) in eset, tok
        elif tok[0] == "chain":
            ids = [_resolve(mg, names, t) for t in tok[1:]]
            for a, b in zip(ids, ids[1:]):
                assert (a, b, "data") in eset
    assert _full_check(preds, mg, V) >= 1


def _parse_figure1():
    mg_names, facts = [], []
    mg = M.MemGraph(n_task=6, cap=0)
    for line in open(os.path.join(GOLDEN, "figure1_memgraph.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        tok = line.split()
        if tok[0] == "vertex":
            _, name, kind, tensor, loc, ops = tok
            mg_names.append(name)
            facts.append((kind, int(tensor), None if loc == "-" else (int(loc), 1), [] if ops == "-" else ops.split(",")))
        elif tok[0] == "cap":
            mg.cap = int(tok[1])
        else:
            facts.append(tok)
    return mg, mg_names, facts


def test_figure1_either_kernel_may_go_first():
    """Section 2: after 1 and 2 have run, 4 waits only for offload_1 and 5 only for reload_3."""
    mg, names, facts = _parse_figure1()
    idx = {n: i for i, n in enumerate(names)}
    # tensors are numbered by first appearance so that taskgraph ids are dense
    tensor_ids = {}
    unordered = None
    for f in facts:
        if isinstance(f, tuple):
            kind, tensor, loc, ops = f
            t = tensor_ids.setdefault(tensor, len(tensor_ids))
            mg.add_vertex(kind, t, loc, [idx[o] for o in ops])
        elif f[0] == "edge":
            mg.edges.append((idx[f[1]], idx[f[2]], f[3]))
        elif f[0] == "unordered":
            unordered = (idx[f[1]], idx[f[2]])
    mg.order = list(range(len(mg)))
    M.check_forward_edges(mg)
    M.check_race_free(mg)
    desc = M._reach_bitsets(mg)
    a, b = unordered
    assert not (desc[a] >> b) & 1 and not (desc[b] >> a) & 1
    firsts = set()
    for order in M.all_topological_orders(mg):
        firsts.add(min((a, b), key=order.index))
    assert firsts == {a, b}
    # without the memory dependency offload_1 -> 4 the graph has a race, and the checker says so
    mg.edges.remove((idx["off1"], idx["4"], "mem"))
    with pytest.raises(M.MemgraphError):
        M.check_race_free(mg)


@pytest.mark.parametrize("seed", range(40))
def test_all_orders_on_tiny_random_graphs(seed):
    rng = np.random.default_rng(1000 + seed)
    n = int(rng.integers(4, 8))
    preds, _, _ = random_dag(seed, n, max_fanin=2, n_inputs=int(rng.integers(1, 3)))
    V = list(range(n))
    min_slots = max(len(set(p)) + 1 for p in preds)
    slots = min_slots + int(rng.integers(0, 2))
    mg = M.build_memgraph_uniform(preds, V, slots)
    if len(mg) > 11:
        pytest.skip("too many orders to enumerate")
    assert _full_check(preds, mg, V) >= 1


@pytest.mark.parametrize("seed", range(30))
def test_random_orders_on_larger_graphs(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(20, 80))
    preds, _, _ = random_dag(seed, n, max_fanin=4, n_inputs=3)
    V = list(range(n))
    min_slots = max(len(set(p)) + 1 for p in preds)
    mg = M.build_memgraph_uniform(preds, V, min_slots + int(rng.integers(0, 3)))
    assert any(k == "offload" for k in mg.kind) or n < 30
    _full_check(preds, mg, V, exhaustive=False, n_random=25, seed=seed)


def test_degenerate_memory_sizes():
    preds, _, _ = random_dag(7, 30, max_fanin=3, n_inputs=2)
    V = list(range(30))
    # plenty of memory: nothing is offloaded, nothing shares a slot, and the memgraph's edges
    # are exactly the taskgraph's
    mg = M.build_memgraph_uniform(preds, V, 30)
    assert all(k in ("load", "op") for k in mg.kind)
    assert sorted((a, b) for a, b, _ in mg.edges) == sorted({(u, v) for v in V for u in preds[v]})
    assert all(k == "data" for _, _, k in mg.edges)
    # the exact minimum still compiles; one slot fewer cannot hold some vertex's operands
    min_slots = max(len(set(p)) + 1 for p in preds)
    mg = M.build_memgraph_uniform(preds, V, min_slots)
    _full_check(preds, mg, V, exhaustive=False, n_random=20)
    with pytest.raises(M.CapTooSmall):
        M.build_memgraph_uniform(preds, V, min_slots - 1)


def test_chain_of_two_with_one_slot_too_few_is_rejected_and_with_two_is_plain():
    preds = [[], [0]]
    mg = M.build_memgraph_uniform(preds, [0, 1], 2)
    assert mg.edges == [(0, 1, "data")]
    with pytest.raises(M.CapTooSmall):
        M.build_memgraph_uniform(preds, [0, 1], 1)


def _copy(mg, edges=None):
    return M.MemGraph(mg.n_task, mg.cap, list(mg.kind), list(mg.src), list(mg.loc),
                      [list(o) for o in mg.operands], list(mg.edges if edges is None else edges),
                      list(mg.order))


def test_planted_mistakes_are_caught_both_ways():
    """Dropping a single memory dependency either leaves the graph correct (the edge was implied
    by others) or creates a race.  The structural race check and the brute-force run of every
    order must agree on which, edge by edge: the two detection methods pin each other."""
    flagged = kept = 0
    for seed in range(60):
        n = 6
        preds, _, _ = random_dag(300 + seed, n, max_fanin=2, n_inputs=2)
        V = list(range(n))
        mg = M.build_memgraph_uniform(preds, V, max(len(set(p)) + 1 for p in preds))
        if len(mg) > 10:
            continue
        expected = M.taskgraph_values(preds, V)
        for e in [e for e in mg.edges if e[2] == "mem"]:
            broken = _copy(mg, [x for x in mg.edges if x != e])
            try:
                M.check_race_free(broken)
                structural_ok = True
            except M.MemgraphError:
                structural_ok = False
            dynamic_ok = True
            for order in M.all_topological_orders(broken):
                try:
                    M.simulate(broken, order, preds, expected)
                except M.MemgraphError:
                    dynamic_ok = False
                    break
            assert structural_ok == dynamic_ok, (seed, e, structural_ok, dynamic_ok)
            flagged += (not structural_ok)
            kept += structural_ok
    assert flagged >= 20, (flagged, kept)


def test_backward_edge_and_misplaced_vertex_are_caught():
    preds, _, _ = random_dag(11, 20, max_fanin=3, n_inputs=2)
    V = list(range(20))
    mg = M.build_memgraph_uniform(preds, V, max(len(set(p)) + 1 for p in preds))
    a, b = mg.order[3], mg.order[12]
    with pytest.raises(M.MemgraphError):
        M.check_forward_edges(_copy(mg, mg.edges + [(b, a, "mem")]))
    moved = _copy(mg)
    v = next(v for v in range(len(mg)) if mg.loc[v] is not None)
    moved.loc[v] = (mg.cap, 1)
    with pytest.raises(M.MemgraphError):
        M.check_race_free(moved)


def test_data_dependency_checker_catches_a_dropped_and_a_rewired_edge():
    preds, _, _ = random_dag(5, 25, max_fanin=3, n_inputs=2)
    V = list(range(25))
    mg = M.build_memgraph_uniform(preds, V, max(len(set(p)) + 1 for p in preds))
    M.check_data_deps(preds, mg)
    data_edges = [e for e in mg.edges if e[2] == "data"]
    e = data_edges[len(data_edges) // 2]
    mg.edges.remove(e)
    with pytest.raises(M.MemgraphError):
        M.check_data_deps(preds, mg)
    mg.edges.append(e)
    v = next(v for v in range(25) if len(preds[v]) >= 1 and mg.operands[v])
    wrong = next(u for u in range(25) if u not in preds[v] and u != v)
    mg.operands[v][0] = wrong
    with pytest.raises(M.MemgraphError):
        M.check_data_deps(preds, mg)
