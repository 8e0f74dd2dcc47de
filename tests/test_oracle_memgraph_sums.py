"""The oracle's own BuildMemgraph with sum vertices (Appendix A, resources: a reduction as
increments into a write-locked output): uniform slots, random graphs in which some vertices are
sums, every slot count from roomy down to the smallest that compiles.  Each result must pass the
three structural requirements of Section 6 and run correctly on the address-level memory model in
every order (all orders for tiny graphs, sampled ones otherwise); planted mistakes must be caught;
the library compiling the same graphs must agree on what is unique (number of increments, clears
and joins) and pass the same checks."""
import numpy as np
import pytest

from oracle import memgraph as M
from paper_2405_16283_amd import binding as B
from workloads import random_dag

from util import check_all, oracle_memgraph, task_preds


def _graph_with_sums(seed, n, max_fanin=3):
    """A random DAG; every vertex with two or more distinct producers becomes a sum with probability 1/2."""
    preds, _, _ = random_dag(seed, n, max_fanin=max_fanin, n_inputs=2)
    rng = np.random.default_rng(1000 + seed)
    sums = [v for v in range(n) if len(set(preds[v])) >= 2 and len(set(preds[v])) == len(preds[v]) and rng.random() < 0.5]
    return preds, sums


def _smallest_slots(preds, sums, V):
    lo = None
    for slots in range(len(preds), 1, -1):
        try:
            M.build_memgraph_uniform(preds, V, slots, sums=sums)
            lo = slots
        except M.CapTooSmall:
            break
    return lo


@pytest.mark.parametrize("seed", range(12))
def test_tiny_graphs_with_sums_run_correctly_in_every_order(seed):
    n = 7
    preds, sums = _graph_with_sums(seed, n, max_fanin=3)
    V = list(range(n))
    lo = _smallest_slots(preds, sums, V)
    assert lo is not None
    for slots in sorted({n, lo + 1, lo}):
        mg = M.build_memgraph_uniform(preds, V, slots, sums=sums)
        assert [mg.kind[s] for s in sums] == ["join"] * len(sums)
        assert mg.kind.count("zero") == len(sums)
        assert mg.kind.count("increment") == sum(len(preds[s]) for s in sums)
        count, _ = check_all(preds, mg, exhaustive=len(mg) <= 11, n_random=200, seed=seed)
        assert count > 0


@pytest.mark.parametrize("seed", range(8))
def test_larger_graphs_with_sums_under_pressure(seed):
    n = 40
    preds, sums = _graph_with_sums(50 + seed, n, max_fanin=4)
    assert sums
    V = list(range(n))
    lo = _smallest_slots(preds, sums, V)
    offloads = 0
    for slots in (lo + 4, lo + 1, lo):
        mg = M.build_memgraph_uniform(preds, V, slots, sums=sums)
        offloads += mg.kind.count("offload")
        check_all(preds, mg, n_random=25, seed=seed)
    assert offloads > 0  # the small slot counts do force evictions


def test_an_open_accumulator_is_never_evicted():
    """While increments are outstanding the slot holds a partial sum: every offload of a sum's
    tensor must come after the join."""
    for seed in range(20):
        preds, sums = _graph_with_sums(200 + seed, 25, max_fanin=4)
        V = list(range(25))
        lo = _smallest_slots(preds, sums, V)
        mg = M.build_memgraph_uniform(preds, V, lo, sums=sums)
        at = {m: i for i, m in enumerate(mg.order)}
        for m in range(len(mg)):
            if mg.kind[m] == "offload" and mg.src[m] in sums:
                assert mg.kind[mg.operands[m][0]] in ("join", "reload") and at[m] > at[mg.src[m]]


def test_planted_mistakes_in_a_sum_are_caught():
    preds = [[], [], [], [0], [1], [2], [3, 4, 5], [6, 0]]
    V = list(range(8))
    mg = M.build_memgraph_uniform(preds, V, 8, sums=[6])  # roomy: no memory dependency stands in for the edge taken out
    check_all(preds, mg, n_random=50)
    z = mg.kind.index("zero")
    incs = [m for m in range(len(mg)) if mg.kind[m] == "increment"]
    expected = M.taskgraph_values(preds, V)

    def broken(edges):
        bad = M.MemGraph(n_task=mg.n_task, cap=mg.cap)
        bad.kind, bad.src, bad.loc, bad.operands, bad.order = mg.kind, mg.src, mg.loc, mg.operands, mg.order
        bad.edges = edges
        return bad

    # an increment that may run before the output is cleared
    bad = broken([e for e in mg.edges if (e[0], e[1]) != (z, incs[1])])
    with pytest.raises(M.MemgraphError):
        M.check_data_deps(preds, bad)
    caught = 0
    for i in range(200):
        order = M.random_topological_order(bad, np.random.default_rng(i))
        try:
            r = M.simulate(bad, order, preds, expected)
            caught += r["results"] != M.simulate(mg, mg.order, preds, expected)["results"]
        except M.MemgraphError:
            caught += 1
    assert caught > 0
    # a join that does not wait for one of its increments
    bad = broken([e for e in mg.edges if (e[0], e[1]) != (incs[2], 6)])
    with pytest.raises(M.MemgraphError):
        M.check_data_deps(preds, bad)


@pytest.mark.parametrize("seed", range(6))
def test_the_library_agrees_on_what_is_unique(seed):
    """Same graph, one allocation unit per tensor, the same serial order: the library's memgraph has
    the same number of clears, increments and joins, and passes the same checks at the oracle's
    smallest slot count plus the room the library's own reading needs (it never revokes below the
    operands of the vertex about to run)."""
    n = 24
    preds, sums = _graph_with_sums(400 + seed, n, max_fanin=3)
    V = list(range(n))
    # what the library's vertex kinds can express: a sum of all its operands, or an add of two
    lib_preds = [list(preds[v]) if v in sums else sorted(set(preds[v][:2])) for v in range(n)]
    lo = _smallest_slots(lib_preds, sums, V)
    tg = B.tn_taskgraph_create()
    try:
        for v in range(n):
            if not preds[v]:
                B.tn_taskgraph_add_input(tg, B.TN_F32, 8, 8, B.TN_HOST)
            elif v in sums:
                B.tn_taskgraph_add_op(tg, B.TN_OP_SUM, B.tn_op_params(), preds[v], B.TN_F32, 8, 8)
            else:
                B.tn_taskgraph_add_op(tg, B.TN_OP_ADD, B.tn_op_params(), (lib_preds[v] * 2)[:2], B.TN_F32, 8, 8)
        consumed = {u for ps in lib_preds for u in ps}
        for v in range(n):
            if v not in consumed:
                B.tn_taskgraph_mark_output(tg, v)
        want = M.build_memgraph_uniform(lib_preds, V, lo + 2, sums=sums)
        mg = B.tn_compile(tg, V, (lo + 2) * 256, B.tn_compile_opts(max_lookahead_bytes=B.UINT64_MAX, drop_clean_inputs=0))
        try:
            got = oracle_memgraph(mg)
            for kind in ("zero", "increment", "join"):
                assert got.kind.count(kind) == want.kind.count(kind)
            check_all(task_preds(tg), got, n_random=25, seed=seed)
        finally:
            B.tn_memgraph_destroy(mg)
    finally:
        B.tn_taskgraph_destroy(tg)
