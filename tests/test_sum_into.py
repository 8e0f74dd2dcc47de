"""Sum vertices: a reduction run as increments into a write-locked output (Appendix A, resources),
and the k-split form of the projections built on it.  CPU tests: the oracle's definition against
plain sums and error bounds, the library's tiler against the oracle's, and the compiled memgraphs
(clear, increments in any order, join) against the oracle's checkers and address-level simulator."""
import itertools

import numpy as np
import pytest

from oracle import llama_ref as R
from oracle import memgraph as M
from oracle import tiled as T
from paper_2405_16283_amd import binding as B
from paper_2405_16283_amd import harness as H
from workloads import config, make_llama_inputs

from util import check_all, oracle_memgraph, oracle_taskgraph, task_preds


# ---------------------------------------------------------------------------------------------
# the oracle's sum vertex
# ---------------------------------------------------------------------------------------------

def _sum_graph(n, shape, dtype):
    tg = T.TaskGraph()
    ins = [tg.add("input", [], shape, dtype) for _ in range(n)]
    s = tg.add("sum", ins, shape, dtype)
    tg.outputs.append(s)
    return tg, ins, s


def test_sum_of_exactly_representable_values_is_the_plain_sum_in_every_order():
    rng = np.random.default_rng(0)
    tg, ins, s = _sum_graph(4, (5, 7), "bf16")
    vals = {v: rng.integers(-8, 9, size=(5, 7)).astype(np.float64) for v in ins}  # small integers: no rounding
    want = sum(vals.values())
    for perm in itertools.permutations(range(4)):
        got = T.evaluate(tg, vals, increment_order=lambda v, n: perm)[s]
        np.testing.assert_array_equal(got, want)


def test_sum_depends_on_the_order_by_rounding_only():
    rng = np.random.default_rng(1)
    tg, ins, s = _sum_graph(5, (64, 64), "bf16")
    vals = {v: T.round_bf16(rng.standard_normal((64, 64)) * 10.0 ** rng.integers(-1, 2)) for v in ins}
    exact = sum(vals.values())
    # each of the n increments rounds a partial sum no larger than sum |p_i| to 8 significant bits:
    # half a unit in the last place is at most 2**-8 of the value
    bound = 5 * 2.0 ** -8 * sum(np.abs(a) for a in vals.values())
    results = []
    for perm in itertools.permutations(range(5)):
        got = T.evaluate(tg, vals, increment_order=lambda v, n: perm)[s]
        assert np.all(np.abs(got - exact) <= bound)
        np.testing.assert_array_equal(got, T.round_bf16(got))  # the output is a bf16 tensor
        results.append(got)
    assert any(not np.array_equal(results[0], r) for r in results[1:])
    # the default is ascending operand order
    np.testing.assert_array_equal(T.evaluate(tg, vals)[s], results[0])
    with pytest.raises(AssertionError):
        T.evaluate(tg, vals, increment_order=lambda v, n: [0] * n)


@pytest.mark.parametrize("name,k_split,tol", [("c1", 2, 1e-5), ("c1", 3, 1e-5), ("ragged_f32", 3, 1e-5),
                                              ("ragged_bf16", 2, 2e-2)])
def test_k_split_forward_equals_the_untiled_model(name, k_split, tol):
    cfg = config(name)
    w = R.widen(cfg, make_llama_inputs(cfg, 0))
    tg = T.build_llama_taskgraph(cfg, k_split=k_split)
    assert "sum" in tg.kind
    y_exact = R.forward(cfg, w)
    y = T.assemble_outputs(tg, T.evaluate(tg, T.cut_inputs(tg, w)), cfg.tokens, cfg.d_model)
    assert R.rel_err(y, y_exact) < tol
    rev = T.assemble_outputs(tg, T.evaluate(tg, T.cut_inputs(tg, w), increment_order=lambda v, n: range(n - 1, -1, -1)),
                             cfg.tokens, cfg.d_model)
    assert R.rel_err(rev, y_exact) < tol


# ---------------------------------------------------------------------------------------------
# the library's taskgraph
# ---------------------------------------------------------------------------------------------

def test_add_op_validates_sums():
    tg = B.tn_taskgraph_create()
    try:
        a = B.tn_taskgraph_add_input(tg, B.TN_F32, 4, 4, B.TN_HOST)
        b = B.tn_taskgraph_add_input(tg, B.TN_F32, 4, 4, B.TN_HOST)
        c = B.tn_taskgraph_add_input(tg, B.TN_F32, 4, 5, B.TN_HOST)
        h = B.tn_taskgraph_add_input(tg, B.TN_BF16, 4, 4, B.TN_HOST)
        p = B.tn_op_params()
        s = B.tn_taskgraph_add_op(tg, B.TN_OP_SUM, p, [a, b], B.TN_F32, 4, 4)
        assert B.tn_taskgraph_vertex(tg, s).kind == B.TN_OP_SUM
        B.tn_taskgraph_add_op(tg, B.TN_OP_SUM, p, [a], B.TN_F32, 4, 4)  # a sum of one tensor is allowed
        for bad in ([a, c], [a, h], [a, a]):
            with pytest.raises(B.TurnipError):
                B.tn_taskgraph_add_op(tg, B.TN_OP_SUM, p, bad, B.TN_F32, 4, 4)
        for memgraph_only in (B.TN_OP_ZERO, B.TN_OP_SUM_INTO):
            with pytest.raises(B.TurnipError, match="memgraphs only"):
                B.tn_taskgraph_add_op(tg, memgraph_only, p, [a, b], B.TN_F32, 4, 4)
    finally:
        B.tn_taskgraph_destroy(tg)


@pytest.mark.parametrize("name,k_split", [("c1", 2), ("ragged_bf16", 3)])
def test_library_k_split_taskgraph_equals_the_oracles(name, k_split):
    cfg = config(name)
    w = R.widen(cfg, make_llama_inputs(cfg, 0))
    tg = B.tn_build_llama(H.llama_config_struct(cfg, weights_transposed=False, v_transposed=False, k_split=k_split))
    try:
        otg = oracle_taskgraph(tg)
        mine = T.build_llama_taskgraph(cfg, k_split=k_split)
        assert otg.kind.count("sum") == mine.kind.count("sum") > 0
        assert otg.kind.count("gemm") == mine.kind.count("gemm")
        y_lib = T.assemble_outputs(otg, T.evaluate(otg, T.cut_inputs(otg, w)), cfg.tokens, cfg.d_model)
        y_own = T.assemble_outputs(mine, T.evaluate(mine, T.cut_inputs(mine, w)), cfg.tokens, cfg.d_model)
        np.testing.assert_array_equal(y_lib, y_own)
    finally:
        B.tn_taskgraph_destroy(tg)


# ---------------------------------------------------------------------------------------------
# compiled memgraphs
# ---------------------------------------------------------------------------------------------

def _chain_with_a_sum(n_parts, residency=B.TN_HOST):
    """x -> n_parts products p_i = x @ w_i -> sum -> + x: every operand of the sum is an op result."""
    tg = B.tn_taskgraph_create()
    x = B.tn_taskgraph_add_input(tg, B.TN_F32, 8, 8, residency)
    parts = []
    for _ in range(n_parts):
        w = B.tn_taskgraph_add_input(tg, B.TN_F32, 8, 8, residency)
        parts.append(B.tn_taskgraph_add_op(tg, B.TN_OP_GEMM, B.tn_op_params(nk=1), [x, w], B.TN_F32, 8, 8))
    s = B.tn_taskgraph_add_op(tg, B.TN_OP_SUM, B.tn_op_params(), parts, B.TN_F32, 8, 8)
    y = B.tn_taskgraph_add_op(tg, B.TN_OP_ADD, B.tn_op_params(), [s, x], B.TN_F32, 8, 8)
    B.tn_taskgraph_mark_output(tg, y)
    return tg, s


@pytest.mark.parametrize("n_parts,extra_units", [(2, 0), (2, 2), (3, 1)])
def test_every_order_of_a_small_graph_with_a_sum(n_parts, extra_units):
    tg, s = _chain_with_a_sum(n_parts)
    unit = 8 * 8 * 4
    try:
        # x, one weight, one product and the sum's output must fit; little more is given
        mg = B.tn_compile(tg, None, (4 + extra_units) * unit,
                          B.tn_compile_opts(max_lookahead_bytes=B.UINT64_MAX, drop_clean_inputs=1, alignment=64))
        st = B.tn_memgraph_stats(mg)
        assert st.n_increment == n_parts
        omg = oracle_memgraph(mg)
        assert omg.kind[s] == "join" and omg.kind.count("zero") == 1 and omg.kind.count("increment") == n_parts
        B.tn_memgraph_simulate(mg)
        B.tn_memgraph_destroy(mg)
        count, _ = check_all(task_preds(tg), omg, exhaustive=len(omg) <= 14, n_random=300)
        assert count >= 2
    finally:
        B.tn_taskgraph_destroy(tg)


@pytest.mark.parametrize("name,k_split", [("c1", 2), ("c1", 3), ("ragged_bf16", 2), ("batch2_f32", 2)])
def test_k_split_memgraph_under_the_cap_is_correct_in_every_sampled_order(name, k_split):
    cfg = config(name)
    tg = B.tn_build_llama(H.llama_config_struct(cfg, k_split=k_split))
    cap = H.cap_for(cfg, tg)
    mg = B.tn_compile(tg, None, cap)
    try:
        st = B.tn_memgraph_stats(mg)
        assert st.n_increment > 0 and st.n_offload > 0 and st.high_water <= cap
        omg = oracle_memgraph(mg)
        preds = task_preds(tg)
        count, ref = check_all(preds, omg, n_random=30, seed=11)
        assert ref["hw_live"] <= cap
        B.tn_memgraph_simulate(mg)
        rng = np.random.default_rng(5)
        for _ in range(10):
            B.tn_memgraph_simulate(mg, M.random_topological_order(omg, rng))
        # an increment never waits for another increment of the same sum: the order among them is free
        inc = [v for v in range(len(omg)) if omg.kind[v] == "increment"]
        target = {v: omg.operands[v][1] for v in inc}
        for a, b, _ in omg.edges:
            assert not (a in target and b in target and target[a] == target[b])
    finally:
        B.tn_memgraph_destroy(mg)
        B.tn_taskgraph_destroy(tg)


def test_fixed_order_leaves_the_increments_free():
    cfg = config("c1")
    tg = B.tn_build_llama(H.llama_config_struct(cfg, k_split=2))
    mg = B.tn_compile(tg, None, H.cap_for(cfg, tg), B.tn_compile_opts(max_lookahead_bytes=B.UINT64_MAX,
                                                                         drop_clean_inputs=1, fix_order=1))
    try:
        omg = oracle_memgraph(mg)
        inc = {v for v in range(len(omg)) if omg.kind[v] == "increment"}
        assert inc and not any(k == "order" and (a in inc or b in inc) for a, b, k in omg.edges)
        M.check_forward_edges(omg)
    finally:
        B.tn_memgraph_destroy(mg)
        B.tn_taskgraph_destroy(tg)


def test_a_join_that_runs_before_an_increment_is_caught():
    tg, s = _chain_with_a_sum(2)
    try:
        mg = B.tn_compile(tg, None, 1 << 20)
        omg = oracle_memgraph(mg)
        B.tn_memgraph_destroy(mg)
        inc = [v for v in range(len(omg)) if omg.kind[v] == "increment"]
        # plant the mistake in the copy the oracle checks: drop the edge from one increment to the join
        broken = M.MemGraph(n_task=omg.n_task, cap=omg.cap, kind=omg.kind, src=omg.src, loc=omg.loc,
                            operands=omg.operands, edges=[e for e in omg.edges if (e[0], e[1]) != (inc[0], s)],
                            order=omg.order)
        with pytest.raises(M.MemgraphError):
            M.check_data_deps(task_preds(tg), broken)
        order = [v for v in omg.order if v != inc[0]]
        order.insert(order.index(s) + 1, inc[0])
        preds = task_preds(tg)
        expected = M.taskgraph_values(preds, [v for v in omg.order if v < omg.n_task])
        with pytest.raises(M.MemgraphError):
            M.simulate(broken, order, preds, expected)
    finally:
        B.tn_taskgraph_destroy(tg)


@pytest.mark.parametrize("opts", [
    dict(max_lookahead_bytes=0, drop_clean_inputs=1),
    dict(max_lookahead_bytes=64 * 1024, drop_clean_inputs=0),
    dict(max_lookahead_bytes=B.UINT64_MAX, drop_clean_inputs=1, next_fit=1, evict_ahead_bytes=32 * 1024),
    dict(max_lookahead_bytes=B.UINT64_MAX, drop_clean_inputs=1, prune_superfluous=1, alignment=4096),
])
def test_compile_options_keep_a_k_split_memgraph_correct(opts):
    cfg = config("c1")
    tg = B.tn_build_llama(H.llama_config_struct(cfg, k_split=3))
    cap = H.cap_for(cfg, tg)
    mg = B.tn_compile(tg, None, cap, B.tn_compile_opts(**opts))
    try:
        st = B.tn_memgraph_stats(mg)
        assert st.n_increment > 0 and st.high_water <= cap
        omg = oracle_memgraph(mg)
        check_all(task_preds(tg), omg, n_random=15, seed=2)
        B.tn_memgraph_simulate(mg)
    finally:
        B.tn_memgraph_destroy(mg)
        B.tn_taskgraph_destroy(tg)


def test_k_split_lowers_the_smallest_cap_that_compiles():
    """What the split buys: a partial product needs only its share of the K tiles next to the
    output, so the largest per-vertex footprint -- the floor of the cap -- shrinks."""
    cfg = config("c1").with_(weights_resident=False, x_resident=False)

    def smallest_cap(k_split):
        tg = B.tn_build_llama(H.llama_config_struct(cfg, k_split=k_split))
        lo, hi = 1024, 1 << 24
        try:
            while hi - lo > 1024:
                mid = (lo + hi) // 2
                try:
                    B.tn_memgraph_destroy(B.tn_compile(tg, None, mid, B.tn_compile_opts(max_lookahead_bytes=0, drop_clean_inputs=1)))
                    hi = mid
                except B.TurnipError:
                    lo = mid
        finally:
            B.tn_taskgraph_destroy(tg)
        return hi

    whole, split = smallest_cap(0), smallest_cap(4)
    assert split < 0.75 * whole, (whole, split)
