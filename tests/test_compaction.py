"""BuildMemgraph's answer to fragmentation (not in the paper, which presents uniform slots,
Section 6): when pinned tensors scattered over memory leave no hole although the bytes suffice,
memory is emptied and the vertex at hand is placed compactly.  Each of the three places that can
get there -- the allocation of a vertex's own output, the reload of an evicted operand, and the
allocation of a sum's output when its first operand arrives -- is forced by a hand-laid memory
layout and judged by the oracle's checkers and by runs of many orders on the memory model."""
import numpy as np
import pytest

from oracle import memgraph as M
from paper_2405_16283_amd import binding as B

from util import check_all, oracle_memgraph, task_preds

F = B.TN_F32
KB = 1024


def _inp(tg, rows, cols):
    return B.tn_taskgraph_add_input(tg, F, rows, cols, B.TN_HOST)


def _op(tg, kind, ins, rows, cols, **params):
    p = B.tn_op_params()
    for k, v in params.items():
        setattr(p, k, v)
    return B.tn_taskgraph_add_op(tg, kind, p, ins, F, rows, cols)


def _compile_and_check(tg, order, cap, outputs, n_random=200):
    for v in outputs:
        B.tn_taskgraph_mark_output(tg, v)
    mg = B.tn_compile(tg, order, cap, B.tn_compile_opts(max_lookahead_bytes=0, drop_clean_inputs=1))
    try:
        st = B.tn_memgraph_stats(mg)
        omg = oracle_memgraph(mg)
        assert all(o >= 0 for ops in omg.operands for o in ops), "an operand names no vertex"
        check_all(task_preds(tg), omg, n_random=n_random, seed=5)
        B.tn_memgraph_simulate(mg)
        rng = np.random.default_rng(11)
        for _ in range(20):
            B.tn_memgraph_simulate(mg, M.random_topological_order(omg, rng))
        assert st.high_water <= cap
        return st, omg
    finally:
        B.tn_memgraph_destroy(mg)


def test_compaction_when_a_vertex_output_finds_no_hole():
    """[a 256K][p 128K][b 256K][q 128K][stat 1K]: once p and q are dead, a + b needs 256 KiB and finds
    two holes of 128 and 129 KiB between its own operands, which cannot be evicted."""
    tg = B.tn_taskgraph_create()
    try:
        a, p, b, q = _inp(tg, 256, 256), _inp(tg, 256, 128), _inp(tg, 256, 256), _inp(tg, 256, 128)
        z = _op(tg, B.TN_OP_RMS_STAT, [p, q], 256, 1, d=256, eps=1e-6)
        v = _op(tg, B.TN_OP_ADD, [a, b], 256, 256)
        st, omg = _compile_and_check(tg, [a, p, b, q, z, v], 2 * 256 * KB + 2 * 128 * KB + KB, [z, v])
        assert st.n_compactions == 1
        # a and b were dropped and loaded a second time, next to the output
        assert st.n_drop == 2 and st.n_load == 6
    finally:
        B.tn_taskgraph_destroy(tg)


def test_compaction_while_an_evicted_operand_comes_back():
    """Six tensors, 768 KiB: when a + b is about to run, b is out, and the room for it exists only
    as two separate 128 KiB holes between a and the output; the compaction happens inside the loop
    that reloads operands and pushes a out, which that loop then brings back as well."""
    tg = B.tn_taskgraph_create()
    try:
        p, b, q, a, c = (_inp(tg, 256, 128), _inp(tg, 256, 256), _inp(tg, 256, 128), _inp(tg, 256, 256),
                         _inp(tg, 256, 256))
        v = _op(tg, B.TN_OP_ADD, [a, b], 256, 256)
        z1 = _op(tg, B.TN_OP_ADD, [p, q], 256, 128)
        z2 = _op(tg, B.TN_OP_TRANSPOSE, [c], 256, 256)
        st, omg = _compile_and_check(tg, [p, b, q, a, c, v, z1, z2], 768 * KB, [v, z1, z2])
        assert st.n_compactions == 1
        # b was out before the step began; a was resident, pushed out by the compaction and brought back by
        # the same loop: the vertex reads second loads of both
        ops = omg.operands[v]
        assert sorted(omg.src[o] for o in ops) == sorted([a, b]) and all(o >= omg.n_task for o in ops)
    finally:
        B.tn_taskgraph_destroy(tg)


def test_compaction_when_a_sum_output_is_placed_brings_the_operand_back():
    """The first operand u of a sum arrives while the only room for the sum's output is in pieces:
    emptying the memory pushes u out too, and the increment must read a reload of u, not nothing."""
    tg = B.tn_taskgraph_create()
    try:
        a, p, q, b = (_inp(tg, 128, 128) for _ in range(4))
        stat = _op(tg, B.TN_OP_RMS_STAT, [p, q], 128, 1, d=256, eps=1e-6)
        u, u2 = _inp(tg, 128, 256), _inp(tg, 128, 256)
        s = _op(tg, B.TN_OP_SUM, [u, u2], 128, 256)
        c = _op(tg, B.TN_OP_ADD, [a, b], 128, 128)
        cap = 2 * 128 * 256 * 4 + 512
        st, omg = _compile_and_check(tg, [a, p, q, b, stat, u, u2, s, c], cap, [stat, s, c])
        assert st.n_compactions == 1 and st.n_increment == 2
        incs = [m for m in range(len(omg)) if omg.kind[m] == "increment"]
        first = min(incs, key=omg.order.index)
        # the first increment reads the second load of u (u itself was pushed out by the compaction)
        assert omg.kind[omg.operands[first][0]] == "load" and omg.operands[first][0] >= omg.n_task
        assert omg.src[omg.operands[first][0]] == u
    finally:
        B.tn_taskgraph_destroy(tg)


def test_sum_whose_operand_and_output_do_not_fit_together_is_an_error_not_a_crash():
    tg = B.tn_taskgraph_create()
    try:
        a, p, q, b = (_inp(tg, 128, 128) for _ in range(4))
        stat = _op(tg, B.TN_OP_RMS_STAT, [p, q], 128, 1, d=256, eps=1e-6)
        u, u2 = _inp(tg, 128, 256), _inp(tg, 128, 256)
        s = _op(tg, B.TN_OP_SUM, [u, u2], 128, 256)
        c = _op(tg, B.TN_OP_ADD, [a, b], 128, 128)
        for v in (stat, s, c):
            B.tn_taskgraph_mark_output(tg, v)
        with pytest.raises(B.TurnipError) as e:
            B.tn_compile(tg, [a, p, q, b, stat, u, u2, s, c], 2 * 128 * 256 * 4 - 256,
                         B.tn_compile_opts(max_lookahead_bytes=0, drop_clean_inputs=1))
        assert e.value.status == B.TN_ERR_CAP_TOO_SMALL
    finally:
        B.tn_taskgraph_destroy(tg)


@pytest.mark.parametrize("seed", range(30))
def test_random_graphs_with_sums_at_tight_caps(seed):
    """Random mixes of elementwise vertices and sums over tensors of three sizes, compiled at the
    smallest cap that works: whatever path the compiler takes, the memgraph must be sound."""
    rng = np.random.default_rng(1000 + seed)
    tg = B.tn_taskgraph_create()
    try:
        shapes = [(128, 128), (128, 256), (256, 256)]
        by_shape = {s: [] for s in shapes}
        sizes = {}
        n_in = int(rng.integers(4, 8))
        for _ in range(n_in):
            s = shapes[int(rng.integers(0, 3))]
            v = _inp(tg, *s)
            by_shape[s].append(v)
            sizes[v] = s[0] * s[1] * 4
        for s in shapes:  # at least two tensors of every shape
            while len(by_shape[s]) < 2:
                v = _inp(tg, *s)
                by_shape[s].append(v)
                sizes[v] = s[0] * s[1] * 4
        preds = {}
        for _ in range(int(rng.integers(8, 30))):
            s = shapes[int(rng.integers(0, 3))]
            pool = by_shape[s]
            if rng.random() < 0.4 and len(pool) >= 3:
                k = int(rng.integers(2, min(4, len(pool)) + 1))
                ins = [int(x) for x in rng.choice(pool, size=k, replace=False)]
                v = _op(tg, B.TN_OP_SUM, ins, *s)
            else:
                ins = [int(x) for x in rng.choice(pool, size=2, replace=False)]
                v = _op(tg, B.TN_OP_ADD, ins, *s)
            preds[v] = ins
            pool.append(v)
            sizes[v] = s[0] * s[1] * 4
        n = B.tn_taskgraph_num_vertices(tg)
        consumed = {u for ins in preds.values() for u in ins}
        for v in range(n):
            if v not in consumed:
                B.tn_taskgraph_mark_output(tg, v)
        opts = B.tn_compile_opts(max_lookahead_bytes=0 if seed % 2 else B.UINT64_MAX, drop_clean_inputs=seed % 3 != 0,
                                 next_fit=seed % 4 == 1)
        # smallest cap, found by trying: start at the largest footprint of one vertex
        cap = max(sum(sizes[u] for u in set(ins)) + sizes[v] for v, ins in preds.items())
        mg = None
        for _ in range(40):
            try:
                mg = B.tn_compile(tg, None, cap, opts)
                break
            except B.TurnipError as e:
                assert e.status == B.TN_ERR_CAP_TOO_SMALL
                cap += 64 * KB
        assert mg is not None
        try:
            omg = oracle_memgraph(mg)
            assert all(o >= 0 for ops in omg.operands for o in ops)
            check_all(task_preds(tg), omg, n_random=25, seed=seed)
            B.tn_memgraph_simulate(mg)
        finally:
            B.tn_memgraph_destroy(mg)
    finally:
        B.tn_taskgraph_destroy(tg)
