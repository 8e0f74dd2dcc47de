"""The library's taskgraph builder and BuildMemgraph, judged on the CPU by the oracle's checkers
(no GPU, no compute calls)."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import llama_ref as R
from oracle import memgraph as M
from oracle import tiled as T
from paper_2405_16283_amd import binding as B
from paper_2405_16283_amd import harness as H
from workloads import config, make_llama_inputs, random_dag

from util import check_all, oracle_memgraph, oracle_taskgraph, task_preds

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_loads_and_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "turnip.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(tn_[a-z0-9_]+)\s*\(", header))
    assert len(declared) >= 25
    lib = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), f"{name} is declared in turnip.h but not exported"
    assert declared == set(B.SIGNATURES), declared ^ set(B.SIGNATURES)


# ---------------------------------------------------------------------------------------------
# the LLaMA tiler
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("name", ["c1", "ragged_f32", "ragged_bf16", "batch2_f32"])
def test_library_taskgraph_evaluated_by_the_oracle_equals_the_untiled_model(name):
    cfg = config(name)
    tg = B.tn_build_llama(H.llama_config_struct(cfg))
    try:
        otg = oracle_taskgraph(tg)
    finally:
        B.tn_taskgraph_destroy(tg)
    w = R.widen(cfg, make_llama_inputs(cfg, 0))
    y_lib = T.assemble_outputs(otg, T.evaluate(otg, T.cut_inputs(otg, w)), cfg.tokens, cfg.d_model)
    own = T.build_llama_taskgraph(cfg)
    y_own = T.assemble_outputs(own, T.evaluate(own, T.cut_inputs(own, w)), cfg.tokens, cfg.d_model)
    # same decomposition, same vertex semantics: the two tilers must agree to the bit
    np.testing.assert_array_equal(y_lib, y_own)
    assert R.rel_err(y_lib, R.forward(cfg, w)) < (2e-6 if cfg.dtype == "f32" else 5e-2)
    kinds = lambda g: sorted((k, g.kind.count(k)) for k in set(g.kind))
    assert kinds(otg) == kinds(own)


@pytest.mark.parametrize("name,fuse", [("ragged_f32", 3), ("ragged_bf16", 1), ("ragged_bf16", 2), ("decode_f32", 3)])
def test_library_taskgraph_with_fused_epilogues_equals_the_oracles(name, fuse):
    """fuse_epilogues: the library's graph, interpreted by the oracle, gives the bits of the oracle's own fused
    graph and stays at the untiled model; the fused kinds replace exactly the vertices they stand for."""
    cfg = config(name)
    tg = B.tn_build_llama(H.llama_config_struct(cfg, fuse_epilogues=fuse))
    try:
        otg = oracle_taskgraph(tg)
    finally:
        B.tn_taskgraph_destroy(tg)
    w = R.widen(cfg, make_llama_inputs(cfg, 0))
    y_lib = T.assemble_outputs(otg, T.evaluate(otg, T.cut_inputs(otg, w)), cfg.tokens, cfg.d_model)
    own = T.build_llama_taskgraph(cfg, fuse_epilogues=fuse)
    y_own = T.assemble_outputs(own, T.evaluate(own, T.cut_inputs(own, w)), cfg.tokens, cfg.d_model)
    np.testing.assert_array_equal(y_lib, y_own)
    assert R.rel_err(y_lib, R.forward(cfg, w)) < (2e-6 if cfg.dtype == "f32" else 5e-2)
    kinds = lambda g: sorted((k, g.kind.count(k)) for k in set(g.kind))
    assert kinds(otg) == kinds(own)
    modes = lambda g: sorted(p.get("mode", 0) for k, p in zip(g.kind, g.params) if k == "gemm")
    assert modes(otg) == modes(own) and set(modes(otg)) == {0} | ({1} if fuse & 1 else set()) | ({2} if fuse & 2 else set())
    assert ("add" in otg.kind) == (not fuse & 1) and ("silu_mul" in otg.kind) == (not fuse & 2)


def test_fused_epilogues_are_checked():
    for kw in (dict(train=True, lora_rank=4), dict(k_split=2)):
        with pytest.raises(B.TurnipError) as e:
            B.tn_build_llama(H.llama_config_struct(config("c1"), fuse_epilogues=1, **kw))
        assert e.value.status == B.TN_ERR_INVALID
    c = H.llama_config_struct(config("c1"))
    c.fuse_epilogues = 4
    with pytest.raises(B.TurnipError):
        B.tn_build_llama(c)
    # a hand-built vertex: operand counts and shapes of the two modes
    tg = B.tn_taskgraph_create()
    try:
        inp = lambda r, c_: B.tn_taskgraph_add_input(tg, B.TN_F32, r, c_, B.TN_DEVICE)
        a, b, u, r, bad = inp(4, 8), inp(8, 6), inp(8, 6), inp(4, 6), inp(4, 5)
        B.tn_taskgraph_add_op(tg, B.TN_OP_GEMM, B.tn_op_params(nk=1, mode=1), [a, b, r], B.TN_F32, 4, 6)
        B.tn_taskgraph_add_op(tg, B.TN_OP_GEMM, B.tn_op_params(nk=1, mode=2), [a, b, u], B.TN_F32, 4, 6)
        for params, ins in ((B.tn_op_params(nk=1, mode=1), [a, b]), (B.tn_op_params(nk=1, mode=1), [a, b, bad]),
                            (B.tn_op_params(nk=1, mode=2), [a, b, r]), (B.tn_op_params(nk=1, mode=1, trans_c=1), [a, b, r]),
                            (B.tn_op_params(nk=1, mode=3), [a, b])):
            with pytest.raises(B.TurnipError) as e:
                B.tn_taskgraph_add_op(tg, B.TN_OP_GEMM, params, ins, B.TN_F32, 4, 6)
            assert e.value.status == B.TN_ERR_SHAPE
    finally:
        B.tn_taskgraph_destroy(tg)


def test_kv_outputs_are_marked():
    cfg = config("c1")
    tg = B.tn_build_llama(H.llama_config_struct(cfg, kv_outputs=True))
    try:
        names = [b[1] for b in H.bindings(tg)]
        assert B.tn_taskgraph_num_outputs(tg) == 8 + 2 * 2 * 8
        assert sum(n.startswith("k.") for n in names) == 16 and sum(n.startswith("v.") for n in names) == 16
    finally:
        B.tn_taskgraph_destroy(tg)


def test_tiler_rejects_inconsistent_shapes():
    cfg = H.llama_config_struct(config("c1"))
    cfg.n_heads = 3
    with pytest.raises(B.TurnipError) as e:
        B.tn_build_llama(cfg)
    assert e.value.status == B.TN_ERR_SHAPE
    cfg = H.llama_config_struct(config("c1"))
    cfg.attn_block = 96
    with pytest.raises(B.TurnipError):
        B.tn_build_llama(cfg)


def test_add_op_validates_operands():
    tg = B.tn_taskgraph_create()
    try:
        a = B.tn_taskgraph_add_input(tg, B.TN_F32, 8, 8, B.TN_HOST)
        b = B.tn_taskgraph_add_input(tg, B.TN_F32, 8, 4, B.TN_HOST)
        p = B.tn_op_params()
        with pytest.raises(B.TurnipError) as e:
            B.tn_taskgraph_add_op(tg, B.TN_OP_ADD, p, [a, b], B.TN_F32, 8, 8)
        assert e.value.status == B.TN_ERR_SHAPE
        p.nk = 1
        c = B.tn_taskgraph_add_op(tg, B.TN_OP_GEMM, p, [a, b], B.TN_F32, 8, 4)
        with pytest.raises(B.TurnipError):
            B.tn_taskgraph_add_op(tg, B.TN_OP_GEMM, p, [b, a], B.TN_F32, 8, 8)
        with pytest.raises(B.TurnipError) as e:
            B.tn_taskgraph_add_op(tg, B.TN_OP_ADD, B.tn_op_params(), [c, 99], B.TN_F32, 8, 4)
        assert e.value.status == B.TN_ERR_INVALID
        B.tn_taskgraph_mark_output(tg, c)
        with pytest.raises(B.TurnipError):
            B.tn_taskgraph_mark_output(tg, c)
        assert B.tn_taskgraph_num_vertices(tg) == 3 and B.tn_taskgraph_num_outputs(tg) == 1
    finally:
        B.tn_taskgraph_destroy(tg)


# ---------------------------------------------------------------------------------------------
# BuildMemgraph on the LLaMA graphs
# ---------------------------------------------------------------------------------------------

def _compile_llama(name, cap=None, opts=None, resident=None):
    cfg = config(name)
    if resident is not None:
        cfg = cfg.with_(weights_resident=resident, x_resident=resident)
    tg = B.tn_build_llama(H.llama_config_struct(cfg))
    cap = cap if cap is not None else H.cap_for(cfg, tg)
    mg = B.tn_compile(tg, None, cap, opts) if cap else None
    return cfg, tg, mg, cap


@pytest.mark.parametrize("name,n_orders", [("c1", 60), ("ragged_f32", 40), ("ragged_bf16", 40), ("batch2_f32", 40)])
def test_llama_memgraph_under_the_cap_is_correct_in_every_sampled_order(name, n_orders):
    cfg, tg, mg, cap = _compile_llama(name)
    try:
        omg = oracle_memgraph(mg)
        preds = task_preds(tg)
        count, ref = check_all(preds, omg, n_random=n_orders, seed=7)
        st = B.tn_memgraph_stats(mg)
        assert st.n_offload > 0 and st.n_reload > 0, "the cap must force offload on this workload"
        assert st.high_water <= cap and ref["hw_live"] <= cap
        assert set(ref["results"]) == set(H.export_taskgraph(tg)["outputs"])
        # the library's own dry run agrees on orders the oracle accepts
        B.tn_memgraph_simulate(mg)
        rng = np.random.default_rng(3)
        for _ in range(10):
            B.tn_memgraph_simulate(mg, M.random_topological_order(omg, rng))
    finally:
        B.tn_memgraph_destroy(mg)
        B.tn_taskgraph_destroy(tg)


def test_c1_thousand_random_orders():
    cfg, tg, mg, cap = _compile_llama("c1")
    try:
        check_all(task_preds(tg), oracle_memgraph(mg), n_random=1000, seed=100)
    finally:
        B.tn_memgraph_destroy(mg)
        B.tn_taskgraph_destroy(tg)


@pytest.mark.parametrize("name", ["c1", "batch2_f32", "ragged_bf16"])
def test_fine_tuning_memgraph_under_the_cap_is_correct_in_every_sampled_order(name):
    """Forward with adapters + reverse pass: saved activations are what the cap pushes out."""
    cfg = config(name)
    tg = B.tn_build_llama(H.llama_config_struct(cfg, lora_rank=8, train=True))
    try:
        cap = H.cap_for(cfg, tg)
        for opts in (None, B.tn_compile_opts(max_lookahead_bytes=B.UINT64_MAX, drop_clean_inputs=1, next_fit=1,
                                             evict_ahead_bytes=cap // 16)):
            mg = B.tn_compile(tg, None, cap, opts)
            try:
                st = B.tn_memgraph_stats(mg)
                assert st.n_offload > 0 and st.high_water <= cap
                check_all(task_preds(tg), oracle_memgraph(mg), n_random=12, seed=3)
            finally:
                B.tn_memgraph_destroy(mg)
    finally:
        B.tn_taskgraph_destroy(tg)


@pytest.mark.parametrize("opts", [
    dict(max_lookahead_bytes=0, drop_clean_inputs=1),
    dict(max_lookahead_bytes=B.UINT64_MAX, drop_clean_inputs=0),
    dict(max_lookahead_bytes=200_000, drop_clean_inputs=1, prune_superfluous=1),
    dict(max_lookahead_bytes=B.UINT64_MAX, drop_clean_inputs=1, fix_order=1),
    dict(max_lookahead_bytes=B.UINT64_MAX, drop_clean_inputs=1, alignment=4096),
    dict(max_lookahead_bytes=B.UINT64_MAX, drop_clean_inputs=1, next_fit=1),
    dict(max_lookahead_bytes=B.UINT64_MAX, drop_clean_inputs=1, evict_ahead_bytes=100_000),
    dict(max_lookahead_bytes=B.UINT64_MAX, drop_clean_inputs=0, evict_ahead_bytes=300_000, next_fit=1),
])
def test_compile_options_keep_the_memgraph_correct(opts):
    cfg, tg, mg, cap = _compile_llama("ragged_f32", opts=B.tn_compile_opts(**opts))
    try:
        omg = oracle_memgraph(mg)
        check_all(task_preds(tg), omg, n_random=25, seed=1)
        st = B.tn_memgraph_stats(mg)
        if not opts.get("drop_clean_inputs"):
            assert st.n_drop == 0
        if opts.get("prune_superfluous"):
            data = {(a, b) for a, b, k in omg.edges if k == "data"}
            assert not any((a, b) in data for a, b, k in omg.edges if k == "mem")
        if opts.get("fix_order"):
            # kernels are totally ordered by dependencies
            desc = M._reach_bitsets(omg)
            ops = [v for v in omg.order if omg.kind[v] == "op"]
            assert all((desc[a] >> b) & 1 for a, b in zip(ops, ops[1:]))
    finally:
        B.tn_memgraph_destroy(mg)
        B.tn_taskgraph_destroy(tg)


def test_device_resident_inputs_are_placed_first_and_offloaded_for_real():
    cfg, tg, mg, cap = _compile_llama("batch2_f32", resident=True, cap=1_400_000)
    try:
        omg = oracle_memgraph(mg)
        check_all(task_preds(tg), omg, n_random=25)
        inputs = [v for v in range(omg.n_task) if omg.kind[v] == "input"]
        assert inputs and omg.order[:len(inputs)] == inputs
        # nothing else may ever have lain where an input lies at the start
        first_writer = {}
        for v in omg.order:
            if omg.loc[v] is not None:
                first_writer.setdefault(omg.loc[v][0], v)
        st = B.tn_memgraph_stats(mg)
        assert st.n_drop == 0 and st.n_load == 0
    finally:
        B.tn_memgraph_destroy(mg)
        B.tn_taskgraph_destroy(tg)
    with pytest.raises(B.TurnipError) as e:
        _compile_llama("batch2_f32", resident=True, cap=500_000)
    assert e.value.status == B.TN_ERR_CAP_TOO_SMALL


def test_plenty_of_memory_means_no_transfers_and_only_data_edges():
    cfg, tg, mg, cap = _compile_llama("c1", cap=1 << 30, opts=B.tn_compile_opts(max_lookahead_bytes=B.UINT64_MAX))
    try:
        omg = oracle_memgraph(mg)
        preds = task_preds(tg)
        st = B.tn_memgraph_stats(mg)
        assert st.n_offload == st.n_reload == st.n_drop == 0 and st.n_mem_edges == 0
        stores = {v for v in range(len(omg)) if omg.kind[v] == "store"}
        got = sorted((a, b) for a, b, k in omg.edges if b not in stores)
        assert got == sorted({(u, v) for v in range(len(preds)) for u in preds[v]})
        check_all(preds, omg, n_random=5)
    finally:
        B.tn_memgraph_destroy(mg)
        B.tn_taskgraph_destroy(tg)


def test_c2_fits_its_cap_without_offload_and_offloads_at_forty_percent():
    cfg, tg, mg, cap = _compile_llama("c2")
    try:
        st = B.tn_memgraph_stats(mg)
        assert st.n_offload == 0 and st.high_water <= cap
    finally:
        B.tn_memgraph_destroy(mg)
        B.tn_taskgraph_destroy(tg)
    # with everything streamed from the host, 40 % of the uncapped peak forces real offloads
    cfg, tg, mg, small = _compile_llama("c2", resident=False, cap=0)
    B.tn_memgraph_destroy(mg) if mg else None
    small = (int(0.4 * H.uncapped_peak(tg)) + 255) // 256 * 256
    mg = B.tn_compile(tg, None, small, None)
    try:
        st = B.tn_memgraph_stats(mg)
        assert st.n_offload > 0 and st.high_water <= small
        check_all(task_preds(tg), oracle_memgraph(mg), n_random=3)
    finally:
        B.tn_memgraph_destroy(mg)
        B.tn_taskgraph_destroy(tg)


# ---------------------------------------------------------------------------------------------
# BuildMemgraph on random dataflow graphs (generic taskgraph API)
# ---------------------------------------------------------------------------------------------

def _random_taskgraph(seed, n, rows=16, uniform=False, n_inputs=2, residency=B.TN_HOST, max_fanin=3):
    """Vertices are rms_stat reductions (any fan-in); inputs are fp32 [rows, c] of varying width."""
    preds, _, outputs = random_dag(seed, n, max_fanin=max_fanin, n_inputs=n_inputs)
    rng = np.random.default_rng(seed)
    tg = B.tn_taskgraph_create()
    cols = []
    for v in range(n):
        if not preds[v]:
            c = 1 if uniform else int(rng.integers(1, 9))
            B.tn_taskgraph_add_input(tg, B.TN_F32, rows, c, residency)
            cols.append(c)
        else:
            p = B.tn_op_params(d=sum(cols[u] for u in preds[v]), eps=1e-6)
            B.tn_taskgraph_add_op(tg, B.TN_OP_RMS_STAT, p, preds[v], B.TN_F32, rows, 1)
            cols.append(1)
    for v in outputs:
        B.tn_taskgraph_mark_output(tg, v)
    unit = rows * 4
    return tg, preds, [c * unit for c in cols], unit


@pytest.mark.parametrize("seed", range(30))
def test_every_order_of_tiny_random_graphs(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(4, 7))
    tg, preds, sizes, unit = _random_taskgraph(seed, n, uniform=True, max_fanin=2)
    need = max(sum(sizes[u] for u in set(preds[v])) + sizes[v] for v in range(n))
    try:
        mg = B.tn_compile(tg, None, need + unit * int(rng.integers(0, 2)),
                          B.tn_compile_opts(max_lookahead_bytes=B.UINT64_MAX, drop_clean_inputs=seed % 2, alignment=64,
                                            next_fit=(seed // 2) % 2, evict_ahead_bytes=unit * ((seed // 4) % 2)))
        omg = oracle_memgraph(mg)
        B.tn_memgraph_destroy(mg)
        if len(omg) > 11:
            pytest.skip("too many orders to enumerate")
        count, _ = check_all(preds, omg, exhaustive=True)
        assert count >= 1
    finally:
        B.tn_taskgraph_destroy(tg)


@pytest.mark.parametrize("seed", range(40))
def test_random_graphs_with_variable_sizes(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(15, 120))
    resid = B.TN_DEVICE if seed % 5 == 0 else B.TN_HOST
    tg, preds, sizes, unit = _random_taskgraph(seed, n, n_inputs=int(rng.integers(2, 6)), residency=resid, max_fanin=4)
    need = max(sum(sizes[u] for u in set(preds[v])) + sizes[v] for v in range(n))
    if resid == B.TN_DEVICE:
        need = max(need, sum(sizes[v] for v in range(n) if not preds[v]) + 2 * unit)
    try:
        mg = B.tn_compile(tg, None, 2 * need, B.tn_compile_opts(max_lookahead_bytes=B.UINT64_MAX,
                                                               drop_clean_inputs=seed % 2, alignment=64))
        omg = oracle_memgraph(mg)
        B.tn_memgraph_simulate(mg)
        B.tn_memgraph_destroy(mg)
        check_all(preds, omg, n_random=20, seed=seed)
    finally:
        B.tn_taskgraph_destroy(tg)


@pytest.mark.parametrize("seed", range(12))
def test_variable_sizes_compile_at_the_exact_minimum(seed):
    """cap = the largest (operands + output) footprint always compiles, however fragmented."""
    tg, preds, sizes, unit = _random_taskgraph(900 + seed, 60, n_inputs=4, max_fanin=4)
    need = max(sum(sizes[u] for u in set(preds[v])) + sizes[v] for v in range(60))
    try:
        mg = B.tn_compile(tg, None, need, B.tn_compile_opts(max_lookahead_bytes=B.UINT64_MAX,
                                                           drop_clean_inputs=seed % 2, alignment=64))
        check_all(preds, oracle_memgraph(mg), n_random=15, seed=seed)
        B.tn_memgraph_destroy(mg)
        with pytest.raises(B.TurnipError) as e:
            B.tn_compile(tg, None, need - 64, B.tn_compile_opts(max_lookahead_bytes=B.UINT64_MAX, alignment=64))
        assert e.value.status == B.TN_ERR_CAP_TOO_SMALL
    finally:
        B.tn_taskgraph_destroy(tg)


def test_exact_minimum_compiles_and_one_unit_less_does_not():
    for seed in range(10):
        tg, preds, sizes, unit = _random_taskgraph(50 + seed, 40, uniform=True, max_fanin=3)
        need = max(sum(sizes[u] for u in set(preds[v])) + sizes[v] for v in range(40))
        try:
            mg = B.tn_compile(tg, None, need, B.tn_compile_opts(max_lookahead_bytes=B.UINT64_MAX, alignment=64))
            check_all(preds, oracle_memgraph(mg), n_random=10)
            B.tn_memgraph_destroy(mg)
            with pytest.raises(B.TurnipError) as e:
                B.tn_compile(tg, None, need - unit, B.tn_compile_opts(max_lookahead_bytes=B.UINT64_MAX, alignment=64))
            assert e.value.status == B.TN_ERR_CAP_TOO_SMALL
            assert "vertex" in e.value.message
        finally:
            B.tn_taskgraph_destroy(tg)


def test_given_order_is_validated_and_used():
    tg, preds, sizes, unit = _random_taskgraph(3, 12, uniform=True)
    try:
        bad = list(range(12))[::-1]
        with pytest.raises(B.TurnipError) as e:
            B.tn_compile(tg, bad, 1 << 20, None)
        assert e.value.status == B.TN_ERR_NOT_TOPOLOGICAL
        with pytest.raises(B.TurnipError) as e:
            B.tn_compile(tg, [0] * 12, 1 << 20, None)
        assert e.value.status == B.TN_ERR_INVALID
        order = list(range(12))
        mg = B.tn_compile(tg, order, 1 << 20, None)
        omg = oracle_memgraph(mg)
        assert [v for v in omg.order if v < 12] == order
        with pytest.raises(B.TurnipError) as e:
            B.tn_memgraph_simulate(mg, omg.order[::-1])
        assert e.value.status == B.TN_ERR_NOT_TOPOLOGICAL
        B.tn_memgraph_destroy(mg)
    finally:
        B.tn_taskgraph_destroy(tg)


def test_two_vertex_chain_may_become_offload_reload(tmp_path):
    """Section 4: v1 -> v2 can always be compiled to v1 -> offload -> reload -> v2."""
    tg = B.tn_taskgraph_create()
    try:
        a = B.tn_taskgraph_add_input(tg, B.TN_F32, 16, 4, B.TN_DEVICE)   # v1: 256 B
        b = B.tn_taskgraph_add_input(tg, B.TN_F32, 16, 4, B.TN_DEVICE)
        s1 = B.tn_taskgraph_add_op(tg, B.TN_OP_RMS_STAT, B.tn_op_params(d=4, eps=1e-6), [b], B.TN_F32, 16, 1)
        s2 = B.tn_taskgraph_add_op(tg, B.TN_OP_RMS_STAT, B.tn_op_params(d=1, eps=1e-6), [s1], B.TN_F32, 16, 1)
        c = B.tn_taskgraph_add_input(tg, B.TN_F32, 16, 4, B.TN_HOST)
        s3 = B.tn_taskgraph_add_op(tg, B.TN_OP_RMS_STAT, B.tn_op_params(d=5, eps=1e-6), [c, s2], B.TN_F32, 16, 1)
        mid = B.tn_taskgraph_add_op(tg, B.TN_OP_RMS_STAT, B.tn_op_params(d=5, eps=1e-6), [b, s3], B.TN_F32, 16, 1)
        v2 = B.tn_taskgraph_add_op(tg, B.TN_OP_RMS_STAT, B.tn_op_params(d=5, eps=1e-6), [a, mid], B.TN_F32, 16, 1)
        B.tn_taskgraph_mark_output(tg, v2)
        # a, b and s2 fill the memory when c has to come in; b is needed sooner than a, so a
        # must leave and come back before v2
        mg = B.tn_compile(tg, None, 256 + 256 + 64 + 64, B.tn_compile_opts(max_lookahead_bytes=0, alignment=64))
        omg = oracle_memgraph(mg)
        check_all(task_preds(tg), omg, exhaustive=len(omg) <= 11, n_random=50)
        off = [v for v in range(len(omg)) if omg.kind[v] == "offload" and omg.src[v] == a]
        rel = [v for v in range(len(omg)) if omg.kind[v] == "reload" and omg.src[v] == a]
        assert len(off) == 1 and len(rel) == 1
        es = set(omg.edges)
        assert (a, off[0], "data") in es and (off[0], rel[0], "data") in es and (rel[0], v2, "data") in es
        path = str(tmp_path / "mg.json")
        B.tn_memgraph_dump_json(mg, path)
        import json
        j = json.load(open(path))
        assert len(j["vertices"]) == len(omg) and len(j["edges"]) == len(omg.edges)
        B.tn_memgraph_destroy(mg)
    finally:
        B.tn_taskgraph_destroy(tg)


@pytest.mark.parametrize("name,kw", [("c1", {}), ("ragged_bf16", dict(lora_rank=8, train=True)), ("batch2_f32", dict(k_split=2))])
def test_level_order_runs_the_graph_level_by_level_and_compiles(name, kw):
    cfg = config(name)
    tg = B.tn_build_llama(H.llama_config_struct(cfg, **kw))
    try:
        order = B.tn_taskgraph_level_order(tg)
        preds = task_preds(tg)
        n = len(preds)
        assert sorted(order) == list(range(n))
        pos = {v: i for i, v in enumerate(order)}
        assert all(pos[u] < pos[v] for v in range(n) for u in preds[v])
        # levels worked out here from the definition: longest chain of kernel vertices ending at v
        level = [0] * n
        for v in range(n):
            if preds[v]:
                level[v] = 1 + max((level[u] for u in preds[v] if preds[u]), default=0)
        ops = [v for v in order if preds[v]]
        assert all(level[a] <= level[b] for a, b in zip(ops, ops[1:]))
        assert all(a < b for a, b in zip(ops, ops[1:]) if level[a] == level[b]), "a level keeps its numbering"
        for v in order:  # an input sits directly before the first level that reads it
            if not preds[v]:
                first = min((level[w] for w in range(n) if v in preds[w]), default=1)
                later_ops = [level[w] for w in order[pos[v]:] if preds[w]]
                earlier_ops = [level[w] for w in order[:pos[v]] if preds[w]]
                assert (not later_ops or later_ops[0] == first) and (not earlier_ops or earlier_ops[-1] < first)
        # (outputs of unfinished sums cannot move, and a level opens all of its sums at once: more room there)
        cap = H.cap_for(cfg, tg) * (2 if kw.get("k_split") else 1)
        mg = B.tn_compile(tg, order, cap, None)
        try:
            check_all(preds, oracle_memgraph(mg), n_random=10, seed=2)
        finally:
            B.tn_memgraph_destroy(mg)
        with pytest.raises(B.TurnipError):
            buf = (ctypes.c_int32 * 4)()
            B._check(B.lib().tn_taskgraph_level_order(tg, buf, 4))
    finally:
        B.tn_taskgraph_destroy(tg)


@pytest.mark.parametrize("name,kw", [("c1", {}), ("ragged_bf16", {}), ("batch2_f32", {}), ("ragged_f32", {"k_split": 2}),
                                     ("c1", {"train": True, "lora_rank": 4}), ("decode_f32", {})])
def test_clustered_order_keeps_reductions_next_to_their_operands_and_compiles(name, kw):
    """tn_taskgraph_clustered_order: a valid order; every combine directly behind its partials (and the
    partials of one combine together), every SiLU-mul directly behind its two products; an input right
    before its first reader; vertices of a level that read inputs ordered by the first input they read;
    the memgraph compiled for it under the cap passes the checks of Section 6 and moves no more bytes to
    the host than the one compiled for the level order."""
    cfg = config(name)
    tg = B.tn_build_llama(H.llama_config_struct(cfg, **kw))
    try:
        order = B.tn_taskgraph_clustered_order(tg)
        preds = task_preds(tg)
        n = len(preds)
        assert sorted(order) == list(range(n))
        pos = {v: i for i, v in enumerate(order)}
        assert all(pos[u] < pos[v] for v in range(n) for u in preds[v])
        kinds = [B.tn_taskgraph_vertex(tg, v).kind for v in range(n)]
        readers = [[] for _ in range(n)]
        for v in range(n):
            for u in dict.fromkeys(preds[v]):
                readers[u].append(v)
        ops_only = [v for v in order if preds[v]]
        opos = {v: i for i, v in enumerate(ops_only)}  # positions among the kernel vertices alone
        seen = 0
        for v in range(n):
            if kinds[v] not in (B.TN_OP_ATTN_COMBINE, B.TN_OP_SILU_MUL):
                continue
            group = sorted(w for w in range(n) if preds[w] == preds[v])  # the vertices with this operand list
            if v != group[0] or any(not preds[u] for u in preds[v]) or any(set(readers[u]) != set(group) for u in preds[v]):
                continue
            if any(kinds[u] == B.TN_OP_SUM for u in preds[v]):
                continue  # the operands are reductions themselves (placed with their own operands): no chains
            block = sorted(opos[u] for u in set(preds[v])) + sorted(opos[w] for w in group)
            assert block == list(range(block[0], block[0] + len(block))), (v, block)  # one uninterrupted run
            assert max(opos[u] for u in preds[v]) < min(opos[w] for w in group)
            seen += 1
        assert seen > 0
        for v in range(n):  # an input sits right before its first reader (other inputs of that reader may lie between)
            if not preds[v] and readers[v]:
                first = min(readers[v], key=pos.get)
                assert all(not preds[w] for w in order[pos[v] + 1:pos[first]])
        cap = H.cap_for(cfg, tg) * (2 if kw.get("k_split") else 1)
        mg = B.tn_compile(tg, order, cap, None)
        mg_level = B.tn_compile(tg, B.tn_taskgraph_level_order(tg), cap, None)
        try:
            check_all(preds, oracle_memgraph(mg), n_random=10, seed=2)
            st, st_level = B.tn_memgraph_stats(mg), B.tn_memgraph_stats(mg_level)
            assert st.offload_bytes <= st_level.offload_bytes
            print(f"{name} {kw}: offloaded {st.offload_bytes} against {st_level.offload_bytes} bytes in level order; "
                  f"loaded {st.load_bytes} against {st_level.load_bytes}")
        finally:
            B.tn_memgraph_destroy(mg)
            B.tn_memgraph_destroy(mg_level)
        with pytest.raises(B.TurnipError):
            buf = (ctypes.c_int32 * 4)()
            B._check(B.lib().tn_taskgraph_clustered_order(tg, buf, 4))
    finally:
        B.tn_taskgraph_destroy(tg)
