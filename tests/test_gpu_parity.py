"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs; across dispatch orders and injected transfer delays; on the offload path."""
import numpy as np
import pytest

from oracle import llama_ref as R
from oracle import tiled as T
from paper_2405_16283_amd import binding as B
from paper_2405_16283_amd import harness as H
from workloads import bf16_bits_to_f32, config, make_llama_inputs

from util import check_layer_rows, oracle_taskgraph

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}  # max relative error allowed against the oracle, per storage type


def _as_f64(cfg, a):
    return (bf16_bits_to_f32(a) if cfg.dtype == "bf16" else a).astype(np.float64)


def _oracle(cfg, full, tg_handle=None):
    """Tiled oracle (same rounding points as the taskgraph) and untiled float64 reference."""
    w = R.widen(cfg, full)
    own = T.build_llama_taskgraph(cfg)
    y_tiled = T.assemble_outputs(own, T.evaluate(own, T.cut_inputs(own, w)), cfg.tokens, cfg.d_model)
    return y_tiled, R.forward(cfg, w)


@pytest.mark.parametrize("name", ["c1", "ragged_f32", "batch2_f32", "ragged_bf16", "mid_bf16"])
@pytest.mark.parametrize("seed", [0, 1])
def test_forward_matches_oracle_under_the_cap(name, seed):
    cfg = config(name)
    full = make_llama_inputs(cfg, seed)
    y_tiled, y_ref = _oracle(cfg, full)
    print(f"[case] {name} seed {seed}", flush=True)
    s = H.GpuSession(cfg, full)
    try:
        assert s.stats.n_offload > 0, "cap must force offload"
        out, rep = s.run()
        y = _as_f64(cfg, out["y"])
        assert np.isfinite(y).all()
        err = R.rel_err(y, y_tiled)
        print(f"  rel err vs tiled oracle {err:.3e}, vs untiled {R.rel_err(y, y_ref):.3e}; "
              f"{rep.n_offload} offloads, {rep.n_reload} reloads, {rep.n_launches} launches", flush=True)
        assert err < TOL[cfg.dtype]
        assert rep.n_offload == s.stats.n_offload and rep.n_reload == s.stats.n_reload
        assert rep.n_vertices == s.stats.n_vertices
    finally:
        s.close()


@pytest.mark.parametrize("name", ["c1", "ragged_bf16", "mid_bf16"])
def test_twenty_dispatch_orders_and_transfer_delays_give_identical_bits(name):
    """Any dependency-respecting order must produce the same output (Introduction); the vertex
    kernels have a fixed summation order, so 'same' means bit for bit."""
    cfg = config(name)
    full = make_llama_inputs(cfg, 0)
    y_tiled, _ = _oracle(cfg, full)
    s = H.GpuSession(cfg, full)
    try:
        ref, _ = s.run(B.tn_exec_opts(policy=B.TN_POLICY_BY_ORDER, max_batch=1))
        assert R.rel_err(_as_f64(cfg, ref["y"]), y_tiled) < TOL[cfg.dtype]
        orders = set()
        for seed in range(20):
            delay = (0, 50, 500)[seed % 3]
            batch = (1, 4, 0)[(seed // 3) % 3]
            print(f"[case] {name} order_seed {seed} delay {delay} batch {batch}", flush=True)
            depth = (1, 3, 8)[(seed // 2) % 3]
            out, rep = s.run(B.tn_exec_opts(policy=B.TN_POLICY_RANDOM, order_seed=seed, delay_seed=100 + seed,
                                            max_delay_us=delay, max_batch=batch, queue_depth=depth))
            np.testing.assert_array_equal(out["y"], ref["y"])
            orders.add(tuple(s.last_order()))
        assert len(orders) >= 15, "the seeds must really perturb the dispatch order"
        for policy in (B.TN_POLICY_FIFO, B.TN_POLICY_LIFO, B.TN_POLICY_IN_ORDER):
            for depth in (1, 3):
                out, _ = s.run(B.tn_exec_opts(policy=policy, queue_depth=depth, max_delay_us=50, delay_seed=policy))
                np.testing.assert_array_equal(out["y"], ref["y"])
    finally:
        s.close()


def test_launch_order_respects_every_dependency():
    cfg = config("c1")
    s = H.GpuSession(cfg, make_llama_inputs(cfg, 0))
    try:
        s.run(B.tn_exec_opts(policy=B.TN_POLICY_RANDOM, order_seed=5, max_batch=3))
        order = s.last_order()
        B.tn_memgraph_simulate(s.mg, order)
        # with kernels enqueued ahead of the completion of their predecessors, too
        s.run(B.tn_exec_opts(policy=B.TN_POLICY_RANDOM, order_seed=6, max_batch=5, queue_depth=4))
        order = s.last_order()
        e = H.export_memgraph(s.mg)
        assert sorted(order) == list(range(len(e["kind"])))
        # the launch order is a valid order for the library's own dry run, too
        B.tn_memgraph_simulate(s.mg, order)
        # the in-order policy launches kernels, and the transfers of each direction, exactly in
        # the serial order the memgraph was compiled for
        s.run(B.tn_exec_opts(policy=B.TN_POLICY_IN_ORDER, max_batch=7, queue_depth=2, max_delay_us=100, delay_seed=3))
        order = s.last_order()
        pos = {v: i for i, v in enumerate(e["order"])}
        for kinds in (("op",), ("load", "reload"), ("offload", "store")):
            launched = [v for v in order if e["kind"][v] in kinds]
            assert launched == sorted(launched, key=pos.get), kinds
        B.tn_memgraph_simulate(s.mg, order)
    finally:
        s.close()


@pytest.mark.parametrize("opts", [
    dict(max_lookahead_bytes=0, drop_clean_inputs=1),
    dict(max_lookahead_bytes=B.UINT64_MAX, drop_clean_inputs=0),
    dict(max_lookahead_bytes=B.UINT64_MAX, drop_clean_inputs=1, fix_order=1),
    dict(max_lookahead_bytes=B.UINT64_MAX, drop_clean_inputs=1, next_fit=1, evict_ahead_bytes=200_000),
])
def test_compile_variants_on_the_gpu(opts):
    cfg = config("ragged_f32")
    full = make_llama_inputs(cfg, 3)
    y_tiled, _ = _oracle(cfg, full)
    s = H.GpuSession(cfg, full, compile_opts=B.tn_compile_opts(**opts))
    try:
        out, rep = s.run(B.tn_exec_opts(policy=B.TN_POLICY_RANDOM, order_seed=1))
        assert R.rel_err(out["y"].astype(np.float64), y_tiled) < TOL["f32"]
    finally:
        s.close()


def test_device_resident_inputs_and_untransposed_weights():
    cfg = config("batch2_f32").with_(weights_resident=True, x_resident=True)
    full = make_llama_inputs(cfg, 0)
    y_tiled, _ = _oracle(cfg, full)
    for tr in (True, False):
        s = H.GpuSession(cfg, full, cap=760_000, weights_transposed=tr)
        try:
            assert s.stats.n_offload > 0 and s.stats.n_load == 0
            for _ in range(2):  # inputs are re-placed before every run
                out, rep = s.run()
                assert R.rel_err(out["y"].astype(np.float64), y_tiled) < TOL["f32"]
        finally:
            s.close()


def test_kv_outputs_match_the_oracle():
    cfg = config("c1")
    full = make_llama_inputs(cfg, 0)
    w = R.widen(cfg, full)
    s = H.GpuSession(cfg, full, kv_outputs=True)
    try:
        out, _ = s.run()
        x = w["x"]
        for l in range(cfg.layers):
            y, k, v = R.decoder_layer(x, w, l, cfg.n_heads, cfg.head_dim, cfg.eps, cfg.rope_base, return_kv=True)
            assert R.rel_err(out[f"k.{l}"].astype(np.float64), k) < TOL["f32"]
            assert R.rel_err(out[f"v.{l}"].astype(np.float64), v) < TOL["f32"]
            x = y
    finally:
        s.close()


@pytest.mark.parametrize("engine", [B.TN_COPY_MEMCPY, B.TN_COPY_KERNEL, B.TN_COPY_KERNEL_IN])
def test_all_copy_engines_give_identical_bits(engine):
    cfg = config("ragged_bf16")
    s = H.GpuSession(cfg, make_llama_inputs(cfg, 0))
    try:
        ref, _ = s.run(B.tn_exec_opts(policy=B.TN_POLICY_BY_ORDER))
        out, rep = s.run(B.tn_exec_opts(policy=B.TN_POLICY_RANDOM, order_seed=3, copy_engine=engine, max_transfers=5))
        np.testing.assert_array_equal(out["y"], ref["y"])
        assert rep.n_offload == s.stats.n_offload > 0
    finally:
        s.close()


@pytest.mark.parametrize("name", ["c1", "mid_bf16", "decode_bf16"])
def test_offloads_gathered_in_staging_slots_give_identical_bits(name):
    """TN_COPY_KERNEL_IN: the offloads of a group are gathered into a staging slot in GPU memory and leave
    with one copy into adjacent arena slots, from where each tensor is reloaded on its own; stores go
    one by one.  Group sizes from one tensor to as many as fit, orders, delays and depths perturbed; K/V
    outputs (stores) mixed in."""
    cfg = config(name)
    s = H.GpuSession(cfg, make_llama_inputs(cfg, 0), kv_outputs=True)
    try:
        assert s.stats.n_offload > 0
        ref, rep0 = s.run(B.tn_exec_opts(policy=B.TN_POLICY_BY_ORDER, copy_engine=B.TN_COPY_KERNEL))
        for seed in range(12):
            mt, depth, td = (1, 3, 32, 128)[seed % 4], (1, 3, 8)[seed % 3], (1, 3, 8)[(seed // 2) % 3]
            print(f"[case] {name} staged offloads, order_seed {seed}, max_transfers {mt}, queue_depth {depth}, "
                  f"transfer_depth {td}", flush=True)
            out, rep = s.run(B.tn_exec_opts(policy=B.TN_POLICY_RANDOM, order_seed=seed, copy_engine=B.TN_COPY_KERNEL_IN,
                                            max_transfers=mt, queue_depth=depth, transfer_depth=td,
                                            max_delay_us=(0, 100)[seed % 2], delay_seed=seed))
            assert rep.n_offload == s.stats.n_offload and rep.n_reload == s.stats.n_reload
            assert rep.d2h_bytes == rep0.d2h_bytes and rep.h2d_bytes == rep0.h2d_bytes
            assert rep.arena_high_water <= s.stats.host_arena_bytes
            for k in ref:
                np.testing.assert_array_equal(out[k], ref[k])
    finally:
        s.close()


def test_pageable_host_buffers_fall_back_to_memcpy_and_kernel_engine_refuses_them():
    import torch
    rng = np.random.default_rng(1)
    a = rng.standard_normal((64, 32)).astype(np.float32)  # plain, pageable memory
    tg = B.tn_taskgraph_create()
    va = B.tn_taskgraph_add_input(tg, B.TN_F32, 64, 32, B.TN_HOST)
    s = B.tn_taskgraph_add_op(tg, B.TN_OP_ADD, B.tn_op_params(), [va, va], B.TN_F32, 64, 32)
    B.tn_taskgraph_mark_output(tg, s)
    mg = B.tn_compile(tg, None, 1 << 20, None)
    dev = torch.empty(1 << 20, dtype=torch.uint8, device="cuda:0")
    streams = [torch.cuda.Stream() for _ in range(3)]
    out = np.zeros((64, 32), dtype=np.float32)
    ex = B.tn_executor_create(mg, dev.data_ptr(), 1 << 20, 0, 0, [streams[0].cuda_stream],
                              streams[1].cuda_stream, streams[2].cuda_stream)
    try:
        B.tn_execute(ex, [a.ctypes.data, 0], [out.ctypes.data])
        np.testing.assert_array_equal(out, 2 * a)
        with pytest.raises(B.TurnipError) as e:
            B.tn_execute(ex, [a.ctypes.data, 0], [out.ctypes.data], B.tn_exec_opts(copy_engine=B.TN_COPY_KERNEL))
        assert e.value.status == B.TN_ERR_INVALID
    finally:
        B.tn_executor_destroy(ex)
        B.tn_memgraph_destroy(mg)
        B.tn_taskgraph_destroy(tg)


def test_exhausted_host_arena_is_an_error_not_a_hang():
    cfg = config("c1")
    s = H.GpuSession(cfg, make_llama_inputs(cfg, 0), arena_bytes=4096)
    try:
        s.place_inputs()
        with pytest.raises(B.TurnipError) as e:
            s.execute()
        assert e.value.status == B.TN_ERR_ARENA
    finally:
        s.close()


def test_generic_taskgraph_through_the_abi():
    """A hand-built graph (not the LLaMA tiler): C = A B^T + A B^T, one output, fp32."""
    import torch
    rng = np.random.default_rng(0)
    a = rng.standard_normal((40, 24)).astype(np.float32)
    b = rng.standard_normal((56, 24)).astype(np.float32)
    tg = B.tn_taskgraph_create()
    va = B.tn_taskgraph_add_input(tg, B.TN_F32, 40, 24, B.TN_HOST)
    vb = B.tn_taskgraph_add_input(tg, B.TN_F32, 56, 24, B.TN_HOST)
    g = B.tn_taskgraph_add_op(tg, B.TN_OP_GEMM, B.tn_op_params(nk=1, trans_b=1), [va, vb], B.TN_F32, 40, 56)
    s = B.tn_taskgraph_add_op(tg, B.TN_OP_ADD, B.tn_op_params(), [g, g], B.TN_F32, 40, 56)
    B.tn_taskgraph_mark_output(tg, s)
    mg = B.tn_compile(tg, None, 1 << 20, None)
    dev = torch.empty(1 << 20, dtype=torch.uint8, device="cuda:0")
    streams = [torch.cuda.Stream() for _ in range(3)]
    ta, tb = torch.from_numpy(a).pin_memory(), torch.from_numpy(b).pin_memory()
    out = torch.zeros(40, 56).pin_memory()
    ex = B.tn_executor_create(mg, dev.data_ptr(), 1 << 20, 0, 0, [streams[0].cuda_stream],
                              streams[1].cuda_stream, streams[2].cuda_stream)
    try:
        B.tn_execute(ex, [ta.data_ptr(), tb.data_ptr(), 0, 0], [out.data_ptr()])
        ref = 2.0 * (a.astype(np.float64) @ b.astype(np.float64).T)
        assert R.rel_err(out.numpy().astype(np.float64), ref) < 1e-5
    finally:
        B.tn_executor_destroy(ex)
        B.tn_memgraph_destroy(mg)
        B.tn_taskgraph_destroy(tg)


@pytest.mark.parametrize("name,layers", [("ragged_bf16", 2), ("c1", 2), ("batch2_f32", 1), ("mid_bf16", 3)])
def test_every_layer_alone_against_the_oracle(name, layers):
    """The check used on the deep workloads, on shapes where everything else is checked too: each
    layer's input rows as the GPU produced them through one oracle layer, the GPU's stored keys and
    values as the context of late rows."""
    cfg = config(name).with_(layers=layers)
    full = make_llama_inputs(cfg, 2)
    s = H.GpuSession(cfg, full, kv_outputs=True, hidden_outputs=True)
    try:
        print(f"[case] per-layer check {name}", flush=True)
        out, rep = s.run(B.tn_exec_opts(policy=B.TN_POLICY_RANDOM, order_seed=9, queue_depth=2))
        rows = np.array(sorted({0, 1, 5, cfg.seq // 2, cfg.seq // 2 + 1, cfg.seq - 34, cfg.seq - 2, cfg.seq - 1}))
        for layer in range(cfg.layers):
            for b in range(cfg.batch):
                check_layer_rows(cfg, full, out, layer, b, rows, TOL[cfg.dtype], True, name)
                check_layer_rows(cfg, full, out, layer, b, np.arange(8), TOL[cfg.dtype], False, name)
    finally:
        s.close()


@pytest.mark.parametrize("name", ["c1", "mid_bf16", "ragged_bf16"])
def test_serial_orders_change_the_memgraph_and_not_the_bits(name):
    """The same taskgraph compiled for the tiler's order, the level order and the clustered order, under the
    same cap: three different memgraphs (other transfers, other memory dependencies), identical outputs."""
    cfg = config(name)
    full = make_llama_inputs(cfg, 0)
    tg = B.tn_build_llama(H.llama_config_struct(cfg, kv_outputs=True))
    orders = {"tiler": None, "level": B.tn_taskgraph_level_order(tg), "clustered": B.tn_taskgraph_clustered_order(tg)}
    B.tn_taskgraph_destroy(tg)
    ref, moved = None, {}
    for label, order in orders.items():
        s = H.GpuSession(cfg, full, kv_outputs=True, order=order)
        try:
            print(f"[case] {name} serial order {label}: {s.stats.n_offload} offloads, {s.stats.n_load} loads", flush=True)
            out, rep = s.run(B.tn_exec_opts(policy=B.TN_POLICY_RANDOM, order_seed=4, max_delay_us=50))
            moved[label] = (s.stats.n_offload, s.stats.n_load, s.stats.n_mem_edges)
            if ref is None:
                ref = out
            for k in ref:
                np.testing.assert_array_equal(out[k], ref[k])
        finally:
            s.close()
    assert len(set(moved.values())) > 1


@pytest.mark.parametrize("name", ["c1", "ragged_bf16", "mid_bf16"])
def test_whole_row_attention_vertices_match_the_oracle(name):
    """Tiler option attn_whole_rows: one attention vertex per query block over all earlier keys (the MFMA
    kernel then walks through up to 1440 keys with the diagonal inside its last blocks) against the oracle's
    tiling of the same kind, under the cap, and the same bits in another order."""
    cfg = config(name)
    full = make_llama_inputs(cfg, 0)
    w = R.widen(cfg, full)
    own = T.build_llama_taskgraph(cfg, attn_whole_rows=True)
    y_tiled = T.assemble_outputs(own, T.evaluate(own, T.cut_inputs(own, w)), cfg.tokens, cfg.d_model)
    s = H.GpuSession(cfg, full, attn_whole_rows=True)
    try:
        assert s.stats.n_offload > 0
        out, _ = s.run()
        err = R.rel_err(_as_f64(cfg, out["y"]), y_tiled)
        print(f"[case] {name} whole-row attention: rel err {err:.3e}", flush=True)
        assert err < TOL[cfg.dtype]
        o2, _ = s.run(B.tn_exec_opts(policy=B.TN_POLICY_RANDOM, order_seed=3, max_batch=2, max_delay_us=100))
        np.testing.assert_array_equal(o2["y"], out["y"])
    finally:
        s.close()


@pytest.mark.parametrize("k_second,launches", [(1024, 1), (8192, 2), (16384, 2)])
def test_tile_products_of_different_depth_do_not_share_a_launch(k_second, launches):
    """Two independent 512x512 products that are ready together: of the same depth class they go out as one
    launch of two vertices, of different classes (up to 6144, up to 12288, deeper) as two launches -- workgroups
    that do not walk along K in step lose the sharing in the L2s.  Both results against the oracle's vertex."""
    import torch
    from workloads import to_bf16_bits
    rng = np.random.default_rng(k_second)
    tg = B.tn_taskgraph_create()
    host, wide, outs = {}, {}, []
    for k in (1024, k_second):
        ins = []
        for _ in range(2):
            a = to_bf16_bits(np.ascontiguousarray(rng.standard_normal((512, k)) / np.sqrt(np.sqrt(k)), dtype=np.float32)).reshape(512, k)
            v = B.tn_taskgraph_add_input(tg, B.TN_BF16, 512, k, B.TN_HOST)
            host[v] = torch.from_numpy(a.view(np.int16)).pin_memory()
            wide[v] = bf16_bits_to_f32(a).astype(np.float64)
            ins.append(v)
        o = B.tn_taskgraph_add_op(tg, B.TN_OP_GEMM, B.tn_op_params(nk=1, trans_b=1), ins, B.TN_BF16, 512, 512)
        B.tn_taskgraph_mark_output(tg, o)
        outs.append((o, ins))
    cap = 256 << 20
    mg = B.tn_compile(tg, None, cap, None)
    dev = torch.empty(cap, dtype=torch.uint8, device="cuda:0")
    streams = [torch.cuda.Stream() for _ in range(3)]
    bufs = [torch.zeros(512 * 512, dtype=torch.int16).pin_memory() for _ in outs]
    ex = B.tn_executor_create(mg, dev.data_ptr(), cap, 0, 0, [streams[0].cuda_stream], streams[1].cuda_stream, streams[2].cuda_stream)
    try:
        n = B.tn_taskgraph_num_vertices(tg)
        print(f"[case] two products, depths 1024 and {k_second}", flush=True)
        # small copy groups, so that nothing but the products' readiness decides; the products wait for all loads
        B.tn_execute(ex, [host[v].data_ptr() if v in host else 0 for v in range(n)], [b.data_ptr() for b in bufs],
                     B.tn_exec_opts(policy=B.TN_POLICY_BY_ORDER, max_batch=1920, profile=1, max_gemm_inflight=1, max_delay_us=2000,
                                    delay_seed=1))
        rec = B.tn_executor_last_launches(ex)
        gemm = rec[rec["family"] == 0]
        print("  tile-product launches:", [(int(x["n_vertices"]), int(x["work"])) for x in gemm], flush=True)
        assert int(gemm["n_vertices"].sum()) == 2
        if launches == 2:
            assert len(gemm) == 2  # never together, whatever the timing
        for (o, ins), b in zip(outs, bufs):
            ref = T._eval_vertex("gemm", dict(nk=1, trans_b=1), [wide[v] for v in ins])
            got = bf16_bits_to_f32(b.numpy().view(np.uint16)).astype(np.float64).reshape(512, 512)
            assert R.rel_err(got, T.round_bf16(ref)) < 2.0 ** -7
    finally:
        B.tn_executor_destroy(ex)
        B.tn_memgraph_destroy(mg)
        B.tn_taskgraph_destroy(tg)
