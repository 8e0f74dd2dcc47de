"""tn_execute_static: the entry point for callers that cannot allocate.  Its kernels read their
operand tables from the region that is part of the loaded library instead of the executor's own
GPU allocation; results must equal tn_execute's bit for bit.  Two calls in a row, the second on a
smaller memgraph, so that what the first call left in the shared region is still there when the
second one runs; then the first again, and a memgraph whose tables do not fit the region."""
import ctypes

import numpy as np
import pytest

from oracle import llama_ref as R
from oracle import tiled as T
from paper_2405_16283_amd import binding as B
from paper_2405_16283_amd import harness as H
from workloads import bf16_bits_to_f32, config, make_llama_inputs

pytestmark = pytest.mark.gpu


def _session(name, seed):
    cfg = config(name)
    return cfg, H.GpuSession(cfg, make_llama_inputs(cfg, seed))


def _run(s, static, opts):
    s.out_slab.fill_(0xFF)
    s.place_inputs()
    rep = s.execute_static(opts) if static else s.execute(opts)
    return s.outputs()["y"].copy(), rep


def test_static_tables_give_the_bits_of_the_allocated_tables_on_two_calls_in_a_row():
    big_cfg, big = _session("c1", 0)               # 1438 memgraph vertices, fp32 kernels, 40 % cap
    small_cfg, small = _session("ragged_bf16", 1)  # 604 vertices, a smaller cap, bf16 MFMA kernels
    try:
        assert B.tn_memgraph_num_vertices(small.mg) < B.tn_memgraph_num_vertices(big.mg)
        assert big.stats.n_offload > 0 and small.stats.n_offload > 0 and small.cap < big.cap
        opts = B.tn_exec_opts(policy=B.TN_POLICY_RANDOM, order_seed=3, max_delay_us=50, delay_seed=4, queue_depth=3)
        ref_big, _ = _run(big, False, opts)
        ref_small, _ = _run(small, False, opts)
        print("[case] static tables: c1, then ragged_bf16, then c1 again", flush=True)
        import torch
        torch.cuda.synchronize()
        free0, _ = torch.cuda.mem_get_info()
        got_big, rep_big = _run(big, True, opts)
        got_small, rep_small = _run(small, True, opts)   # the region still holds the larger graph's tables
        np.testing.assert_array_equal(got_big, ref_big)
        np.testing.assert_array_equal(got_small, ref_small)
        assert rep_big.n_vertices == big.stats.n_vertices and rep_small.n_vertices == small.stats.n_vertices
        assert rep_big.n_offload == big.stats.n_offload
        # and back: the larger tables over the smaller ones, under another dispatch order and with timing on
        opts2 = B.tn_exec_opts(policy=B.TN_POLICY_LIFO, profile=1, queue_depth=2)
        again, rep = _run(big, True, opts2)
        np.testing.assert_array_equal(again, ref_big)
        assert rep.untimed_launches == 0 and rep.kernel_busy_ms > 0
        torch.cuda.synchronize()
        assert torch.cuda.mem_get_info()[0] == free0, "free GPU memory moved during the static calls"
        # the executor's own tables were not disturbed
        plain, _ = _run(big, False, opts)
        np.testing.assert_array_equal(plain, ref_big)
        # against the oracle as well (the bar of the parity tests)
        for cfg, s, y in ((big_cfg, big, got_big), (small_cfg, small, got_small)):
            full = make_llama_inputs(cfg, 0 if cfg is big_cfg else 1)
            own = T.build_llama_taskgraph(cfg)
            w = R.widen(cfg, full)
            y_tiled = T.assemble_outputs(own, T.evaluate(own, T.cut_inputs(own, w)), cfg.tokens, cfg.d_model)
            yy = (bf16_bits_to_f32(y) if cfg.dtype == "bf16" else y).astype(np.float64)
            assert R.rel_err(yy, y_tiled) < (2e-2 if cfg.dtype == "bf16" else 1e-4)
    finally:
        big.close()
        small.close()


def test_tables_larger_than_the_region_are_refused():
    import torch
    # a chain of 70 000 tiny additions: about 10 MB of descriptors and operand addresses
    tg = B.tn_taskgraph_create()
    mg = ex = None
    try:
        a = B.tn_taskgraph_add_input(tg, B.TN_F32, 8, 8, B.TN_HOST)
        v = a
        for _ in range(70_000):
            v = B.tn_taskgraph_add_op(tg, B.TN_OP_ADD, B.tn_op_params(), [v, a], B.TN_F32, 8, 8)
        B.tn_taskgraph_mark_output(tg, v)
        cap = 1 << 20
        mg = B.tn_compile(tg, None, cap, None)
        dev = torch.empty(cap, dtype=torch.uint8, device="cuda:0")
        streams = [torch.cuda.Stream(device="cuda:0") for _ in range(3)]
        h = [s.cuda_stream for s in streams]
        ex = B.tn_executor_create(mg, dev.data_ptr(), cap, 0, 0, h[:1], h[1], h[2])
        x = torch.ones(64, dtype=torch.float32).pin_memory()
        y = torch.zeros(64, dtype=torch.float32).pin_memory()
        ins = [0] * B.tn_taskgraph_num_vertices(tg)
        ins[a] = x.data_ptr()
        print("[case] static tables: 70 000-vertex chain is refused, then runs through tn_execute", flush=True)
        with pytest.raises(B.TurnipError) as e:
            B.tn_execute_static(ex, ins, [y.data_ptr()], None)
        assert e.value.status == B.TN_ERR_INVALID and "static table region" in str(e.value)
        # the refusal leaves the executor usable
        B.tn_execute(ex, ins, [y.data_ptr()], B.tn_exec_opts(max_batch=1, queue_depth=8))
        assert float(y[0]) == 70_001.0 and float(y[63]) == 70_001.0
    finally:
        if ex:
            torch.cuda.synchronize()
            B.tn_executor_destroy(ex)
        if mg:
            B.tn_memgraph_destroy(mg)
        B.tn_taskgraph_destroy(tg)
