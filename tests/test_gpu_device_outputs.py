"""Results that stay on the GPU, and inputs that are already there: the buffers handed to
tn_execute and tn_executor_place_inputs lie in GPU memory outside the capped device buffer, so
the store and load vertices are copies inside GPU memory.  The bits must be those of the run that
goes through pinned host memory, with either copy engine, and the oracle's."""
import numpy as np
import pytest

from oracle import llama_ref as R
from oracle import tiled as T
from paper_2405_16283_amd import binding as B
from paper_2405_16283_amd import harness as H
from workloads import bf16_bits_to_f32, config, make_llama_inputs

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,tol", [("c1", 1e-4), ("ragged_bf16", 2e-2)])
def test_outputs_in_gpu_memory_carry_the_same_bits(name, tol):
    cfg = config(name)
    full = make_llama_inputs(cfg, 0)
    tg = T.build_llama_taskgraph(cfg)
    ref = T.assemble_outputs(tg, T.evaluate(tg, T.cut_inputs(tg, R.widen(cfg, full))), cfg.tokens, cfg.d_model)
    s = H.GpuSession(cfg, full, kv_outputs=True)
    try:
        want, _ = s.run(B.tn_exec_opts(policy=B.TN_POLICY_BY_ORDER, max_batch=64))
    finally:
        s.close()
    s = H.GpuSession(cfg, full, kv_outputs=True, device_outputs=True)
    try:
        assert s.out_slab.is_cuda and s.stats.n_offload > 0
        for engine in (B.TN_COPY_AUTO, B.TN_COPY_KERNEL, B.TN_COPY_MEMCPY, B.TN_COPY_KERNEL_IN):
            for seed in (0, 1):
                print(f"[case] {name} device outputs, copy engine {engine}, order_seed {seed}", flush=True)
                out, rep = s.run(B.tn_exec_opts(policy=B.TN_POLICY_RANDOM, order_seed=seed, copy_engine=engine,
                                                max_delay_us=50 * seed))
                assert rep.n_vertices == s.stats.n_vertices and out.keys() == want.keys()
                for k in want:
                    np.testing.assert_array_equal(out[k], want[k])
        y = (bf16_bits_to_f32(out["y"]) if cfg.dtype == "bf16" else out["y"]).astype(np.float64)
        assert R.rel_err(y, ref) < tol
    finally:
        s.close()


@pytest.mark.parametrize("resident", [False, True])
def test_inputs_in_gpu_memory_carry_the_same_bits(resident):
    """resident=False: every input is a load vertex reading GPU memory; True: the inputs are placed
    by tn_executor_place_inputs from GPU memory."""
    cfg = config("ragged_bf16").with_(weights_resident=resident, x_resident=resident)
    full = make_llama_inputs(cfg, 0)
    cap = 64 << 20 if resident else None  # resident inputs alone exceed the workload's own 40 % cap
    s = H.GpuSession(cfg, full, cap=cap)
    try:
        want, _ = s.run(B.tn_exec_opts(policy=B.TN_POLICY_BY_ORDER, max_batch=64))
    finally:
        s.close()
    s = H.GpuSession(cfg, full, cap=cap, device_inputs=True, device_outputs=True)
    try:
        assert s.in_slab.is_cuda and s.out_slab.is_cuda
        assert (s.stats.n_load == 0) == resident
        for engine in (B.TN_COPY_AUTO, B.TN_COPY_MEMCPY):
            print(f"[case] ragged_bf16 inputs in GPU memory, resident {resident}, copy engine {engine}", flush=True)
            out, rep = s.run(B.tn_exec_opts(policy=B.TN_POLICY_RANDOM, order_seed=3, copy_engine=engine))
            assert rep.n_vertices == s.stats.n_vertices
            np.testing.assert_array_equal(out["y"], want["y"])
    finally:
        s.close()


def test_an_output_buffer_inside_the_device_buffer_is_refused():
    """The host-side check turns the mistake into an error before anything is launched."""
    cfg = config("c1")
    full = make_llama_inputs(cfg, 0)
    s = H.GpuSession(cfg, full, device_outputs=True)
    try:
        bad = list(s.out_ptrs)
        bad[0] = s.dev.data_ptr() + 256  # inside the capped buffer the memgraph's locations refer to
        s.place_inputs()
        with pytest.raises(B.TurnipError, match="overlaps"):
            B.tn_execute(s.ex, s.in_ptrs, B.ptr_array(bad), None)
        out, rep = s.run()  # the executor is still usable
        assert rep.n_vertices == s.stats.n_vertices
    finally:
        s.close()
