"""Section 5: every tensor's place is fixed by the compile, so a run of the memgraph calls no
allocator.  What a test inside the process can see without trusting the library's own word is the
GPU's free memory as the driver reports it: it must not move over repeated runs, profiled or not,
with offloads and reloads going on.  (The per-call list of HIP functions a run makes comes from the
profiler's trace of the benchmark at two step counts, kept with the other profiles.)"""
import numpy as np
import pytest

from paper_2405_16283_amd import binding as B
from paper_2405_16283_amd import harness as H
from workloads import config, make_llama_inputs

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["c1", "ragged_bf16"])
def test_free_gpu_memory_does_not_move_while_memgraphs_run(name):
    import torch
    cfg = config(name)
    s = H.GpuSession(cfg, make_llama_inputs(cfg, 0))
    try:
        assert s.stats.n_offload > 0
        ref, _ = s.run(B.tn_exec_opts(profile=1))  # first run: lazy initialisations of the runtime happen here
        torch.cuda.synchronize()
        free0, _ = torch.cuda.mem_get_info()
        for k in range(12):
            print(f"[case] steady memory {name} run {k}", flush=True)
            opts = B.tn_exec_opts(policy=B.TN_POLICY_RANDOM, order_seed=k, profile=k % 2, queue_depth=1 + k % 4,
                                  max_delay_us=(0, 50)[k % 2], delay_seed=k, max_batch=(0, 1, 5)[k % 3])
            s.place_inputs()
            rep = s.execute(opts)
            assert rep.untimed_launches == 0
            torch.cuda.synchronize()
            free, _ = torch.cuda.mem_get_info()
            assert free == free0, f"free GPU memory moved by {free0 - free} bytes in run {k}"
        np.testing.assert_array_equal(s.outputs()["y"], ref["y"])
    finally:
        s.close()
