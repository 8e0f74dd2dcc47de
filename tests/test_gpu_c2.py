"""GPU parity at the benchmark's full size (one LLaMA-7B-shaped layer, seq 4096, bf16) and in the
launch configuration bench.py times: whole output against the tiled CPU oracle, identical bits
across dispatch orders, and the offload path at 40 % of the uncapped peak."""
import numpy as np
import pytest

from oracle import llama_ref as R
from oracle import tiled as T
from paper_2405_16283_amd import binding as B
from paper_2405_16283_amd import harness as H
from workloads import bf16_bits_to_f32, config, make_llama_inputs

pytestmark = pytest.mark.gpu


FUSE = H.BENCH_FUSE.get("c2", 0)  # the benchmark tiles this workload with fused epilogues


def _case(seed, fuse=FUSE):
    cfg = config("c2")
    full = make_llama_inputs(cfg, seed)
    w = R.widen(cfg, full)
    tg = T.build_llama_taskgraph(cfg, fuse_epilogues=fuse)
    y = T.assemble_outputs(tg, T.evaluate(tg, T.cut_inputs(tg, w)), cfg.tokens, cfg.d_model)
    return cfg, full, y


@pytest.fixture(scope="module")
def c2():
    return _case(0)


@pytest.fixture(scope="module")
def c2_plain():
    return _case(0, 0) if FUSE else None


def bench_opts(**kw):
    return B.tn_exec_opts(policy=B.TN_POLICY_BY_ORDER, max_batch=1920, max_gemm_inflight=1, queue_depth=3, **kw)


def test_c2_bench_configuration_matches_the_oracle_everywhere(c2):
    cfg, full, y_oracle = c2
    print("[case] c2 full size, bench configuration", flush=True)
    s = H.GpuSession(cfg, full, n_compute=H.BENCH_COMPUTE_STREAMS, device_outputs=True, fuse_epilogues=FUSE)  # as bench.py runs it
    try:
        out, rep = s.run(bench_opts())
        y = bf16_bits_to_f32(out["y"]).astype(np.float64)
        err = R.rel_err(y, y_oracle)
        print(f"  rel err vs tiled oracle over all {y.size} outputs: {err:.3e}", flush=True)
        assert np.isfinite(y).all() and err < 2e-2
        assert rep.n_vertices == s.stats.n_vertices
        # other dispatch orders, group sizes and copy engines: same bits
        for seed, (batch, engine) in enumerate([(64, B.TN_COPY_KERNEL), (7, B.TN_COPY_MEMCPY), (240, B.TN_COPY_AUTO)]):
            print(f"[case] c2 random order seed {seed} batch {batch}", flush=True)
            o2, _ = s.run(B.tn_exec_opts(policy=B.TN_POLICY_RANDOM, order_seed=seed, max_batch=batch, copy_engine=engine,
                                         delay_seed=seed, max_delay_us=100))
            np.testing.assert_array_equal(o2["y"], out["y"])
    finally:
        s.close()


@pytest.mark.parametrize("seed", [1, 2])
def test_c2_other_seeds_match_the_oracle_everywhere(seed):
    """The bar is 2e-2 over all 16.7 M outputs; the margin is printed for every seed."""
    cfg, full, y_oracle = _case(seed)
    print(f"[case] c2 full size, seed {seed}", flush=True)
    s = H.GpuSession(cfg, full, n_compute=H.BENCH_COMPUTE_STREAMS, device_outputs=True, fuse_epilogues=FUSE)
    try:
        out, rep = s.run(bench_opts())
        y = bf16_bits_to_f32(out["y"]).astype(np.float64)
        err = R.rel_err(y, y_oracle)
        print(f"  seed {seed}: rel err vs tiled oracle over all {y.size} outputs: {err:.3e} (bar 2e-2)", flush=True)
        assert np.isfinite(y).all() and err < 2e-2
    finally:
        s.close()


@pytest.mark.parametrize("percent,order", [(40, "clustered"), (25, "clustered"), (40, "level")])
def test_c2_streamed_under_a_fraction_of_its_peak_gives_the_same_bits(c2, c2_plain, percent, order):
    """The benchmark's capped runs of the one-layer workload (everything streamed from the host; cap 40 % and
    25 % of the uncapped peak, clustered serial order, epilogues fused as the benchmark has them) and the level
    order at 40 %, which offloads: the oracle's result at the one-layer bar, and the same bits in another order."""
    fuse = H.BENCH_FUSE.get(f"c2_capped{percent}", 0) if order == "clustered" else 0
    cfg, full, y_oracle = c2 if fuse == FUSE else c2_plain
    capped = cfg.with_(cap_bytes=0, cap_frac=percent / 100.0, weights_resident=False, x_resident=False)
    print(f"[case] c2 streamed, cap = {percent} % of the uncapped peak, serial order {order}, fuse_epilogues {fuse}", flush=True)
    tg = B.tn_build_llama(H.llama_config_struct(capped, fuse_epilogues=fuse))
    cap = H.cap_for(capped, tg)
    B.tn_taskgraph_destroy(tg)
    # the serial order, compile options and stream count of the benchmark's capped runs
    s = H.GpuSession(capped, full, cap=cap, compile_opts=H.bench_compile_opts(cap, False, pressed=True),
                     n_compute=H.BENCH_COMPUTE_STREAMS, order=order, fuse_epilogues=fuse)
    try:
        print(f"  {s.stats.n_offload} offloads, {s.stats.n_load} loads", flush=True)
        assert s.stats.n_load > 0 and s.stats.high_water <= cap
        assert (s.stats.n_offload > 0) == (percent == 25 or order == "level")
        # the benchmark's transfer options for these runs (and, under 40 %, no 128x128 launch form)
        out, rep = s.run(bench_opts(max_transfers=32, copy_workgroups=16, small_gemm_tiles=-1 if percent == 40 else 0))
        y = bf16_bits_to_f32(out["y"]).astype(np.float64)
        assert R.rel_err(y, y_oracle) < 2e-2
        assert rep.n_offload == s.stats.n_offload and (rep.arena_high_water > 0) == (s.stats.n_offload > 0)
        o2, _ = s.run(B.tn_exec_opts(policy=B.TN_POLICY_RANDOM, order_seed=11, max_batch=32, max_delay_us=200))
        np.testing.assert_array_equal(o2["y"], out["y"])
    finally:
        s.close()
