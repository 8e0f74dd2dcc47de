"""GPU parity of the fine-tuning workload c5 at its real widths (LLaMA-7B shape, bf16, rank-16
adapters on q and v, 4096-token sequences, saved activations offloaded for the reverse pass).

One layer on one sequence is small enough for the float64 oracle to differentiate, so every
gradient of that slice is compared element by element, under a cap that forces offloads.  At
these widths the largest of 16.7 million bf16 errors exceeds the small-shape bar, so the bar is
the oracle's own: its form with bf16 storage rounding shows how far a correct bf16 pipeline
stands from the exact gradients, and the GPU result has to be as close (within NOISE_FACTOR).  The
whole 32-layer, 4-sequence step is beyond the oracle; there the test runs the configuration the
benchmark times and checks what can be known without it: the first rows of the final hidden
state (causal attention: they depend on the first rows of the input alone, and with B = 0 the
adapters do not change the forward pass), the gradient of A (identically zero while B = 0), the
byte counts of the transfers, finiteness, and the same bits under another dispatch order.
"""
import time

import numpy as np
import pytest

from oracle import llama_ref as R
from oracle import lora_ref as L
from oracle import tiled as T
from paper_2405_16283_amd import binding as B
from paper_2405_16283_amd import harness as H
from workloads import bf16_bits_to_f32, config, make_llama_inputs, make_lora_inputs

from util import check_layer_rows

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(1500)]
RANK = 16
NOISE_FACTOR = 1.5  # see test_gpu_deep: distance to the exact result, relative to the bf16 oracle's own


def _f64(a):
    return bf16_bits_to_f32(a).astype(np.float64)


def test_one_layer_one_sequence_matches_the_oracle_under_a_cap_that_forces_offloads():
    cfg = config("c5").with_(layers=1, batch=1, cap_bytes=0, cap_frac=0.40)
    t0 = time.time()
    full = make_llama_inputs(cfg, 0, workers=16)
    full.update(make_lora_inputs(cfg, 0, rank=RANK, b_std=0.02))
    w = R.widen(cfg, full)
    lora = {k: a for k, a in w.items() if k.split(".")[0] in ("aq", "bq", "av", "bv")}
    y_ref, g_ref = L.loss_and_grads(cfg, w, lora, w["x"], w["probe"])
    # how far a bf16 pipeline of this depth and width stands from the exact result: the oracle
    # with every stored tensor (and the gradient arriving at it) rounded to bf16
    y_b, g_b = L.loss_and_grads(cfg, w, lora, w["x"], w["probe"], storage="bf16")
    print(f"[c5 layer] oracle done {time.time() - t0:.1f}s", flush=True)
    s = H.GpuSession(cfg, full, lora_rank=RANK, train=True)
    try:
        print(f"[c5 layer] cap {s.cap}, {s.stats.n_vertices} vertices, {s.stats.n_offload} offloads, "
              f"{s.stats.n_reload} reloads {time.time() - t0:.1f}s", flush=True)
        assert s.stats.n_offload > 0
        out, rep = s.run(B.tn_exec_opts(policy=B.TN_POLICY_BY_ORDER, max_batch=1920, max_gemm_inflight=1, queue_depth=3))
        assert rep.n_vertices == s.stats.n_vertices

        def rms_err(a, b):
            return float(np.sqrt(np.mean((a - b) ** 2)) / np.sqrt(np.mean(b ** 2)))

        cases = [("y", _f64(out["y"]), y_b, y_ref), ("dx", _f64(out["dx"]), g_b["x"], g_ref["x"])]
        for k in ("aq", "bq", "av", "bv"):
            cases.append((f"d{k}", _f64(out[f"d{k}.0"]), g_b[f"{k}.0"], g_ref[f"{k}.0"]))
        for name, got, noisy, exact in cases:
            max_o, max_g = R.rel_err(noisy, exact), R.rel_err(got, exact)
            rms_o, rms_g = rms_err(noisy, exact), rms_err(got, exact)
            print(f"[c5 layer] {name}: max-measure oracle(bf16) vs exact {max_o:.3e}, gpu vs exact {max_g:.3e}; "
                  f"rms {rms_o:.3e}, {rms_g:.3e}", flush=True)
            assert max_g < NOISE_FACTOR * max_o and rms_g < NOISE_FACTOR * rms_o, name
        o2, _ = s.run(B.tn_exec_opts(policy=B.TN_POLICY_RANDOM, order_seed=3, max_batch=64, delay_seed=3, max_delay_us=50))
        for k in out:
            np.testing.assert_array_equal(o2[k], out[k])
    finally:
        s.close()


def test_full_step_in_the_benchmark_configuration():
    cfg = config("c5")
    PREFIX, distinct = 16, 4
    last = cfg.layers - 1
    t0 = time.time()
    full = make_llama_inputs(cfg, 0, distinct_layers=distinct, workers=16)
    full.update(make_lora_inputs(cfg, 0, rank=RANK, b_std=0.0))
    print(f"[c5] inputs generated {time.time() - t0:.1f}s", flush=True)
    stride = 8  # hidden states of pairs of neighbouring layers through the depth of the stack are outputs
    probe = [0] + [l for l in range(stride, cfg.layers - 1, stride)] + [last]
    s = H.GpuSession(cfg, full, lora_rank=RANK, train=True, compile_opts=H.bench_compile_opts(cfg.cap_bytes, True), n_compute=H.BENCH_COMPUTE_STREAMS,
                     hidden_outputs=True, output_layer_stride=stride,
                     progress=lambda m: print(f"[c5] {m} {time.time() - t0:.1f}s", flush=True))
    st = s.stats
    print(f"[c5] compiled and placed {time.time() - t0:.1f}s: {st.n_vertices} vertices, {st.n_load} loads "
          f"({st.load_bytes / 1e9:.1f} GB), {st.n_offload} offloads ({st.offload_bytes / 1e9:.1f} GB)", flush=True)
    try:
        assert st.n_offload > 0 and st.high_water <= cfg.cap_bytes
        names = ["y", "dx", "daq.0", "dbq.0", "dav.0", "dbv.0", f"daq.{last}", f"dbq.{last}", f"dav.{last}", f"dbv.{last}"]
        names += [f"h.{l}" for l in probe if l != last] + [f"h.{l - 1}" for l in probe if l > 0]
        opts = B.tn_exec_opts(policy=B.TN_POLICY_BY_ORDER, max_batch=1920, max_gemm_inflight=1, queue_depth=3,
                              small_gemm_tiles=-1)  # the launch configuration the benchmark times this workload in
        out, rep = s.run(opts, only=names)
        print(f"[c5] executed in {rep.wall_ms:.1f} ms ({cfg.tokens / rep.wall_ms * 1e3:.0f} tokens/s), "
              f"h2d {rep.h2d_bytes / 1e9:.2f} GB, d2h {rep.d2h_bytes / 1e9:.2f} GB {time.time() - t0:.1f}s", flush=True)
        assert rep.n_vertices == st.n_vertices
        assert rep.h2d_bytes == st.load_bytes + st.reload_bytes
        assert rep.d2h_bytes == st.offload_bytes + st.store_bytes
        for n in names:
            assert np.isfinite(bf16_bits_to_f32(out[n])).all(), n
        for n in names:
            if n.startswith(("daq", "dav")):
                assert np.abs(bf16_bits_to_f32(out[n])).max() == 0.0, n  # B = 0: no gradient reaches A
            elif n != "y":
                assert np.abs(bf16_bits_to_f32(out[n])).max() > 0.0, n

        # forward result on the first rows of the first and the last sequence
        wide = {}

        def layer_weights(l):
            w = {}
            for k, a in full.items():
                if k.endswith(f".{l}") and k.split(".")[0] in ("wq", "wk", "wv", "wo", "w1", "w2", "w3", "g1", "g2"):
                    if id(a) not in wide:
                        wide[id(a)] = R.widen_array(a)
                    w[k] = wide[id(a)]
            return w

        # Forward pass layer by layer at the one-layer tolerance (B = 0: the adapters add nothing to it):
        # the GPU's own input rows of a layer, the first 32 positions of the first and the last sequence,
        # through one oracle layer with the storage rounding of the tiled execution
        for l in probe:
            for b in (0, cfg.batch - 1):
                check_layer_rows(cfg, full, out, l, b, np.arange(32), 2e-2, False, "[c5]", wide)
        print(f"[c5] layers {probe} checked one by one {time.time() - t0:.1f}s", flush=True)

        def rms_err(a, b):
            return float(np.sqrt(np.mean((a - b) ** 2)) / np.sqrt(np.mean(b ** 2)))

        pcfg = cfg.with_(seq=PREFIX, batch=1)
        tgp = T.build_llama_taskgraph(pcfg)
        for b in (0, cfg.batch - 1):
            rows = slice(b * cfg.seq, b * cfg.seq + PREFIX)
            y_exact = R.widen_array(full["x"][rows])
            for l in range(cfg.layers):
                y_exact = R.decoder_layer(y_exact, layer_weights(l), l, cfg.n_heads, cfg.head_dim, cfg.eps, cfg.rope_base)
            pfull = {k: a for k, a in full.items() if k.split(".")[0] in ("wq", "wk", "wv", "wo", "w1", "w2", "w3", "g1", "g2")}
            pfull["x"] = full["x"][rows]
            vals = T.evaluate(tgp, T.LazyInputs(tgp, pfull, R.widen_array, cache_bytes=16 << 30))
            y_tiled = T.assemble_outputs(tgp, vals, PREFIX, cfg.d_model)
            y_gpu = _f64(out["y"][rows])
            max_o, max_g = R.rel_err(y_tiled, y_exact), R.rel_err(y_gpu, y_exact)
            rms_o, rms_g = rms_err(y_tiled, y_exact), rms_err(y_gpu, y_exact)
            print(f"[c5] sequence {b}, first {PREFIX} rows of y after {cfg.layers} layers: max-measure oracle(bf16) vs exact "
                  f"{max_o:.3e}, gpu vs exact {max_g:.3e}; rms {rms_o:.3e}, {rms_g:.3e} {time.time() - t0:.1f}s", flush=True)
            assert rms_g < NOISE_FACTOR * rms_o and max_g < NOISE_FACTOR * max_o

        o2, rep2 = s.run(B.tn_exec_opts(policy=B.TN_POLICY_RANDOM, order_seed=1, max_batch=64, delay_seed=1,
                                        max_delay_us=50, queue_depth=1), only=names)
        print(f"[c5] random order executed in {rep2.wall_ms:.1f} ms {time.time() - t0:.1f}s", flush=True)
        for n in names:
            np.testing.assert_array_equal(o2[n], out[n])
    finally:
        s.close()
    # The same step as the benchmark compiles it by default: the normalised layer inputs and the gate and up
    # products are formed again in the reverse pass instead of kept, which leaves nothing to offload under this
    # cap; two groups of tile products in flight.  Every output carries the bits of the step above.
    import gc
    gc.collect()
    lean, regate = H.BENCH_RECOMPUTE_NORMED.get("c5", False), H.BENCH_RECOMPUTE_GATE_UP.get("c5", False)
    if not (lean or regate):
        return
    s = H.GpuSession(cfg, full, lora_rank=RANK, train=True, compile_opts=H.bench_compile_opts(cfg.cap_bytes, True),
                     n_compute=H.BENCH_COMPUTE_STREAMS, hidden_outputs=True, output_layer_stride=stride,
                     recompute_normed=lean, recompute_gate_up=regate)
    try:
        print(f"[c5] recompute options: {s.stats.n_vertices} vertices, {s.stats.n_offload} offloads "
              f"({s.stats.offload_bytes / 1e9:.1f} GB) {time.time() - t0:.1f}s", flush=True)
        assert s.stats.offload_bytes < st.offload_bytes and s.stats.high_water <= cfg.cap_bytes
        o3, rep3 = s.run(B.tn_exec_opts(policy=B.TN_POLICY_BY_ORDER, max_batch=1920, max_gemm_inflight=2, queue_depth=3,
                                        small_gemm_tiles=-1), only=names)
        print(f"[c5] executed in {rep3.wall_ms:.1f} ms ({cfg.tokens / rep3.wall_ms * 1e3:.0f} tokens/s) {time.time() - t0:.1f}s", flush=True)
        for n in names:
            np.testing.assert_array_equal(o3[n], out[n])
    finally:
        s.close()
