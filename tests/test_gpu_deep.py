"""GPU parity on the deep workloads, whose weights live in host memory and are streamed in under
the cap: c3 (32 LLaMA-7B-shaped layers, 16384 tokens, 16 GB, K/V of every layer and the final
hidden state as outputs) and c4 (80 LLaMA-65B-shaped layers, 8192 tokens, 48 GB).

The CPU oracle cannot run these models on all tokens, but attention is causal and every other
step works row by row, so the first rows of the output depend on the first rows of the input
alone: the oracle runs the same model on a prefix and must agree with the prefix of the GPU
result.  Properties that hold at any size cover the rest: nothing non-finite, the byte counts of
the transfers, and the same bits under another dispatch order.

Layers share weights (layer l reads the arrays of layer l mod k) to keep generation time and
pinned memory small; shapes, vertex count and transfers are those of distinct layers.
"""
import time

import numpy as np
import pytest

from oracle import llama_ref as R
from oracle import tiled as T
from paper_2405_16283_amd import binding as B
from paper_2405_16283_amd import harness as H
from workloads import bf16_bits_to_f32, config, make_llama_inputs

from util import check_layer_rows

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(1500)]

# Through {cfg.layers} layers a bf16 pipeline drifts from the exact result by far more than the one-layer
# bound: each side rounds every tensor to bf16, a last-bit difference in one layer perturbs the
# next, and after a few layers the rounding decisions of two correct bf16 implementations are
# unrelated.  The oracle itself shows how large that drift is: its tiled, bf16-rounding form is
# compared with its exact float64 form, and the GPU result has to be as close to the exact one
# as that (within this factor), in the root-mean-square and in the maximum measure.
NOISE_FACTOR = 1.5


def _f64(a):
    return bf16_bits_to_f32(a).astype(np.float64)


@pytest.mark.parametrize("name,PREFIX,distinct,stride", [("c3", 256, 4, 8), ("c4", 16, 2, 20)])
def test_prefix_matches_the_oracle_and_orders_agree(name, PREFIX, distinct, stride):
    kv = True
    cfg = config(name)
    last = cfg.layers - 1
    t0 = time.time()
    full = make_llama_inputs(cfg, 0, distinct_layers=distinct, workers=16)
    print(f"[{name}] inputs generated {time.time() - t0:.1f}s", flush=True)
    # K/V and the hidden state of pairs of neighbouring layers through the depth of the stack are outputs
    # the serial order, attention tiling and fused epilogues the benchmark compiles this workload with
    whole_rows, fuse = H.BENCH_WHOLE_ROWS.get(name, False), H.BENCH_FUSE.get(name, 0)
    s = H.GpuSession(cfg, full, kv_outputs=kv, hidden_outputs=True, output_layer_stride=stride,
                     order=H.BENCH_ORDER.get(name), attn_whole_rows=whole_rows, fuse_epilogues=fuse)
    probe = [0] + [l for l in range(stride, cfg.layers - 1, stride)] + [last]  # layers checked one by one
    print(f"[{name}] compiled and placed {time.time() - t0:.1f}s: {s.stats.n_vertices} vertices, "
          f"{s.stats.n_load} loads, {s.stats.n_offload} offloads, {s.stats.n_store} stores", flush=True)
    try:
        names = ["y"] + [f"{t}.{l}" for l in probe for t in ("k", "v")] + [f"h.{l}" for l in probe if l != last] \
            + [f"h.{l - 1}" for l in probe if l > 0]
        opts = B.tn_exec_opts(policy=B.TN_POLICY_BY_ORDER, max_batch=1920, max_gemm_inflight=1, queue_depth=3)
        if name == "c4":  # the launch configuration the benchmark times this workload in
            opts.max_transfers, opts.copy_workgroups, opts.small_gemm_tiles = 128, 14, -1
        out, rep = s.run(opts, only=names)
        print(f"[{name}] executed in {rep.wall_ms:.1f} ms ({cfg.tokens / rep.wall_ms * 1e3:.0f} tokens/s), "
              f"h2d {rep.h2d_bytes / 1e9:.2f} GB, d2h {rep.d2h_bytes / 1e9:.2f} GB {time.time() - t0:.1f}s", flush=True)
        assert rep.n_vertices == s.stats.n_vertices
        assert rep.h2d_bytes == s.stats.load_bytes + s.stats.reload_bytes
        for n in names:
            assert np.isfinite(bf16_bits_to_f32(out[n])).all(), n

        # layer 0: K (after the rotation) and V of the prefix against the untiled definition
        wide = {}  # layers that share their arrays share the float64 copy

        def layer_weights(l):
            w = {}
            for k, a in full.items():
                if k.endswith(f".{l}") and k != "x":
                    if id(a) not in wide:
                        wide[id(a)] = R.widen_array(a)
                    w[k] = wide[id(a)]
            return w

        x = R.widen_array(full["x"][:PREFIX])
        if kv:
            _, k0, v0 = R.decoder_layer(x, layer_weights(0), 0, cfg.n_heads, cfg.head_dim, cfg.eps, cfg.rope_base,
                                        return_kv=True)
            for tensor, ref in (("k.0", k0), ("v.0", v0)):
                err = R.rel_err(_f64(out[tensor][:PREFIX]), ref)
                print(f"[{name}] {tensor} prefix rel err {err:.3e}", flush=True)
                assert err < 2e-2

        # Layer by layer at the one-layer tolerance: the GPU's own input rows of a layer through one
        # oracle layer (storage rounding as in the tiled execution); late rows attend to the GPU's
        # stored keys and values of that layer, which are held to the same bar on those rows
        rng = np.random.default_rng(11)
        rows = np.unique(np.concatenate([np.arange(8), rng.integers(8, cfg.seq - 8, size=8), np.arange(cfg.seq - 8, cfg.seq)]))
        for l in probe:
            check_layer_rows(cfg, full, out, l, 0, rows, 2e-2, True, f"[{name}]", wide, fuse_epilogues=fuse)
        print(f"[{name}] layers {probe} checked one by one {time.time() - t0:.1f}s", flush=True)

        # the whole stack on the prefix: exact (float64, untiled), and tiled with the GPU path's
        # rounding points
        y_exact = x
        for l in range(cfg.layers):
            y_exact = R.decoder_layer(y_exact, layer_weights(l), l, cfg.n_heads, cfg.head_dim, cfg.eps, cfg.rope_base)
        print(f"[{name}] exact prefix forward done {time.time() - t0:.1f}s", flush=True)
        pcfg = cfg.with_(seq=PREFIX)
        tgp = T.build_llama_taskgraph(pcfg, attn_whole_rows=whole_rows, fuse_epilogues=fuse)
        pfull = dict(full)
        pfull["x"] = full["x"][:PREFIX]
        vals = T.evaluate(tgp, T.LazyInputs(tgp, pfull, R.widen_array, cache_bytes=16 << 30))
        y_tiled = T.assemble_outputs(tgp, vals, PREFIX, cfg.d_model)
        y_gpu = _f64(out["y"][:PREFIX])

        def rms_err(a, b):
            return float(np.sqrt(np.mean((a - b) ** 2)) / np.sqrt(np.mean(b ** 2)))

        max_o, max_g, max_go = R.rel_err(y_tiled, y_exact), R.rel_err(y_gpu, y_exact), R.rel_err(y_gpu, y_tiled)
        rms_o, rms_g = rms_err(y_tiled, y_exact), rms_err(y_gpu, y_exact)
        print(f"[{name}] y prefix ({PREFIX} rows, {cfg.layers} layers): max-measure oracle(bf16) vs exact {max_o:.3e}, "
              f"gpu vs exact {max_g:.3e}, gpu vs oracle(bf16) {max_go:.3e}; rms oracle(bf16) vs exact {rms_o:.3e}, "
              f"gpu vs exact {rms_g:.3e} {time.time() - t0:.1f}s", flush=True)
        assert rms_g < NOISE_FACTOR * rms_o and max_g < NOISE_FACTOR * max_o

        # another dispatch order, transfers delayed: same bits everywhere we look
        o2, rep2 = s.run(B.tn_exec_opts(policy=B.TN_POLICY_RANDOM, order_seed=1, max_batch=64, delay_seed=1,
                                        max_delay_us=50, queue_depth=1), only=names)
        print(f"[{name}] random order executed in {rep2.wall_ms:.1f} ms {time.time() - t0:.1f}s", flush=True)
        for n in names:
            np.testing.assert_array_equal(o2[n], out[n])
    finally:
        s.close()
