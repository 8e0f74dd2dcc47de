"""GPU parity of the fused product vertices (fuse_epilogues: the residual as a last operand of the product
before it; the gated pair of products with silu * up), through the C ABI, against the oracle's own fused
graph: small shapes on the generic kernel, the mid-size shapes on the 256-tile MFMA kernel, under caps that
offload, across dispatch orders.  (The one-layer workload at full size runs fused in test_gpu_c2.py, as the
benchmark tiles it.)"""
import numpy as np
import pytest

from oracle import llama_ref as R
from oracle import tiled as T
from paper_2405_16283_amd import binding as B
from paper_2405_16283_amd import harness as H
from workloads import bf16_bits_to_f32, config, make_llama_inputs

from test_gpu_backward_ops import Graph

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


def _as_f64(cfg, a):
    return (bf16_bits_to_f32(a) if cfg.dtype == "bf16" else a).astype(np.float64)


def _oracle(cfg, full, fuse):
    w = R.widen(cfg, full)
    own = T.build_llama_taskgraph(cfg, fuse_epilogues=fuse)
    return T.assemble_outputs(own, T.evaluate(own, T.cut_inputs(own, w)), cfg.tokens, cfg.d_model)


@pytest.mark.parametrize("name,fuse", [("ragged_f32", 3), ("batch2_f32", 1), ("ragged_bf16", 3), ("mid_bf16", 1),
                                       ("mid_bf16", 2), ("mid_bf16", 3), ("decode_f32", 3), ("decode_bf16", 3)])
def test_fused_forward_matches_the_oracle_under_the_cap(name, fuse):
    cfg = config(name)
    full = make_llama_inputs(cfg, 0)
    y_tiled = _oracle(cfg, full, fuse)
    print(f"[case] {name} fuse_epilogues {fuse}", flush=True)
    s = H.GpuSession(cfg, full, fuse_epilogues=fuse)
    try:
        assert s.stats.n_offload > 0, "cap must force offload"
        out, rep = s.run()
        y = _as_f64(cfg, out["y"])
        err = R.rel_err(y, y_tiled)
        print(f"  rel err vs the oracle's fused graph {err:.3e}; {rep.n_offload} offloads, {rep.n_launches} launches", flush=True)
        assert np.isfinite(y).all() and err < TOL[cfg.dtype]
        # other dispatch orders and group sizes: the same bits
        for seed in range(6):
            o2, _ = s.run(B.tn_exec_opts(policy=B.TN_POLICY_RANDOM, order_seed=seed, delay_seed=seed, max_delay_us=(0, 100)[seed % 2],
                                         max_batch=(1, 5, 0)[seed % 3], queue_depth=(1, 3)[seed % 2]))
            np.testing.assert_array_equal(o2["y"], out["y"])
    finally:
        s.close()


@pytest.mark.parametrize("mode", [1, 2])
@pytest.mark.parametrize("shape", [(256, 256, 64), (384, 640, 96), (300, 264, 32), (512, 1024, 128), (128, 136, 40),
                                   (128, 136, 64), (72, 40, 32), (40, 72, 32)])
def test_fused_product_vertex_alone(mode, shape):
    """One vertex of each fused mode on hand-built graphs, two k tiles, weights stored [out, in]: shapes the
    256-tile kernel takes whole, ragged in rows and columns and smaller than one tile (its clamped loads and
    guarded stores), and shapes that go to the generic kernel (K not a multiple of 32, fewer than 64 rows),
    against the oracle's vertex in float64."""
    m, n, k = shape
    rng = np.random.default_rng(m + n + mode)
    g = Graph("bf16")
    a = [g.inp(rng.standard_normal((m, k))) for _ in range(2)]
    b = [g.inp(rng.standard_normal((n, k)) / np.sqrt(2 * k)) for _ in range(2)]
    extra = [g.inp(rng.standard_normal((m, n)))] if mode == 1 else [g.inp(rng.standard_normal((n, k)) / np.sqrt(2 * k)) for _ in range(2)]
    ins = a + b + extra
    print(f"[case] fused gemm mode {mode} shape {shape}", flush=True)
    v = g.op(B.TN_OP_GEMM, [i[0] for i in ins], m, n, nk=2, trans_b=1, mode=mode)
    (got,) = g.run([v])
    ref = T._eval_vertex("gemm", dict(nk=2, trans_b=1, mode=mode), [i[1] for i in ins])
    err = R.rel_err(got, T.round_bf16(ref))
    print(f"  rel err after the bf16 store {err:.2e}", flush=True)
    assert err < 2.0 ** -7  # one bf16 rounding step where fp32 and float64 round apart, nothing more
