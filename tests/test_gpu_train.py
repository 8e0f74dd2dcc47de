"""GPU parity of the fine-tuning step (forward with low-rank adapters on q and v, probe loss,
reverse pass through the frozen base weights) against the float64 oracle, under the memory cap."""
import numpy as np
import pytest

from oracle import llama_ref as R
from oracle import lora_ref as L
from paper_2405_16283_amd import binding as B
from paper_2405_16283_amd import harness as H
from workloads import bf16_bits_to_f32, config, make_llama_inputs, make_lora_inputs

pytestmark = pytest.mark.gpu
RANK = 16


def _f64(cfg, a):
    return (bf16_bits_to_f32(a) if cfg.dtype == "bf16" else a).astype(np.float64)


def _case(name, b_std, **session):
    cfg = config(name)
    full = make_llama_inputs(cfg, 0)
    full.update(make_lora_inputs(cfg, 0, rank=RANK, b_std=b_std))
    w = R.widen(cfg, full)
    lora = {k: a for k, a in w.items() if k.split(".")[0] in ("aq", "bq", "av", "bv")}
    y_ref, g_ref = L.loss_and_grads(cfg, w, lora, w["x"], w["probe"])
    s = H.GpuSession(cfg, full, lora_rank=RANK, train=True, **session)
    return cfg, s, y_ref, g_ref


@pytest.mark.parametrize("name,b_std,tol", [("c1", 0.02, 1e-4), ("c1", 0.0, 1e-4), ("ragged_f32", 0.02, 1e-4),
                                            ("batch2_f32", 0.02, 1e-4), ("ragged_bf16", 0.02, 4e-2),
                                            ("mid_bf16", 0.02, 4e-2)])
def test_adapter_gradients_match_the_oracle_under_the_cap(name, b_std, tol):
    cfg, s, y_ref, g_ref = _case(name, b_std)
    try:
        print(f"[case] {name} b_std {b_std}: cap {s.cap}, {s.stats.n_vertices} vertices, {s.stats.n_offload} offloads, "
              f"{s.stats.n_reload} reloads", flush=True)
        out, rep = s.run(B.tn_exec_opts(policy=B.TN_POLICY_RANDOM, order_seed=2, max_delay_us=50))
        assert rep.n_vertices == s.stats.n_vertices
        assert R.rel_err(_f64(cfg, out["y"]), y_ref) < tol
        errs = {}
        for l in range(cfg.layers):
            for k in ("aq", "bq", "av", "bv"):
                got, ref = _f64(cfg, out[f"d{k}.{l}"]), g_ref[f"{k}.{l}"]
                if b_std == 0.0 and k in ("aq", "av"):
                    assert not ref.any() and np.abs(got).max() == 0.0  # B = 0: the gradient of A vanishes identically
                    continue
                errs[f"d{k}.{l}"] = R.rel_err(got, ref)
        errs["dx"] = R.rel_err(_f64(cfg, out["dx"]), g_ref["x"])
        print("  " + ", ".join(f"{k} {v:.2e}" for k, v in errs.items()), flush=True)
        assert max(errs.values()) < tol, errs
        # another dispatch order: the same bits
        o2, _ = s.run(B.tn_exec_opts(policy=B.TN_POLICY_BY_ORDER, max_batch=1920, queue_depth=3))
        for k in out:
            np.testing.assert_array_equal(o2[k], out[k])
    finally:
        s.close()


@pytest.mark.parametrize("name", ["ragged_bf16", "mid_bf16"])
def test_twenty_dispatch_orders_of_the_fine_tuning_step_give_identical_bits(name):
    """The reverse pass through the MFMA kernels (attention statistics, dQ, dK, dV at head size 128; on
    mid_bf16 also the 256x256 tile products with ragged blocks and transposed operands) under the
    cap: any dependency-respecting order, group size, queue depth and transfer delay gives the same
    bits in y, dx and every adapter gradient."""
    cfg, s, y_ref, g_ref = _case(name, 0.02)
    try:
        assert s.stats.n_offload > 0
        ref, _ = s.run(B.tn_exec_opts(policy=B.TN_POLICY_BY_ORDER, max_batch=1))
        assert R.rel_err(_f64(cfg, ref["y"]), y_ref) < 4e-2 and R.rel_err(_f64(cfg, ref["dx"]), g_ref["x"]) < 4e-2
        orders = set()
        for seed in range(20):
            delay, batch, depth = (0, 50, 500)[seed % 3], (1, 4, 0)[(seed // 3) % 3], (1, 3, 8)[(seed // 2) % 3]
            print(f"[case] {name} train order_seed {seed} delay {delay} batch {batch} depth {depth}", flush=True)
            out, _ = s.run(B.tn_exec_opts(policy=B.TN_POLICY_RANDOM, order_seed=seed, delay_seed=100 + seed,
                                          max_delay_us=delay, max_batch=batch, queue_depth=depth))
            for k in ref:
                np.testing.assert_array_equal(out[k], ref[k])
            orders.add(tuple(s.last_order()))
        assert len(orders) >= 15
    finally:
        s.close()


@pytest.mark.parametrize("name,options", [("c1", dict(recompute_normed=True)), ("ragged_bf16", dict(recompute_normed=True)),
                                          ("c1", dict(recompute_gate_up=True)), ("ragged_bf16", dict(recompute_gate_up=True)),
                                          ("mid_bf16", dict(recompute_normed=True, recompute_gate_up=True)),
                                          ("ragged_bf16", dict(recompute_gate_up=True, checkpoint=True, checkpoint_layers=1))])
def test_recomputed_tensors_give_the_same_bits(name, options):
    """Tiler options recompute_normed and recompute_gate_up (the reverse pass forms the normalised layer input,
    or the gate and up products, again instead of keeping them): every output carries the bits of the step that
    kept them, in other dispatch orders too."""
    cfg, s, _, _ = _case(name, 0.02)
    try:
        want, _ = s.run(B.tn_exec_opts(policy=B.TN_POLICY_BY_ORDER, max_batch=1920, queue_depth=3))
        kept = s.stats.n_vertices
    finally:
        s.close()
    cfg, s, _, _ = _case(name, 0.02, **options)
    try:
        print(f"[case] {name} {options}: {s.stats.n_vertices} vertices ({kept} without), {s.stats.n_offload} offloads", flush=True)
        for seed in range(3):
            out, rep = s.run(B.tn_exec_opts(policy=B.TN_POLICY_RANDOM, order_seed=seed, max_delay_us=(0, 50)[seed % 2],
                                            max_batch=(1, 0, 7)[seed]))
            assert out.keys() == want.keys()
            for k in want:
                np.testing.assert_array_equal(out[k], want[k])
    finally:
        s.close()


@pytest.mark.parametrize("name,tol,first", [("c1", 1e-4, 0), ("batch2_f32", 1e-4, 0), ("ragged_bf16", 4e-2, 0),
                                            ("c1", 1e-4, 1), ("ragged_bf16", 4e-2, 1)])
def test_checkpointed_step_gives_the_same_bits_as_the_saved_activation_step(name, tol, first):
    """Activation checkpointing (Section 8, the fine-tuning experiment's setting): the layer's
    forward vertices run a second time before its reverse pass.  The kernels are deterministic, so
    every output must carry the bits of the step that saved its activations, and with them the
    oracle's gradients within the tolerance.  first > 0: only that many of the first layers are checkpointed,
    the others keep their saved activations."""
    cfg, s, y_ref, g_ref = _case(name, 0.02)
    try:
        want, _ = s.run(B.tn_exec_opts(policy=B.TN_POLICY_BY_ORDER, max_batch=1920, queue_depth=3))
    finally:
        s.close()
    cfg, s, _, _ = _case(name, 0.02, checkpoint=True, checkpoint_layers=first)
    try:
        print(f"[case] {name} checkpointed: cap {s.cap}, {s.stats.n_vertices} vertices, {s.stats.n_offload} offloads, "
              f"{s.stats.n_reload} reloads", flush=True)
        for seed in range(4):
            print(f"[case] {name} checkpointed order_seed {seed}", flush=True)
            out, rep = s.run(B.tn_exec_opts(policy=B.TN_POLICY_RANDOM, order_seed=seed, max_delay_us=(0, 50)[seed % 2],
                                            max_batch=(1, 0)[seed // 2]))
            assert rep.n_vertices == s.stats.n_vertices
            assert out.keys() == want.keys()
            for k in want:
                np.testing.assert_array_equal(out[k], want[k])
        assert R.rel_err(_f64(cfg, out["dx"]), g_ref["x"]) < tol
        for l in range(cfg.layers):
            for k in ("aq", "bq", "av", "bv"):
                assert R.rel_err(_f64(cfg, out[f"d{k}.{l}"]), g_ref[f"{k}.{l}"]) < tol
    finally:
        s.close()


@pytest.mark.parametrize("name,tol,checkpoint", [("c1", 1e-4, False), ("c1", 1e-4, True), ("ragged_bf16", 4e-2, True)])
def test_fine_tuning_step_with_k_split_projections(name, tol, checkpoint):
    """The tiler's options together: projections of the forward pass as partial products joined by
    sums (two per sum, so the order of the increments cannot matter), with and without
    checkpointing; gradients against the oracle, a second dispatch order bit for bit."""
    cfg, s, y_ref, g_ref = _case(name, 0.02, k_split=2, checkpoint=checkpoint)
    try:
        print(f"[case] {name} k_split 2 checkpoint {checkpoint}: {s.stats.n_increment} increments, {s.stats.n_offload} offloads", flush=True)
        assert s.stats.n_increment > 0 and s.stats.n_offload > 0
        out, rep = s.run(B.tn_exec_opts(policy=B.TN_POLICY_RANDOM, order_seed=1, max_delay_us=50))
        assert rep.n_vertices == s.stats.n_vertices
        assert R.rel_err(_f64(cfg, out["y"]), y_ref) < tol
        assert R.rel_err(_f64(cfg, out["dx"]), g_ref["x"]) < tol
        for l in range(cfg.layers):
            for k in ("aq", "bq", "av", "bv"):
                assert R.rel_err(_f64(cfg, out[f"d{k}.{l}"]), g_ref[f"{k}.{l}"]) < tol
        o2, _ = s.run(B.tn_exec_opts(policy=B.TN_POLICY_BY_ORDER, max_batch=1920, queue_depth=3))
        for k in out:
            np.testing.assert_array_equal(o2[k], out[k])
    finally:
        s.close()
