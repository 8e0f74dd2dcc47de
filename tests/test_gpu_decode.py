"""GPU parity of the decode memgraph (Section 9, limitations: generation with the number of steps
fixed beforehand): prefill, then single-row steps whose keys and values join the cache as
single-row tiles, compiled once under a cap that moves cached keys and values to the host and
back, against the oracle's decode (one row at a time against a growing cache)."""
import numpy as np
import pytest

from oracle import llama_ref as R
from oracle import tiled as T
from paper_2405_16283_amd import binding as B
from paper_2405_16283_amd import harness as H
from workloads import bf16_bits_to_f32, config, make_llama_inputs

from util import assemble_named, oracle_taskgraph

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


def _f64(cfg, a):
    return (bf16_bits_to_f32(a) if cfg.dtype == "bf16" else a).astype(np.float64)


@pytest.mark.parametrize("name,seed", [("decode_f32", 0), ("decode_f32", 1), ("decode_bf16", 0), ("decode_bf16", 1)])
def test_decode_steps_match_the_oracle_under_a_cap_that_moves_the_cache(name, seed):
    cfg = config(name)
    assert cfg.decode_steps >= 8
    full = make_llama_inputs(cfg, seed)
    w = R.widen(cfg, full)
    P, N = cfg.seq, cfg.decode_steps
    store = (lambda z: T.round_store(z, cfg.dtype))
    y_dec, kc, vc = R.decode(cfg, w, store=store)     # row by row, rounding where the tiled run stores
    y_exact, _, _ = R.decode(cfg, w)
    print(f"[case] {name} seed {seed}: prefill {P}, {N} steps", flush=True)
    s = H.GpuSession(cfg, full, kv_outputs=True)
    try:
        # the library's graph, run by the oracle's interpreter: same rounding points as the GPU run
        otg = oracle_taskgraph(s.tg)
        vals = T.evaluate(otg, T.cut_inputs(otg, w))
        y_tiled = assemble_named(otg, vals, "y", cfg.tokens, cfg.d_model)
        assert R.rel_err(y_tiled, y_dec) < (2.0 ** -6 if cfg.dtype == "bf16" else 1e-6)

        # the cap really moves cached keys and values out and back
        e = H.export_memgraph(s.mg)
        kv_vertices = {v for v, nm, *_ in H.bindings(s.tg) if nm.startswith(("k.", "v."))}
        back = [v for v in range(len(e["kind"])) if e["kind"][v] in ("reload", "load") and e["src"][v] in kv_vertices]
        decode_rows_back = [v for v in back if otg.shape[e["src"][v]][0] == 1 or otg.shape[e["src"][v]][1] == 1]
        print(f"  {s.stats.n_offload} offloads, {s.stats.n_reload} reloads; {len(back)} of the transfers bring cached K/V "
              f"back, {len(decode_rows_back)} of them single-row tiles of decode steps", flush=True)
        assert s.stats.n_offload > 0 and len(back) > 0

        out, rep = s.run()
        y = _f64(cfg, out["y"])
        assert y.shape == (P + N, cfg.d_model) and np.isfinite(y).all()
        err_all, err_dec = R.rel_err(y, y_tiled), R.rel_err(y[P:], y_tiled[P:])
        print(f"  y against the interpreted graph: all rows {err_all:.3e}, decode rows {err_dec:.3e}; decode rows against "
              f"the row-by-row oracle {R.rel_err(y[P:], y_dec[P:]):.3e}, against exact float64 {R.rel_err(y[P:], y_exact[P:]):.3e}",
              flush=True)
        assert err_all < TOL[cfg.dtype] and err_dec < TOL[cfg.dtype]
        assert R.rel_err(y[P:], y_dec[P:]) < TOL[cfg.dtype]
        for u in range(N):  # step by step: a late step must be as good as the first
            assert R.rel_err(y[P + u], y_dec[P + u]) < TOL[cfg.dtype], u
        # the caches at the end: every layer's keys and values, prefill rows and decode rows
        for l in range(cfg.layers):
            for nm, ref in ((f"k.{l}", kc[l]), (f"v.{l}", vc[l])):
                got = _f64(cfg, out[nm])
                assert got.shape == ref.shape
                err = R.rel_err(got[P:], ref[P:])
                assert R.rel_err(got, ref) < TOL[cfg.dtype] and err < TOL[cfg.dtype], nm
        assert rep.n_offload == s.stats.n_offload and rep.n_reload == s.stats.n_reload

        # other dispatch orders, transfers delayed: the same bits in every row and cache
        for order_seed in range(6):
            o2, _ = s.run(B.tn_exec_opts(policy=B.TN_POLICY_RANDOM, order_seed=order_seed, delay_seed=7 + order_seed,
                                         max_delay_us=(0, 50, 300)[order_seed % 3], max_batch=(1, 4, 0)[order_seed % 3],
                                         queue_depth=(1, 3)[order_seed % 2]))
            for nm in out:
                np.testing.assert_array_equal(o2[nm], out[nm])
    finally:
        s.close()
