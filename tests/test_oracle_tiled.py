"""Pins for the oracle's tiled taskgraph interpreter (CPU only): the tiled evaluation equals the
untiled layer math, is independent of the execution order bit for bit, and its vertex kinds
reduce to the untiled routines on single tiles."""
import numpy as np
import pytest

from oracle import llama_ref as R
from oracle import tiled as T
from workloads import config, make_llama_inputs


def _random_topological_order(tg, rng):
    n = len(tg)
    indeg = [len(tg.inputs[v]) for v in range(n)]
    succ = [[] for _ in range(n)]
    for v in range(n):
        for u in tg.inputs[v]:
            succ[u].append(v)
    ready = [v for v in range(n) if indeg[v] == 0]
    out = []
    while ready:
        i = int(rng.integers(len(ready)))
        ready[i], ready[-1] = ready[-1], ready[i]
        v = ready.pop()
        out.append(v)
        for w in succ[v]:
            indeg[w] -= 1
            if indeg[w] == 0:
                ready.append(w)
    return out


@pytest.mark.parametrize("name", ["c1", "ragged_f32", "batch2_f32"])
def test_tiled_equals_untiled_fp32_storage(name):
    cfg = config(name)
    w = R.widen(cfg, make_llama_inputs(cfg, 0))
    y1 = R.forward(cfg, w)
    tg = T.build_llama_taskgraph(cfg)
    y2 = T.assemble_outputs(tg, T.evaluate(tg, T.cut_inputs(tg, w)), cfg.tokens, cfg.d_model)
    assert not np.isnan(y2).any()
    assert R.rel_err(y2, y1) < 2e-6  # fp32 rounding at every tensor boundary


def test_tiled_equals_untiled_without_storage_rounding(monkeypatch):
    cfg = config("ragged_f32")
    w = R.widen(cfg, make_llama_inputs(cfg, 1))
    monkeypatch.setattr(T, "round_store", lambda x, dtype: np.asarray(x, dtype=np.float64))
    tg = T.build_llama_taskgraph(cfg)
    y2 = T.assemble_outputs(tg, T.evaluate(tg, T.cut_inputs(tg, w)), cfg.tokens, cfg.d_model)
    assert R.rel_err(y2, R.forward(cfg, w)) < 1e-12  # only re-association is left


def test_bf16_storage_stays_close_to_untiled():
    cfg = config("ragged_bf16")
    w = R.widen(cfg, make_llama_inputs(cfg, 0))
    tg = T.build_llama_taskgraph(cfg)
    y2 = T.assemble_outputs(tg, T.evaluate(tg, T.cut_inputs(tg, w)), cfg.tokens, cfg.d_model)
    assert R.rel_err(y2, R.forward(cfg, w)) < 5e-2


@pytest.mark.parametrize("name", ["c1", "ragged_bf16"])
def test_every_order_gives_identical_bits(name):
    cfg = config(name)
    w = R.widen(cfg, make_llama_inputs(cfg, 2))
    tg = T.build_llama_taskgraph(cfg)
    tiles = T.cut_inputs(tg, w)
    ref = T.evaluate(tg, tiles)
    rng = np.random.default_rng(0)
    for _ in range(5):
        got = T.evaluate(tg, tiles, order=_random_topological_order(tg, rng))
        for v in tg.outputs:
            np.testing.assert_array_equal(got[v], ref[v])
    with pytest.raises(ValueError):
        T.evaluate(tg, tiles, order=list(range(len(tg)))[::-1])


def test_vertex_kinds_reduce_to_untiled_routines():
    rng = np.random.default_rng(5)
    hd = 8
    # rope on a tile of two heads starting at sequence position 7
    x = rng.standard_normal((5, 2 * hd))
    y = T._eval_vertex("rope", dict(pos0=7, col0=0, head_dim=hd, base=1e4), [x])
    for h in range(2):
        np.testing.assert_allclose(y[:, h * hd:(h + 1) * hd], R.rope(x[:, h * hd:(h + 1) * hd], 7 + np.arange(5), 1e4), rtol=1e-13)
    # a tile that starts in the middle of a head
    y2 = T._eval_vertex("rope", dict(pos0=7, col0=4, head_dim=hd, base=1e4), [x[:, 4:8]])
    np.testing.assert_allclose(y2, y[:, 4:8], rtol=1e-13)
    # blocked attention with partial/combine equals the one-shot routine
    n, bs = 12, 4
    q, k, v = (rng.standard_normal((n, hd)) for _ in range(3))
    full = R.causal_attention_head(q, k, v)
    for bi in range(n // bs):
        parts = []
        for bj in range(bi + 1):
            parts.append(T._eval_vertex("attn_block", dict(n_q_tiles=1, n_kv_tiles=1, n_col_tiles=1, head_dim=hd,
                                                            q_pos0=bi * bs, k_pos0=bj * bs, causal=(bi == bj),
                                                            scale=1 / np.sqrt(hd)),
                                        [q[bi * bs:(bi + 1) * bs], k[bj * bs:(bj + 1) * bs], v[bj * bs:(bj + 1) * bs]]))
        o = T._eval_vertex("attn_combine", dict(row0=0, col0=0, rows=bs, cols=hd, head_dim=hd, hpg=1), parts)
        np.testing.assert_allclose(o, full[bi * bs:(bi + 1) * bs], rtol=1e-12)
    # rms_stat over column tiles, then apply
    xs = rng.standard_normal((3, 10))
    g = rng.standard_normal(10)
    st = T._eval_vertex("rms_stat", dict(eps=1e-6, d=10), [xs[:, :4], xs[:, 4:]])
    ya = T._eval_vertex("rms_apply", {}, [xs[:, 4:], st, g[4:].reshape(1, -1)])
    np.testing.assert_allclose(ya, R.rmsnorm(xs, g, 1e-6)[:, 4:], rtol=1e-13)
    # gemm over k tiles
    a, b = rng.standard_normal((3, 10)), rng.standard_normal((10, 4))
    c = T._eval_vertex("gemm", dict(nk=2), [a[:, :6], a[:, 6:], b[:6], b[6:]])
    np.testing.assert_allclose(c, a @ b, rtol=1e-13)


def test_graph_sizes_match_the_workload_arithmetic():
    cfg = config("c1")
    tg = T.build_llama_taskgraph(cfg)
    kinds = {k: tg.kind.count(k) for k in set(tg.kind)}
    # per layer: 2 row blocks x (4+4+4+4+11+11+4) gemm output tiles = 84; 3 of 4 causal block pairs x 4 heads
    assert kinds["gemm"] == 2 * 84
    assert kinds["attn_block"] == 2 * 3 * 4
    assert kinds["input"] == 2 * 4 + 2 * (196 + 8)
    assert len(tg.outputs) == 8
