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


def test_fused_gemm_modes_are_the_separate_vertices_in_one():
    """Mode 1 (the product plus a residual operand) and mode 2 (silu(A G) * (A U)) against the routines they
    replace: the plain product, an addition, the scipy logistic function."""
    from scipy.special import expit
    rng = np.random.default_rng(11)
    a, g, u, r = rng.standard_normal((5, 10)), rng.standard_normal((10, 4)), rng.standard_normal((10, 4)), rng.standard_normal((5, 4))
    ins = [a[:, :6], a[:, 6:], g[:6], g[6:]]
    np.testing.assert_allclose(T._eval_vertex("gemm", dict(nk=2, mode=1), ins + [r]), a @ g + r, rtol=1e-13)
    gate, up = a @ g, a @ u
    got = T._eval_vertex("gemm", dict(nk=2, mode=2), ins + [u[:6], u[6:]])
    np.testing.assert_allclose(got, gate * expit(gate) * up, rtol=1e-12)
    # weights stored [out, in]
    got_t = T._eval_vertex("gemm", dict(nk=2, mode=2, trans_b=1), [a[:, :6], a[:, 6:], g[:6].T, g[6:].T, u[:6].T, u[6:].T])
    np.testing.assert_allclose(got_t, got, rtol=1e-13)
    # separate vertices give the same numbers
    sep = T._eval_vertex("silu_mul", {}, [T._eval_vertex("gemm", dict(nk=2), ins), T._eval_vertex("gemm", dict(nk=2), [a[:, :6], a[:, 6:], u[:6], u[6:]])])
    np.testing.assert_allclose(got, sep, rtol=1e-13)


@pytest.mark.parametrize("fuse", [1, 2, 3])
def test_fused_graph_equals_the_untiled_model(monkeypatch, fuse):
    """Without storage rounding the fused graph is the same function as the untiled layers (and so as the
    unfused graph); with fp32 storage it stays as close as the unfused one; it has fewer vertices."""
    cfg = config("ragged_f32")
    w = R.widen(cfg, make_llama_inputs(cfg, 3))
    tg = T.build_llama_taskgraph(cfg, fuse_epilogues=fuse)
    plain = T.build_llama_taskgraph(cfg)
    y1 = R.forward(cfg, w)
    y2 = T.assemble_outputs(tg, T.evaluate(tg, T.cut_inputs(tg, w)), cfg.tokens, cfg.d_model)
    assert R.rel_err(y2, y1) < 2e-6
    assert tg.kind.count("add") == (0 if fuse & 1 else plain.kind.count("add"))
    assert tg.kind.count("silu_mul") == (0 if fuse & 2 else plain.kind.count("silu_mul"))
    n_ffn_tiles = plain.kind.count("silu_mul")
    assert plain.kind.count("gemm") - tg.kind.count("gemm") == (n_ffn_tiles if fuse & 2 else 0)
    monkeypatch.setattr(T, "round_store", lambda x, dtype: np.asarray(x, dtype=np.float64))
    y3 = T.assemble_outputs(tg, T.evaluate(tg, T.cut_inputs(tg, w)), cfg.tokens, cfg.d_model)
    assert R.rel_err(y3, y1) < 1e-12


def test_fused_decode_steps_give_the_rows_of_the_whole_sequence():
    cfg = config("decode_f32")
    w = R.widen(cfg, make_llama_inputs(cfg, 0))
    tg = T.build_llama_taskgraph(cfg, fuse_epilogues=3)
    y = T.assemble_outputs(tg, T.evaluate(tg, T.cut_inputs(tg, w)), cfg.tokens, cfg.d_model)
    assert R.rel_err(y, R.forward(cfg, w)) < 2e-6


def test_graph_sizes_match_the_workload_arithmetic():
    cfg = config("c1")
    tg = T.build_llama_taskgraph(cfg)
    kinds = {k: tg.kind.count(k) for k in set(tg.kind)}
    # per layer: 2 row blocks x (4+4+4+4+11+11+4) gemm output tiles = 84; 3 of 4 causal block pairs x 4 heads
    assert kinds["gemm"] == 2 * 84
    assert kinds["attn_block"] == 2 * 3 * 4
    assert kinds["input"] == 2 * 4 + 2 * (196 + 8)
    assert len(tg.outputs) == 8
