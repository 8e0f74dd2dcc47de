"""Pins for the oracle's untiled layer math (CPU only): closed forms, invariants, and special
cases that reduce to a library routine.  Each would fail for a plausible mistake (dropped scale,
wrong mask direction, wrong rotation sign or pairing, missing eps, transposed weight)."""
import numpy as np
import pytest
from scipy.special import expit, softmax

from oracle import llama_ref as R
from workloads import config, make_llama_inputs


def test_rmsnorm_closed_forms():
    # (3, 4): mean square 12.5
    y = R.rmsnorm(np.array([[3.0, 4.0]]), np.array([1.0, 2.0]), 1e-6)
    np.testing.assert_allclose(y, [[3 / np.sqrt(12.5 + 1e-6), 8 / np.sqrt(12.5 + 1e-6)]], rtol=1e-15)
    # unit-RMS rows and unit gain: identity up to eps
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 64))
    x /= np.sqrt(np.mean(x * x, axis=1, keepdims=True))
    np.testing.assert_allclose(R.rmsnorm(x, np.ones(64), 1e-6), x, rtol=1e-6)
    # eps matters for a zero row (no division by zero) and scale invariance holds otherwise
    assert np.all(R.rmsnorm(np.zeros((1, 8)), np.ones(8), 1e-6) == 0)
    np.testing.assert_allclose(R.rmsnorm(1e3 * x, np.ones(64), 1e-6), R.rmsnorm(x, np.ones(64), 1e-6), rtol=1e-6)


def test_rope_closed_forms():
    hd = 8
    rng = np.random.default_rng(1)
    x = rng.standard_normal((6, hd))
    pos = np.arange(6) + 3
    y = R.rope(x, pos, 10000.0)
    # position 0 is the identity
    np.testing.assert_array_equal(R.rope(x, np.zeros(6), 10000.0), x)
    # pair 0 has frequency 1: (1, 0) at position 1 goes to (cos 1, sin 1)
    e = np.zeros((1, hd)); e[0, 0] = 1.0
    r = R.rope(e, np.array([1]), 10000.0)
    np.testing.assert_allclose(r[0, :2], [np.cos(1.0), np.sin(1.0)], rtol=1e-15)
    # the last pair has frequency base**(-(hd-2)/hd)
    e = np.zeros((1, hd)); e[0, hd - 2] = 1.0
    r = R.rope(e, np.array([5]), 10000.0)
    th = 5 * 10000.0 ** (-(hd - 2) / hd)
    np.testing.assert_allclose(r[0, hd - 2:], [np.cos(th), np.sin(th)], rtol=1e-14)
    # the same thing as multiplication of complex numbers x_{2i} + i x_{2i+1} by exp(i pos theta_i)
    z = (x[:, 0::2] + 1j * x[:, 1::2]) * np.exp(1j * pos[:, None] * 10000.0 ** (-np.arange(0, hd, 2) / hd)[None, :])
    np.testing.assert_allclose(y[:, 0::2], z.real, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(y[:, 1::2], z.imag, rtol=1e-13, atol=1e-14)
    # pair norms are preserved and q.k depends only on the position difference
    np.testing.assert_allclose(y[:, 0::2] ** 2 + y[:, 1::2] ** 2, x[:, 0::2] ** 2 + x[:, 1::2] ** 2, rtol=1e-13)
    k = rng.standard_normal((6, hd))
    d1 = R.rope(x, pos, 1e4) @ R.rope(k, pos, 1e4).T
    d2 = R.rope(x, pos + 11, 1e4) @ R.rope(k, pos + 11, 1e4).T
    np.testing.assert_allclose(d1, d2, rtol=1e-10, atol=1e-12)


def test_attention_closed_forms():
    rng = np.random.default_rng(2)
    n, hd = 7, 4
    v = rng.standard_normal((n, hd))
    # zero queries: every allowed key weighs the same, so row r is the mean of v[0..r]
    o = R.causal_attention_head(np.zeros((n, hd)), rng.standard_normal((n, hd)), v)
    np.testing.assert_allclose(o, np.cumsum(v, axis=0) / np.arange(1, n + 1)[:, None], rtol=1e-13)
    # row 0 sees only key 0
    q, k = rng.standard_normal((n, hd)), rng.standard_normal((n, hd))
    o = R.causal_attention_head(q, k, v)
    np.testing.assert_allclose(o[0], v[0], rtol=1e-14)
    # the scale: with hd = 4, q.k1/2 = ln 3 and q.k2/2 = 0 give weights (3/4, 1/4) on row 1
    q2 = np.zeros((2, 4)); q2[1, 0] = 2.0
    k2 = np.zeros((2, 4)); k2[0, 0] = np.log(3.0)
    v2 = np.array([[1.0, 0, 0, 0], [0, 1.0, 0, 0]])
    o2 = R.causal_attention_head(q2, k2, v2)
    np.testing.assert_allclose(o2[1, :2], [0.75, 0.25], rtol=1e-14)
    # the mask direction: a huge score on a *later* key must be ignored, on an earlier key it wins
    kk = np.eye(n, hd * 2)[:, :hd] * 0
    kk = rng.standard_normal((n, hd)); kk /= np.linalg.norm(kk, axis=1, keepdims=True)
    qq = np.zeros((n, hd)); qq[2] = 1e4 * kk[5]; qq[6] = 1e4 * kk[1]
    oo = R.causal_attention_head(qq, kk, v)
    assert not np.allclose(oo[2], v[5], atol=1e-3)
    sc = (qq[6] @ kk.T) / 2
    np.testing.assert_allclose(oo[6], softmax(sc) @ v, rtol=1e-12)
    # against the library softmax on explicitly masked scores
    s = q @ k.T / np.sqrt(hd)
    s[np.triu_indices(n, 1)] = -np.inf
    np.testing.assert_allclose(o, softmax(s, axis=1) @ v, rtol=1e-12)


def test_silu_closed_forms():
    z = np.linspace(-20, 20, 401)
    np.testing.assert_allclose(R.silu(z), z * expit(z), rtol=1e-13, atol=1e-300)
    np.testing.assert_allclose(R.silu(z) - R.silu(-z), z, rtol=1e-12, atol=1e-13)
    assert R.silu(np.array([0.0]))[0] == 0.0
    np.testing.assert_allclose(R.silu(np.array([np.log(3.0)])), [np.log(3.0) * 0.75], rtol=1e-14)


def _small_layer(seed=0, seq=12, d=16, heads=2, f=24):
    rng = np.random.default_rng(seed)
    w = {f"{k}.0": rng.standard_normal((d, d)) * 0.3 for k in ("wq", "wk", "wv", "wo")}
    w["w1.0"] = rng.standard_normal((d, f)) * 0.3
    w["w3.0"] = rng.standard_normal((d, f)) * 0.3
    w["w2.0"] = rng.standard_normal((f, d)) * 0.3
    w["g1.0"] = 1 + 0.1 * rng.standard_normal(d)
    w["g2.0"] = 1 + 0.1 * rng.standard_normal(d)
    x = rng.standard_normal((seq, d))
    return x, w, heads, d // heads


def test_layer_special_cases():
    x, w, heads, hd = _small_layer()
    # zero output projections leave only the residual path
    w0 = dict(w); w0["wo.0"] = np.zeros_like(w["wo.0"]); w0["w2.0"] = np.zeros_like(w["w2.0"])
    np.testing.assert_array_equal(R.decoder_layer(x, w0, 0, heads, hd, 1e-6, 1e4), x)
    # zero feed-forward output: y = x + attention, and with wq = wk = 0 attention is a running
    # mean of v = rmsnorm(x) wv, which pins weight orientation (x @ W) and the order of the steps
    w1 = dict(w); w1["w2.0"] = np.zeros_like(w["w2.0"]); w1["wq.0"] = np.zeros_like(w["wq.0"])
    a = x / np.sqrt(np.mean(x * x, axis=1, keepdims=True) + 1e-6) * w["g1.0"]
    vv = a @ w["wv.0"]
    run_mean = np.cumsum(vv, axis=0) / np.arange(1, x.shape[0] + 1)[:, None]
    np.testing.assert_allclose(R.decoder_layer(x, w1, 0, heads, hd, 1e-6, 1e4), x + run_mean @ w["wo.0"], rtol=1e-12)
    # zero attention output: y = x + (silu(b w1) * (b w3)) w2 with b = rmsnorm(x; g2)
    w2 = dict(w); w2["wo.0"] = np.zeros_like(w["wo.0"])
    b = x / np.sqrt(np.mean(x * x, axis=1, keepdims=True) + 1e-6) * w["g2.0"]
    g = b @ w["w1.0"]
    np.testing.assert_allclose(R.decoder_layer(x, w2, 0, heads, hd, 1e-6, 1e4),
                               x + ((g * expit(g)) * (b @ w["w3.0"])) @ w["w2.0"], rtol=1e-12)


def test_causality_and_prefix_property():
    x, w, heads, hd = _small_layer(3)
    y = R.decoder_layer(x, w, 0, heads, hd, 1e-6, 1e4)
    x2 = x.copy(); x2[8:] += 1.0
    y2 = R.decoder_layer(x2, w, 0, heads, hd, 1e-6, 1e4)
    np.testing.assert_array_equal(y[:8], y2[:8])
    assert not np.allclose(y[8:], y2[8:])
    np.testing.assert_allclose(R.decoder_layer(x[:5], w, 0, heads, hd, 1e-6, 1e4), y[:5], rtol=1e-12)


def test_heads_are_independent_column_groups():
    # permuting whole heads of wq, wk, wv (columns) and wo (rows) together leaves y unchanged
    x, w, heads, hd = _small_layer(4)
    y = R.decoder_layer(x, w, 0, heads, hd, 1e-6, 1e4)
    perm = np.concatenate([np.arange(hd, 2 * hd), np.arange(0, hd)])
    wp = dict(w)
    for k in ("wq", "wk", "wv"):
        wp[f"{k}.0"] = w[f"{k}.0"][:, perm]
    wp["wo.0"] = w["wo.0"][perm, :]
    np.testing.assert_allclose(R.decoder_layer(x, wp, 0, heads, hd, 1e-6, 1e4), y, rtol=1e-11)


def test_batch_elements_are_independent():
    cfg = config("batch2_f32")
    w = R.widen(cfg, make_llama_inputs(cfg, 0))
    y = R.forward(cfg, w)
    one = cfg.with_(batch=1)
    w1 = dict(w); w1["x"] = w["x"][cfg.seq:]
    np.testing.assert_array_equal(R.forward(one, w1), y[cfg.seq:])


def test_error_measure():
    b = np.array([1.0, -2.0, 0.0, 1e-9])
    a = b + np.array([0.0, 0.02, 0.001, 0.0])
    rms = np.sqrt(np.mean(b * b))
    assert R.rel_err(a, b) == pytest.approx(max(0.02 / 2.0, 0.001 / rms))
    assert R.rel_err(b, b) == 0.0


def test_input_generator_is_counter_based_and_normal():
    from workloads import normal, to_bf16_bits, bf16_bits_to_f32
    a = normal(3, 17, 1000)
    np.testing.assert_array_equal(normal(3, 17, 300, start=200), a[200:500])
    assert not np.array_equal(normal(4, 17, 1000), a)
    big = normal(0, 1, 200000)
    assert abs(big.mean()) < 0.01 and abs(big.std() - 1) < 0.01
    # bf16 rounding: nearest, ties to even
    f = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -7], dtype=np.float32)
    np.testing.assert_array_equal(bf16_bits_to_f32(to_bf16_bits(f)), [1.0, 1.0, 1.0 + 2 ** -6, 1.0 + 2 ** -7])


def test_layer_on_sampled_rows_is_the_layer():
    """decoder_layer_rows is pinned to decoder_layer: all rows as a prefix, a sample of rows with the
    full run's keys and values as context, and -- with storage rounding -- to the tiled interpreter,
    whose rounding points it repeats."""
    from oracle import tiled as T
    cfg = config("ragged_bf16")
    w = R.widen(cfg, make_llama_inputs(cfg, 5))
    x = w["x"][:cfg.seq]
    args = (cfg.n_heads, cfg.head_dim, cfg.eps, cfg.rope_base)
    y, k, v = R.decoder_layer(x, w, 1, *args, return_kv=True)
    # every row, no context given
    y2, k2, v2 = R.decoder_layer_rows(x, np.arange(cfg.seq), w, 1, *args)
    for a, b in ((y2, y), (k2, k), (v2, v)):
        np.testing.assert_allclose(a, b, rtol=1e-11, atol=1e-12)
    # a few rows, early and late, against the full run's keys and values
    rows = np.array([0, 1, 77, 200, cfg.seq - 1])
    y3, k3, v3 = R.decoder_layer_rows(x[rows], rows, w, 1, *args, k_ctx=k, v_ctx=v)
    for a, b in ((y3, y[rows]), (k3, k[rows]), (v3, v[rows])):
        np.testing.assert_allclose(a, b, rtol=1e-11, atol=1e-12)
    # a wrong position, a context from another layer, a swapped context must all show
    bad, _, _ = R.decoder_layer_rows(x[rows], rows + 1, w, 1, *args, k_ctx=k, v_ctx=v)
    assert R.rel_err(bad[2:], y[rows][2:]) > 1e-3
    _, k0, v0 = R.decoder_layer(x, w, 0, *args, return_kv=True)
    assert R.rel_err(R.decoder_layer_rows(x[rows], rows, w, 1, *args, k_ctx=k0, v_ctx=v0)[0][2:], y[rows][2:]) > 1e-3
    assert R.rel_err(R.decoder_layer_rows(x[rows], rows, w, 1, *args, k_ctx=v, v_ctx=k)[0][2:], y[rows][2:]) > 1e-3
    # with the storage rounding of the tiled execution: one layer of the tiled interpreter
    one = cfg.with_(layers=1)
    tg = T.build_llama_taskgraph(one)
    w1 = {n: a for n, a in w.items() if n == "x" or n.endswith(".0")}
    y_tiled = T.assemble_outputs(tg, T.evaluate(tg, T.cut_inputs(tg, w1)), one.tokens, one.d_model)
    y_rows, _, _ = R.decoder_layer_rows(x, np.arange(cfg.seq), w, 0, *args, store=lambda z: T.round_store(z, "bf16"))
    # blocked and unblocked softmax differ in the last bits of float64, which moves a rounding now and then
    assert np.mean(y_rows != y_tiled) < 2e-3 and R.rel_err(y_rows, y_tiled) < 2.0 ** -7
    assert R.rel_err(y_rows, R.decoder_layer(x, w, 0, *args)) > 1e-4  # the rounding is really applied
    # the same with fused epilogues: the tensors the fused graph never stores are not rounded
    for fuse in (1, 2, 3):
        tgf = T.build_llama_taskgraph(one, fuse_epilogues=fuse)
        y_tf = T.assemble_outputs(tgf, T.evaluate(tgf, T.cut_inputs(tgf, w1)), one.tokens, one.d_model)
        y_rf, _, _ = R.decoder_layer_rows(x, np.arange(cfg.seq), w, 0, *args, store=lambda z: T.round_store(z, "bf16"),
                                          fuse_epilogues=fuse)
        assert np.mean(y_rf != y_tf) < 2e-3 and R.rel_err(y_rf, y_tf) < 2.0 ** -7
        assert np.mean(y_rf != y_rows) > 0.01  # ... and that moves roundings: the unfused rows are another result
    exact, _, _ = R.decoder_layer_rows(x, np.arange(cfg.seq), w, 0, *args, fuse_epilogues=3)
    np.testing.assert_array_equal(exact, R.decoder_layer_rows(x, np.arange(cfg.seq), w, 0, *args)[0])


def test_decode_steps_give_the_rows_of_the_whole_sequence():
    """decode() (prefill, then one row at a time against a cache that grows) is pinned by causality:
    its rows are those of the plain layer-by-layer forward pass over all positions at once, and its
    caches are that pass's keys and values.  A step that skips its own key, reads a stale cache or
    sits at the wrong position must show."""
    cfg = config("decode_f32")
    w = R.widen(cfg, make_llama_inputs(cfg, 2))
    assert w["x"].shape[0] == cfg.seq + cfg.decode_steps
    y, kc, vc = R.decode(cfg, w)
    ref = R.forward(cfg, w)  # decoder_layer on all seq + steps positions
    assert ref.shape == y.shape == (cfg.seq + cfg.decode_steps, cfg.d_model)
    np.testing.assert_allclose(y, ref, rtol=1e-10, atol=1e-11)
    h = w["x"]
    args = (cfg.n_heads, cfg.head_dim, cfg.eps, cfg.rope_base)
    for l in range(cfg.layers):
        h, k, v = R.decoder_layer(h, w, l, *args, return_kv=True)
        np.testing.assert_allclose(kc[l], k, rtol=1e-10, atol=1e-11)
        np.testing.assert_allclose(vc[l], v, rtol=1e-10, atol=1e-11)
    # the decode rows really depend on the cache and on their own position
    P = cfg.seq
    row = w["x"][P + 3:P + 4]
    _, k0, v0 = R.decoder_layer(w["x"], w, 0, *args, return_kv=True)
    good = R.decoder_layer(w["x"][:P + 4], w, 0, *args)[-1:]
    ok, _, _ = R.decoder_layer_rows(row, [P + 3], w, 0, *args, k_ctx=k0[:P + 3], v_ctx=v0[:P + 3], own_follow_ctx=True)
    np.testing.assert_allclose(ok, good, rtol=1e-10, atol=1e-11)
    stale, _, _ = R.decoder_layer_rows(row, [P + 2], w, 0, *args, k_ctx=k0[:P + 2], v_ctx=v0[:P + 2], own_follow_ctx=True)
    assert R.rel_err(stale, good) > 1e-4
    no_own, _, _ = R.decoder_layer_rows(row, [P + 3], w, 0, *args, k_ctx=k0[:P + 3], v_ctx=v0[:P + 3])
    assert R.rel_err(no_own, good) > 1e-4
