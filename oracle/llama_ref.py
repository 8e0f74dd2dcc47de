"""CPU ORACLE (test infrastructure, not the product) -- untiled decoder-layer math in float64.

This file defines the result that the tiled, memory-capped GPU execution must reproduce.  The
paper does not define the layer math itself: its workloads are LLaMA prefill passes (Experiments,
item 1, and the Introduction's attention example), so the definitions here are the standard
pre-norm decoder layer with RMSNorm, rotary position embedding, causal softmax attention and a
SwiGLU feed-forward block, with the constants of the workload list (eps 1e-6, rotary base 10000).

Everything is plain NumPy in float64, written for reading, with no blocking or fusion.  Only
tests, the smoke check and the benchmark's CPU-baseline leg may import this package; the
product path never does.
"""
from __future__ import annotations

import numpy as np


def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    """y[r, :] = x[r, :] / sqrt(mean_c x[r, c]^2 + eps) * g."""
    x = np.asarray(x, dtype=np.float64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(g, dtype=np.float64)


def rope(x: np.ndarray, positions: np.ndarray, base: float) -> np.ndarray:
    """Rotary embedding on one head, x [rows, hd], interleaved pairs.

    Pair i = (x[:, 2i], x[:, 2i+1]) is rotated counter-clockwise by the angle
    positions[r] * base**(-2i/hd).
    """
    x = np.asarray(x, dtype=np.float64)
    hd = x.shape[-1]
    i = np.arange(hd // 2, dtype=np.float64)
    theta = base ** (-2.0 * i / hd)
    ang = np.asarray(positions, dtype=np.float64)[:, None] * theta[None, :]
    c, s = np.cos(ang), np.sin(ang)
    xe, xo = x[:, 0::2], x[:, 1::2]
    y = np.empty_like(x)
    y[:, 0::2] = xe * c - xo * s
    y[:, 1::2] = xe * s + xo * c
    return y


def causal_attention_head(q: np.ndarray, k: np.ndarray, v: np.ndarray) -> np.ndarray:
    """softmax_rows(q k^T / sqrt(hd), entries with column > row excluded) v for one head."""
    q, k, v = (np.asarray(a, dtype=np.float64) for a in (q, k, v))
    n, hd = q.shape
    s = (q @ k.T) / np.sqrt(hd)
    r = np.arange(n)
    s = np.where(r[None, :] > r[:, None], -np.inf, s)
    s = s - np.max(s, axis=-1, keepdims=True)
    p = np.exp(s)
    p = p / np.sum(p, axis=-1, keepdims=True)
    return p @ v


def silu(z: np.ndarray) -> np.ndarray:
    z = np.asarray(z, dtype=np.float64)
    return z / (1.0 + np.exp(-z))


def decoder_layer(x, w, layer: int, n_heads: int, head_dim: int, eps: float, base: float,
                  return_kv: bool = False):
    """One pre-norm decoder layer on a single sequence x [seq, d]; w maps names to float64 arrays."""
    x = np.asarray(x, dtype=np.float64)
    seq = x.shape[0]
    a = rmsnorm(x, w[f"g1.{layer}"], eps)
    q, k, v = a @ w[f"wq.{layer}"], a @ w[f"wk.{layer}"], a @ w[f"wv.{layer}"]
    pos = np.arange(seq)
    o = np.empty_like(q)
    for h in range(n_heads):
        sl = slice(h * head_dim, (h + 1) * head_dim)
        q[:, sl] = rope(q[:, sl], pos, base)
        k[:, sl] = rope(k[:, sl], pos, base)
        o[:, sl] = causal_attention_head(q[:, sl], k[:, sl], v[:, sl])
    h1 = x + o @ w[f"wo.{layer}"]
    b = rmsnorm(h1, w[f"g2.{layer}"], eps)
    y = h1 + (silu(b @ w[f"w1.{layer}"]) * (b @ w[f"w3.{layer}"])) @ w[f"w2.{layer}"]
    if return_kv:
        return y, k, v
    return y


def decoder_layer_rows(h_rows, positions, w, layer: int, n_heads: int, head_dim: int, eps: float, base: float,
                       k_ctx=None, v_ctx=None, store=None, own_follow_ctx=False, fuse_epilogues=0):
    """One decoder layer for a sample of the rows of one sequence.

    Every step of the layer works row by row except attention, in which the row at position p reads
    the keys and values of positions 0..p.  h_rows [n, d] are the layer's input rows at `positions`.
    k_ctx, v_ctx [n_ctx, d]: the keys (after the rotation) and values of positions 0..n_ctx-1 as the
    run under test stored them, so that a late row can be checked without running the whole sequence;
    None: the rows are positions 0..n-1 and their own keys and values are all there is to attend to
    (a causal prefix).  store: the rounding applied wherever the tiled execution stores a tensor (every
    taskgraph tensor is rounded to its storage type; attention partials and statistics are not);
    None: exact.  own_follow_ctx: the context holds positions 0..n_ctx-1 and the rows given are the
    positions n_ctx..n_ctx+n-1 that follow it, so each row attends to the context and to the given rows
    up to itself (a decode step: the cache, then the new row).  fuse_epilogues: which tensors the tiled
    execution never stores, and so never rounds -- bit 0: the Wo and W2 products (the residual is added inside
    their vertices), bit 1: the gate and up products (silu * up happens inside theirs).  Returns (output rows,
    key rows after the rotation, value rows).
    """
    st = store if store is not None else (lambda z: z)
    h = np.asarray(h_rows, dtype=np.float64)
    positions = np.asarray(positions)
    n = h.shape[0]
    a = st(rmsnorm(h, w[f"g1.{layer}"], eps))
    q, k, v = st(a @ w[f"wq.{layer}"]), st(a @ w[f"wk.{layer}"]), st(a @ w[f"wv.{layer}"])
    for hh in range(n_heads):
        sl = slice(hh * head_dim, (hh + 1) * head_dim)
        q[:, sl] = rope(q[:, sl], positions, base)
        k[:, sl] = rope(k[:, sl], positions, base)
    q, k = st(q), st(k)
    if k_ctx is None:
        assert np.array_equal(positions, np.arange(n)), "without a context the rows must be a prefix"
        kc, vc = k, v
    else:
        kc, vc = np.asarray(k_ctx, dtype=np.float64), np.asarray(v_ctx, dtype=np.float64)
        if own_follow_ctx:
            assert np.array_equal(positions, kc.shape[0] + np.arange(n)), "the rows must follow the context"
            kc, vc = np.concatenate([kc, k]), np.concatenate([vc, v])
    o = np.empty_like(q)
    for r in range(n):
        p = int(positions[r])
        for hh in range(n_heads):
            sl = slice(hh * head_dim, (hh + 1) * head_dim)
            s = (kc[:p + 1, sl] @ q[r, sl]) / np.sqrt(head_dim)
            e = np.exp(s - np.max(s))
            o[r, sl] = (e / np.sum(e)) @ vc[:p + 1, sl]
    o = st(o)
    st_res = (lambda z: z) if fuse_epilogues & 1 else st  # the products that a residual is added to
    st_gate = (lambda z: z) if fuse_epilogues & 2 else st  # the gate and up products
    h1 = st(h + st_res(o @ w[f"wo.{layer}"]))
    b = st(rmsnorm(h1, w[f"g2.{layer}"], eps))
    gate, up = st_gate(b @ w[f"w1.{layer}"]), st_gate(b @ w[f"w3.{layer}"])
    act = st(silu(gate) * up)
    y = st(h1 + st_res(act @ w[f"w2.{layer}"]))
    return y, k, v


def forward(cfg, inputs_f64, n_tokens_prefix=None):
    """All layers, all sequences of the batch.  inputs_f64: name -> float64 array (full tensors).

    n_tokens_prefix: evaluate only the first that many tokens of each sequence (a causal
    prefill's rows [0, r) equal the model run on the first r tokens).
    """
    out = []
    n = cfg.seq + getattr(cfg, "decode_steps", 0)  # positions per sequence
    for b in range(cfg.batch):
        x = inputs_f64["x"][b * n:(b + 1) * n]
        if n_tokens_prefix is not None:
            x = x[:n_tokens_prefix]
        for l in range(cfg.layers):
            x = decoder_layer(x, inputs_f64, l, cfg.n_heads, cfg.head_dim, cfg.eps, cfg.rope_base)
        out.append(x)
    return np.concatenate(out, axis=0)


def decode(cfg, inputs_f64, store=None):
    """Prefill of the first cfg.seq positions of the one sequence, then cfg.decode_steps steps of one
    position each (Section 9, limitations: generation with the number of steps fixed beforehand).

    A step takes the embedding of its position (row seq + u of x: there is no vocabulary here, so the
    row is given rather than sampled), and runs it through every layer against that layer's cache:
    the keys and values of all earlier positions, to which the step appends its own.  Returns
    (y [seq + steps, d], k, v) with k[l], v[l] [seq + steps, d] the caches at the end.  store: as in
    decoder_layer_rows.  Since attention is causal, y equals forward() on all seq + steps positions.
    """
    assert cfg.batch == 1
    P, N = cfg.seq, cfg.decode_steps
    args = (cfg.n_heads, cfg.head_dim, cfg.eps, cfg.rope_base)
    x = np.asarray(inputs_f64["x"], dtype=np.float64)
    h = x[:P]
    kc, vc = [], []
    for l in range(cfg.layers):
        h, k, v = decoder_layer_rows(h, np.arange(P), inputs_f64, l, *args, store=store)
        kc.append(k)
        vc.append(v)
    ys = [h]
    for u in range(N):
        r = x[P + u:P + u + 1]
        for l in range(cfg.layers):
            r, k, v = decoder_layer_rows(r, [P + u], inputs_f64, l, *args, k_ctx=kc[l], v_ctx=vc[l], store=store,
                                         own_follow_ctx=True)
            kc[l], vc[l] = np.concatenate([kc[l], k]), np.concatenate([vc[l], v])
        ys.append(r)
    return np.concatenate(ys), kc, vc


def widen_array(a: np.ndarray) -> np.ndarray:
    """One storage-dtype buffer (float32, or bfloat16 bit patterns as uint16) -> exact float64."""
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def widen(cfg, inputs):
    """Storage-dtype host buffers -> exact float64 copies."""
    return {k: widen_array(a) for k, a in inputs.items()}


def rel_err(a: np.ndarray, b: np.ndarray) -> float:
    """max_i |a_i - b_i| / max(|b_i|, rms(b)): the error measure the parity thresholds refer to."""
    a = np.asarray(a, dtype=np.float64).ravel()
    b = np.asarray(b, dtype=np.float64).ravel()
    if b.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(b * b)))
    den = np.maximum(np.abs(b), rms if rms > 0 else 1.0)
    return float(np.max(np.abs(a - b) / den))
