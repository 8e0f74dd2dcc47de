"""CPU ORACLE (test infrastructure, not the product) -- tiled taskgraph of the decoder and its
interpreter.

A taskgraph is a dataflow DAG: a vertex without inputs holds an input tensor, every other
vertex is one kernel call with one output tensor, and an edge means "consumes the output of"
(Section 4, first paragraph).  The paper leaves the production of the taskgraph to an outside
framework (Section 4, second paragraph) and prints no vertex catalogue, so the catalogue below
is this build's: each kind is a pure function of its inputs with a fixed summation order, which
is what makes every dependency-respecting execution order give the same output (Introduction,
fourth paragraph).

This module has its own tiler (it does not read the library's) and evaluates any graph given
in the plain format below -- including one exported by the library, so the library's tiler can
be checked on the CPU.  float64 arithmetic inside a vertex; every vertex output is rounded to
the vertex's storage type ("f32" or "bf16"), which reproduces the rounding points of the tiled
execution.  Only tests, the smoke check and the benchmark's CPU-baseline leg import this.

Vertex kinds (inputs -> output):
  input         ()                                   -> the tile itself
  gemm          A_0..A_{nk-1}, B_0..B_{nk-1}         -> sum_k A_k @ B_k, k ascending (B_k held transposed if trans_b;
                                                        result stored transposed if trans_c)
  rms_stat      X_0..X_{n-1} (tiles of one row block)-> [rows,1] 1/sqrt(mean over all columns of x^2 + eps)
  rms_apply     X, stat, gain[1,c]                   -> x * stat * gain
  rope          X                                    -> rotary embedding; params pos0, col0, head_dim, base
  attn_block    Q tiles, K tiles, V tiles            -> packed [rows, gw + 2*hpg]: O (unnormalised), m, l
                                                        (V tiles hold V^T if v_trans)
  attn_combine  partial_0..partial_j                 -> normalised attention output tile
  silu_mul      gate, up                             -> gate/(1+exp(-gate)) * up
  add           a, b                                 -> a + b
  softmax_stat  S_0..S_{n-1} (score tiles of one row   -> [rows, 2]: per row the maximum m of scale * s over the visible
                block, left to right)                   entries and l = sum exp(scale * s - m) over them; entry (r, c)
                                                        is visible unless causal and k_pos0 + c > q_pos0 + r, c counted
                                                        across the tiles.  With softmax_apply this is the softmax "in
                                                        portions" of materialised attention scores (Introduction,
                                                        second paragraph; Appendix A, hand-written kernels)
  softmax_apply S, stat                              -> exp(scale * s - m) / l where visible, else 0; k_pos0 is the
                                                        position of this tile's first column
  sum           p_0..p_{n-1}                         -> their sum, formed the way Appendix A (resources) describes a
                                                        reduction: an output that starts at zero and receives the
                                                        n operands as n increments, each increment rounding the
                                                        output to its storage type.  The increments hold a write
                                                        lock on the output and may come in any order, so this is
                                                        the one kind whose result depends on the execution order
                                                        (by rounding only); `evaluate` takes the order as an
                                                        argument and uses ascending operand order by default.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np


# ---------------------------------------------------------------------------------------------
# storage rounding
# ---------------------------------------------------------------------------------------------

def round_bf16(x: np.ndarray) -> np.ndarray:
    """Nearest-even rounding of float64 values to bfloat16, returned as float64."""
    f = np.ascontiguousarray(x, dtype=np.float32)  # double -> single first, as a store would
    b = f.view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return r.view(np.float32).astype(np.float64)


def round_store(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return round_bf16(x)
    return np.asarray(x, dtype=np.float32).astype(np.float64)


# ---------------------------------------------------------------------------------------------
# graph container
# ---------------------------------------------------------------------------------------------

@dataclass
class TaskGraph:
    kind: List[str] = field(default_factory=list)
    params: List[dict] = field(default_factory=list)
    inputs: List[List[int]] = field(default_factory=list)
    shape: List[Tuple[int, int]] = field(default_factory=list)
    dtype: List[str] = field(default_factory=list)
    outputs: List[int] = field(default_factory=list)
    # vid -> (tensor name, row0, row1, col0, col1[, transposed]) for input tiles and marked outputs
    binding: Dict[int, tuple] = field(default_factory=dict)

    def add(self, kind, inputs, shape, dtype, **params) -> int:
        self.kind.append(kind)
        self.inputs.append(list(inputs))
        self.shape.append((int(shape[0]), int(shape[1])))
        self.dtype.append(dtype)
        self.params.append(params)
        return len(self.kind) - 1

    def __len__(self):
        return len(self.kind)


# ---------------------------------------------------------------------------------------------
# vertex semantics
# ---------------------------------------------------------------------------------------------

def _eval_vertex(kind: str, p: dict, ins: Sequence[np.ndarray]) -> np.ndarray:
    if kind == "gemm":
        nk = p["nk"]

        def product(first):  # sum over k of A_k times the operand at first + k
            acc = None
            for k in range(nk):
                t = ins[k] @ (ins[first + k].T if p.get("trans_b") else ins[first + k])
                acc = t if acc is None else acc + t
            return acc

        mode = p.get("mode", 0)
        if mode == 1:  # the product plus one more operand of the output's shape (a residual)
            return product(nk) + ins[2 * nk]
        if mode == 2:  # two products from the same A tiles, gate and up: silu(gate) * up
            gate, up = product(nk), product(2 * nk)
            return gate / (1.0 + np.exp(-gate)) * up
        acc = product(nk)
        return acc.T if p.get("trans_c") else acc
    if kind == "rms_stat":
        ss = sum(np.sum(x * x, axis=1, keepdims=True) for x in ins)
        return 1.0 / np.sqrt(ss / p["d"] + p["eps"])
    if kind == "rms_apply":
        x, stat, g = ins
        return x * stat * g.reshape(1, -1)
    if kind == "rope":
        (x,) = ins
        hd, base = p["head_dim"], p["base"]
        rows, cols = x.shape
        pos = p["pos0"] + np.arange(rows, dtype=np.float64)
        c = p["col0"] + np.arange(0, cols, 2)  # column of the even member of each pair, in its head
        theta = base ** (-(c % hd).astype(np.float64) / hd)  # (c % hd) = 2i
        ang = pos[:, None] * theta[None, :]
        cs, sn = np.cos(ang), np.sin(ang)
        y = np.empty_like(x)
        y[:, 0::2] = x[:, 0::2] * cs - x[:, 1::2] * sn
        y[:, 1::2] = x[:, 0::2] * sn + x[:, 1::2] * cs
        return y
    if kind == "attn_block":
        nq, nkv, nc, hd = p["n_q_tiles"], p["n_kv_tiles"], p["n_col_tiles"], p["head_dim"]
        def gather(off, nr, transposed=False):
            tiles = [[ins[off + r * nc + c].T if transposed else ins[off + r * nc + c] for c in range(nc)]
                     for r in range(nr)]
            return np.concatenate([np.concatenate(row, axis=1) for row in tiles], axis=0)
        q = gather(0, nq)
        k = gather(nq * nc, nkv)
        v = gather(nq * nc + nkv * nc, nkv, bool(p.get("v_trans")))
        gw = q.shape[1]
        hpg = gw // hd
        rows = q.shape[0]
        out = np.zeros((rows, gw + 2 * hpg))
        qpos = p["q_pos0"] + np.arange(rows)
        kpos = p["k_pos0"] + np.arange(k.shape[0])
        for h in range(hpg):
            sl = slice(h * hd, (h + 1) * hd)
            s = (q[:, sl] @ k[:, sl].T) * p["scale"]
            if p["causal"]:
                s = np.where(kpos[None, :] > qpos[:, None], -np.inf, s)
            m = np.max(s, axis=1)
            msafe = np.where(np.isfinite(m), m, 0.0)
            pr = np.exp(s - msafe[:, None])
            out[:, sl] = pr @ v[:, sl]
            out[:, gw + h] = m
            out[:, gw + hpg + h] = np.sum(pr, axis=1)
        return out
    if kind == "attn_combine":
        hd, hpg = p["head_dim"], p["hpg"]
        gw = hd * hpg
        r0, c0, rows, cols = p["row0"], p["col0"], p["rows"], p["cols"]
        m = np.stack([x[r0:r0 + rows, gw:gw + hpg] for x in ins])  # [j, rows, hpg]
        l = np.stack([x[r0:r0 + rows, gw + hpg:gw + 2 * hpg] for x in ins])
        mstar = np.max(m, axis=0)
        w = np.exp(m - mstar[None])  # exp(-inf) = 0 for empty partials
        lstar = np.sum(l * w, axis=0)
        out = np.zeros((rows, cols))
        head_of_col = (c0 + np.arange(cols)) // hd
        for j, x in enumerate(ins):
            out += x[r0:r0 + rows, c0:c0 + cols] * w[j][:, head_of_col]
        return out / lstar[:, head_of_col]
    if kind == "silu_mul":
        g, u = ins
        return g / (1.0 + np.exp(-g)) * u
    if kind == "add":
        return ins[0] + ins[1]
    if kind == "softmax_stat":
        s = np.concatenate(ins, axis=1) * p["scale"]
        if p["causal"]:
            r = p["q_pos0"] + np.arange(s.shape[0])
            c = p["k_pos0"] + np.arange(s.shape[1])
            s = np.where(c[None, :] > r[:, None], -np.inf, s)
        m = np.max(s, axis=1)
        msafe = np.where(np.isfinite(m), m, 0.0)
        return np.stack([m, np.sum(np.exp(s - msafe[:, None]), axis=1)], axis=1)
    if kind == "softmax_apply":
        s, stat = ins
        s = s * p["scale"]
        if p["causal"]:
            r = p["q_pos0"] + np.arange(s.shape[0])
            c = p["k_pos0"] + np.arange(s.shape[1])
            s = np.where(c[None, :] > r[:, None], -np.inf, s)
        m = np.where(np.isfinite(stat[:, 0]), stat[:, 0], 0.0)
        return np.exp(s - m[:, None]) / stat[:, 1][:, None]
    if kind == "sum":
        acc = np.zeros_like(ins[0])
        for i in p.get("_increment_order", range(len(ins))):
            acc = round_store(acc + ins[i], p["_storage"])
        return acc
    raise ValueError(f"unknown vertex kind {kind}")


def evaluate(tg: TaskGraph, input_values: Dict[int, np.ndarray],
             order: Optional[Sequence[int]] = None, keep_all: bool = False,
             increment_order=None) -> Dict[int, np.ndarray]:
    """Run the graph in `order` (default: vertex numbering, which must be topological).

    increment_order: optional function (sum vertex id, number of operands) -> permutation of the
    operand indices, the order in which that sum's increments take place.

    input_values: vid -> float64 tile for every input vertex.  Returns vid -> float64 value for
    the marked outputs (or for every vertex with keep_all).  Every value is rounded to its
    vertex's storage type, except attention partials and RMS statistics, which are "f32".
    """
    n = len(tg)
    order = range(n) if order is None else order
    remaining = [0] * n
    for v in range(n):
        for u in tg.inputs[v]:
            remaining[u] += 1
    keep = set(tg.outputs)
    val: Dict[int, np.ndarray] = {}
    done = [False] * n
    for v in order:
        if tg.kind[v] == "input":
            if not keep_all and v not in keep:
                done[v] = True  # fetched when its first consumer runs, so that unused tiles hold no memory
                continue
            r = np.asarray(input_values[v], dtype=np.float64).reshape(tg.shape[v])
        else:
            for u in tg.inputs[v]:
                if not done[u]:
                    raise ValueError(f"order is not topological at vertex {v}")
                if u not in val:
                    val[u] = round_store(np.asarray(input_values[u], dtype=np.float64).reshape(tg.shape[u]),
                                         tg.dtype[u])
            p = tg.params[v]
            if tg.kind[v] == "sum":
                p = dict(p, _storage=tg.dtype[v])
                if increment_order is not None:
                    perm = list(increment_order(v, len(tg.inputs[v])))
                    assert sorted(perm) == list(range(len(tg.inputs[v])))
                    p["_increment_order"] = perm
            r = _eval_vertex(tg.kind[v], p, [val[u] for u in tg.inputs[v]])
            assert r.shape == tg.shape[v], (tg.kind[v], r.shape, tg.shape[v])
        val[v] = round_store(r, tg.dtype[v])
        done[v] = True
        if not keep_all:
            for u in tg.inputs[v]:
                remaining[u] -= 1
                if remaining[u] == 0 and u not in keep:
                    del val[u]
    return val if keep_all else {v: val[v] for v in tg.outputs}


# ---------------------------------------------------------------------------------------------
# the oracle's own tiler
# ---------------------------------------------------------------------------------------------

def _splits(n: int, t: int) -> List[Tuple[int, int]]:
    return [(s, min(s + t, n)) for s in range(0, n, t)]


def build_llama_taskgraph(cfg, k_split: int = 1, materialize_scores: bool = False,
                          attn_whole_rows: bool = False, fuse_epilogues: int = 0) -> TaskGraph:
    """Tile the decoder of `cfg` (a workloads.LlamaConfig) into a taskgraph.

    k_split > 1: every projection is cut along K into that many partial products (contiguous runs
    of ceil(nk / k_split) K tiles, each a gemm vertex stored in the storage type) joined by a sum
    vertex -- the k-split + sum-into form of a matrix product.

    materialize_scores (needs tile == head_dim, so that a column tile is one head): attention with
    the scores and probabilities as tensors of the graph -- per head and pair of row tiles (i, j <= i)
    a gemm S = Q_i K_j^T, per head and row tile a softmax_stat over S_i0..S_ii, a softmax_apply per
    score tile, and O_i = sum_j P_ij V_j as one gemm -- instead of the fused blocks and combines.

    Tensors are cut into tile x tile pieces (ragged at the right and bottom edges); row blocks
    never straddle sequences.  Attention runs per (sequence, head group, q block, kv block <= q
    block) with one partial per pair and one combine per output tile; blocks above the diagonal
    are never created.  A head group is the set of heads covering max(tile, head_dim) columns.

    attn_whole_rows: one attention vertex per (sequence, head group, q block) over all keys from
    position 0 to the end of the q block (its softmax runs over the whole range at once) instead of one
    per kv block; the combine then has a single partial to normalise.

    fuse_epilogues (needs k_split == 1): bit 0 -- the two residual additions of a layer become the last
    operand of the products before them (gemm, mode 1); bit 1 -- the W1 and W3 products and silu * up
    become one vertex (gemm, mode 2).  The fused vertices round to the storage type once, where the
    separate ones round after every step.

    cfg.decode_steps > 0 (one sequence): after the prefill of cfg.seq positions, that many steps of one
    row each (Section 9, limitations: the number of generated tokens is fixed when the graph is
    built).  A step's key and value rows are single-row tiles that join the layer's cache; its
    attention is one block per prefill block plus one block over the single-row tiles so far.  The
    step's embedding is row seq + u of the input "x", its result row seq + u of "y".
    """
    tg = TaskGraph()
    dt, t, d, f, hd = cfg.dtype, cfg.tile, cfg.d_model, cfg.ffn, cfg.head_dim
    assert (t % hd == 0 or hd % t == 0) and cfg.attn_block % t == 0
    dcols, fcols = _splits(d, t), _splits(f, t)
    gw = max(t, hd)
    hpg = gw // hd
    ctg = gw // t  # column tiles per head group

    def input_tiles(name, rows, cols, r_off=0):
        """Grid of input vertices for the matrix `name`, cut by `rows` x `cols` ranges."""
        grid = []
        for (r0, r1) in rows:
            line = []
            for (c0, c1) in cols:
                v = tg.add("input", [], (r1 - r0, c1 - c0), dt)
                tg.binding[v] = (name, r_off + r0, r_off + r1, c0, c1)
                line.append(v)
            grid.append(line)
        return grid

    def gain_tiles(name, cols):
        out = []
        for (c0, c1) in cols:
            v = tg.add("input", [], (1, c1 - c0), dt)
            tg.binding[v] = (name, 0, 1, c0, c1)
            out.append(v)
        return out

    assert fuse_epilogues == 0 or k_split <= 1

    def gemm(a_grid, b_grid, out_cols, residual=None, up_grid=None):
        """a_grid [row tiles][k tiles], b_grid [k tiles][col tiles]; residual [row tiles][col tiles] is added
        inside the vertex; up_grid (like b_grid) makes it the gated pair of products."""
        res = []
        for i, arow in enumerate(a_grid):
            line = []
            m = tg.shape[arow[0]][0]
            nk = len(arow)
            per = -(-nk // max(1, k_split))
            for j, (c0, c1) in enumerate(out_cols):
                if residual is not None or up_grid is not None:
                    ins = list(arow) + [b_grid[k][j] for k in range(nk)]
                    ins += [residual[i][j]] if residual is not None else [up_grid[k][j] for k in range(nk)]
                    line.append(tg.add("gemm", ins, (m, c1 - c0), dt, nk=nk, mode=1 if residual is not None else 2))
                    continue
                parts = []
                for k0 in range(0, nk, per):
                    ks = range(k0, min(k0 + per, nk))
                    ins = [arow[k] for k in ks] + [b_grid[k][j] for k in ks]
                    parts.append(tg.add("gemm", ins, (m, c1 - c0), dt, nk=len(ks)))
                line.append(parts[0] if len(parts) == 1 else tg.add("sum", parts, (m, c1 - c0), dt))
            res.append(line)
        return res

    def rmsnorm(x_grid, gains, cols):
        res = []
        for xrow in x_grid:
            m = tg.shape[xrow[0]][0]
            st = tg.add("rms_stat", xrow, (m, 1), "f32", eps=cfg.eps, d=d)
            res.append([tg.add("rms_apply", [xv, st, gains[j]], tg.shape[xv], dt)
                        for j, xv in enumerate(xrow)])
        return res

    def ewise(kind, a_grid, b_grid):
        return [[tg.add(kind, [a, b], tg.shape[a], dt) for a, b in zip(ar, br)]
                for ar, br in zip(a_grid, b_grid)]

    rows = _splits(cfg.seq, t)
    blocks = _splits(cfg.seq, cfg.attn_block)
    tiles_of_block = [[i for i, (r0, _) in enumerate(rows) if b0 <= r0 < b1] for (b0, b1) in blocks]
    xs = [input_tiles("x", rows, dcols, r_off=b * cfg.seq) for b in range(cfg.batch)]

    def roped(grid):
        return [[tg.add("rope", [xv], tg.shape[xv], dt, pos0=rows[i][0], col0=dcols[j][0] % hd,
                        head_dim=hd, base=cfg.rope_base)
                 for j, xv in enumerate(line)] for i, line in enumerate(grid)]

    def attention_materialized(q, k, v):
        assert t == hd
        o = [[None] * len(dcols) for _ in rows]
        scale = 1.0 / np.sqrt(hd)
        for i, (r0, r1) in enumerate(rows):
            for h in range(len(dcols)):
                sc = [tg.add("gemm", [q[i][h], k[j][h]], (r1 - r0, rows[j][1] - rows[j][0]), dt, nk=1, trans_b=1)
                      for j in range(i + 1)]
                st = tg.add("softmax_stat", sc, (r1 - r0, 2), "f32", scale=scale, causal=1, q_pos0=r0, k_pos0=0)
                pr = [tg.add("softmax_apply", [sc[j], st], tg.shape[sc[j]], dt, scale=scale, causal=1, q_pos0=r0,
                             k_pos0=rows[j][0]) for j in range(i + 1)]
                o[i][h] = tg.add("gemm", pr + [v[j][h] for j in range(i + 1)], (r1 - r0, hd), dt, nk=i + 1)
        return o

    def attention(q, k, v):
        """Blocked causal attention of one sequence; returns the grid of output tiles."""
        if materialize_scores:
            return attention_materialized(q, k, v)
        o = [[None] * len(dcols) for _ in rows]
        for g in range(d // gw):
            cts = list(range(g * ctg, (g + 1) * ctg))
            for bi, (q0, q1) in enumerate(blocks):
                parts = []
                for bj in ([bi] if attn_whole_rows else range(bi + 1)):
                    k0 = 0 if attn_whole_rows else blocks[bj][0]
                    qi = tiles_of_block[bi]
                    kj = [r for b2 in range(bi + 1) for r in tiles_of_block[b2]] if attn_whole_rows else tiles_of_block[bj]
                    ins = ([q[r][c] for r in qi for c in cts] + [k[r][c] for r in kj for c in cts]
                           + [v[r][c] for r in kj for c in cts])
                    parts.append(tg.add("attn_block", ins, (q1 - q0, gw + 2 * hpg), "f32",
                                        n_q_tiles=len(qi), n_kv_tiles=len(kj), n_col_tiles=ctg,
                                        head_dim=hd, q_pos0=q0, k_pos0=k0, causal=(bj == bi),
                                        scale=1.0 / np.sqrt(hd)))
                for r in tiles_of_block[bi]:
                    for ci, c in enumerate(cts):
                        m, n_ = rows[r][1] - rows[r][0], dcols[c][1] - dcols[c][0]
                        o[r][c] = tg.add("attn_combine", parts, (m, n_), dt, row0=rows[r][0] - q0,
                                         col0=ci * t, rows=m, cols=n_, head_dim=hd, hpg=hpg)
        return o

    def after_attention(x, o, w, g2):
        """Output projection, residual, feed-forward, residual; returns (h1, its normalised form, the layer's result)."""
        if fuse_epilogues & 1:
            h1 = gemm(o, w["wo"], dcols, residual=x)
        else:
            h1 = ewise("add", x, gemm(o, w["wo"], dcols))
        bn = rmsnorm(h1, g2, dcols)
        if fuse_epilogues & 2:
            act = gemm(bn, w["w1"], fcols, up_grid=w["w3"])
        else:
            act = ewise("silu_mul", gemm(bn, w["w1"], fcols), gemm(bn, w["w3"], fcols))
        if fuse_epilogues & 1:
            return h1, bn, gemm(act, w["w2"], dcols, residual=h1)
        return h1, bn, ewise("add", h1, gemm(act, w["w2"], dcols))

    steps = getattr(cfg, "decode_steps", 0)
    assert steps == 0 or (cfg.batch == 1 and not materialize_scores)
    weights, cache = [], []  # per layer: the weight grids, and the prefill's K (rotated) and V grids
    for l in range(cfg.layers):
        w = {k: input_tiles(f"{k}.{l}", dcols, dcols) for k in ("wq", "wk", "wv", "wo")}
        w["w1"] = input_tiles(f"w1.{l}", dcols, fcols)
        w["w3"] = input_tiles(f"w3.{l}", dcols, fcols)
        w["w2"] = input_tiles(f"w2.{l}", fcols, dcols)
        g1, g2 = gain_tiles(f"g1.{l}", dcols), gain_tiles(f"g2.{l}", dcols)
        weights.append((w, g1, g2))
        for b in range(cfg.batch):
            x = xs[b]
            a = rmsnorm(x, g1, dcols)
            q, k, v = gemm(a, w["wq"], dcols), gemm(a, w["wk"], dcols), gemm(a, w["wv"], dcols)
            k = roped(k)
            cache.append((k, v))
            o = attention(roped(q), k, v)
            h1, bn, xs[b] = after_attention(x, o, w, g2)
    for b in range(cfg.batch):
        for i, line in enumerate(xs[b]):
            for j, vtx in enumerate(line):
                tg.outputs.append(vtx)
                tg.binding[vtx] = ("y", b * cfg.seq + rows[i][0], b * cfg.seq + rows[i][1],
                                   dcols[j][0], dcols[j][1])

    # decode steps: position P + u, one row, through every layer against the layer's cache
    P = cfg.seq
    new_k = [[] for _ in range(cfg.layers)]  # per layer: one line of single-row tiles per step so far
    new_v = [[] for _ in range(cfg.layers)]
    for u in range(steps):
        pos = P + u
        x = input_tiles("x", [(pos, pos + 1)], dcols)
        for l in range(cfg.layers):
            w, g1, g2 = weights[l]
            pk, pv = cache[l]
            a = rmsnorm(x, g1, dcols)
            q, k, v = gemm(a, w["wq"], dcols), gemm(a, w["wk"], dcols), gemm(a, w["wv"], dcols)
            turn = lambda line: [tg.add("rope", [xv], tg.shape[xv], dt, pos0=pos, col0=dcols[j][0] % hd, head_dim=hd,
                                        base=cfg.rope_base) for j, xv in enumerate(line)]
            q, k = turn(q[0]), turn(k[0])
            new_k[l].append(k)
            new_v[l].append(v[0])
            o = [None] * len(dcols)
            for g in range(d // gw):
                cts = list(range(g * ctg, (g + 1) * ctg))
                common = dict(n_q_tiles=1, n_col_tiles=ctg, head_dim=hd, q_pos0=pos, causal=0, scale=1.0 / np.sqrt(hd))
                parts = []
                for bj, (k0, _) in enumerate(blocks):  # the prefill's blocks: all of their positions are earlier
                    kj = tiles_of_block[bj]
                    ins = [q[c] for c in cts] + [pk[r][c] for r in kj for c in cts] + [pv[r][c] for r in kj for c in cts]
                    parts.append(tg.add("attn_block", ins, (1, gw + 2 * hpg), "f32", n_kv_tiles=len(kj), k_pos0=k0, **common))
                ins = ([q[c] for c in cts] + [line[c] for line in new_k[l] for c in cts]
                       + [line[c] for line in new_v[l] for c in cts])
                parts.append(tg.add("attn_block", ins, (1, gw + 2 * hpg), "f32", n_kv_tiles=u + 1, k_pos0=P, **common))
                for ci, c in enumerate(cts):
                    n_ = dcols[c][1] - dcols[c][0]
                    o[c] = tg.add("attn_combine", parts, (1, n_), dt, row0=0, col0=ci * t, rows=1, cols=n_, head_dim=hd, hpg=hpg)
            h1, bn, x = after_attention(x, [o], w, g2)
        for j, vtx in enumerate(x[0]):
            tg.outputs.append(vtx)
            tg.binding[vtx] = ("y", pos, pos + 1, dcols[j][0], dcols[j][1])
    return tg


def cut_inputs(tg: TaskGraph, full_f64: Dict[str, np.ndarray]) -> Dict[int, np.ndarray]:
    """Slice the full input tensors into the tiles the graph's input vertices name."""
    out = {}
    for v, bnd in tg.binding.items():
        if tg.kind[v] != "input":
            continue
        name, r0, r1, c0, c1 = bnd[:5]
        a = full_f64[name]
        a = a.reshape(1, -1) if a.ndim == 1 else a
        out[v] = a[r0:r1, c0:c1].T if len(bnd) > 5 and bnd[5] else a[r0:r1, c0:c1]
    return out


class LazyInputs:
    """Mapping vid -> float64 tile that slices and widens the full storage-type tensors on demand
    (for inputs too large to hold widened all at once).  `widen` turns a storage-type array into
    float64 exactly.  Tiles cut from the same region of the same array (layers that share their
    weights) are kept and reused while they fit `cache_bytes`."""

    def __init__(self, tg: TaskGraph, full_storage: Dict[str, np.ndarray], widen, cache_bytes: int = 0):
        self.tg, self.full, self.widen = tg, full_storage, widen
        self.cache, self.room = {}, cache_bytes

    def __getitem__(self, v: int) -> np.ndarray:
        bnd = self.tg.binding[v]
        name, r0, r1, c0, c1 = bnd[:5]
        a = self.full[name]
        key = (id(a), r0, r1, c0, c1)
        t = self.cache.get(key)
        if t is None:
            a = a.reshape(1, -1) if a.ndim == 1 else a
            t = self.widen(np.ascontiguousarray(a[r0:r1, c0:c1]))
            if t.nbytes <= self.room:
                self.room -= t.nbytes
                self.cache[key] = t
        return t.T if len(bnd) > 5 and bnd[5] else t


def assemble_outputs(tg: TaskGraph, values: Dict[int, np.ndarray], tokens: int, d: int) -> np.ndarray:
    y = np.full((tokens, d), np.nan)
    for v in tg.outputs:
        _, r0, r1, c0, c1 = tg.binding[v][:5]
        y[r0:r1, c0:c1] = values[v]
    return y
