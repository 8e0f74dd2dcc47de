"""Glue used by tests only: converts what the library exports (plain lists) into the oracle's
containers, so that the oracle's checkers and interpreter can judge the library's graphs."""
import numpy as np

from oracle import memgraph as M
from oracle import tiled as T
from paper_2405_16283_amd import binding as B
from paper_2405_16283_amd import harness as H


def oracle_memgraph(mg_handle) -> M.MemGraph:
    e = H.export_memgraph(mg_handle)
    mg = M.MemGraph(n_task=e["n_task"], cap=e["cap"])
    mg.kind, mg.src, mg.loc = e["kind"], e["src"], e["loc"]
    mg.operands, mg.edges, mg.order = e["operands"], e["edges"], e["order"]
    return mg


def oracle_taskgraph(tg_handle) -> T.TaskGraph:
    e = H.export_taskgraph(tg_handle)
    tg = T.TaskGraph()
    tg.kind, tg.inputs, tg.shape, tg.dtype = e["kind"], e["inputs"], e["shape"], e["dtype"]
    tg.outputs = e["outputs"]
    for k, p in zip(e["kind"], e["params"]):
        q = dict(p)
        q["base"] = q.pop("rope_base")
        tg.params.append(q)
    for v, name, r0, r1, c0, c1, tr in e["bindings"]:
        tg.binding[v] = (name, r0, r1, c0, c1, tr)
    # combine vertices need their own output shape
    for v, k in enumerate(tg.kind):
        if k == "attn_combine":
            tg.params[v]["rows"], tg.params[v]["cols"] = tg.shape[v]
    return tg


def assemble_named(tg: T.TaskGraph, values, name: str, rows: int, cols: int) -> np.ndarray:
    """The output tensor `name` of an interpreted graph (a library graph may have several outputs, some
    of them stored transposed), put together from its tiles; NaN where no tile lies."""
    a = np.full((rows, cols), np.nan)
    for v in tg.outputs:
        b = tg.binding[v]
        if b[0] == name:
            a[b[1]:b[2], b[3]:b[4]] = values[v].T if len(b) > 5 and b[5] else values[v]
    return a


def task_preds(tg_handle):
    n = B.tn_taskgraph_num_vertices(tg_handle)
    return [B.tn_taskgraph_inputs(tg_handle, v) if B.tn_taskgraph_vertex(tg_handle, v).n_inputs else []
            for v in range(n)]


def serial_order_of(mg: M.MemGraph):
    return [v for v in mg.order if v < mg.n_task]


def check_all(preds, mg: M.MemGraph, n_random=20, seed=0, exhaustive=False):
    """The three requirements of Section 6 plus the run of many orders on the memory model."""
    M.check_forward_edges(mg)
    M.check_data_deps(preds, mg)
    M.check_race_free(mg)
    expected = M.taskgraph_values(preds, serial_order_of(mg))
    ref = M.simulate(mg, mg.order, preds, expected)
    assert ref["hw_live"] <= mg.cap
    orders = M.all_topological_orders(mg) if exhaustive else (
        M.random_topological_order(mg, np.random.default_rng(seed + i)) for i in range(n_random))
    count = 0
    for order in orders:
        r = M.simulate(mg, order, preds, expected)
        assert r["hw_live"] <= mg.cap
        assert r["results"] == ref["results"]
        count += 1
    return count, ref


def check_layer_rows(cfg, full, out, layer, seq_index, rows, tol, use_context, label="", wide_cache=None,
                     fuse_epilogues=0):
    """One layer of a deep stack held to the one-layer tolerance: the GPU run's own input rows of
    `layer` (x, or its hidden state after layer - 1) go through one oracle layer with the tiled
    execution's storage rounding, and the GPU's output rows of that layer (hidden state after it,
    or y) must agree within `tol`.  fuse_epilogues: the tiler option the run was compiled with (which
    tensors are never stored).  use_context: late rows attend to the GPU's stored keys and values
    of that layer, which are themselves held to `tol` on the sampled rows; otherwise `rows` must be
    a prefix 0..n-1.  `out` maps "h.l", "k.l", "v.l", "y" to the GPU's full tensors (storage type)."""
    from oracle import llama_ref as R
    from workloads import bf16_bits_to_f32

    def f64(a):
        return (bf16_bits_to_f32(a) if a.dtype == np.uint16 else a).astype(np.float64)

    base = seq_index * cfg.seq
    rows = np.asarray(rows)
    src = full["x"] if layer == 0 else out[f"h.{layer - 1}"]
    dst = out["y"] if layer == cfg.layers - 1 else out[f"h.{layer}"]
    wide_cache = {} if wide_cache is None else wide_cache  # layers that share their arrays share the float64 copy
    w = {}
    for k, a in full.items():
        if k.endswith(f".{layer}") and k.split(".")[0] in ("wq", "wk", "wv", "wo", "w1", "w2", "w3", "g1", "g2"):
            if id(a) not in wide_cache:
                wide_cache[id(a)] = R.widen_array(a)
            w[k] = wide_cache[id(a)]
    store = (lambda z: T.round_store(z, cfg.dtype))
    kc = vc = None
    if use_context:
        kc = f64(out[f"k.{layer}"][base:base + cfg.seq])
        vc = f64(out[f"v.{layer}"][base:base + cfg.seq])
    y, k, v = R.decoder_layer_rows(f64(src[base + rows]), rows, w, layer, cfg.n_heads, cfg.head_dim, cfg.eps,
                                   cfg.rope_base, k_ctx=kc, v_ctx=vc, store=store, fuse_epilogues=fuse_epilogues)
    errs = {"h": R.rel_err(f64(dst[base + rows]), y)}
    if use_context:
        errs["k"] = R.rel_err(kc[rows], k)
        errs["v"] = R.rel_err(vc[rows], v)
    print(f"{label} layer {layer}, sequence {seq_index}, {len(rows)} rows up to position {int(rows.max())}: "
          + ", ".join(f"{n} {e:.3e}" for n, e in errs.items()), flush=True)
    for n, e in errs.items():
        assert e < tol, (label, layer, n, e)
    return errs
