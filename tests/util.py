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
