"""ctypes binding of include/turnip.h: same names, argument marshalling only.

Functions raise TurnipError(status, message) instead of returning a negative status.  Handles
are opaque ctypes pointers; the caller releases them with the matching *_destroy.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
# TURNIP_LIB names another build of the same library (a build with different compile-time tuning)
LIB_PATH = os.environ.get("TURNIP_LIB") or os.path.join(_HERE, "libturnip.so")

TN_OK, TN_ERR_INVALID, TN_ERR_NOT_TOPOLOGICAL, TN_ERR_CYCLE = 0, -1, -2, -3
TN_ERR_CAP_TOO_SMALL, TN_ERR_ARENA, TN_ERR_HIP, TN_ERR_SHAPE = -4, -5, -6, -7
TN_F32, TN_BF16 = 0, 1
TN_HOST, TN_DEVICE = 0, 1
(TN_OP_INPUT, TN_OP_GEMM, TN_OP_RMS_STAT, TN_OP_RMS_APPLY, TN_OP_ROPE, TN_OP_ATTN_BLOCK,
 TN_OP_ATTN_COMBINE, TN_OP_SILU_MUL, TN_OP_ADD, TN_OP_SILU_MUL_BWD, TN_OP_RMS_BWD_STAT, TN_OP_RMS_BWD_APPLY,
 TN_OP_ATTN_BWD, TN_OP_TRANSPOSE, TN_OP_SUM, TN_OP_ZERO, TN_OP_SUM_INTO, TN_OP_SOFTMAX_STAT, TN_OP_SOFTMAX_APPLY) = range(19)
(TN_T_X, TN_T_WQ, TN_T_WK, TN_T_WV, TN_T_WO, TN_T_W1, TN_T_W3, TN_T_W2, TN_T_G1, TN_T_G2, TN_T_Y, TN_T_K, TN_T_V,
 TN_T_AQ, TN_T_BQ, TN_T_AV, TN_T_BV, TN_T_PROBE, TN_T_DAQ, TN_T_DBQ, TN_T_DAV, TN_T_DBV, TN_T_DX, TN_T_H) = range(24)
(TN_MG_INPUT, TN_MG_LOAD, TN_MG_OP, TN_MG_OFFLOAD, TN_MG_RELOAD, TN_MG_DROP, TN_MG_STORE, TN_MG_JOIN) = range(8)
TN_EDGE_DATA, TN_EDGE_MEM, TN_EDGE_ORDER = 0, 1, 2
TN_POLICY_FIFO, TN_POLICY_LIFO, TN_POLICY_RANDOM, TN_POLICY_BY_ORDER, TN_POLICY_IN_ORDER = 0, 1, 2, 3, 4
TN_COPY_AUTO, TN_COPY_MEMCPY, TN_COPY_KERNEL = 0, 1, 2
TN_COPY_KERNEL_IN = 3
UINT64_MAX = (1 << 64) - 1


class TurnipError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"[{status}] {message}")
        self.status = status
        self.message = message


class tn_tensor_desc(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("rows", C.c_int32), ("cols", C.c_int32)]


class tn_op_params(C.Structure):
    _fields_ = [("nk", C.c_int32), ("d", C.c_int32), ("eps", C.c_float), ("pos0", C.c_int32),
                ("col0", C.c_int32), ("head_dim", C.c_int32), ("rope_base", C.c_float),
                ("n_q_tiles", C.c_int32), ("n_kv_tiles", C.c_int32), ("n_col_tiles", C.c_int32),
                ("q_pos0", C.c_int32), ("k_pos0", C.c_int32), ("causal", C.c_int32),
                ("scale", C.c_float), ("row0", C.c_int32), ("hpg", C.c_int32), ("trans_b", C.c_int32),
                ("trans_c", C.c_int32), ("v_trans", C.c_int32), ("trans_a", C.c_int32), ("mode", C.c_int32)]


class tn_tg_vertex(C.Structure):
    _fields_ = [("kind", C.c_int32), ("residency", C.c_int32), ("n_inputs", C.c_int32),
                ("output_index", C.c_int32), ("desc", tn_tensor_desc), ("params", tn_op_params)]


class tn_llama_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("layers", "d_model", "n_heads", "head_dim", "ffn", "seq", "batch",
                                          "dtype", "tile", "attn_block")] + \
               [("eps", C.c_float), ("rope_base", C.c_float), ("weights_residency", C.c_int32),
                ("x_residency", C.c_int32), ("kv_outputs", C.c_int32), ("weights_transposed", C.c_int32),
                ("v_transposed", C.c_int32), ("lora_rank", C.c_int32), ("train", C.c_int32), ("k_split", C.c_int32), ("materialize_scores", C.c_int32),
                ("checkpoint", C.c_int32), ("hidden_outputs", C.c_int32),
                ("output_layer_stride", C.c_int32), ("decode_steps", C.c_int32),
                ("attn_whole_rows", C.c_int32), ("checkpoint_layers", C.c_int32), ("fuse_epilogues", C.c_int32), ("recompute_normed", C.c_int32), ("recompute_gate_up", C.c_int32)]


class tn_llama_binding(C.Structure):
    _fields_ = [("vid", C.c_int32), ("tensor", C.c_int32), ("layer", C.c_int32), ("row0", C.c_int32),
                ("row1", C.c_int32), ("col0", C.c_int32), ("col1", C.c_int32), ("transposed", C.c_int32)]


class tn_compile_opts(C.Structure):
    _fields_ = [("max_lookahead_bytes", C.c_uint64), ("drop_clean_inputs", C.c_int32),
                ("fix_order", C.c_int32), ("prune_superfluous", C.c_int32), ("alignment", C.c_uint32),
                ("evict_ahead_bytes", C.c_uint64), ("next_fit", C.c_int32)]


class tn_mg_vertex(C.Structure):
    _fields_ = [("kind", C.c_int32), ("op_kind", C.c_int32), ("src", C.c_int32), ("offset", C.c_int64),
                ("bytes", C.c_uint64), ("n_operands", C.c_int32), ("order_pos", C.c_int64)]


class tn_mg_edge(C.Structure):
    _fields_ = [("from_", C.c_int64), ("to", C.c_int64), ("kind", C.c_int32)]


class tn_mg_stats(C.Structure):
    _fields_ = [("cap", C.c_uint64), ("high_water", C.c_uint64), ("peak_live_bytes", C.c_uint64),
                ("host_arena_bytes", C.c_uint64)] + \
               [(n, C.c_int64) for n in ("n_task", "n_vertices", "n_edges", "n_mem_edges", "n_offload",
                                         "n_reload", "n_drop", "n_load", "n_store")] + \
               [(n, C.c_uint64) for n in ("offload_bytes", "reload_bytes", "load_bytes", "store_bytes")] + \
               [("n_revoked", C.c_int64), ("n_compactions", C.c_int64), ("n_increment", C.c_int64)]


class tn_exec_opts(C.Structure):
    _fields_ = [("policy", C.c_int32), ("order_seed", C.c_uint64), ("delay_seed", C.c_uint64),
                ("max_delay_us", C.c_uint32), ("max_batch", C.c_int32), ("profile", C.c_int32),
                ("max_transfers", C.c_int32), ("copy_engine", C.c_int32),
                ("max_gemm_inflight", C.c_int32), ("queue_depth", C.c_int32), ("transfer_depth", C.c_int32),
                ("copy_workgroups", C.c_int32), ("d2h_workgroups", C.c_int32), ("small_gemm_tiles", C.c_int32)]


class tn_launch_record(C.Structure):
    _fields_ = [("family", C.c_int32), ("n_vertices", C.c_int32), ("work", C.c_int64), ("amount", C.c_double),
                ("start_ms", C.c_float), ("end_ms", C.c_float)]


class tn_exec_report(C.Structure):
    _fields_ = [("wall_ms", C.c_double), ("h2d_bytes", C.c_uint64), ("d2h_bytes", C.c_uint64),
                ("n_vertices", C.c_int64), ("n_launches", C.c_int64), ("n_kernel_launches", C.c_int64),
                ("n_offload", C.c_int64), ("n_reload", C.c_int64), ("arena_high_water", C.c_uint64),
                ("gemm_ms", C.c_double), ("attn_ms", C.c_double), ("ewise_ms", C.c_double),
                ("h2d_ms", C.c_double), ("d2h_ms", C.c_double),
                ("gemm_launches", C.c_int64), ("attn_launches", C.c_int64), ("ewise_launches", C.c_int64),
                ("gemm_flops", C.c_double), ("attn_flops", C.c_double), ("ewise_bytes", C.c_double),
                ("kernel_busy_ms", C.c_double), ("idle_frac", C.c_double), ("idle_frac_wall", C.c_double),
                ("untimed_launches", C.c_int64)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


_P = C.c_void_p
# name -> (restype, argtypes); every symbol include/turnip.h declares
SIGNATURES = {
    "tn_last_error": (C.c_char_p, []),
    "tn_taskgraph_create": (C.c_int32, [C.POINTER(_P)]),
    "tn_taskgraph_destroy": (None, [_P]),
    "tn_taskgraph_add_input": (C.c_int32, [_P, C.POINTER(tn_tensor_desc), C.c_int32, C.POINTER(C.c_int32)]),
    "tn_taskgraph_add_op": (C.c_int32, [_P, C.c_int32, C.POINTER(tn_op_params), C.POINTER(C.c_int32), C.c_int32,
                                        C.POINTER(tn_tensor_desc), C.POINTER(C.c_int32)]),
    "tn_taskgraph_mark_output": (C.c_int32, [_P, C.c_int32]),
    "tn_taskgraph_num_vertices": (C.c_int64, [_P]),
    "tn_taskgraph_num_outputs": (C.c_int64, [_P]),
    "tn_taskgraph_vertex": (C.c_int32, [_P, C.c_int32, C.POINTER(tn_tg_vertex)]),
    "tn_taskgraph_inputs": (C.c_int32, [_P, C.c_int32, C.POINTER(C.c_int32), C.c_int32]),
    "tn_taskgraph_level_order": (C.c_int32, [_P, C.POINTER(C.c_int32), C.c_int64]),
    "tn_taskgraph_clustered_order": (C.c_int32, [_P, C.POINTER(C.c_int32), C.c_int64]),
    "tn_build_llama": (C.c_int32, [C.POINTER(tn_llama_config), C.POINTER(_P)]),
    "tn_taskgraph_num_bindings": (C.c_int64, [_P]),
    "tn_taskgraph_binding": (C.c_int32, [_P, C.c_int64, C.POINTER(tn_llama_binding)]),
    "tn_compile": (C.c_int32, [_P, C.POINTER(C.c_int32), C.c_uint64, C.POINTER(tn_compile_opts), C.POINTER(_P)]),
    "tn_memgraph_destroy": (None, [_P]),
    "tn_memgraph_num_vertices": (C.c_int64, [_P]),
    "tn_memgraph_vertex": (C.c_int32, [_P, C.c_int64, C.POINTER(tn_mg_vertex)]),
    "tn_memgraph_operands": (C.c_int32, [_P, C.c_int64, C.POINTER(C.c_int64), C.c_int32]),
    "tn_memgraph_num_edges": (C.c_int64, [_P]),
    "tn_memgraph_edge": (C.c_int32, [_P, C.c_int64, C.POINTER(tn_mg_edge)]),
    "tn_memgraph_stats": (C.c_int32, [_P, C.POINTER(tn_mg_stats)]),
    "tn_memgraph_dump_json": (C.c_int32, [_P, C.c_char_p]),
    "tn_memgraph_simulate": (C.c_int32, [_P, C.POINTER(C.c_int64), C.c_int64]),
    "tn_executor_create": (C.c_int32, [_P, _P, C.c_uint64, _P, C.c_uint64, C.POINTER(_P), C.c_int32, _P, _P,
                                       C.POINTER(_P)]),
    "tn_executor_destroy": (None, [_P]),
    "tn_executor_place_inputs": (C.c_int32, [_P, C.POINTER(_P)]),
    "tn_execute": (C.c_int32, [_P, C.POINTER(_P), C.POINTER(_P), C.POINTER(tn_exec_opts), C.POINTER(tn_exec_report)]),
    "tn_execute_static": (C.c_int32, [_P, C.POINTER(_P), C.POINTER(_P), C.POINTER(tn_exec_opts),
                                      C.POINTER(tn_exec_report)]),
    "tn_executor_last_order": (C.c_int64, [_P, C.POINTER(C.c_int64), C.c_int64]),
    "tn_executor_last_launches": (C.c_int64, [_P, C.POINTER(tn_launch_record), C.c_int64]),
}

_lib: Optional[C.CDLL] = None


def lib() -> C.CDLL:
    """Loads libturnip.so; there is no fallback when it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_2405_16283_amd.build`")
        l = C.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(l, name)
            fn.restype, fn.argtypes = res, args
        _lib = l
    return _lib


def _check(status: int):
    if status < 0:
        raise TurnipError(int(status), lib().tn_last_error().decode(errors="replace"))
    return status


def tn_last_error() -> str:
    return lib().tn_last_error().decode(errors="replace")


# ---- taskgraph -------------------------------------------------------------------------------
def tn_taskgraph_create():
    h = _P()
    _check(lib().tn_taskgraph_create(C.byref(h)))
    return h


def tn_taskgraph_destroy(tg):
    lib().tn_taskgraph_destroy(tg)


def tn_taskgraph_add_input(tg, dtype: int, rows: int, cols: int, residency: int) -> int:
    out = C.c_int32()
    d = tn_tensor_desc(dtype, rows, cols)
    _check(lib().tn_taskgraph_add_input(tg, C.byref(d), residency, C.byref(out)))
    return out.value


def tn_taskgraph_add_op(tg, kind: int, params: tn_op_params, inputs: Sequence[int], dtype: int, rows: int,
                        cols: int) -> int:
    out = C.c_int32()
    arr = (C.c_int32 * max(1, len(inputs)))(*inputs)
    d = tn_tensor_desc(dtype, rows, cols)
    _check(lib().tn_taskgraph_add_op(tg, kind, C.byref(params), arr, len(inputs), C.byref(d), C.byref(out)))
    return out.value


def tn_taskgraph_mark_output(tg, v: int):
    _check(lib().tn_taskgraph_mark_output(tg, v))


def tn_taskgraph_num_vertices(tg) -> int:
    return _check(lib().tn_taskgraph_num_vertices(tg))


def tn_taskgraph_num_outputs(tg) -> int:
    return _check(lib().tn_taskgraph_num_outputs(tg))


def tn_taskgraph_vertex(tg, v: int) -> tn_tg_vertex:
    out = tn_tg_vertex()
    _check(lib().tn_taskgraph_vertex(tg, v, C.byref(out)))
    return out


def tn_taskgraph_inputs(tg, v: int) -> List[int]:
    n = _check(lib().tn_taskgraph_inputs(tg, v, None, 0))
    buf = (C.c_int32 * max(1, n))()
    _check(lib().tn_taskgraph_inputs(tg, v, buf, n))
    return list(buf[:n])


def tn_build_llama(cfg: tn_llama_config):
    h = _P()
    _check(lib().tn_build_llama(C.byref(cfg), C.byref(h)))
    return h


def tn_taskgraph_num_bindings(tg) -> int:
    return _check(lib().tn_taskgraph_num_bindings(tg))


def tn_taskgraph_binding(tg, i: int) -> tn_llama_binding:
    out = tn_llama_binding()
    _check(lib().tn_taskgraph_binding(tg, i, C.byref(out)))
    return out


# ---- compile ---------------------------------------------------------------------------------
def tn_taskgraph_level_order(tg) -> List[int]:
    n = tn_taskgraph_num_vertices(tg)
    buf = (C.c_int32 * max(1, n))()
    _check(lib().tn_taskgraph_level_order(tg, buf, n))
    return list(buf[:n])


def tn_taskgraph_clustered_order(tg) -> List[int]:
    n = tn_taskgraph_num_vertices(tg)
    buf = (C.c_int32 * max(1, n))()
    _check(lib().tn_taskgraph_clustered_order(tg, buf, n))
    return list(buf[:n])


def tn_compile(tg, order: Optional[Sequence[int]], gpu_cap_bytes: int, opts: Optional[tn_compile_opts] = None):
    h = _P()
    arr = None
    if order is not None:
        arr = (C.c_int32 * len(order))(*order)
    _check(lib().tn_compile(tg, arr, gpu_cap_bytes, C.byref(opts) if opts is not None else None, C.byref(h)))
    return h


def tn_memgraph_destroy(mg):
    lib().tn_memgraph_destroy(mg)


def tn_memgraph_num_vertices(mg) -> int:
    return _check(lib().tn_memgraph_num_vertices(mg))


def tn_memgraph_vertex(mg, i: int) -> tn_mg_vertex:
    out = tn_mg_vertex()
    _check(lib().tn_memgraph_vertex(mg, i, C.byref(out)))
    return out


def tn_memgraph_operands(mg, i: int, n: Optional[int] = None) -> List[int]:
    if n is None:
        n = _check(lib().tn_memgraph_operands(mg, i, None, 0))
    buf = (C.c_int64 * max(1, n))()
    _check(lib().tn_memgraph_operands(mg, i, buf, n))
    return list(buf[:n])


def tn_memgraph_num_edges(mg) -> int:
    return _check(lib().tn_memgraph_num_edges(mg))


def tn_memgraph_edge(mg, i: int) -> tn_mg_edge:
    out = tn_mg_edge()
    _check(lib().tn_memgraph_edge(mg, i, C.byref(out)))
    return out


def tn_memgraph_stats(mg) -> tn_mg_stats:
    out = tn_mg_stats()
    _check(lib().tn_memgraph_stats(mg, C.byref(out)))
    return out


def tn_memgraph_dump_json(mg, path: str):
    _check(lib().tn_memgraph_dump_json(mg, path.encode()))


def tn_memgraph_simulate(mg, order: Optional[Sequence[int]] = None):
    if order is None:
        _check(lib().tn_memgraph_simulate(mg, None, 0))
    else:
        arr = (C.c_int64 * len(order))(*order)
        _check(lib().tn_memgraph_simulate(mg, arr, len(order)))


# ---- execute ---------------------------------------------------------------------------------
def tn_executor_create(mg, device_base: int, device_bytes: int, pinned_arena: int, arena_bytes: int,
                       compute_streams: Sequence[int], h2d_stream: int, d2h_stream: int):
    h = _P()
    cs = (_P * len(compute_streams))(*[_P(s) for s in compute_streams])
    _check(lib().tn_executor_create(mg, _P(device_base), device_bytes, _P(pinned_arena) if pinned_arena else None,
                                    arena_bytes, cs, len(compute_streams), _P(h2d_stream), _P(d2h_stream),
                                    C.byref(h)))
    return h


def tn_executor_destroy(ex):
    lib().tn_executor_destroy(ex)


def ptr_array(ptrs: Sequence[int]):
    """A C array of pointers from integer addresses (0 = NULL).  Callers that execute the same
    graph many times build it once and pass it in place of the list."""
    a = (_P * max(1, len(ptrs)))()
    for i, p in enumerate(ptrs):
        if p:
            a[i] = p
    return a


def _ptr_array(ptrs):
    return ptrs if isinstance(ptrs, C.Array) else ptr_array(ptrs)


def tn_executor_place_inputs(ex, host_inputs: Sequence[int]):
    _check(lib().tn_executor_place_inputs(ex, _ptr_array(host_inputs)))


def tn_execute(ex, host_inputs: Sequence[int], host_outputs: Sequence[int],
               opts: Optional[tn_exec_opts] = None) -> tn_exec_report:
    rep = tn_exec_report()
    _check(lib().tn_execute(ex, _ptr_array(host_inputs), _ptr_array(host_outputs),
                            C.byref(opts) if opts is not None else None, C.byref(rep)))
    return rep


def tn_execute_static(ex, host_inputs: Sequence[int], host_outputs: Sequence[int],
                      opts: Optional[tn_exec_opts] = None) -> tn_exec_report:
    rep = tn_exec_report()
    _check(lib().tn_execute_static(ex, _ptr_array(host_inputs), _ptr_array(host_outputs),
                                   C.byref(opts) if opts is not None else None, C.byref(rep)))
    return rep


def tn_executor_last_launches(ex):
    """The timed launches of the last profiled run as a structured numpy array
    (family, n_vertices, work, amount, start_ms, end_ms)."""
    import numpy as np
    n = lib().tn_executor_last_launches(ex, None, 0)
    _check(min(n, 0))
    buf = (tn_launch_record * max(1, n))()
    k = lib().tn_executor_last_launches(ex, buf, n)
    dt = np.dtype([("family", "<i4"), ("n_vertices", "<i4"), ("work", "<i8"), ("amount", "<f8"), ("start_ms", "<f4"),
                   ("end_ms", "<f4")])
    return np.frombuffer(buf, dtype=dt, count=max(0, k)).copy()


def tn_executor_last_order(ex, n: int) -> List[int]:
    buf = (C.c_int64 * max(1, n))()
    k = lib().tn_executor_last_order(ex, buf, n)
    return list(buf[:max(0, k)])
