"""Shapes and seeded random buffers of the synthetic LLaMA-shaped workloads.

Random numbers come from a counter-based generator: every element is a pure
function of (seed, tensor id, element index), so a buffer can be regenerated
anywhere, in any chunking, with the same bits.  Values are drawn in float64 and
rounded once to the storage type (fp32, or bf16 kept as uint16 bit patterns).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List, Tuple

import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


@dataclass(frozen=True)
class LlamaConfig:
    """One synthetic decoder workload (forward prefill)."""

    name: str
    layers: int
    d_model: int
    n_heads: int
    head_dim: int
    ffn: int
    seq: int
    batch: int
    dtype: str  # storage type of taskgraph tensors: "f32" or "bf16"
    tile: int  # edge of a GEMM / elementwise tile
    attn_block: int  # edge of a blocked-attention block (multiple of `tile`)
    cap_bytes: int  # GPU memory cap; 0 = derive as cap_frac x uncapped peak
    cap_frac: float
    weights_resident: bool  # True: weights pre-placed in GPU memory; False: streamed from host
    x_resident: bool  # same for the input embeddings
    eps: float = 1e-6
    rope_base: float = 10000.0
    decode_steps: int = 0  # single-row steps after the prefill of `seq` positions (one sequence only)

    @property
    def total_seq(self) -> int:
        """Positions per sequence: the prefill's plus the decode steps'."""
        return self.seq + self.decode_steps

    @property
    def tokens(self) -> int:
        return self.total_seq * self.batch

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def with_(self, **kw) -> "LlamaConfig":
        return replace(self, **kw)


CONFIGS: Dict[str, LlamaConfig] = {
    # 2-layer toy decoder, fp32, cap = 40 % of the uncapped peak working set
    "c1": LlamaConfig("c1", 2, 256, 4, 64, 688, 128, 1, "f32", 64, 64, 0, 0.40, False, False),
    # one LLaMA-7B-shaped layer, bf16 storage / fp32 accumulate, 2 GB cap
    "c2": LlamaConfig("c2", 1, 4096, 32, 128, 11008, 4096, 1, "bf16", 512, 1024,
                      2_000_000_000, 0.0, True, True),
    # 32-layer 7B prefill, weights streamed from pinned host memory, 16 GB cap
    "c3": LlamaConfig("c3", 32, 4096, 32, 128, 11008, 16384, 1, "bf16", 512, 1024,
                      16_000_000_000, 0.0, False, False),
    # 65B-shaped prefill, 48 GB cap
    "c4": LlamaConfig("c4", 80, 8192, 64, 128, 22016, 8192, 1, "bf16", 1024, 1024,
                      48_000_000_000, 0.0, False, False),
    # LoRA fine-tuning step on the 7B shape: 4 sequences of 4096 tokens, forward + backward, 32 GB cap
    "c5": LlamaConfig("c5", 32, 4096, 32, 128, 11008, 4096, 4, "bf16", 512, 1024,
                      32_000_000_000, 0.0, False, False),
    # small shapes with ragged row, column and K tails, used by the parity tests
    "ragged_f32": LlamaConfig("ragged_f32", 2, 192, 3, 64, 272, 160, 1, "f32", 64, 128,
                              0, 0.40, False, False),
    "ragged_bf16": LlamaConfig("ragged_bf16", 2, 256, 2, 128, 432, 320, 1, "bf16", 128, 256,
                               0, 0.40, False, False),
    # mid-size bf16 shape whose tiles (384, last ones 288) are cut by the 256x256 MFMA GEMM kernel into
    # blocks with ragged rows and columns, and whose attention blocks (768 = two row tiles, then 672)
    # go through the MFMA attention kernel with head size 128
    "mid_bf16": LlamaConfig("mid_bf16", 1, 1152, 9, 128, 1440, 1440, 1, "bf16", 384, 768,
                            0, 0.40, False, False),
    # prefill, then decode steps fixed in number: each step's keys and values join the cache as
    # single-row tiles (prefill lengths that leave ragged last tiles and, for bf16, two stripes)
    "decode_f32": LlamaConfig("decode_f32", 2, 256, 4, 64, 688, 120, 1, "f32", 64, 64,
                              0, 0.40, False, False, decode_steps=8),
    "decode_bf16": LlamaConfig("decode_bf16", 2, 256, 2, 128, 432, 320, 1, "bf16", 128, 256,
                               0, 0.40, False, False, decode_steps=9),
    "batch2_f32": LlamaConfig("batch2_f32", 1, 128, 2, 64, 176, 128, 2, "f32", 64, 64,
                              0, 0.50, False, False),
}


def config(name: str) -> LlamaConfig:
    return CONFIGS[name]


# --------------------------------------------------------------------------------------
# counter-based normal generator
# --------------------------------------------------------------------------------------

def _mix64(z: np.ndarray) -> np.ndarray:
    """splitmix64 finaliser on uint64 arrays (wrap-around arithmetic)."""
    z = (z + np.uint64(0x9E3779B97F4A7C15)) & _M64
    z = ((z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)) & _M64
    z = ((z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)) & _M64
    return z ^ (z >> np.uint64(31))


def normal(seed: int, tensor_id: int, n: int, start: int = 0) -> np.ndarray:
    """n standard-normal float64 values: elements start..start+n-1 of stream (seed, tensor_id)."""
    with np.errstate(over="ignore"):
        key = _mix64(np.array([(seed * 0x100000001B3 + tensor_id) & 0xFFFFFFFFFFFFFFFF], dtype=np.uint64))
        idx = np.arange(start, start + n, dtype=np.uint64)
        h1 = _mix64(key ^ (idx * np.uint64(2)))
        h2 = _mix64(key ^ (idx * np.uint64(2) + np.uint64(1)))
    u1 = ((h1 >> np.uint64(11)).astype(np.float64) + 1.0) * (1.0 / 9007199254740992.0)  # (0,1]
    u2 = (h2 >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)  # [0,1)
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float values to bfloat16 (nearest, ties to even); returns uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------------------
# LLaMA-shaped inputs
# --------------------------------------------------------------------------------------

_KIND_ID = {"x": 1, "wq": 2, "wk": 3, "wv": 4, "wo": 5, "w1": 6, "w3": 7, "w2": 8, "g1": 9, "g2": 10,
            "aq": 11, "bq": 12, "av": 13, "bv": 14, "probe": 15}


def _tensor(seed, cfg, kind, layer, shape, mean, std, chunk=1 << 22):
    n = int(np.prod(shape))
    tid = _KIND_ID[kind] + 16 * (layer + 1)
    if cfg.dtype == "f32":
        out = np.empty(n, dtype=np.float32)
    else:
        out = np.empty(n, dtype=np.uint16)
    for s in range(0, n, chunk):
        m = min(chunk, n - s)
        v = mean + std * normal(seed, tid, m, s)
        out[s:s + m] = v.astype(np.float32) if cfg.dtype == "f32" else to_bf16_bits(v)
    return out.reshape(shape)


def make_llama_inputs(cfg: LlamaConfig, seed: int, distinct_layers: int = 0, workers: int = 0) -> Dict[str, np.ndarray]:
    """Full (untiled) input tensors in storage dtype.

    Keys: "x" [tokens, d]; per layer l: "wq.l", "wk.l", "wv.l", "wo.l" [d, d], "w1.l", "w3.l"
    [d, F], "w2.l" [F, d] (all right-multiplied: y = x @ W, row-major [in, out]); "g1.l",
    "g2.l" [d].  Weights ~ N(0, 0.02), x ~ N(0, 1), gains 1 + 0.02 N(0, 1).  bf16 tensors are
    uint16 bit patterns.

    distinct_layers = k > 0: only the first k layers get tensors of their own; layer l uses the
    very arrays of layer l mod k (same objects), which keeps the host footprint of the deep
    workloads small without changing any shape, vertex count or transfer.
    workers > 1 generates the tensors on that many threads (same bits: every element is a pure
    function of its index).
    """
    d, f = cfg.d_model, cfg.ffn
    k = cfg.layers if distinct_layers <= 0 else min(distinct_layers, cfg.layers)
    jobs = [("x", "x", -1, (cfg.tokens, d), 0.0, 1.0)]
    for l in range(k):
        for kind, shape in (("wq", (d, d)), ("wk", (d, d)), ("wv", (d, d)), ("wo", (d, d)),
                            ("w1", (d, f)), ("w3", (d, f)), ("w2", (f, d))):
            jobs.append((f"{kind}.{l}", kind, l, shape, 0.0, 0.02))
        jobs.append((f"g1.{l}", "g1", l, (d,), 1.0, 0.02))
        jobs.append((f"g2.{l}", "g2", l, (d,), 1.0, 0.02))

    def make(j):
        return _tensor(seed, cfg, j[1], j[2], j[3], j[4], j[5])

    if workers > 1:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(workers) as pool:
            arrays = list(pool.map(make, jobs))
    else:
        arrays = [make(j) for j in jobs]
    t: Dict[str, np.ndarray] = {j[0]: a for j, a in zip(jobs, arrays)}
    for l in range(k, cfg.layers):
        for kind in ("wq", "wk", "wv", "wo", "w1", "w3", "w2", "g1", "g2"):
            t[f"{kind}.{l}"] = t[f"{kind}.{l % k}"]
    return t


def make_lora_inputs(cfg: LlamaConfig, seed: int, rank: int = 16, b_std: float = 0.0) -> Dict[str, np.ndarray]:
    """Adapter matrices and the probe of the fine-tuning workload, in storage dtype.

    Keys per layer l: "aq.l", "av.l" [d, rank] ~ N(0, 0.02); "bq.l", "bv.l" [rank, d], zero as at
    the start of fine-tuning unless b_std > 0 (then N(0, b_std): a later step, where the gradient
    of A does not vanish); "probe" [tokens, d] ~ N(0, 1), the fixed tensor the loss sums y against.
    """
    d = cfg.d_model
    t: Dict[str, np.ndarray] = {"probe": _tensor(seed, cfg, "probe", -1, (cfg.tokens, d), 0.0, 1.0)}
    for l in range(cfg.layers):
        for kind in ("aq", "av"):
            t[f"{kind}.{l}"] = _tensor(seed, cfg, kind, l, (d, rank), 0.0, 0.02)
        for kind in ("bq", "bv"):
            t[f"{kind}.{l}"] = _tensor(seed, cfg, kind, l, (rank, d), 0.0, b_std)
    return t


# --------------------------------------------------------------------------------------
# random dataflow graphs for the memory-planning tests
# --------------------------------------------------------------------------------------

def random_dag(seed: int, n: int, max_fanin: int = 3, n_inputs: int = 2,
               sizes: Tuple[int, ...] = (1,), p_output: float = 0.15
               ) -> Tuple[List[List[int]], List[int], List[int]]:
    """A seeded random dataflow graph in topological numbering.

    Returns (preds, size, outputs): preds[v] lists the producers vertex v reads (all < v; empty
    for the first n_inputs vertices), size[v] is the size of v's output in allocation units, and
    outputs lists the vertices whose result the caller wants back (every sink plus a few more).
    """
    rng = np.random.default_rng(seed)
    preds: List[List[int]] = []
    for v in range(n):
        if v < n_inputs:
            preds.append([])
        else:
            k = int(rng.integers(1, min(max_fanin, v) + 1))
            # bias towards recent producers so lifetimes are a mix of short and long
            cand = np.unique(np.concatenate([rng.integers(0, v, size=k), rng.integers(max(0, v - 3), v, size=1)]))
            preds.append([int(c) for c in cand[:max_fanin]])
    size = [int(rng.choice(sizes)) for _ in range(n)]
    consumed = {p for ps in preds for p in ps}
    outputs = [v for v in range(n) if v not in consumed]
    outputs += [v for v in range(n_inputs, n) if v in consumed and rng.random() < p_output]
    return preds, size, sorted(set(outputs))
