"""GPU parity of the reverse-mode vertex kinds, one kind at a time, through the C ABI on
hand-built taskgraphs.  Expected values come from the float64 oracle: the forward definitions of
oracle/llama_ref.py and oracle/lora_ref.py differentiated by torch on the CPU."""
import numpy as np
import pytest
import torch

from oracle import llama_ref as R
from oracle import lora_ref as L
from paper_2405_16283_amd import binding as B
from workloads import bf16_bits_to_f32, to_bf16_bits

pytestmark = pytest.mark.gpu
TOL = {"f32": 1e-4, "bf16": 2e-2}


class Graph:
    """A taskgraph under construction together with the host buffers of its inputs."""

    def __init__(self, dtype):
        self.dtype = dtype
        self.code = B.TN_F32 if dtype == "f32" else B.TN_BF16
        self.tg = B.tn_taskgraph_create()
        self.host = {}

    def store(self, a):
        a = np.ascontiguousarray(a, dtype=np.float32)
        return a if self.dtype == "f32" else to_bf16_bits(a).reshape(a.shape)

    def widen(self, a):
        return (a if a.dtype == np.float32 else bf16_bits_to_f32(a)).astype(np.float64)

    def inp(self, a, f32=False):
        """Adds an input holding `a` rounded to the graph's storage type (or kept fp32); returns
        (vertex, the values as the GPU sees them, float64)."""
        a = np.atleast_2d(a)
        s = np.ascontiguousarray(a, dtype=np.float32) if f32 else self.store(a)
        v = B.tn_taskgraph_add_input(self.tg, B.TN_F32 if f32 else self.code, a.shape[0], a.shape[1], B.TN_HOST)
        self.host[v] = torch.from_numpy(s.view(np.int16) if s.dtype == np.uint16 else s).pin_memory()
        return v, self.widen(s)

    def op(self, kind, ins, rows, cols, f32=False, **params):
        return B.tn_taskgraph_add_op(self.tg, kind, B.tn_op_params(**params), ins, B.TN_F32 if f32 else self.code,
                                     rows, cols)

    def run(self, outs):
        shapes = []
        for v in outs:
            B.tn_taskgraph_mark_output(self.tg, v)
            x = B.tn_taskgraph_vertex(self.tg, v)
            shapes.append((x.desc.rows, x.desc.cols, x.desc.dtype))
        n = B.tn_taskgraph_num_vertices(self.tg)
        cap = 64 << 20
        mg = B.tn_compile(self.tg, None, cap, None)
        dev = torch.empty(cap, dtype=torch.uint8, device="cuda:0")
        streams = [torch.cuda.Stream() for _ in range(3)]
        bufs = [torch.zeros(r * c, dtype=torch.float32 if dt == B.TN_F32 else torch.int16).pin_memory()
                for r, c, dt in shapes]
        ex = B.tn_executor_create(mg, dev.data_ptr(), cap, 0, 0, [streams[0].cuda_stream], streams[1].cuda_stream,
                                  streams[2].cuda_stream)
        try:
            ptrs = [self.host[v].data_ptr() if v in self.host else 0 for v in range(n)]
            B.tn_execute(ex, ptrs, [b.data_ptr() for b in bufs], B.tn_exec_opts(policy=B.TN_POLICY_RANDOM, order_seed=1))
        finally:
            B.tn_executor_destroy(ex)
            B.tn_memgraph_destroy(mg)
            B.tn_taskgraph_destroy(self.tg)
        res = []
        for b, (r, c, dt) in zip(bufs, shapes):
            a = b.numpy()
            a = a.astype(np.float64) if dt == B.TN_F32 else bf16_bits_to_f32(a.view(np.uint16)).astype(np.float64)
            res.append(a.reshape(r, c))
        return res


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_gemm_with_transposed_a(dtype):
    rng = np.random.default_rng(0)
    g = Graph(dtype)
    a0, A0 = g.inp(rng.standard_normal((40, 24)))   # stored [K, rows]
    a1, A1 = g.inp(rng.standard_normal((56, 24)))
    b0, B0 = g.inp(rng.standard_normal((40, 72)))   # [K, cols]
    b1, B1 = g.inp(rng.standard_normal((56, 72)))
    c = g.op(B.TN_OP_GEMM, [a0, a1, b0, b1], 24, 72, nk=2, trans_a=1)
    (out,) = g.run([c])
    assert R.rel_err(out, A0.T @ B0 + A1.T @ B1) < TOL[dtype]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_inverse_rotation(dtype):
    rng = np.random.default_rng(1)
    g = Graph(dtype)
    x, X = g.inp(rng.standard_normal((48, 128)))
    y = g.op(B.TN_OP_ROPE, [x], 48, 128, pos0=100, col0=0, head_dim=64, rope_base=10000.0, mode=1)
    (out,) = g.run([y])
    pos = np.arange(100, 148)
    ref = np.concatenate([R.rope(X[:, :64], -pos, 10000.0), R.rope(X[:, 64:], -pos, 10000.0)], axis=1)
    assert R.rel_err(out, ref) < TOL[dtype]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_silu_mul_backward(dtype):
    rng = np.random.default_rng(2)
    g = Graph(dtype)
    da, DA = g.inp(rng.standard_normal((37, 50)))
    ga, GA = g.inp(2.0 * rng.standard_normal((37, 50)))
    up, UP = g.inp(rng.standard_normal((37, 50)))
    dg = g.op(B.TN_OP_SILU_MUL_BWD, [da, ga, up], 37, 50, mode=0)
    du = g.op(B.TN_OP_SILU_MUL_BWD, [da, ga, up], 37, 50, mode=1)
    out_g, out_u = g.run([dg, du])
    tg_, tu = torch.tensor(GA, requires_grad=True), torch.tensor(UP, requires_grad=True)
    (tg_ * torch.sigmoid(tg_) * tu * torch.tensor(DA)).sum().backward()
    assert R.rel_err(out_g, tg_.grad.numpy()) < TOL[dtype]
    assert R.rel_err(out_u, tu.grad.numpy()) < TOL[dtype]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("residual", [False, True])
def test_rmsnorm_backward(dtype, residual):
    rng = np.random.default_rng(3)
    g = Graph(dtype)
    rows, cols, eps = 21, [32, 32, 24], 1e-6
    d = sum(cols)
    xs = [g.inp(rng.standard_normal((rows, c))) for c in cols]
    dys = [g.inp(rng.standard_normal((rows, c))) for c in cols]
    gs = [g.inp(1.0 + 0.1 * rng.standard_normal((1, c))) for c in cols]
    rs = [g.inp(rng.standard_normal((rows, c))) for c in cols]
    stat = g.op(B.TN_OP_RMS_STAT, [v for v, _ in xs], rows, 1, f32=True, d=d, eps=eps)
    dot = g.op(B.TN_OP_RMS_BWD_STAT, [v for v, _ in dys] + [v for v, _ in xs] + [v for v, _ in gs], rows, 1, f32=True,
               nk=len(cols))
    outs = []
    for j, c in enumerate(cols):
        ins = [dys[j][0], xs[j][0], stat, dot, gs[j][0]] + ([rs[j][0]] if residual else [])
        outs.append(g.op(B.TN_OP_RMS_BWD_APPLY, ins, rows, c, d=d))
    got = np.concatenate(g.run(outs), axis=1)
    X = torch.tensor(np.concatenate([a for _, a in xs], axis=1), requires_grad=True)
    G = torch.tensor(np.concatenate([a for _, a in gs], axis=1))
    DY = torch.tensor(np.concatenate([a for _, a in dys], axis=1))
    (L._rmsnorm(X, G, eps) * DY).sum().backward()
    ref = X.grad.numpy() + (np.concatenate([a for _, a in rs], axis=1) if residual else 0.0)
    assert R.rel_err(got, ref) < TOL[dtype]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_transpose(dtype):
    rng = np.random.default_rng(5)
    # odd shapes (element by element), multiples of 8 that are ragged against the 64x64 pieces (16-byte
    # pieces for bf16), and the skinny shapes of the adapter tiles
    for rows, cols in ((70, 150), (72, 152), (512, 16), (16, 512), (128, 64)):
        g = Graph(dtype)
        x, X = g.inp(rng.standard_normal((rows, cols)))
        (out,) = g.run([g.op(B.TN_OP_TRANSPOSE, [x], cols, rows)])
        np.testing.assert_array_equal(out, X.T)


@pytest.mark.parametrize("dtype,hd,v_trans,aux", [("f32", 64, 0, 0), ("f32", 64, 1, 0), ("bf16", 128, 1, 0), ("bf16", 64, 0, 0),
                                                  ("bf16", 128, 0, 1), ("bf16", 64, 0, 1), ("f32", 64, 0, 1)])
def test_attention_backward(dtype, hd, v_trans, aux):
    """Two heads, 96 queries at positions 64.. against 160 keys from position 0, causal; Q rows in
    tiles of 64 (ragged), K/V rows in tiles of 64, one column tile per head."""
    rng = np.random.default_rng(4)
    g = Graph(dtype)
    nq_rows, nkv_rows, q_pos0, hpg = 96, 160, 64, 2
    gw, scale = hpg * hd, 1.0 / np.sqrt(hd)
    qt, kt = [(0, 64), (64, 96)], [(0, 64), (64, 128), (128, 160)]

    def grid(rows, ranges, std, transpose=False):
        full = std * rng.standard_normal((rows, gw))
        vs, wide = [], np.zeros((rows, gw))
        for (r0, r1) in ranges:
            for h in range(hpg):
                tile = full[r0:r1, h * hd:(h + 1) * hd]
                v, w = g.inp(tile.T if transpose else tile)
                vs.append(v)
                wide[r0:r1, h * hd:(h + 1) * hd] = w.T if transpose else w
        return vs, wide

    q, Q = grid(nq_rows, qt, 1.0)
    k, K = grid(nkv_rows, kt, 1.0)
    v, V = grid(nkv_rows, kt, 1.0, transpose=bool(v_trans))
    do, DO = grid(nq_rows, qt, 1.0)
    common = dict(n_q_tiles=len(qt), n_kv_tiles=len(kt), n_col_tiles=hpg, head_dim=hd, q_pos0=q_pos0, k_pos0=0,
                  causal=1, scale=scale, v_trans=v_trans)
    # statistics per Q row tile
    stats = []
    for i, (r0, r1) in enumerate(qt):
        ins = q[i * hpg:(i + 1) * hpg] + k + v + do[i * hpg:(i + 1) * hpg]
        p = dict(common, n_q_tiles=1, q_pos0=q_pos0 + r0)
        stats.append(g.op(B.TN_OP_ATTN_BWD, ins, r1 - r0, 2 * hpg, f32=True, mode=0, **p))
    def tr(vs, ranges):  # transposes of a grid's tiles, as vertices (aux: what the MFMA kernels read)
        out = []
        for i, (r0, r1) in enumerate(ranges):
            for h in range(hpg):
                out.append(g.op(B.TN_OP_TRANSPOSE, [vs[i * hpg + h]], hd, r1 - r0))
        return out

    base = q + k + v + do + stats
    dq = g.op(B.TN_OP_ATTN_BWD, base + (tr(k, kt) if aux else []), nq_rows, gw, mode=1, trans_a=aux, **common)
    dk = g.op(B.TN_OP_ATTN_BWD, base + (tr(q, qt) if aux else []), nkv_rows, gw, mode=2, trans_a=aux, **common)
    dv = g.op(B.TN_OP_ATTN_BWD, base + (tr(do, qt) if aux else []), nkv_rows, gw, mode=3, trans_a=aux, **common)
    got = g.run(stats + [dq, dk, dv])
    got_stats = np.concatenate(got[:len(qt)], axis=0)
    tq, tk, tv = (torch.tensor(a, requires_grad=True) for a in (Q, K, V))
    lse_ref, d_ref = np.zeros((nq_rows, hpg)), np.zeros((nq_rows, hpg))
    loss = 0.0
    for h in range(hpg):
        sl = slice(h * hd, (h + 1) * hd)
        s = tq[:, sl] @ tk[:, sl].T * scale
        mask = torch.arange(nkv_rows)[None, :] > (q_pos0 + torch.arange(nq_rows))[:, None]
        s = s.masked_fill(mask, float("-inf"))
        p = torch.softmax(s, dim=-1)
        o = p @ tv[:, sl]
        loss = loss + (o * torch.tensor(DO[:, sl])).sum()
        lse_ref[:, h] = torch.logsumexp(s, dim=-1).detach().numpy()
        d_ref[:, h] = (o.detach().numpy() * DO[:, sl]).sum(axis=1)
    loss.backward()
    tol = TOL[dtype]
    assert R.rel_err(got_stats[:, :hpg], lse_ref) < tol
    assert R.rel_err(got_stats[:, hpg:], d_ref) < tol
    assert R.rel_err(got[-3], tq.grad.numpy()) < tol
    assert R.rel_err(got[-2], tk.grad.numpy()) < tol
    assert R.rel_err(got[-1], tv.grad.numpy()) < tol
