"""GPU parity of the attention-block vertex alone (and of block + combine), through the C ABI on
hand-built taskgraphs, against the oracle's vertex semantics in float64.

A partial (unnormalised sums, a reference maximum m, the sum l of exp(s - m)) is not unique -- any
m serves as long as the three belong together -- so what is compared is what the partial stands
for: the normalised rows O / l and the log-sum-exp m + log l, per head.  The inputs are bf16 on
both sides, so the only differences are fp32 accumulation, the exponential, and the 16 bits the
kernel keeps of each probability: the bar is far below the bf16 tolerance of the whole layer."""
import numpy as np
import pytest

from oracle import llama_ref as R
from oracle import tiled as T
from paper_2405_16283_amd import binding as B

from test_gpu_backward_ops import Graph

pytestmark = pytest.mark.gpu


def _ranges(rows, tile):
    return [(a, min(a + tile, rows)) for a in range(0, rows, tile)]


def _block(hd, hpg, q_rows, kv_rows, tq, tk, q_pos0, k_pos0, causal, q_std=1.0, seed=0, combine_with=None):
    """Builds Q / K / V^T tile grids (one column tile holding hpg heads), one attn_block vertex, runs
    it, and returns (GPU partial, oracle partial, gw)."""
    rng = np.random.default_rng(seed)
    g = Graph("bf16")
    gw = hpg * hd
    scale = 1.0 / np.sqrt(hd)
    qt, kt = _ranges(q_rows, tq), _ranges(kv_rows, tk)

    def grid(rows, ranges, std, transpose=False):
        full = std * rng.standard_normal((rows, gw))
        vs, tiles = [], []
        for (r0, r1) in ranges:
            v, w = g.inp(full[r0:r1].T if transpose else full[r0:r1])
            vs.append(v)
            tiles.append(w)
        return vs, tiles

    q, Q = grid(q_rows, qt, q_std)
    k, K = grid(kv_rows, kt, 1.0)
    v, V = grid(kv_rows, kt, 1.0, transpose=True)
    params = dict(n_q_tiles=len(qt), n_kv_tiles=len(kt), n_col_tiles=1, head_dim=hd, q_pos0=q_pos0, k_pos0=k_pos0,
                  causal=int(causal), scale=scale, v_trans=1)
    blk = g.op(B.TN_OP_ATTN_BLOCK, q + k + v, q_rows, gw + 2 * hpg, f32=True, **params)
    (got,) = g.run([blk])
    ref = T._eval_vertex("attn_block", params, Q + K + V)
    return got, ref, gw


def _compare(got, ref, gw, hd, hpg, tol=1e-4):
    for h in range(hpg):
        sl = slice(h * hd, (h + 1) * hd)
        m_g, l_g = got[:, gw + h], got[:, gw + hpg + h]
        m_r, l_r = ref[:, gw + h], ref[:, gw + hpg + h]
        seen = l_r > 0
        # rows that see no key of this block: nothing summed, and marked as such
        assert np.all(l_g[~seen] == 0) and np.all(got[:, sl][~seen] == 0) and np.all(np.isneginf(m_g[~seen]))
        assert np.all(np.isfinite(got[seen])) and np.all(l_g[seen] > 0)
        o_g = got[:, sl][seen] / l_g[seen][:, None]
        o_r = ref[:, sl][seen] / l_r[seen][:, None]
        err_o = R.rel_err(o_g, o_r)
        err_lse = float(np.max(np.abs((m_g[seen] + np.log(l_g[seen])) - (m_r[seen] + np.log(l_r[seen])))))
        print(f"  head {h}: {int(seen.sum())} rows, O/l rel err {err_o:.2e}, log-sum-exp abs err {err_lse:.2e}", flush=True)
        assert err_o < tol and err_lse < tol


CASES = [
    # hd, hpg, q_rows, kv_rows, tq, tk, q_pos0, k_pos0, causal, q_std
    (128, 2, 256, 384, 128, 128, 0, 0, False, 1.0),      # plain block, several chunks of keys
    (128, 1, 200, 328, 128, 128, 200, 64, True, 1.0),    # ragged rows both ways, the diagonal crosses the block
    (64, 2, 192, 320, 64, 64, 0, 0, True, 1.0),          # head size 64; keys beyond the last query are all masked
    (128, 4, 1024, 1024, 512, 512, 2048, 2048, True, 1.0),  # a diagonal block of the one-layer workload
    (128, 4, 1024, 1024, 512, 512, 2048, 0, True, 1.0),     # a block below the diagonal (the mask lets everything through)
    (128, 1, 128, 1024, 128, 256, 0, 0, False, 8.0),     # scores spread over hundreds of units: the running maximum moves a lot
    (64, 1, 96, 72, 64, 64, 0, 0, False, 4.0),           # fewer keys than a chunk, fewer rows than a workgroup
    (128, 1, 160, 256, 128, 128, 0, 96, True, 1.0),      # the first 96 queries see no key of this block
    (128, 2, 384, 448, 384, 64, 0, 0, False, 1.0),       # key tiles of one chunk each
]


@pytest.mark.parametrize("case", CASES)
def test_attention_block_against_the_oracle(case):
    hd, hpg, q_rows, kv_rows, tq, tk, q_pos0, k_pos0, causal, q_std = case
    print(f"[case] attn_block {case}", flush=True)
    got, ref, gw = _block(hd, hpg, q_rows, kv_rows, tq, tk, q_pos0, k_pos0, causal, q_std, seed=hd + q_rows)
    _compare(got, ref, gw, hd, hpg)


def test_blocks_and_combine_give_the_attention_of_the_whole_row():
    """Three key blocks of one query block (the last on the diagonal), merged by the combine vertex,
    against softmax attention over all keys at once."""
    hd, hpg, tile = 128, 2, 256
    gw, scale = hd * hpg, 1.0 / np.sqrt(128)
    rng = np.random.default_rng(3)
    g = Graph("bf16")
    q, Q = g.inp(rng.standard_normal((tile, gw)))
    ks, vs, K, V = [], [], [], []
    for j in range(3):
        kv, kw = g.inp(rng.standard_normal((tile, gw)))
        vv, vw = g.inp(rng.standard_normal((tile, gw)).T)
        ks.append(kv); vs.append(vv); K.append(kw); V.append(vw.T)
    parts = []
    for j in range(3):
        parts.append(g.op(B.TN_OP_ATTN_BLOCK, [q, ks[j], vs[j]], tile, gw + 2 * hpg, f32=True, n_q_tiles=1, n_kv_tiles=1,
                          n_col_tiles=1, head_dim=hd, q_pos0=2 * tile, k_pos0=j * tile, causal=int(j == 2), scale=scale,
                          v_trans=1))
    out = g.op(B.TN_OP_ATTN_COMBINE, parts, tile, gw, row0=0, col0=0, head_dim=hd, hpg=hpg)
    print("[case] attn_block x3 + combine", flush=True)
    (got,) = g.run([out])
    Kall, Vall = np.concatenate(K), np.concatenate(V)
    ref = np.zeros((tile, gw))
    for h in range(hpg):
        sl = slice(h * hd, (h + 1) * hd)
        s = Q[:, sl] @ Kall[:, sl].T * scale
        s = np.where(np.arange(3 * tile)[None, :] > (2 * tile + np.arange(tile))[:, None], -np.inf, s)
        p = np.exp(s - s.max(axis=1, keepdims=True))
        ref[:, sl] = (p / p.sum(axis=1, keepdims=True)) @ Vall[:, sl]
    err = R.rel_err(got, T.round_bf16(ref))
    print(f"  rel err after the bf16 store {err:.2e}", flush=True)
    assert err < 2.0 ** -7  # one bf16 rounding step now and then, nothing more
