"""CPU ORACLE (test infrastructure, not the product) -- LoRA fine-tuning step: forward, a linear
probe loss and the gradients of the adapter matrices, in float64.

The paper's training experiment (Experiments, item 2) fine-tunes LLaMA with low-rank adapters on
frozen base weights; it does not spell the math out.  Reading used here (the workload list's):
adapters of rank r on the query and value projections only,

    q = a Wq + (a Aq) Bq,        v = a Wv + (a Av) Bv,        a = RMSNorm(x; g1),

everything else as in `llama_ref.decoder_layer`; the loss is L = sum(y_final * probe) with a fixed
probe tensor, so that dL/dy_final = probe; the wanted results are dL/dAq, dL/dBq, dL/dAv, dL/dBv
of every layer (and dL/dx, which costs nothing extra and pins the whole backward chain).

The forward pass is written out in plain PyTorch CPU ops in float64, step by step like
`llama_ref`; the gradients are those of torch's reverse-mode differentiation of exactly that
forward.  Pins (tests/test_oracle_lora.py): the forward equals `llama_ref`'s NumPy forward on
merged weights W + A B; gradients against central finite differences; dA == 0 exactly when
B == 0, and dB == (a A)^T dq in that case; gradients are linear in the probe.

Storage rounding.  The tiled execution keeps every taskgraph tensor in the storage type, so with
bf16 storage each stored tensor -- and, in the reverse pass, the gradient that arrives at it -- is
rounded to bf16 (round to nearest, ties to even).  `loss_and_grads(..., storage="bf16")` models
that: `_Stored` rounds a tensor on the way forward and the gradient on the way back, at the
tensors the layer stores (norm outputs, projections, low-rank activations, rotated q and k, the
attention output, residual sums, gate, up, their product).  It does not model the tiling (partial
sums of the reverse pass that the tiled form stores separately), so it measures how far a bf16
pipeline of this depth may stand from the exact result, not the bits of any one of them.  Pins:
the rounding against hand-worked bit patterns, and storage=None equal to the plain form.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this package.
"""
from __future__ import annotations

from typing import Dict, Tuple

import numpy as np
import torch


def round_bf16(t: torch.Tensor) -> torch.Tensor:
    """float64 -> nearest bfloat16 (ties to even) -> float64, on the bit pattern of the float32 value."""
    f = t.to(torch.float32)
    bits = f.view(torch.int32)
    rounded = (bits + 0x7FFF + ((bits >> 16) & 1)) & ~0xFFFF
    out = rounded.view(torch.float32)
    return torch.where(torch.isfinite(f), out, f).to(torch.float64)


class _Stored(torch.autograd.Function):
    """A tensor written to bf16 storage: rounded going forward, its gradient rounded coming back."""

    @staticmethod
    def forward(ctx, t):
        return round_bf16(t)

    @staticmethod
    def backward(ctx, g):
        return round_bf16(g)


def _rmsnorm(x, g, eps):
    return x / torch.sqrt(torch.mean(x * x, dim=-1, keepdim=True) + eps) * g


def _rope(x, base):
    """x [seq, heads, hd]: pair (2i, 2i+1) of every head rotated by position * base**(-2i/hd)."""
    seq, _, hd = x.shape
    i = torch.arange(hd // 2, dtype=torch.float64)
    ang = torch.arange(seq, dtype=torch.float64)[:, None] * (base ** (-2.0 * i / hd))[None, :]
    c, s = torch.cos(ang)[:, None, :], torch.sin(ang)[:, None, :]
    xe, xo = x[..., 0::2], x[..., 1::2]
    return torch.stack((xe * c - xo * s, xe * s + xo * c), dim=-1).reshape(x.shape)


def _layer(x, w, lora, l, n_heads, hd, eps, base, S=lambda t: t):
    """One layer; S is applied to every tensor the layer stores (identity, or `_Stored.apply`)."""
    seq, d = x.shape
    a = S(_rmsnorm(x, w[f"g1.{l}"], eps))
    q = S(S(a @ w[f"wq.{l}"]) + S(S(a @ lora[f"aq.{l}"]) @ lora[f"bq.{l}"]))
    k = S(a @ w[f"wk.{l}"])
    v = S(S(a @ w[f"wv.{l}"]) + S(S(a @ lora[f"av.{l}"]) @ lora[f"bv.{l}"]))
    q = S(_rope(q.reshape(seq, n_heads, hd), base))
    k = S(_rope(k.reshape(seq, n_heads, hd), base))
    v = v.reshape(seq, n_heads, hd)
    s = torch.einsum("qhc,khc->hqk", q, k) / np.sqrt(hd)
    r = torch.arange(seq)
    s = s.masked_fill(r[None, None, :] > r[None, :, None], float("-inf"))
    p = torch.softmax(s, dim=-1)
    o = S(torch.einsum("hqk,khc->qhc", p, v).reshape(seq, d))
    h1 = S(x + S(o @ w[f"wo.{l}"]))
    b = S(_rmsnorm(h1, w[f"g2.{l}"], eps))
    g, u = S(b @ w[f"w1.{l}"]), S(b @ w[f"w3.{l}"])
    return S(h1 + S(S(g * torch.sigmoid(g) * u) @ w[f"w2.{l}"]))


def forward(cfg, w: Dict[str, np.ndarray], lora: Dict[str, np.ndarray], x: np.ndarray) -> np.ndarray:
    """All layers and sequences; arrays in, float64 array out."""
    y, _ = loss_and_grads(cfg, w, lora, x, None)
    return y


def loss_and_grads(cfg, w: Dict[str, np.ndarray], lora: Dict[str, np.ndarray], x: np.ndarray,
                   probe, storage=None) -> Tuple[np.ndarray, Dict[str, np.ndarray]]:
    """Returns (y_final, grads) with grads["aq.l"], ["bq.l"], ["av.l"], ["bv.l"] for every layer
    and grads["x"]; grads is empty when probe is None.  storage: None (exact) or "bf16" (every
    stored tensor and the gradient arriving at it rounded to bf16, see the module text)."""
    if storage not in (None, "bf16"):
        raise ValueError(f"unknown storage {storage!r}")
    S = _Stored.apply if storage == "bf16" else (lambda t: t)
    tw = {k: torch.tensor(np.asarray(a, dtype=np.float64)) for k, a in w.items() if k != "x"}
    tl = {k: torch.tensor(np.asarray(a, dtype=np.float64), requires_grad=probe is not None) for k, a in lora.items()}
    tx = torch.tensor(np.asarray(x, dtype=np.float64), requires_grad=probe is not None)
    outs = []
    for b in range(cfg.batch):
        h = tx[b * cfg.seq:(b + 1) * cfg.seq]
        for l in range(cfg.layers):
            h = _layer(h, tw, tl, l, cfg.n_heads, cfg.head_dim, cfg.eps, cfg.rope_base, S)
        outs.append(h)
    y = torch.cat(outs, dim=0)
    if probe is None:
        return y.detach().numpy(), {}
    loss = torch.sum(y * torch.tensor(np.asarray(probe, dtype=np.float64)))
    loss.backward()
    grads = {k: t.grad.numpy() for k, t in tl.items()}
    grads["x"] = tx.grad.numpy()
    return y.detach().numpy(), grads
