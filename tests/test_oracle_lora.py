"""Pins for the fine-tuning oracle (oracle/lora_ref.py): its forward against the NumPy layer
oracle, its gradients against finite differences and closed forms."""
import numpy as np
import pytest

from oracle import llama_ref as R
from oracle import lora_ref as L
from workloads import LlamaConfig, make_llama_inputs, make_lora_inputs

CFG = LlamaConfig(name="tiny", layers=2, d_model=32, n_heads=2, head_dim=16, ffn=40, seq=12, batch=2, dtype="f32",
                  tile=16, attn_block=16, cap_bytes=0, cap_frac=0.5, weights_resident=False, x_resident=False)


def _inputs(b_std):
    w = R.widen(CFG, make_llama_inputs(CFG, 3))
    lo = R.widen(CFG, make_lora_inputs(CFG, 3, rank=4, b_std=b_std))
    probe = lo.pop("probe")
    return w, lo, probe


def test_forward_with_zero_b_is_the_base_model():
    w, lo, _ = _inputs(0.0)
    np.testing.assert_allclose(L.forward(CFG, w, lo, w["x"]), R.forward(CFG, w), rtol=1e-11, atol=1e-12)


def test_forward_equals_the_base_model_on_merged_weights():
    """q = a Wq + (a A) B = a (Wq + A B): folding the adapters into the weights must not change y."""
    w, lo, _ = _inputs(0.05)
    merged = dict(w)
    for l in range(CFG.layers):
        merged[f"wq.{l}"] = w[f"wq.{l}"] + lo[f"aq.{l}"] @ lo[f"bq.{l}"]
        merged[f"wv.{l}"] = w[f"wv.{l}"] + lo[f"av.{l}"] @ lo[f"bv.{l}"]
    y = L.forward(CFG, w, lo, w["x"])
    np.testing.assert_allclose(y, R.forward(CFG, merged), rtol=1e-10, atol=1e-11)
    assert np.max(np.abs(y - R.forward(CFG, w))) > 1e-3  # and the adapters do something


@pytest.mark.parametrize("b_std", [0.0, 0.05])
def test_gradients_match_central_differences(b_std):
    w, lo, probe = _inputs(b_std)
    _, g = L.loss_and_grads(CFG, w, lo, w["x"], probe)

    def loss(lo_, x_):
        return float(np.sum(L.forward(CFG, w, lo_, x_) * probe))

    rng = np.random.default_rng(0)
    h = 1e-5
    for name in ["aq.0", "bq.0", "av.1", "bv.1", "aq.1", "bv.0"]:
        for _ in range(4):
            idx = tuple(rng.integers(0, n) for n in lo[name].shape)
            up, dn = {k: a.copy() for k, a in lo.items()}, {k: a.copy() for k, a in lo.items()}
            up[name][idx] += h
            dn[name][idx] -= h
            fd = (loss(up, w["x"]) - loss(dn, w["x"])) / (2 * h)
            assert abs(fd - g[name][idx]) <= 1e-6 * max(1.0, abs(fd)), (name, idx, fd, g[name][idx])
    for _ in range(6):
        idx = tuple(rng.integers(0, n) for n in w["x"].shape)
        xu, xd = w["x"].copy(), w["x"].copy()
        xu[idx] += h
        xd[idx] -= h
        fd = (loss(lo, xu) - loss(lo, xd)) / (2 * h)
        assert abs(fd - g["x"][idx]) <= 1e-6 * max(1.0, abs(fd))


def test_zero_b_closed_forms():
    """With B = 0 the adapters do not reach the output: dA vanishes identically, and dB is the
    outer product of the low-rank activations with the gradient arriving at the projection."""
    w, lo, probe = _inputs(0.0)
    _, g = L.loss_and_grads(CFG, w, lo, w["x"], probe)
    for l in range(CFG.layers):
        assert not g[f"aq.{l}"].any() and not g[f"av.{l}"].any()
        assert np.abs(g[f"bq.{l}"]).max() > 0 and np.abs(g[f"bv.{l}"]).max() > 0
    # last layer, v projection: dL/dv is available in closed form through the base-model oracle,
    # because y is linear in v once the attention probabilities are fixed (B = 0 keeps them fixed)
    l = CFG.layers - 1
    dbv = np.zeros_like(g[f"bv.{l}"])
    for b in range(CFG.batch):
        x = w["x"][b * CFG.seq:(b + 1) * CFG.seq]
        for ll in range(l):
            x = R.decoder_layer(x, w, ll, CFG.n_heads, CFG.head_dim, CFG.eps, CFG.rope_base)
        a = R.rmsnorm(x, w[f"g1.{l}"], CFG.eps)
        t = a @ lo[f"av.{l}"]                       # [seq, rank]
        # dL/dv by central differences of the numpy layer in v-space: perturb Wv along A's range
        # instead: L(B) with B = eps * E_ij is linear in eps for the value path
        for i in range(t.shape[1]):
            for j in range(0, CFG.d_model, 7):
                def run(eps):
                    wv = dict(w)
                    e = np.zeros_like(lo[f"bv.{l}"])
                    e[i, j] = eps
                    wv[f"wv.{l}"] = w[f"wv.{l}"] + lo[f"av.{l}"] @ e
                    y = R.decoder_layer(x, wv, l, CFG.n_heads, CFG.head_dim, CFG.eps, CFG.rope_base)
                    return float(np.sum(y * probe[b * CFG.seq:(b + 1) * CFG.seq]))
                dbv[i, j] += (run(1e-4) - run(-1e-4)) / 2e-4
    cols = np.arange(0, CFG.d_model, 7)
    np.testing.assert_allclose(g[f"bv.{l}"][:, cols], dbv[:, cols], rtol=1e-6, atol=1e-9)


def test_gradients_are_linear_in_the_probe():
    w, lo, probe = _inputs(0.05)
    _, g1 = L.loss_and_grads(CFG, w, lo, w["x"], probe)
    _, g2 = L.loss_and_grads(CFG, w, lo, w["x"], -2.5 * probe)
    for k in g1:
        np.testing.assert_allclose(g2[k], -2.5 * g1[k], rtol=1e-12, atol=1e-15)


def test_bf16_rounding_against_hand_worked_values():
    import torch
    # bf16 keeps 8 significant bits: the spacing in [1, 2) is 2**-7
    cases = [(1.0, 1.0),
             (1 + 2.0 ** -8, 1.0),                       # half way, lower neighbour even
             (1 + 3 * 2.0 ** -8, 1 + 2.0 ** -6),         # half way, upper neighbour even
             (1 + 2.0 ** -8 + 2.0 ** -20, 1 + 2.0 ** -7),  # just above half way
             (-(1 + 2.0 ** -8 + 2.0 ** -20), -(1 + 2.0 ** -7)),
             (3.1415926, 3.140625),                      # float32 0x40490FDB -> 0x4049
             (0.0, 0.0), (float("inf"), float("inf"))]
    got = L.round_bf16(torch.tensor([c[0] for c in cases], dtype=torch.float64)).numpy()
    np.testing.assert_array_equal(got, np.array([c[1] for c in cases]))
    # the same as the workload generator's conversion (written independently of this one)
    from workloads import bf16_bits_to_f32, to_bf16_bits
    x = np.random.default_rng(0).standard_normal(10000).astype(np.float32)
    np.testing.assert_array_equal(L.round_bf16(torch.tensor(x.astype(np.float64))).numpy(),
                                  bf16_bits_to_f32(to_bf16_bits(x)).astype(np.float64))


def test_stored_tensor_rounds_the_value_forward_and_the_gradient_back():
    import torch
    x = torch.tensor([1 + 2.0 ** -8 + 2.0 ** -20], dtype=torch.float64, requires_grad=True)
    c = torch.tensor([3.1415926], dtype=torch.float64)
    y = torch.sum(L._Stored.apply(x) * c)
    y.backward()
    assert float(y) == (1 + 2.0 ** -7) * 3.1415926
    assert float(x.grad[0]) == 3.140625


def test_bf16_storage_is_a_small_perturbation_and_none_is_the_plain_form():
    w, lo, probe = _inputs(0.05)
    y0, g0 = L.loss_and_grads(CFG, w, lo, w["x"], probe)
    y1, g1 = L.loss_and_grads(CFG, w, lo, w["x"], probe, storage=None)
    np.testing.assert_array_equal(y0, y1)
    yb, gb = L.loss_and_grads(CFG, w, lo, w["x"], probe, storage="bf16")
    assert 1e-4 < R.rel_err(yb, y0) < 2e-2          # rounded, and by no more than a few bf16 ulps
    for k in g0:
        assert 1e-4 < R.rel_err(gb[k], g0[k]) < 4e-2, k
    with pytest.raises(ValueError):
        L.loss_and_grads(CFG, w, lo, w["x"], probe, storage="fp8")
