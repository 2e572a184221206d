"""Pins for oracle/lora.py (CPU only): the adapted layer and the chain rule through B A."""
import numpy as np
import pytest

from oracle import layer, lora

from test_oracle_layer import make as make_layer


def make(rank=3, seed=0, names=lora.MATRICES, T=6):
    cfg, w, x, dy = make_layer(T=T, seed=seed, pos_offset=1)
    rng = np.random.default_rng(seed + 100)
    ad = {n: (rng.normal(0, 0.3, (rank, w[n].shape[1])), rng.normal(0, 0.3, (w[n].shape[0], rank))) for n in names}
    return cfg, w, ad, x, dy


def loss(x, w, ad, scale, cfg, dy):
    """Scalar functional of the adapted layer whose derivatives the finite differences below take."""
    y, _ = layer.layer_forward(x, lora.effective_weights(w, ad, scale), cfg)
    return float(np.sum(y * dy))


def test_one_linear_map_merged_equals_unmerged():
    rng = np.random.default_rng(0)
    x, W, A, B = rng.normal(size=(5, 7)), rng.normal(size=(4, 7)), rng.normal(size=(2, 7)), rng.normal(size=(4, 2))
    w_eff = lora.effective_weights(dict(wq=W), dict(wq=(A, B)), 0.5)["wq"]
    assert w_eff.shape == W.shape
    np.testing.assert_allclose(x @ w_eff.T, x @ W.T + 0.5 * (x @ A.T) @ B.T, rtol=1e-13)


@pytest.mark.parametrize("name", lora.MATRICES)
def test_adapter_gradients_by_finite_differences(name):
    cfg, w, ad, x, dy = make()
    scale = 0.7
    _, dx, dA, dB = lora.layer_forward_backward(x, w, ad, scale, cfg, dy)
    hstep = 1e-6
    for which, ana in ((0, dA[name]), (1, dB[name])):
        base = ad[name][which]
        num = np.zeros_like(base)
        it = np.nditer(base, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            vals = []
            for sgn in (+1, -1):
                pert = base.copy(); pert[i] += sgn * hstep
                pair = (pert, ad[name][1]) if which == 0 else (ad[name][0], pert)
                vals.append(loss(x, w, {**ad, name: pair}, scale, cfg, dy))
            num[i] = (vals[0] - vals[1]) / (2 * hstep)
        assert np.linalg.norm(num - ana) / np.linalg.norm(num) < 1e-7, (name, which)


def test_input_gradient_by_finite_differences_and_base_case():
    cfg, w, ad, x, dy = make(seed=1)
    scale = 0.4
    y, dx, dA, dB = lora.layer_forward_backward(x, w, ad, scale, cfg, dy)
    num = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        p = x.copy(); p[i] += 1e-6
        m = x.copy(); m[i] -= 1e-6
        num[i] = (loss(p, w, ad, scale, cfg, dy) - loss(m, w, ad, scale, cfg, dy)) / 2e-6
    assert np.linalg.norm(num - dx[0]) / np.linalg.norm(num) < 1e-7
    # B = 0: the adapted layer is the base layer; dA vanishes exactly; dB = s dW A^T with the base layer's dW
    ad0 = {n: (A, np.zeros_like(B)) for n, (A, B) in ad.items()}
    y0, dx0, dA0, dB0 = lora.layer_forward_backward(x, w, ad0, scale, cfg, dy)
    yb, dxb, gb = layer.layer_forward_backward(x, w, cfg, dy)
    assert np.array_equal(y0, yb) and np.array_equal(dx0, dxb)
    for n in ad:
        assert np.all(dA0[n] == 0)
        np.testing.assert_allclose(dB0[n], scale * gb[n] @ ad[n][0].T, rtol=1e-13)


def test_full_rank_identity_adapter_recovers_the_weight_gradient():
    # A = I (rank = fan-in), s = 1: W_eff = W + B, so dB is the ordinary weight gradient at W + B
    cfg, w, _, x, dy = make(seed=2)
    rng = np.random.default_rng(5)
    n = "wup"
    B = rng.normal(0, 0.2, w[n].shape)
    ad = {n: (np.eye(w[n].shape[1]), B)}
    _, _, dA, dB = lora.layer_forward_backward(x, w, ad, 1.0, cfg, dy)
    _, _, g = layer.layer_forward_backward(x, {**w, n: w[n] + B}, cfg, dy)
    np.testing.assert_allclose(dB[n], g[n], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(dA[n], B.T @ g[n], rtol=1e-12, atol=1e-14)


def test_only_some_matrices_adapted_and_batch_sum():
    cfg, w, ad, x, dy = make(names=("wq", "wv"), seed=3)
    x2, dy2 = np.stack([x, x[::-1]]), np.stack([dy, 2 * dy])
    _, dx, dA, dB = lora.layer_forward_backward(x2, w, ad, 0.5, cfg, dy2)
    assert set(dA) == {"wq", "wv"}
    parts = [lora.layer_forward_backward(x2[b], w, ad, 0.5, cfg, dy2[b]) for b in range(2)]
    for n in dA:
        np.testing.assert_allclose(dA[n], parts[0][2][n] + parts[1][2][n], rtol=1e-12)
        np.testing.assert_allclose(dB[n], parts[0][3][n] + parts[1][3][n], rtol=1e-12)
