"""Pins for the mask rules of the oracle beyond plain causality (CPU only): the sliding window and padding in front of
the sequence (Sec. 3.2.2 writes softmax(S, M) with a general mask M and names padding and sliding windows).
Chosen so that an off-by-one in either rule, a mask applied on the wrong side, a forgotten rule in the backward, or a
wrong convention for rows that see nothing fails at least one of them."""
import math

import numpy as np
import pytest

from oracle import attn, layer

from test_oracle_layer import make as make_layer


def make(c=5, s=6, Hq=4, Hkv=2, dh=4, seed=0):
    rng = np.random.default_rng(seed)
    q = rng.normal(size=(c, Hq, dh)); d_o = rng.normal(size=(c, Hq, dh))
    k = rng.normal(size=(s + c, Hkv, dh)); v = rng.normal(size=(s + c, Hkv, dh))
    return q, k, v, d_o


@pytest.mark.parametrize("window,kv_first", [(3, 0), (0, 4), (4, 7), (1, 0), (100, 0), (2, 9)])
def test_forward_matches_scalar_loops(window, kv_first):
    c, s, scale = 5, 6, 0.5
    q, k, v, _ = make(c, s)
    o, lse = attn.chunk_forward(q, k, v, s, scale, window, kv_first)
    for t in range(c):
        pos = s + t
        keys = [u for u in range(pos + 1) if u >= kv_first and (window == 0 or u > pos - window)]
        for h in range(4):
            kv = h // 2
            if not keys:                                  # a padding row: empty softmax
                assert np.all(o[t, h] == 0) and lse[h, t] == -np.inf
                continue
            sc = [scale * sum(q[t, h, j] * k[u, kv, j] for j in range(4)) for u in keys]
            den = sum(math.exp(x) for x in sc)
            assert abs(lse[h, t] - math.log(den)) < 1e-12
            for j in range(4):
                want = sum(math.exp(x) / den * v[u, kv, j] for x, u in zip(sc, keys))
                assert abs(o[t, h, j] - want) < 1e-12


def test_visible_counts_are_the_closed_form():
    # query at position t sees min(t + 1, window) keys, minus those before kv_first
    for window, first in ((0, 0), (3, 0), (0, 5), (4, 5), (1, 0)):
        vis = attn.visible(np.arange(12), np.arange(12), window, first)
        for t in range(12):
            lo = max(first, t - window + 1) if window else first
            assert vis[t].sum() == max(0, t - lo + 1)
            assert not vis[t, t + 1:].any()


@pytest.mark.parametrize("window,kv_first", [(3, 0), (0, 4), (4, 7), (2, 9)])
def test_backward_finite_differences(window, kv_first):
    c, s, scale = 5, 6, 0.5
    q, k, v, d_o = make(c, s, seed=1)
    dq, dk, dv = attn.chunk_backward(q, k, v, d_o, s, scale, window, kv_first)
    f = lambda q, k, v: float(np.sum(attn.chunk_forward(q, k, v, s, scale, window, kv_first)[0] * d_o))
    hstep = 1e-6
    for name, base, ana in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        num = np.zeros_like(base)
        it = np.nditer(base, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            args = dict(q=q, k=k, v=v)
            p = base.copy(); p[i] += hstep
            m = base.copy(); m[i] -= hstep
            num[i] = (f(**{**args, name: p}) - f(**{**args, name: m})) / (2 * hstep)
        assert np.linalg.norm(num - ana) / max(np.linalg.norm(num), 1e-30) < 1e-8, name
    # keys no query of the chunk can see get exactly zero gradient
    hidden = ~attn.visible(s + np.arange(c), np.arange(s + c), window, kv_first).any(axis=0)
    assert hidden.any() and np.all(dk[hidden] == 0) and np.all(dv[hidden] == 0)
    # rows that see nothing send no gradient to q
    empty = ~attn.visible(s + np.arange(c), np.arange(s + c), window, kv_first).any(axis=1)
    assert np.all(dq[empty] == 0)


def test_special_cases():
    c, s, scale = 5, 6, 0.5
    q, k, v, d_o = make(c, s, seed=2)
    base = attn.chunk_forward(q, k, v, s, scale)
    # a window at least as long as the sequence is plain causal attention, bit for bit
    for w in (s + c, 10 ** 6):
        got = attn.chunk_forward(q, k, v, s, scale, w, 0)
        assert np.array_equal(got[0], base[0]) and np.array_equal(got[1], base[1])
    # window 1: every query sees only itself: o_t = v_t, lse = its own score, and q gets no gradient
    o, lse = attn.chunk_forward(q, k, v, s, scale, 1, 0)
    for h in range(4):
        np.testing.assert_allclose(o[:, h], v[s:, h // 2], rtol=1e-14)
        np.testing.assert_allclose(lse[h], scale * np.sum(q[:, h] * k[s:, h // 2], axis=1), rtol=1e-13)
    dq, dk, dv = attn.chunk_backward(q, k, v, d_o, s, scale, 1, 0)
    assert np.all(np.abs(dq) < 1e-15) and np.all(np.abs(dk) < 1e-15)
    np.testing.assert_allclose(dv[s:, 0], d_o[:, 0] + d_o[:, 1], rtol=1e-14)      # dv_t = sum over the group of do_t
    # hidden keys are never read: changing them changes nothing, bit for bit
    k2, v2 = k.copy(), v.copy()
    k2[:4] = 1e6; v2[:4] = -1e6                                                  # before kv_first = 4
    a = attn.chunk_forward(q, k, v, s, scale, 0, 4)
    b = attn.chunk_forward(q, k2, v2, s, scale, 0, 4)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    k3 = k.copy(); k3[:s + 0 - 3 + 1] = 7.0                                       # older than the first query's window of 3
    a = attn.chunk_forward(q, k, v, s, scale, 3, 0)
    b = attn.chunk_forward(q, k3, v, s, scale, 3, 0)
    assert np.array_equal(a[0], b[0])
    # the chunked call agrees with the layer's full-sequence mask: same visibility rule
    T = 9
    full = np.zeros((T, T), bool)
    for t in range(T):
        for u in range(T):
            full[t, u] = u <= t and u > t - 4 and u >= 2
    assert np.array_equal(attn.visible(np.arange(T), np.arange(T), 4, 2), full)


def test_padding_in_front_equals_the_sequence_without_it():
    # f padding positions in front: rows >= f must equal the layer run on the sequence cut at f with positions shifted by
    # f (RoPE sees absolute positions) - forward values and, when no loss sits on the padding rows, every weight gradient.
    cfg, w, x, dy = make_layer(T=9, pos_offset=1, seed=3)
    f = 3
    dy = dy.copy(); dy[:f] = 0.0
    y_pad, cache = layer.layer_forward(x, w, dict(cfg, first_valid=f))
    dx_pad, g_pad = layer.layer_backward(cache, dy)
    y_cut, cache_c = layer.layer_forward(x[f:], w, dict(cfg, pos_offset=cfg["pos_offset"] + f))
    dx_cut, g_cut = layer.layer_backward(cache_c, dy[f:])
    np.testing.assert_allclose(y_pad[f:], y_cut, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(dx_pad[f:], dx_cut, rtol=1e-10, atol=1e-13)
    assert np.all(dx_pad[:f] == 0)
    for n in g_cut:
        np.testing.assert_allclose(g_pad[n], g_cut[n], rtol=1e-10, atol=1e-13, err_msg=n)
    # the padding rows see nothing: their attention output is exactly zero, so h1 = x there
    np.testing.assert_array_equal(cache["o2"][:f], 0.0)


@pytest.mark.parametrize("name", ["x", "wq", "wk", "wv", "wo"])
def test_layer_backward_with_window_and_padding_finite_differences(name):
    cfg, w, x, dy = make_layer(T=7, pos_offset=2, seed=4)
    cfg = dict(cfg, window=3, first_valid=2)
    _, cache = layer.layer_forward(x, w, cfg)
    dx, g = layer.layer_backward(cache, dy)
    analytic = dx if name == "x" else g[name]
    base = x if name == "x" else w[name]

    def loss(arr):
        y, _ = layer.layer_forward(arr if name == "x" else x, w if name == "x" else {**w, name: arr}, cfg)
        return float(np.sum(y * dy))

    num = np.zeros_like(base)
    it = np.nditer(base, flags=["multi_index"])
    hstep = 1e-6
    for _ in it:
        idx = it.multi_index
        p = base.copy(); p[idx] += hstep
        m = base.copy(); m[idx] -= hstep
        num[idx] = (loss(p) - loss(m)) / (2 * hstep)
    assert np.linalg.norm(num - analytic) / np.linalg.norm(num) < 1e-7


def test_layer_window_matches_chunk_attention_rule():
    # the layer's T x T probabilities obey the same rule as oracle/attn.py: zero exactly where `visible` says hidden
    cfg, w, x, _ = make_layer(T=8, seed=5)
    _, cache = layer.layer_forward(x, w, dict(cfg, window=3, first_valid=1))
    vis = attn.visible(np.arange(8), np.arange(8), 3, 1)
    for h in range(cfg["n_q_heads"]):
        assert np.all(cache["P"][h][~vis] == 0) and np.all(cache["P"][h][vis] > 0)
        np.testing.assert_allclose(cache["P"][h][1:].sum(axis=1), 1.0, rtol=1e-13)
