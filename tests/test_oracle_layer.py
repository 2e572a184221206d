"""Pins for oracle/layer.py and oracle/chunked.py (CPU only).

Each test is chosen so that a plausible slip in the oracle (dropped term, wrong
sign or index, transposed operand, wrong head mapping) fails at least one.
"""
import math

import numpy as np
import pytest

from oracle import chunked, layer


def make(T=6, d=8, Hq=4, Hkv=2, dh=4, F=12, seed=0, pos_offset=0, eps=1e-6):
    rng = np.random.default_rng(seed)
    cfg = dict(n_q_heads=Hq, n_kv_heads=Hkv, head_dim=dh, rms_eps=eps, rope_theta=100.0, pos_offset=pos_offset)
    w = dict(wq=rng.normal(0, 0.4, (Hq * dh, d)), wk=rng.normal(0, 0.4, (Hkv * dh, d)),
             wv=rng.normal(0, 0.4, (Hkv * dh, d)), wo=rng.normal(0, 0.4, (d, Hq * dh)),
             wgate=rng.normal(0, 0.4, (F, d)), wup=rng.normal(0, 0.4, (F, d)),
             wdown=rng.normal(0, 0.4, (d, F)), g1=1 + rng.normal(0, 0.2, d), g2=1 + rng.normal(0, 0.2, d))
    x = rng.normal(0, 1, (T, d))
    dy = rng.normal(0, 1, (T, d))
    return cfg, w, x, dy


def scalar_loop_forward(x, w, cfg):
    """Brute force: the layer written with Python scalar loops only (no matmul,
    no broadcasting), straight from the definitions."""
    T, d = x.shape
    Hq, Hkv, dh = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    half = dh // 2
    F = w["wgate"].shape[0]

    def norm(row, g):
        ms = sum(v * v for v in row) / len(row)
        r = 1.0 / math.sqrt(ms + cfg["rms_eps"])
        return [g[j] * row[j] * r for j in range(len(row))]

    def proj(vec, W):
        return [sum(W[o][i] * vec[i] for i in range(len(vec))) for o in range(len(W))]

    def rot(vec, t):   # vec: one head [dh]
        out = [0.0] * dh
        for j in range(half):
            ang = (t + cfg["pos_offset"]) * cfg["rope_theta"] ** (-2.0 * j / dh)
            cs, sn = math.cos(ang), math.sin(ang)
            out[j] = vec[j] * cs - vec[j + half] * sn
            out[j + half] = vec[j + half] * cs + vec[j] * sn
        return out

    a = [norm(list(x[t]), w["g1"]) for t in range(T)]
    q = [proj(a[t], w["wq"]) for t in range(T)]
    k = [proj(a[t], w["wk"]) for t in range(T)]
    v = [proj(a[t], w["wv"]) for t in range(T)]
    qh = [[rot(q[t][h * dh:(h + 1) * dh], t) for h in range(Hq)] for t in range(T)]
    kh = [[rot(k[t][h * dh:(h + 1) * dh], t) for h in range(Hkv)] for t in range(T)]
    y = np.zeros((T, d))
    for t in range(T):
        o = []
        for h in range(Hq):
            kv = h // (Hq // Hkv)
            s = [sum(qh[t][h][j] * kh[u][kv][j] for j in range(dh)) / math.sqrt(dh) for u in range(t + 1)]
            mx = max(s)
            ex = [math.exp(v_ - mx) for v_ in s]
            den = sum(ex)
            for j in range(dh):
                o.append(sum(ex[u] / den * v[u][kv * dh + j] for u in range(t + 1)))
        h1 = [x[t][j] + sum(w["wo"][j][i] * o[i] for i in range(Hq * dh)) for j in range(d)]
        m = norm(h1, w["g2"])
        gate, up = proj(m, w["wgate"]), proj(m, w["wup"])
        act = [gate[f] / (1 + math.exp(-gate[f])) * up[f] for f in range(F)]
        for j in range(d):
            y[t][j] = h1[j] + sum(w["wdown"][j][f] * act[f] for f in range(F))
    return y


def test_forward_matches_scalar_loops():
    cfg, w, x, _ = make(T=5, pos_offset=3)
    y, _ = layer.layer_forward(x, w, cfg)
    np.testing.assert_allclose(y, scalar_loop_forward(x, w, cfg), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("name", ["x", "wq", "wk", "wv", "wo", "wgate", "wup", "wdown", "g1", "g2"])
def test_backward_finite_differences(name):
    cfg, w, x, dy = make(T=6, pos_offset=2)
    _, cache = layer.layer_forward(x, w, cfg)
    dx, g = layer.layer_backward(cache, dy)
    analytic = dx if name == "x" else g[name]

    def loss(xx, ww):
        y, _ = layer.layer_forward(xx, ww, cfg)
        return float(np.sum(y * dy))

    base = x if name == "x" else w[name]
    num = np.zeros_like(base)
    it = np.nditer(base, flags=["multi_index"])
    hstep = 1e-6
    for _ in it:
        idx = it.multi_index
        for sgn in (+1, -1):
            pert = base.copy()
            pert[idx] += sgn * hstep
            val = loss(pert, w) if name == "x" else loss(x, {**w, name: pert})
            num[idx] += sgn * val
        num[idx] /= 2 * hstep
    err = np.linalg.norm(num - analytic) / np.linalg.norm(num)
    assert err < 1e-7, (name, err)


def test_single_token_attention_is_identity_on_v():
    # T = 1: softmax over one key is 1, so o = v and the layer has a closed form.
    cfg, w, x, _ = make(T=1)
    y, c = layer.layer_forward(x, w, cfg)
    a, _ = layer.rmsnorm_forward(x, w["g1"], cfg["rms_eps"])
    v = (a @ w["wv"].T).reshape(1, cfg["n_kv_heads"], cfg["head_dim"])
    o = np.repeat(v, cfg["n_q_heads"] // cfg["n_kv_heads"], axis=1).reshape(1, -1)
    np.testing.assert_allclose(c["o2"], o, rtol=1e-13)
    # first row of any sequence also sees only itself
    cfg, w, x, _ = make(T=5)
    _, c5 = layer.layer_forward(x, w, cfg)
    a, _ = layer.rmsnorm_forward(x[:1], w["g1"], cfg["rms_eps"])
    v0 = np.repeat((a @ w["wv"].T).reshape(1, 2, 4), 2, axis=1).reshape(-1)
    np.testing.assert_allclose(c5["o2"][0], v0, rtol=1e-13)


def test_causality_future_rows_do_not_matter():
    cfg, w, x, dy = make(T=7)
    y0, _ = layer.layer_forward(x, w, cfg)
    x2 = x.copy()
    x2[4:] += 10.0
    y1, _ = layer.layer_forward(x2, w, cfg)
    assert np.array_equal(y0[:4], y1[:4])
    # and gradient wrt a future input of a loss on past rows is zero
    dyp = dy.copy()
    dyp[4:] = 0
    _, c = layer.layer_forward(x, w, cfg)
    dx, _ = layer.layer_backward(c, dyp)
    assert np.all(dx[4:] == 0)


def test_rope_is_a_rotation_with_relative_phase():
    rng = np.random.default_rng(1)
    dh = 8
    q = rng.normal(size=(1, 1, dh))
    k = rng.normal(size=(1, 1, dh))
    dots = []
    for (tq, tk) in [(5, 2), (9, 6), (103, 100)]:
        cq, sq = layer.rope_tables(1, dh, 1e4, tq)
        ck, sk = layer.rope_tables(1, dh, 1e4, tk)
        rq, rk = layer.rope_apply(q, cq, sq), layer.rope_apply(k, ck, sk)
        np.testing.assert_allclose(np.linalg.norm(rq), np.linalg.norm(q), rtol=1e-13)
        dots.append(float(np.sum(rq * rk)))
    np.testing.assert_allclose(dots, dots[0], rtol=1e-10)
    # position 0 is the identity; transposed rotation is the inverse
    c0, s0 = layer.rope_tables(1, dh, 1e4, 0)
    assert np.array_equal(layer.rope_apply(q, c0, s0), q)
    c, s = layer.rope_tables(1, dh, 1e4, 17)
    np.testing.assert_allclose(layer.rope_apply_transposed(layer.rope_apply(q, c, s), c, s), q, rtol=1e-13)
    # pair (j, j + dh/2) with frequency theta^(-2j/dh): a unit vector on pair j=1 at position 1
    e = np.zeros((1, 1, dh)); e[0, 0, 1] = 1.0
    c1, s1 = layer.rope_tables(1, dh, 1e4, 1)
    r = layer.rope_apply(e, c1, s1)[0, 0]
    ang = 1e4 ** (-2.0 / dh)
    assert abs(r[1] - math.cos(ang)) < 1e-15 and abs(r[1 + dh // 2] - math.sin(ang)) < 1e-15


def test_rmsnorm_closed_forms():
    rng = np.random.default_rng(2)
    x = rng.normal(size=(3, 16))
    g = 1 + rng.normal(0, 0.1, 16)
    a, r = layer.rmsnorm_forward(x, g, 0.0)
    np.testing.assert_allclose(np.mean((a / g) ** 2, axis=1), 1.0, rtol=1e-13)   # unit RMS
    a2, _ = layer.rmsnorm_forward(3.7 * x, g, 0.0)                                 # scale invariance
    np.testing.assert_allclose(a2, a, rtol=1e-13)
    da = rng.normal(size=(3, 16))
    dx, dg = layer.rmsnorm_backward(da, x, g, r)
    np.testing.assert_allclose(np.sum(dx * x, axis=1), 0.0, atol=1e-13)           # <x, dx> = 0 when eps = 0
    np.testing.assert_allclose(dg, np.sum(da * a / g, axis=0), rtol=1e-13)
    # constant row: x = c * ones -> a = g * sign(c)
    a3, _ = layer.rmsnorm_forward(np.full((1, 16), -2.0), g, 0.0)
    np.testing.assert_allclose(a3[0], -g, rtol=1e-13)


def test_gqa_consecutive_heads_share_a_kv_head():
    # Zero all V columns except KV head 1: only query heads 2, 3 (of 4, group 2) may produce output.
    cfg, w, x, _ = make(T=4)
    w = dict(w)
    wv = np.zeros_like(w["wv"]); wv[4:8] = w["wv"][4:8]
    w["wv"] = wv
    _, c = layer.layer_forward(x, w, cfg)
    o = c["o2"].reshape(4, 4, 4)
    assert np.all(o[:, :2] == 0) and np.all(np.abs(o[:, 2:]).sum(axis=(0, 2)) > 0)


@pytest.mark.parametrize("chunk", [1, 2, 3, 4, 7, 100])
def test_chunk_loop_reaches_the_full_gradient(chunk):
    # Eq. 1: the per-chunk terms sum to the full-sequence gradient, for any partition.
    cfg, w, x, dy = make(T=7, pos_offset=1)
    _, cache = layer.layer_forward(x, w, cfg)
    dx, g = layer.layer_backward(cache, dy)
    dxc, gc, parts = chunked.layer_backward_chunked(x, w, cfg, dy, chunk, return_partials=True)
    np.testing.assert_allclose(dxc, dx, rtol=1e-11, atol=1e-12)
    for n in g:
        np.testing.assert_allclose(gc[n], g[n], rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(sum(p[n] for p in parts), g[n], rtol=1e-11, atol=1e-12)
    assert len(parts) == len(chunked.chunk_bounds(7, chunk)) + 1


def test_chunk_bounds():
    assert chunked.chunk_bounds(10, 4) == [(0, 4), (4, 8), (8, 10)]
    assert chunked.chunk_bounds(10, 10) == [(0, 10)]
    assert chunked.chunk_bounds(10, 1000) == [(0, 10)]
    assert chunked.chunk_bounds(3, 1) == [(0, 1), (1, 2), (2, 3)]


def test_batch_sums_weight_gradients():
    cfg, w, x, dy = make(T=4)
    cfg2, _, x2, dy2 = make(T=4, seed=5)
    _, dxs, g = layer.layer_forward_backward(np.stack([x, x2]), w, cfg, np.stack([dy, dy2]))
    _, c = layer.layer_forward(x, w, cfg)
    dx_a, g_a = layer.layer_backward(c, dy)
    _, c = layer.layer_forward(x2, w, cfg)
    dx_b, g_b = layer.layer_backward(c, dy2)
    np.testing.assert_allclose(dxs[0], dx_a)
    np.testing.assert_allclose(g["wup"], g_a["wup"] + g_b["wup"])
