"""Pins for oracle/attn.py (CPU only)."""
import math

import numpy as np
import pytest

from oracle import attn, layer


def make(c=3, s=4, Hq=4, Hkv=2, dh=4, seed=0):
    rng = np.random.default_rng(seed)
    q = rng.normal(size=(c, Hq, dh)); d_o = rng.normal(size=(c, Hq, dh))
    k = rng.normal(size=(s + c + 2, Hkv, dh)); v = rng.normal(size=(s + c + 2, Hkv, dh))
    return q, k, v, d_o


def test_forward_matches_scalar_loops():
    q, k, v, _ = make()
    s, scale = 4, 0.5
    o, lse = attn.chunk_forward(q, k, v, s, scale)
    for t in range(3):
        for h in range(4):
            kv = h // 2
            sc = [scale * sum(q[t, h, j] * k[u, kv, j] for j in range(4)) for u in range(s + t + 1)]
            den = sum(math.exp(x) for x in sc)
            assert abs(lse[h, t] - math.log(den)) < 1e-12
            for j in range(4):
                want = sum(math.exp(sc[u]) / den * v[u, kv, j] for u in range(s + t + 1))
                assert abs(o[t, h, j] - want) < 1e-12


def test_backward_finite_differences():
    q, k, v, d_o = make()
    s, scale = 4, 0.5
    dq, dk, dv = attn.chunk_backward(q, k, v, d_o, s, scale)
    f = lambda qq, kk, vv: float(np.sum(attn.chunk_forward(qq, kk, vv, s, scale)[0] * d_o))
    hstep = 1e-6
    for name, base, ana in (("q", q, dq), ("k", k, dk), ("v", v, dv)):
        num = np.zeros_like(base)
        it = np.nditer(base, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            p = base.copy(); p[i] += hstep
            m = base.copy(); m[i] -= hstep
            args_p = dict(q=q, k=k, v=v); args_p[name] = p
            args_m = dict(q=q, k=k, v=v); args_m[name] = m
            num[i] = (f(args_p["q"], args_p["k"], args_p["v"]) - f(args_m["q"], args_m["k"], args_m["v"])) / (2 * hstep)
        n = ana.shape[0]
        assert np.linalg.norm(num[:n] - ana) / np.linalg.norm(num) < 1e-8, name
        assert np.all(num[n:] == 0)            # keys past the chunk end get no gradient


def test_keys_beyond_chunk_end_are_never_read():
    # Property 3.1: chunk i needs only K^(:i), V^(:i).
    q, k, v, d_o = make()
    k2, v2 = k.copy(), v.copy()
    k2[7:] = np.nan; v2[7:] = np.inf
    a = attn.chunk_forward(q, k, v, 4, 0.5)
    b = attn.chunk_forward(q, k2, v2, 4, 0.5)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    ga = attn.chunk_backward(q, k, v, d_o, 4, 0.5)
    gb = attn.chunk_backward(q, k2, v2, d_o, 4, 0.5)
    assert all(np.array_equal(x, y) for x, y in zip(ga, gb))


def test_last_key_only_hears_the_last_query():
    q, k, v, d_o = make()
    _, dk, dv = attn.chunk_backward(q, k, v, d_o, 4, 0.5)
    d2 = d_o.copy(); d2[:-1] = 0
    _, dk2, dv2 = attn.chunk_backward(q, k, v, d2, 4, 0.5)
    np.testing.assert_allclose(dk[-1], dk2[-1], rtol=1e-13)
    np.testing.assert_allclose(dv[-1], dv2[-1], rtol=1e-13)


def test_chunks_tile_the_full_sequence_attention():
    # Full-sequence attention inside oracle.layer == chunks stitched together.
    rng = np.random.default_rng(3)
    T, Hq, Hkv, dh = 9, 4, 2, 4
    q = rng.normal(size=(T, Hq, dh)); k = rng.normal(size=(T, Hkv, dh)); v = rng.normal(size=(T, Hkv, dh))
    d_o = rng.normal(size=(T, Hq, dh))
    full_o, _ = attn.chunk_forward(q, k, v, 0, 0.5)
    full_dq, full_dk, full_dv = attn.chunk_backward(q, k, v, d_o, 0, 0.5)
    dk = np.zeros_like(k); dv = np.zeros_like(v)
    for s, e in [(0, 4), (4, 8), (8, 9)]:
        o, _ = attn.chunk_forward(q[s:e], k, v, s, 0.5)
        np.testing.assert_allclose(o, full_o[s:e], rtol=1e-12)
        dq, dkc, dvc = attn.chunk_backward(q[s:e], k, v, d_o[s:e], s, 0.5)
        np.testing.assert_allclose(dq, full_dq[s:e], rtol=1e-12, atol=1e-14)
        dk[:e] += dkc; dv[:e] += dvc
    np.testing.assert_allclose(dk, full_dk, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(dv, full_dv, rtol=1e-12, atol=1e-14)


def test_softmax_rows_and_ds_rows_sum():
    q, k, v, d_o = make()
    P, _ = attn._probs(q[:, 0], k[:7, 0], 4, 0.5)
    np.testing.assert_allclose(P.sum(axis=1), 1.0, rtol=1e-14)
    assert np.all(np.triu(P, k=5) == 0)      # key u > 4 + t masked to exactly zero
