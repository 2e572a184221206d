"""fp64 oracle twin: the paper's chunk loop, step by step.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

This is the method itself (Sec. 3.2.1 accumulation of g_lm_head and g_H over
sequence chunks; Sec. 3.2.2 partitioned attention / partitioned MLP with K and
V computed once and cached, gradients accumulated over chunks i = 1..D), in
fp64 and in the paper's order, written so that the tests can check the two
invariants the exactness claim rests on: the per-chunk terms of Eq. 1 sum to
the full-sequence gradient, and the chunk size does not change the result.
It reuses only the elementwise primitives of oracle.layer / oracle.attn.
"""
from __future__ import annotations

import numpy as np

from . import attn as _attn
from . import head as _head
from .layer import (F64, rmsnorm_backward, rmsnorm_forward, rope_apply,
                    rope_apply_transposed, rope_tables, silu, silu_grad)


def chunk_bounds(T, chunk):
    """Chunks [i*c, min((i+1)*c, T)); a chunk size >= T means a single chunk
    (Sec. 4.4: no partition when the partition size exceeds the length)."""
    c = max(1, min(int(chunk), T))
    return [(s, min(s + c, T)) for s in range(0, T, c)]


def layer_backward_chunked(x, w, cfg, dy, chunk, return_partials=False):
    """One sequence x [T, d].  Returns (dx, grads) and, if asked, the list of
    per-chunk partial weight gradients (the summands of Eq. 1)."""
    x = np.asarray(x, F64)
    dy = np.asarray(dy, F64)
    T, d = x.shape
    Hq, Hkv, dh = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    eps = cfg.get("rms_eps", 1e-6)
    W = {k: np.asarray(v, F64) for k, v in w.items()}
    scale = 1.0 / np.sqrt(dh)
    cos, sin = rope_tables(T, dh, cfg.get("rope_theta", 1e4), cfg.get("pos_offset", 0))

    # K and V for the whole sequence, once (cached for the layer).
    a_full, r1_full = rmsnorm_forward(x, W["g1"], eps)
    K = rope_apply((a_full @ W["wk"].T).reshape(T, Hkv, dh), cos, sin)
    V = (a_full @ W["wv"].T).reshape(T, Hkv, dh)

    names = ["wq", "wk", "wv", "wo", "wgate", "wup", "wdown", "g1", "g2"]
    g = {n: np.zeros_like(W[n]) for n in names}
    g_hin = np.zeros_like(x)                     # running sum of dL/dH_in
    dK = np.zeros_like(K)
    dV = np.zeros_like(V)
    partials = []

    for (s, e) in chunk_bounds(T, chunk):
        p = {n: np.zeros_like(W[n]) for n in names}
        # ---- partitioned reforward of chunk rows [s, e)
        a, r1 = a_full[s:e], r1_full[s:e]
        q = rope_apply((a @ W["wq"].T).reshape(e - s, Hq, dh), cos[s:e], sin[s:e])
        o, _ = _attn.chunk_forward(q, K, V, s, scale)          # uses K^(:i), V^(:i) only
        o2 = o.reshape(e - s, Hq * dh)
        h1 = x[s:e] + o2 @ W["wo"].T
        m, r2 = rmsnorm_forward(h1, W["g2"], eps)
        gate, up = m @ W["wgate"].T, m @ W["wup"].T
        act = silu(gate) * up
        # ---- backward of the chunk
        dyc = dy[s:e]
        p["wdown"] = dyc.T @ act
        dact = dyc @ W["wdown"]
        dgate = dact * up * silu_grad(gate)
        dup = dact * silu(gate)
        p["wgate"], p["wup"] = dgate.T @ m, dup.T @ m
        dm = dgate @ W["wgate"] + dup @ W["wup"]
        dh1n, p["g2"] = rmsnorm_backward(dm, h1, W["g2"], r2)
        dh1 = dyc + dh1n
        p["wo"] = dh1.T @ o2
        d_o = (dh1 @ W["wo"]).reshape(e - s, Hq, dh)
        dq, dk_c, dv_c = _attn.chunk_backward(q, K, V, d_o, s, scale)
        dK[:e] += dk_c                                         # prefix rows only
        dV[:e] += dv_c
        dq = rope_apply_transposed(dq, cos[s:e], sin[s:e]).reshape(e - s, Hq * dh)
        p["wq"] = dq.T @ a
        da = dq @ W["wq"]
        dxn, pg1 = rmsnorm_backward(da, x[s:e], W["g1"], r1)
        p["g1"] = pg1
        g_hin[s:e] += dh1 + dxn
        for n in names:
            g[n] += p[n]
        partials.append(p)

    # K/V side: the cached K, V depend on every row of H_in through W_k, W_v.
    dKr = rope_apply_transposed(dK, cos, sin).reshape(T, Hkv * dh)
    dVr = dV.reshape(T, Hkv * dh)
    pk = {n: np.zeros_like(W[n]) for n in names}
    pk["wk"], pk["wv"] = dKr.T @ a_full, dVr.T @ a_full
    da = dKr @ W["wk"] + dVr @ W["wv"]
    dxn, pk["g1"] = rmsnorm_backward(da, x, W["g1"], r1_full)
    g_hin += dxn
    for n in names:
        g[n] += pk[n]
    partials.append(pk)
    if return_partials:
        return g_hin, g, partials
    return g_hin, g


def head_backward_chunked(h, w, targets, chunk, objective="sft", **kw):
    """Accumulate g_lm_head and g_H chunk by chunk along the sequence
    (Sec. 3.2.1).  h [B, T, d], targets [B, T].  For GRPO the per-sequence
    response length T_o is a property of the whole sequence, so it is counted
    first and handed to every chunk as a weight."""
    h = np.asarray(h, F64)
    tg = np.asarray(targets)
    B, T, d = h.shape
    dW = np.zeros_like(np.asarray(w, F64))
    dH = np.zeros_like(h)
    loss = 0.0
    n_active = 0
    for (s, e) in chunk_bounds(T, chunk):
        if objective == "sft":
            r = _head.sft(h[:, s:e], w, tg[:, s:e], kw.get("loss_scale", 1.0))
            dH[:, s:e] += r["dh"]
            dW += r["dw"]
            loss += r["loss"]
        elif objective == "grpo":
            # evaluate the chunk with its own token count, then re-weight to T_o of the sequence
            t_o = (tg >= 0).sum(axis=1).astype(F64)
            t_c = (tg[:, s:e] >= 0).sum(axis=1).astype(F64)
            for j in range(B):
                if t_c[j] == 0:
                    continue
                old = kw.get("old_logp")
                r = _head.grpo(h[j:j + 1, s:e], w, tg[j:j + 1, s:e], kw["advantages"][j:j + 1],
                               kw["ref_logp"][j:j + 1, s:e],
                               None if old is None else old[j:j + 1, s:e],
                               kw.get("clip_eps", 0.2), kw.get("kl_beta", 0.04), kw.get("kl_mode", 0))
                f = t_c[j] / (B * t_o[j])
                dH[j:j + 1, s:e] += f * r["dh"]
                dW += f * r["dw"]
                loss += f * r["loss"]
        else:
            raise ValueError(objective)
        n_active += int((tg[:, s:e] >= 0).sum())
    return dict(loss=loss, dh=dH, dw=dW, n_active=n_active)
