"""fp64 oracle: causal attention of one chunk of queries against the prefix.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Partitioned attention (Sec. 3.2.2): S^(i) = Q^(i) K^(:i)^T, P^(i) =
softmax(S^(i), M^(i)), O^(i) = P^(i) V^(:i).  Query row t of the chunk sits at
global position q_start + t and sees key positions 0 .. q_start + t; keys
beyond the chunk end play no part (Property 3.1).  Heads: query head h reads
KV head h // (Hq / Hkv).  q [c, Hq, dh] (already rotated), k, v [n, Hkv, dh]
with n >= q_start + c.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def _probs(qh, kh, q_start, scale):
    c, e = qh.shape[0], kh.shape[0]
    S = (qh @ kh.T) * scale
    qpos = q_start + np.arange(c)[:, None]
    kpos = np.arange(e)[None, :]
    S = np.where(kpos <= qpos, S, -np.inf)
    smax = S.max(axis=1, keepdims=True)
    E = np.exp(S - smax)
    den = E.sum(axis=1, keepdims=True)
    return E / den, (smax + np.log(den))[:, 0]


def chunk_forward(q, k, v, q_start, scale):
    """Returns o [c, Hq, dh] and lse [Hq, c] (natural-log sum-exp of the scaled,
    masked scores)."""
    q, k, v = (np.asarray(t, F64) for t in (q, k, v))
    c, Hq, dh = q.shape
    grp = Hq // k.shape[1]
    e = q_start + c
    o = np.empty_like(q)
    lse = np.empty((Hq, c), F64)
    for h in range(Hq):
        P, lse[h] = _probs(q[:, h], k[:e, h // grp], q_start, scale)
        o[:, h] = P @ v[:e, h // grp]
    return o, lse


def chunk_backward(q, k, v, d_o, q_start, scale):
    """Returns dq [c, Hq, dh] and this chunk's contribution to dk, dv
    [q_start + c, Hkv, dh] (summed over the query heads of each group)."""
    q, k, v, d_o = (np.asarray(t, F64) for t in (q, k, v, d_o))
    c, Hq, dh = q.shape
    Hkv = k.shape[1]
    grp = Hq // Hkv
    e = q_start + c
    dq = np.empty_like(q)
    dk = np.zeros((e, Hkv, dh), F64)
    dv = np.zeros((e, Hkv, dh), F64)
    for h in range(Hq):
        kv = h // grp
        P, _ = _probs(q[:, h], k[:e, kv], q_start, scale)
        dv[:, kv] += P.T @ d_o[:, h]
        dP = d_o[:, h] @ v[:e, kv].T
        dS = P * (dP - np.sum(dP * P, axis=1, keepdims=True)) * scale
        dq[:, h] = dS @ k[:e, kv]
        dk[:, kv] += dS.T @ q[:, h]
    return dq, dk, dv
