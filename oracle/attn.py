"""fp64 oracle: causal attention of one chunk of queries against the prefix.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

Partitioned attention (Sec. 3.2.2): S^(i) = Q^(i) K^(:i)^T, P^(i) =
softmax(S^(i), M^(i)), O^(i) = P^(i) V^(:i).  Query row t of the chunk sits at
global position q_start + t and sees key positions 0 .. q_start + t; keys
beyond the chunk end play no part (Property 3.1).  Heads: query head h reads
KV head h // (Hq / Hkv).  q [c, Hq, dh] (already rotated), k, v [n, Hkv, dh]
with n >= q_start + c.

The mask M of Sec. 3.2.2 is general ("padding / sliding window"); beyond the
causal rule two more rules can be switched on, both plain index comparisons:
  window > 0 : the query at position t sees only the last `window` positions,
               t - window < u <= t (sliding-window attention);
  kv_first   : key positions u < kv_first are padding in front of the sequence
               and are never visible.
A query that sees no key at all (only possible with kv_first) has an empty
softmax: its probabilities and its output are zero, its log-sum-exp is -inf, and
it sends no gradient to any q, k or v.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def visible(qpos, kpos, window=0, kv_first=0):
    """The mask as a boolean array: query positions along rows, key positions along columns."""
    qpos = np.asarray(qpos)[:, None]
    kpos = np.asarray(kpos)[None, :]
    vis = (kpos <= qpos) & (kpos >= kv_first)
    if window > 0:
        vis &= kpos > qpos - window
    return vis


def _probs(qh, kh, q_start, scale, window=0, kv_first=0):
    c, e = qh.shape[0], kh.shape[0]
    S = (qh @ kh.T) * scale
    vis = visible(q_start + np.arange(c), np.arange(e), window, kv_first)
    S = np.where(vis, S, -np.inf)
    smax = S.max(axis=1, keepdims=True)
    empty = ~np.isfinite(smax)                       # rows that see no key
    E = np.where(vis, np.exp(S - np.where(empty, 0.0, smax)), 0.0)
    den = E.sum(axis=1, keepdims=True)
    P = E / np.where(empty, 1.0, den)
    with np.errstate(divide="ignore"):
        lse = np.where(empty, -np.inf, smax + np.log(np.where(empty, 1.0, den)))
    return P, lse[:, 0]


def chunk_forward(q, k, v, q_start, scale, window=0, kv_first=0):
    """Returns o [c, Hq, dh] and lse [Hq, c] (natural-log sum-exp of the scaled,
    masked scores)."""
    q, k, v = (np.asarray(t, F64) for t in (q, k, v))
    c, Hq, dh = q.shape
    grp = Hq // k.shape[1]
    e = q_start + c
    o = np.empty_like(q)
    lse = np.empty((Hq, c), F64)
    for h in range(Hq):
        P, lse[h] = _probs(q[:, h], k[:e, h // grp], q_start, scale, window, kv_first)
        o[:, h] = P @ v[:e, h // grp]
    return o, lse


def chunk_backward(q, k, v, d_o, q_start, scale, window=0, kv_first=0):
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
        P, _ = _probs(q[:, h], k[:e, kv], q_start, scale, window, kv_first)
        dv[:, kv] += P.T @ d_o[:, h]
        dP = d_o[:, h] @ v[:e, kv].T
        dS = P * (dP - np.sum(dP * P, axis=1, keepdims=True)) * scale
        dq[:, h] = dS @ k[:e, kv]
        dk[:, kv] += dS.T @ q[:, h]
    return dq, dk, dv
