"""fp64 oracle: one pre-norm decoder layer, full sequence, ordinary backprop.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

The chunked method reaches exactly the ordinary gradient (Sec. 3.1, Eq. 1:
the sum over any partition of Z_out of the per-chunk terms is the full chain
rule product), so the oracle is the plain definition: a full-sequence forward
with explicit T x T attention matrices, followed by the textbook adjoint.

Layer (Sec. 3.2.2 gives Q,K,V projections, S = QK^T, P = softmax(S, M), O = PV
and the gated MLP; it states that normalisation, heads and residuals are left
out of the presentation only).  The readings taken here:
  * pre-norm layout with two RMSNorms and two residual adds, an output
    projection W_o, grouped-query heads (consecutive query heads share a KV
    head), rotary position embedding in the rotate-half pairing applied to q
    and k before K is cached, scores scaled by 1/sqrt(head_dim), sigma := SiLU.
  * weights are stored [out, in]; y = x W^T.

  * the mask M is causal by default; cfg may add the two further rules of
    oracle/attn.py: "window" (sliding window, 0 = off) and "first_valid"
    (positions before it are padding in front of the sequence: never visible
    as keys; as queries they see nothing, so their attention output is zero).

Shapes: x [T, d]; wq [Hq*dh, d]; wk, wv [Hkv*dh, d]; wo [d, Hq*dh];
wgate, wup [F, d]; wdown [d, F]; g1, g2 [d].
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def rmsnorm_forward(x, g, eps):
    """a_t = g * x_t / sqrt(mean_j x_tj^2 + eps); returns (a, r) with r the
    reciprocal root per row."""
    x = np.asarray(x, F64)
    r = 1.0 / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)
    return np.asarray(g, F64) * x * r, r


def rmsnorm_backward(da, x, g, r):
    """Adjoint of rmsnorm_forward: returns (dx, dg)."""
    x = np.asarray(x, F64)
    g = np.asarray(g, F64)
    d = x.shape[-1]
    dg = np.sum(da * x * r, axis=0)
    u = da * g                                  # gradient wrt the normalised row x*r
    dot = np.sum(u * x, axis=-1, keepdims=True)  # <u_t, x_t>
    dx = u * r - x * (r ** 3) * dot / d
    return dx, dg


def rope_tables(n_pos, head_dim, theta, pos_offset=0):
    """cos/sin [n_pos, head_dim/2] with angle (t + pos_offset) * theta^(-2j/head_dim)."""
    half = head_dim // 2
    j = np.arange(half, dtype=F64)
    inv_freq = theta ** (-2.0 * j / head_dim)
    pos = np.arange(n_pos, dtype=F64) + float(pos_offset)
    ang = pos[:, None] * inv_freq[None, :]
    return np.cos(ang), np.sin(ang)


def rope_apply(x, cos, sin):
    """Rotate pairs (j, j + dh/2) of x [T, H, dh] by the row's angle."""
    half = x.shape[-1] // 2
    x1, x2 = x[..., :half], x[..., half:]
    c, s = cos[:, None, :], sin[:, None, :]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def rope_apply_transposed(dy, cos, sin):
    """Adjoint of rope_apply (rotation by the negative angle)."""
    half = dy.shape[-1] // 2
    d1, d2 = dy[..., :half], dy[..., half:]
    c, s = cos[:, None, :], sin[:, None, :]
    return np.concatenate([d1 * c + d2 * s, d2 * c - d1 * s], axis=-1)


def silu(z):
    return z / (1.0 + np.exp(-z))


def silu_grad(z):
    sg = 1.0 / (1.0 + np.exp(-z))
    return sg * (1.0 + z * (1.0 - sg))


def layer_forward(x, w, cfg):
    """Full-sequence forward.  w: dict of weights; cfg: dict with n_q_heads,
    n_kv_heads, head_dim, rms_eps, rope_theta, pos_offset.  Returns (y, cache)."""
    x = np.asarray(x, F64)
    T, d = x.shape
    Hq, Hkv, dh = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    grp = Hq // Hkv
    eps = cfg.get("rms_eps", 1e-6)
    W = {k: np.asarray(v, F64) for k, v in w.items()}

    a, r1 = rmsnorm_forward(x, W["g1"], eps)
    cos, sin = rope_tables(T, dh, cfg.get("rope_theta", 1e4), cfg.get("pos_offset", 0))
    q = rope_apply((a @ W["wq"].T).reshape(T, Hq, dh), cos, sin)
    k = rope_apply((a @ W["wk"].T).reshape(T, Hkv, dh), cos, sin)
    v = (a @ W["wv"].T).reshape(T, Hkv, dh)

    scale = 1.0 / np.sqrt(dh)
    idx = np.arange(T)
    hidden = idx[None, :] > idx[:, None]                 # key index > query index
    window, first = cfg.get("window", 0), cfg.get("first_valid", 0)
    if window > 0:
        hidden |= idx[None, :] <= idx[:, None] - window  # older than the last `window` positions
    if first > 0:
        hidden |= idx[None, :] < first                   # padding in front of the sequence
    empty = hidden.all(axis=1, keepdims=True)            # queries that see no key (the padding rows themselves)
    P = np.empty((Hq, T, T), F64)
    o = np.empty((T, Hq, dh), F64)
    for h in range(Hq):
        kv = h // grp
        S = (q[:, h, :] @ k[:, kv, :].T) * scale
        S[hidden] = -np.inf
        S = S - np.where(empty, 0.0, S.max(axis=1, keepdims=True))
        E = np.exp(S)
        P[h] = E / np.where(empty, 1.0, E.sum(axis=1, keepdims=True))
        o[:, h, :] = P[h] @ v[:, kv, :]

    o2 = o.reshape(T, Hq * dh)
    h1 = x + o2 @ W["wo"].T
    m, r2 = rmsnorm_forward(h1, W["g2"], eps)
    gate = m @ W["wgate"].T
    up = m @ W["wup"].T
    act = silu(gate) * up
    y = h1 + act @ W["wdown"].T
    cache = dict(x=x, a=a, r1=r1, cos=cos, sin=sin, q=q, k=k, v=v, P=P, o2=o2,
                 h1=h1, m=m, r2=r2, gate=gate, up=up, act=act, W=W, cfg=cfg, scale=scale)
    return y, cache


def layer_backward(cache, dy):
    """Textbook adjoint of layer_forward.  Returns (dx, grads dict)."""
    c = cache
    W, cfg = c["W"], c["cfg"]
    dy = np.asarray(dy, F64)
    T, d = dy.shape
    Hq, Hkv, dh = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    grp = Hq // Hkv
    g = {}

    # y = h1 + act Wd^T
    g["wdown"] = dy.T @ c["act"]
    dact = dy @ W["wdown"]
    dgate = dact * c["up"] * silu_grad(c["gate"])
    dup = dact * silu(c["gate"])
    g["wgate"] = dgate.T @ c["m"]
    g["wup"] = dup.T @ c["m"]
    dm = dgate @ W["wgate"] + dup @ W["wup"]
    dh1_norm, g["g2"] = rmsnorm_backward(dm, c["h1"], W["g2"], c["r2"])
    dh1 = dy + dh1_norm

    # h1 = x + o Wo^T
    g["wo"] = dh1.T @ c["o2"]
    do = (dh1 @ W["wo"]).reshape(T, Hq, dh)

    dq = np.zeros((T, Hq, dh), F64)
    dk = np.zeros((T, Hkv, dh), F64)
    dv = np.zeros((T, Hkv, dh), F64)
    for h in range(Hq):
        kv = h // grp
        P = c["P"][h]
        dv[:, kv, :] += P.T @ do[:, h, :]
        dP = do[:, h, :] @ c["v"][:, kv, :].T
        delta = np.sum(dP * P, axis=1, keepdims=True)
        dS = P * (dP - delta) * c["scale"]
        dq[:, h, :] = dS @ c["k"][:, kv, :]
        dk[:, kv, :] += dS.T @ c["q"][:, h, :]

    dq = rope_apply_transposed(dq, c["cos"], c["sin"]).reshape(T, Hq * dh)
    dk = rope_apply_transposed(dk, c["cos"], c["sin"]).reshape(T, Hkv * dh)
    dv = dv.reshape(T, Hkv * dh)
    g["wq"] = dq.T @ c["a"]
    g["wk"] = dk.T @ c["a"]
    g["wv"] = dv.T @ c["a"]
    da = dq @ W["wq"] + dk @ W["wk"] + dv @ W["wv"]
    dx_norm, g["g1"] = rmsnorm_backward(da, c["x"], W["g1"], c["r1"])
    dx = dh1 + dx_norm
    return dx, g


def layer_forward_backward(x, w, cfg, dy, first_valid=None):
    """Convenience: batch of sequences x [B, T, d], dy [B, T, d]; weight
    gradients are summed over the batch (independent sequences).  first_valid:
    optional per-sequence count of padding positions in front."""
    x = np.asarray(x, F64)
    dy = np.asarray(dy, F64)
    if x.ndim == 2:
        x, dy = x[None], dy[None]
    ys, dxs, gsum = [], [], None
    for b in range(x.shape[0]):
        cfg_b = cfg if first_valid is None else dict(cfg, first_valid=int(first_valid[b]))
        y, cache = layer_forward(x[b], w, cfg_b)
        dx, g = layer_backward(cache, dy[b])
        ys.append(y)
        dxs.append(dx)
        gsum = g if gsum is None else {k: gsum[k] + g[k] for k in g}
    return np.stack(ys), np.stack(dxs), gsum
