"""fp64 oracle: LM head + objective, full sequence, ordinary backprop.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

logits = H W^T with W stored [V, d] (Sec. 3.2.1; the paper writes H W with W
[d, C]).  Every position's logits enter the objective independently, which is
what lets the method chunk along the sequence; the oracle does no chunking.

targets[b, t] is the id the row must predict (the caller has already shifted
labels); a negative target marks an ignored row (prompt / padding / last
position).
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def _logits_logp(h, w, targets):
    h2 = np.asarray(h, F64).reshape(-1, h.shape[-1])
    w = np.asarray(w, F64)
    tg = np.asarray(targets).reshape(-1).astype(np.int64)
    z = h2 @ w.T
    zmax = z.max(axis=1, keepdims=True)
    lse = zmax[:, 0] + np.log(np.exp(z - zmax).sum(axis=1))
    active = tg >= 0
    safe = np.where(active, tg, 0)
    logp = z[np.arange(z.shape[0]), safe] - lse
    soft = np.exp(z - lse[:, None])
    return h2, w, tg, active, safe, logp, soft


def _grads_from_coef(h2, w, active, safe, soft, coef, shape):
    """dz_t = coef_t * (e_{y_t} - softmax(z_t)) with coef_t = dL/dlogp_t;
    dH = dz W, dW = dz^T H."""
    n = h2.shape[0]
    onehot = np.zeros_like(soft)
    onehot[np.arange(n), safe] = 1.0
    dz = coef[:, None] * (onehot - soft)
    dz[~active] = 0.0
    return (dz @ w).reshape(shape), dz.T @ h2


def sft(h, w, targets, loss_scale=1.0):
    """Un-normalised SFT objective times loss_scale (Sec. 3.2.1, SFT
    objective): L = -scale * sum_{active t} log softmax(z_t)[y_t].
    Returns dict(loss, dh, dw, n_active, logp)."""
    h2, w, tg, active, safe, logp, soft = _logits_logp(h, w, targets)
    loss = -loss_scale * np.sum(logp[active])
    coef = np.where(active, -loss_scale, 0.0)
    dh, dw = _grads_from_coef(h2, w, active, safe, soft, coef, np.shape(h))
    return dict(loss=loss, dh=dh, dw=dw, n_active=int(active.sum()),
                logp=logp.reshape(np.shape(targets)))


def grpo(h, w, targets, advantages, ref_logp, old_logp=None,
         clip_eps=0.2, kl_beta=0.04, kl_mode=0):
    """GRPO objective (Sec. 3.2.1, GRPO objective; notation in App. A.2).

    h [G, T, d]; targets [G, T] (negative = not a response token);
    advantages [G] (one per sequence); ref_logp, old_logp [G, T].
    f(j,t) = min(r A_j, clip(r, 1-eps, 1+eps) A_j) - beta * KL_t with
    r = pi_theta / pi_old, and
      kl_mode 0: KL_t = log pi_theta - log pi_ref       (the paper's compact form)
      kl_mode 1: KL_t = exp(ref - logp) - (ref - logp) - 1   (with the
                 compensation term the paper says it leaves out of the display)
    L = -(1/G) sum_j (1/T_o,j) sum_{t in response_j} f(j,t), T_o,j the number of
    response tokens of sequence j.  old_logp=None means the on-policy case
    pi_old = stop_gradient(pi_theta): r = 1 in value, d r / d logp = 1.
    Derivative of the min term wrt logp: r*A when the unclipped term is the
    (weak) minimum, else 0.
    """
    G, T = np.shape(targets)
    h2, w, tg, active, safe, logp, soft = _logits_logp(h, w, targets)
    adv = np.repeat(np.asarray(advantages, F64), T)
    ref = np.asarray(ref_logp, F64).reshape(-1)
    r = np.ones_like(logp) if old_logp is None else np.exp(logp - np.asarray(old_logp, F64).reshape(-1))
    unclipped = r * adv
    clipped = np.clip(r, 1.0 - clip_eps, 1.0 + clip_eps) * adv
    surrogate = np.minimum(unclipped, clipped)
    dsurr = np.where(unclipped <= clipped, unclipped, 0.0)
    if kl_mode == 0:
        kl = logp - ref
        dkl = np.ones_like(logp)
    else:
        kl = np.exp(ref - logp) - (ref - logp) - 1.0
        dkl = 1.0 - np.exp(ref - logp)
    f = surrogate - kl_beta * kl
    df = dsurr - kl_beta * dkl
    t_o = active.reshape(G, T).sum(axis=1).astype(F64)            # response length per sequence
    wgt = np.repeat(np.where(t_o > 0, 1.0 / (G * np.maximum(t_o, 1.0)), 0.0), T)
    loss = -np.sum((wgt * f)[active])
    coef = np.where(active, -wgt * df, 0.0)
    dh, dw = _grads_from_coef(h2, w, active, safe, soft, coef, np.shape(h))
    return dict(loss=loss, dh=dh, dw=dw, n_active=int(active.sum()),
                logp=logp.reshape(G, T))


def dpo(h, w, targets, ref_logp, beta=0.1):
    """DPO objective for one (chosen, rejected) pair (Sec. 3.2.1, DPO
    objective): h [2, T, d], row 0 = chosen y_w, row 1 = rejected y_l.
    ell = sum_t [(logp_w - ref_w) - (logp_l - ref_l)] over active tokens,
    L = -log sigmoid(beta * ell);  dL/dlogp_w,t = (sigmoid(beta ell) - 1) beta,
    dL/dlogp_l,t = -(sigmoid(beta ell) - 1) beta."""
    _, T = np.shape(targets)
    h2, w, tg, active, safe, logp, soft = _logits_logp(h, w, targets)
    ref = np.asarray(ref_logp, F64).reshape(-1)
    sign = np.concatenate([np.ones(T), -np.ones(T)])
    ell = np.sum((sign * (logp - ref))[active])
    sig = 1.0 / (1.0 + np.exp(-beta * ell))
    loss = np.log1p(np.exp(-beta * ell)) if beta * ell > -30 else -beta * ell
    coef = np.where(active, (sig - 1.0) * beta * sign, 0.0)
    dh, dw = _grads_from_coef(h2, w, active, safe, soft, coef, np.shape(h))
    return dict(loss=loss, dh=dh, dw=dw, n_active=int(active.sum()), ell=ell,
                logp=logp.reshape(2, T))
