"""Pins for oracle/head.py and the head part of oracle/chunked.py (CPU only)."""
import math

import numpy as np
import pytest
from scipy.special import log_softmax

from oracle import chunked, head


def make(B=2, T=5, d=6, V=11, seed=0, mask_first=2):
    rng = np.random.default_rng(seed)
    h = rng.normal(0, 1, (B, T, d))
    w = rng.normal(0, 0.5, (V, d))
    tg = rng.integers(0, V, (B, T)).astype(np.int32)
    tg[:, :mask_first] = -1
    return h, w, tg


def fd(fun, base, hstep=1e-6):
    num = np.zeros_like(base)
    it = np.nditer(base, flags=["multi_index"])
    for _ in it:
        idx = it.multi_index
        p = base.copy(); p[idx] += hstep
        m = base.copy(); m[idx] -= hstep
        num[idx] = (fun(p) - fun(m)) / (2 * hstep)
    return num


def relerr(a, b):
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300)


def test_sft_loss_is_library_log_softmax_at_labels():
    h, w, tg = make()
    r = head.sft(h, w, tg, loss_scale=0.37)
    lp = log_softmax(h.reshape(-1, 6) @ w.T, axis=1)
    want = -0.37 * sum(lp[i, t] for i, t in enumerate(tg.reshape(-1)) if t >= 0)
    assert abs(r["loss"] - want) < 1e-12
    assert r["n_active"] == int((tg >= 0).sum())


def test_sft_finite_differences():
    h, w, tg = make()
    r = head.sft(h, w, tg, 0.5)
    assert relerr(r["dh"], fd(lambda hh: head.sft(hh, w, tg, 0.5)["loss"], h)) < 1e-8
    assert relerr(r["dw"], fd(lambda ww: head.sft(h, ww, tg, 0.5)["loss"], w)) < 1e-8


def test_sft_structure():
    h, w, tg = make(V=13)
    r = head.sft(h, w, tg)
    assert np.all(r["dh"][tg < 0] == 0.0)                         # ignored rows: exactly zero
    np.testing.assert_allclose(r["dw"].sum(axis=0), 0.0, atol=1e-13)   # rows of dz sum to zero
    # zero weights: uniform softmax, loss = n_active * ln V, dh = 0
    r0 = head.sft(h, np.zeros_like(w), tg)
    assert abs(r0["loss"] - r0["n_active"] * math.log(13)) < 1e-12
    assert np.all(r0["dh"] == 0)
    # single active row: dz = softmax - onehot, dW = dz^T h written out by hand
    h1, w1, tg1 = make(B=1, T=1, mask_first=0, V=13)
    z = w1 @ h1[0, 0]
    p = np.exp(z - z.max()); p /= p.sum()
    p[tg1[0, 0]] -= 1.0
    r1 = head.sft(h1, w1, tg1)
    np.testing.assert_allclose(r1["dw"], np.outer(p, h1[0, 0]), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(r1["dh"][0, 0], p @ w1, rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("kl_mode", [0, 1])
@pytest.mark.parametrize("on_policy", [True, False])
def test_grpo_finite_differences(kl_mode, on_policy):
    h, w, tg = make(B=3, T=6, seed=3)
    rng = np.random.default_rng(7)
    adv = rng.normal(size=3)
    ref = rng.normal(-2, 0.5, (3, 6))
    base = head.grpo(h, w, tg, adv, ref, None, 0.2, 0.04, kl_mode)
    # pi_old is a constant (no gradient through it).  On-policy: old = current log-probs, frozen.
    old = base["logp"].copy() if on_policy else base["logp"] + rng.normal(0, 0.3, (3, 6))
    r = head.grpo(h, w, tg, adv, ref, None if on_policy else old, 0.2, 0.04, kl_mode)
    f_h = lambda hh: head.grpo(hh, w, tg, adv, ref, old, 0.2, 0.04, kl_mode)["loss"]
    f_w = lambda ww: head.grpo(h, ww, tg, adv, ref, old, 0.2, 0.04, kl_mode)["loss"]
    assert relerr(r["dh"], fd(f_h, h)) < 1e-7
    assert relerr(r["dw"], fd(f_w, w)) < 1e-7
    # value: explicit frozen old = current must give the same loss as old=None
    assert abs(head.grpo(h, w, tg, adv, ref, base["logp"], 0.2, 0.04, kl_mode)["loss"] - base["loss"]) < 1e-12


def test_grpo_value_by_hand_and_clipping():
    # one sequence, two response tokens, written out with scalars
    h, w, tg = make(B=1, T=3, mask_first=1, seed=4)
    adv = np.array([1.5]); ref = np.array([[-2.0, -1.0, -3.0]])
    lp = log_softmax(h.reshape(-1, 6) @ w.T, axis=1)
    logp = np.array([lp[i, max(t, 0)] for i, t in enumerate(tg.reshape(-1))])
    old = logp + np.array([0.0, 0.5, -0.5])        # ratios exp(-0.5) (clipped low), exp(0.5) (clipped high)
    want = 0.0
    for t in (1, 2):
        r = math.exp(logp[t] - old[t])
        f = min(r * 1.5, min(max(r, 0.8), 1.2) * 1.5) - 0.04 * (logp[t] - ref[0, t])
        want -= f / 2.0
    got = head.grpo(h, w, tg, adv, ref, old[None], 0.2, 0.04, 0)
    assert abs(got["loss"] - want) < 1e-12
    # positive advantage with ratio above 1+eps: surrogate is clipped, only the KL term has gradient
    only_kl = head.grpo(h, w, tg, adv, ref, old[None], 0.2, 0.04, 0)
    no_adv = head.grpo(h, w, tg, 0 * adv, ref, old[None], 0.2, 0.04, 0)
    t2 = only_kl["dh"][0, 2]      # ratio exp(0.5) > 1.2, A > 0 -> clipped
    np.testing.assert_allclose(t2, no_adv["dh"][0, 2], rtol=1e-12)
    assert relerr(only_kl["dh"][0, 1], no_adv["dh"][0, 1]) > 1e-3    # ratio < 0.8 with A > 0 is NOT clipped by min


def test_dpo_finite_differences_on_true_loss():
    h, w, tg = make(B=2, T=5, seed=9)
    ref = np.random.default_rng(1).normal(-2, 0.5, (2, 5))
    r = head.dpo(h, w, tg, ref, beta=0.3)
    # the true loss written independently
    def true_loss(hh, ww):
        lp = log_softmax(hh.reshape(-1, 6) @ ww.T, axis=1)
        ell = 0.0
        for i, t in enumerate(tg.reshape(-1)):
            if t >= 0:
                ell += (1 if i < 5 else -1) * (lp[i, t] - ref.reshape(-1)[i])
        return -math.log(1 / (1 + math.exp(-0.3 * ell)))
    assert abs(r["loss"] - true_loss(h, w)) < 1e-12
    assert relerr(r["dh"], fd(lambda hh: true_loss(hh, w), h)) < 1e-7
    assert relerr(r["dw"], fd(lambda ww: true_loss(h, ww), w)) < 1e-7


@pytest.mark.parametrize("chunk", [1, 2, 3, 5, 64])
def test_head_chunk_loop_reaches_the_full_gradient(chunk):
    h, w, tg = make(B=2, T=5)
    full = head.sft(h, w, tg, 0.25)
    ch = chunked.head_backward_chunked(h, w, tg, chunk, "sft", loss_scale=0.25)
    for k in ("dh", "dw", "loss"):
        np.testing.assert_allclose(ch[k], full[k], rtol=1e-12, atol=1e-13)
    assert ch["n_active"] == full["n_active"]
    rng = np.random.default_rng(5)
    adv, ref = rng.normal(size=2), rng.normal(-2, 0.5, (2, 5))
    full = head.grpo(h, w, tg, adv, ref, None, 0.2, 0.04, 1)
    ch = chunked.head_backward_chunked(h, w, tg, chunk, "grpo", advantages=adv, ref_logp=ref, kl_mode=1)
    for k in ("dh", "dw", "loss"):
        np.testing.assert_allclose(ch[k], full[k], rtol=1e-12, atol=1e-13)
