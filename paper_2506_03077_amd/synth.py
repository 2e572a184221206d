"""Seeded synthetic inputs shared by the tests, the smoke check and the bench.

This module holds none of the method's arithmetic: it only draws random
tensors with the shapes and value distributions of the workloads (random-init
weights N(0, 0.02), hidden states N(0, 1), upstream gradients N(0, 1e-3),
uniform token ids, prompt masks) and rounds them to the storage type, so that
the CPU oracle and the HIP path start from bit-identical values and input
quantisation is not counted as error.
"""
from __future__ import annotations

import numpy as np

WEIGHT_NAMES = ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown", "g1", "g2")

# Named workload shapes.
CONFIGS = {
    # tiny fp32 layer + head: F = 172 is deliberately not a multiple of 16
    "tiny": dict(dtype="f32", hidden=64, n_q_heads=4, n_kv_heads=4, head_dim=16, mlp_width=172,
                 vocab=512, seq_len=256, chunk=64, batch=1),
    "llama_layer": dict(dtype="bf16", hidden=4096, n_q_heads=32, n_kv_heads=8, head_dim=128,
                        mlp_width=14336, seq_len=8192, chunk=1024, batch=1),
    "lmhead": dict(dtype="bf16", hidden=3584, vocab=152064, seq_len=32768, chunk=2048, batch=1),
    "7b": dict(dtype="bf16", hidden=3584, n_q_heads=28, n_kv_heads=4, head_dim=128, mlp_width=18944,
               vocab=152064, seq_len=32768, chunk=2048, batch=1, n_layers=28),
    "grpo": dict(dtype="bf16", hidden=3584, n_q_heads=28, n_kv_heads=4, head_dim=128, mlp_width=18944,
                 vocab=152064, seq_len=16384, chunk=2048, batch=8),
}


def round_bf16(a):
    """Round float values to the nearest bfloat16 (ties to even); returns float32."""
    a32 = np.ascontiguousarray(a, dtype=np.float32)
    u = a32.view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    out = ((u + bias) & np.uint32(0xFFFF0000)).view(np.float32)
    return np.where(np.isfinite(a32), out, a32).astype(np.float32)


def to_storage(a, dtype):
    """Values as float32 arrays that are exactly representable in `dtype`."""
    a = np.asarray(a, dtype=np.float32)
    return round_bf16(a) if dtype == "bf16" else a


def _streams(seed, n):
    return [np.random.default_rng(s) for s in np.random.SeedSequence(seed).spawn(n)]


def layer_weights(cfg, seed=0):
    """Matrices N(0, 0.02) stored [out, in]; norm gains 1 + N(0, 0.02)."""
    d, Hq, Hkv, dh, F = (cfg[k] for k in ("hidden", "n_q_heads", "n_kv_heads", "head_dim", "mlp_width"))
    shapes = dict(wq=(Hq * dh, d), wk=(Hkv * dh, d), wv=(Hkv * dh, d), wo=(d, Hq * dh),
                  wgate=(F, d), wup=(F, d), wdown=(d, F), g1=(d,), g2=(d,))
    rngs = _streams(seed, len(WEIGHT_NAMES))
    w = {}
    for name, rng in zip(WEIGHT_NAMES, rngs):
        v = rng.standard_normal(shapes[name], dtype=np.float32) * np.float32(0.02)
        if name in ("g1", "g2"):
            v = v + np.float32(1.0)
        w[name] = to_storage(v, cfg["dtype"])
    return w


def layer_inputs(cfg, seed=0, seq_len=None, batch=None, x_std=1.0, dy_std=1e-3):
    """x [B, T, d] ~ N(0, x_std), dy [B, T, d] ~ N(0, dy_std) plus layer weights."""
    T = seq_len or cfg["seq_len"]
    B = batch or cfg.get("batch", 1)
    d = cfg["hidden"]
    rx, rdy = _streams(seed + 1000003, 2)
    x = to_storage(rx.standard_normal((B, T, d), dtype=np.float32) * np.float32(x_std), cfg["dtype"])
    dy = to_storage(rdy.standard_normal((B, T, d), dtype=np.float32) * np.float32(dy_std), cfg["dtype"])
    return dict(x=x, dy=dy, w=layer_weights(cfg, seed))


def head_inputs(cfg, seed=0, seq_len=None, batch=None, vocab=None, prompt_frac=0.25, h_std=1.0):
    """h [B, T, d] ~ N(0, h_std); W [V, d] ~ N(0, 0.02); targets uniform in
    [0, V) with the first prompt_frac of every sequence set to -1 (ignored)."""
    T = seq_len or cfg["seq_len"]
    B = batch or cfg.get("batch", 1)
    V = vocab or cfg["vocab"]
    d = cfg["hidden"]
    rh, rw, rt = _streams(seed + 2000003, 3)
    h = to_storage(rh.standard_normal((B, T, d), dtype=np.float32) * np.float32(h_std), cfg["dtype"])
    w = to_storage(rw.standard_normal((V, d), dtype=np.float32) * np.float32(0.02), cfg["dtype"])
    targets = rt.integers(0, V, size=(B, T), dtype=np.int32)
    n_prompt = int(round(prompt_frac * T))
    targets[:, :n_prompt] = -1
    return dict(h=h, w=w, targets=targets)


def grpo_extras(batch, seq_len, seed=0):
    """Per-sequence advantages N(0, 1) and reference log-probs N(-2, 0.5)
    (second parameter read as the standard deviation)."""
    ra, rr = _streams(seed + 3000003, 2)
    adv = ra.standard_normal(batch).astype(np.float32)
    ref = (rr.standard_normal((batch, seq_len)) * 0.5 - 2.0).astype(np.float32)
    return dict(advantages=adv, ref_logp=ref)


def token_stream(cfg, seed=0, seq_len=None):
    """Token ids uniform in [0, V), an embedding table N(0, 0.02), and SFT
    targets = ids shifted by one with the last position ignored."""
    T = seq_len or cfg["seq_len"]
    V, d = cfg["vocab"], cfg["hidden"]
    ri, re = _streams(seed + 4000003, 2)
    ids = ri.integers(0, V, size=(T,), dtype=np.int32)
    emb = to_storage(re.standard_normal((V, d), dtype=np.float32) * np.float32(0.02), cfg["dtype"])
    targets = np.concatenate([ids[1:], np.array([-1], dtype=np.int32)])
    return dict(ids=ids, emb=emb, targets=targets)


def attn_inputs(n_q_heads, n_kv_heads, head_dim, q_start, q_len, dtype="bf16", seed=0, std=1.0):
    """q, d_o [c, Hq, dh]; k, v [q_start + c, Hkv, dh], all N(0, std)."""
    rq, rk, rv, rdo = _streams(seed + 5000003, 4)
    n = q_start + q_len
    q = to_storage(rq.standard_normal((q_len, n_q_heads, head_dim), dtype=np.float32) * np.float32(std), dtype)
    k = to_storage(rk.standard_normal((n, n_kv_heads, head_dim), dtype=np.float32) * np.float32(std), dtype)
    v = to_storage(rv.standard_normal((n, n_kv_heads, head_dim), dtype=np.float32) * np.float32(std), dtype)
    d_o = to_storage(rdo.standard_normal((q_len, n_q_heads, head_dim), dtype=np.float32) * np.float32(std), dtype)
    return dict(q=q, k=k, v=v, d_o=d_o)
