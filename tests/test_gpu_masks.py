"""GPU parity of the mask rules beyond plain causality - sliding window and padding in front of the sequence (Sec. 3.2.2:
softmax(S, M) with a general mask M) - against the fp64 oracle: chunk attention forward / backward on the MFMA kernels
and on the shape-agnostic ones, and the whole layer backward with a window and per-sequence padding."""
import numpy as np
import pytest
import torch

from oracle import attn as o_attn
from oracle import layer as o_layer
from paper_2506_03077_amd import binding as sb
from paper_2506_03077_amd import synth

from gpu_util import TOL, assert_close, code, dev, host, lib_layer_cfg, oracle_cfg

pytestmark = pytest.mark.gpu


def masked_attn_case(dtype, Hq, Hkv, dh, s, c, window, kv_first, seed=0):
    inp = synth.attn_inputs(Hq, Hkv, dh, s, c, dtype, seed)
    scale = 1.0 / np.sqrt(dh)
    o_ref, lse_ref = o_attn.chunk_forward(inp["q"], inp["k"], inp["v"], s, scale, window, kv_first)
    dq_ref, dk_ref, dv_ref = o_attn.chunk_backward(inp["q"], inp["k"], inp["v"], inp["d_o"], s, scale, window, kv_first)
    q, k, v, d_o = (dev(inp[n], dtype) for n in ("q", "k", "v", "d_o"))
    ac = sb.attn_cfg(code(dtype), Hq, Hkv, dh, s, c, scale, window, kv_first)
    o, lse = sb.streambp_attn_chunk_forward(ac, q, k, v)
    dq, dk, dv = sb.streambp_attn_chunk_backward(ac, q, k, v, o, lse, d_o)
    torch.cuda.synchronize()
    tol = TOL[dtype]
    empty = ~np.isfinite(lse_ref)                                       # [Hq, c]: queries that see no key
    lse_g = host(lse)
    assert np.array_equal(~np.isfinite(lse_g), empty) and np.all(lse_g[empty] == -np.inf)
    if empty.any():
        assert torch.all(o[torch.from_numpy(empty.T.copy()).cuda()] == 0)        # o = 0 exactly where nothing is visible
        assert torch.all(dq[torch.from_numpy(empty.T.copy()).cuda()] == 0)
    assert_close(host(o), o_ref, tol, "o")
    assert_close(np.where(empty, 0.0, lse_g), np.where(empty, 0.0, lse_ref), 1e-4 if dtype == "f32" else 2e-3, "lse")
    assert_close(host(dq), dq_ref, tol, "dq")
    assert_close(host(dk)[:s + c], dk_ref, tol, "dk")
    assert_close(host(dv)[:s + c], dv_ref, tol, "dv")
    # keys no query of the chunk can see get exactly zero (integer mask: exact)
    hidden = ~o_attn.visible(s + np.arange(c), np.arange(s + c), window, kv_first).any(axis=0)
    hid = torch.from_numpy(hidden).cuda()
    assert torch.all(dk[:s + c][hid] == 0) and torch.all(dv[:s + c][hid] == 0)
    return q, k, v, d_o, ac, o, lse, dq, dk, dv, hidden


@pytest.mark.parametrize("s,c,window,kv_first", [
    (0, 200, 10, 0),          # window shorter than a key tile
    (300, 177, 100, 0),       # window across tiles, ragged chunk, prefix keys wholly outside every window
    (1000, 256, 300, 0),      # whole key tiles skipped on the left edge
    (256, 200, 0, 70),        # padding inside the prefix
    (0, 300, 0, 130),         # padding reaching into the chunk: queries that see nothing
    (500, 130, 64, 520),      # both rules; padding ends inside the chunk
    (513, 255, 1, 0),         # every query sees only itself
    (100, 64, 5000, 0),       # window longer than the sequence: plain causal
])
def test_masked_attention_bf16_dh128(s, c, window, kv_first):
    masked_attn_case("bf16", 8, 2, 128, s, c, window, kv_first)


def test_masked_attention_shape_agnostic_kernels():
    masked_attn_case("f32", 4, 2, 16, 100, 37, 20, 0)
    masked_attn_case("f32", 4, 4, 16, 0, 64, 0, 30)
    masked_attn_case("f32", 6, 2, 24, 300, 50, 17, 310)
    masked_attn_case("bf16", 6, 2, 24, 40, 50, 17, 45)


def test_hidden_keys_are_never_read_or_never_matter():
    # keys and values outside every query's range: whole tiles of them are never loaded (NaN there changes nothing), the
    # ones that share a tile with visible keys are loaded but masked by index (huge finite values change nothing)
    Hq, Hkv, dh, s, c, window = 8, 2, 128, 2000, 200, 300
    q, k, v, d_o, ac, o, lse, dq, dk, dv, hidden = masked_attn_case("bf16", Hq, Hkv, dh, s, c, window, 0, seed=5)
    first_visible = s - window + 1                       # of the chunk's first query
    k2, v2 = k.clone(), v.clone()
    k2[:(first_visible // 128) * 128] = float("nan")     # before the first key block any kernel launches or loads
    v2[:(first_visible // 128) * 128] = float("nan")
    k2[(first_visible // 128) * 128:first_visible] = 3.0e4
    v2[(first_visible // 128) * 128:first_visible] = -3.0e4
    o2, lse2 = sb.streambp_attn_chunk_forward(ac, q, k2, v2)
    dq2, dk2, dv2 = sb.streambp_attn_chunk_backward(ac, q, k2, v2, o2, lse2, d_o)
    torch.cuda.synchronize()
    assert torch.equal(o2, o) and torch.equal(lse2, lse) and torch.equal(dq2, dq)
    vis = torch.from_numpy(~hidden).cuda()
    assert torch.equal(dk2[:s + c][vis], dk[:s + c][vis]) and torch.equal(dv2[:s + c][vis], dv[:s + c][vis])
    assert torch.all(dk2[:(first_visible // 128) * 128] == 0)


MID16 = dict(dtype="bf16", hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=128, mlp_width=512)
TINY = synth.CONFIGS["tiny"]


@pytest.mark.parametrize("cfg,T,chunk,window,first", [
    (MID16, 640, 256, 100, None), (MID16, 333, 100, 0, [50, 0]), (MID16, 500, 128, 200, [130, 7]),
    (TINY, 96, 40, 16, [10, 0, 41]), (TINY, 256, 64, 0, [100]),
])
def test_layer_backward_with_window_and_front_padding(cfg, T, chunk, window, first):
    cfg = dict(cfg, window=window)
    B = len(first) if first else 1
    inp = synth.layer_inputs(cfg, seed=7, seq_len=T, batch=B)
    _, dx_ref, g_ref = o_layer.layer_forward_backward(inp["x"], inp["w"], oracle_cfg(cfg), inp["dy"], first)
    dt = cfg["dtype"]
    w = {k: dev(v, dt) for k, v in inp["w"].items()}
    lc = lib_layer_cfg(cfg, T, chunk, B, seq_first=first)
    dx, dw = sb.streambp_layer_backward(lc, w, dev(inp["x"], dt), dev(inp["dy"], dt))
    torch.cuda.synchronize()
    assert_close(host(dx), dx_ref, TOL[dt], "dx")
    for n in sb.WEIGHT_NAMES:
        assert_close(host(dw[n]), g_ref[n], TOL[dt], f"d{n}")
    # forward with the same masks
    y_ref = np.stack([o_layer.layer_forward(inp["x"][b], inp["w"], dict(oracle_cfg(cfg), first_valid=(first[b] if first else 0)))[0]
                      for b in range(B)])
    y = sb.streambp_layer_forward(lc, w, dev(inp["x"], dt))
    assert_close(host(y), y_ref, TOL[dt] if dt == "f32" else 1e-2, "y")


def test_layer_with_a_window_at_7b_widths_vs_oracle():
    # the bench's launch configuration (chunk 2048, 7B widths) with a 1024-token sliding window and 300 rows of padding
    cfg = dict(synth.CONFIGS["7b"], window=1024)
    T, chunk, first = 4608, 2048, [300]
    inp = synth.layer_inputs(cfg, seed=8, seq_len=T)
    _, dx_ref, g_ref = o_layer.layer_forward_backward(inp["x"], inp["w"], oracle_cfg(cfg), inp["dy"], first)
    w = {k: dev(v, "bf16") for k, v in inp["w"].items()}
    before = sb.streambp_generic_launches()
    dx, dw = sb.streambp_layer_backward(lib_layer_cfg(cfg, T, chunk, seq_first=first), w, dev(inp["x"], "bf16"), dev(inp["dy"], "bf16"))
    torch.cuda.synchronize()
    assert sb.streambp_generic_launches() == before
    assert_close(host(dx), dx_ref, 2e-2, "dx")
    for n in sb.WEIGHT_NAMES:
        assert_close(host(dw[n]), g_ref[n], 2e-2, f"d{n}")
