"""The entry points under HIP graph capture: they allocate nothing, never synchronise and clear memory with fill kernels
(no memset nodes), so a captured call must replay to the eager result - bit for bit, on every replay, with the program's own
eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

from paper_2506_03077_amd import binding as sb
from paper_2506_03077_amd import synth

from gpu_util import dev, lib_layer_cfg

pytestmark = pytest.mark.gpu

MID16 = dict(dtype="bf16", hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=128, mlp_width=512, vocab=1024)


def test_layer_and_head_replay_from_a_captured_graph():
    cfg, T, chunk = MID16, 333, 128
    inp = synth.layer_inputs(cfg, seed=11, seq_len=T, batch=2)
    w = {k: dev(v, "bf16") for k, v in inp["w"].items()}
    x, dy = dev(inp["x"], "bf16"), dev(inp["dy"], "bf16")
    lc = lib_layer_cfg(dict(cfg, window=100), T, chunk, 2, seq_first=[0, 40])
    hin = synth.head_inputs(cfg, seed=11, seq_len=T, batch=2, vocab=cfg["vocab"])
    wh, h, tg = dev(hin["w"], "bf16"), dev(hin["h"], "bf16"), torch.from_numpy(hin["targets"]).cuda()
    hc = sb.head_cfg(sb.SBP_BF16, 2, T, chunk, cfg["hidden"], cfg["vocab"], sb.SBP_OBJ_SFT, 1.0 / 500)

    # eager reference
    dx_e, dw_e = sb.streambp_layer_backward(lc, w, x, dy)
    dh_e, dwh_e, loss_e, na_e = sb.streambp_lmhead_ce_backward(hc, wh, h, tg)
    torch.cuda.synchronize()

    # static buffers of the captured call (everything the calls touch is allocated before the capture)
    dx = torch.empty_like(x)
    dw = sb.new_layer_grads(w)
    ws_l = torch.empty(sb.streambp_layer_workspace_bytes(lc), dtype=torch.uint8, device="cuda")
    dh = torch.empty_like(h)
    dwh = torch.zeros(wh.shape, dtype=torch.float32, device="cuda")
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    na = torch.zeros(1, dtype=torch.int64, device="cuda")
    ws_h = torch.empty(sb.streambp_lmhead_workspace_bytes(hc), dtype=torch.uint8, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            sb.streambp_lmhead_ce_backward(hc, wh, h, tg, dh=dh, dw=dwh, loss=loss, n_active=na, workspace=ws_h, stream=side)
            sb.streambp_layer_backward(lc, w, x, dy, dx=dx, dw=dw, workspace=ws_l, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    for replay in range(3):
        for t in dw.values():           # the accumulators are the caller's: cleared by eager work between the replays
            t.zero_()
        dwh.zero_(); loss.zero_()
        ws_l.fill_(0xAB); ws_h.fill_(0xCD)     # nothing in the workspaces may be expected to survive
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(dx, dx_e), f"replay {replay}: dx"
        assert all(torch.equal(dw[n], dw_e[n]) for n in sb.WEIGHT_NAMES), f"replay {replay}: dw"
        assert torch.equal(dh, dh_e) and torch.equal(dwh, dwh_e) and torch.equal(loss, loss_e) and torch.equal(na, na_e), f"replay {replay}: head"
        _ = (x.float() @ x.float().transpose(1, 2)).sum().item()      # unrelated eager work + a host synchronisation


def test_noalloc_attention_backward_under_capture():
    Hq, Hkv, dh, s, c = 8, 2, 128, 300, 200
    a = synth.attn_inputs(Hq, Hkv, dh, s, c, "bf16", 13)
    q, k, v, d_o = (dev(a[n], "bf16") for n in ("q", "k", "v", "d_o"))
    ac = sb.attn_cfg(sb.SBP_BF16, Hq, Hkv, dh, s, c, 1.0 / np.sqrt(dh))
    o, lse = sb.streambp_attn_chunk_forward(ac, q, k, v)
    dq_e, dk_e, dv_e = sb.streambp_attn_chunk_backward(ac, q, k, v, o, lse, d_o)
    dq = torch.empty_like(q)
    dk = torch.zeros(k.shape, dtype=torch.float32, device="cuda")
    dv = torch.zeros(v.shape, dtype=torch.float32, device="cuda")
    sb.streambp_attn_chunk_backward_noalloc(ac, q, k, v, o, lse, d_o, dq, dk, dv)      # first call on the device: outside capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            sb.streambp_attn_chunk_backward_noalloc(ac, q, k, v, o, lse, d_o, dq, dk, dv, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    for replay in range(3):
        dk.zero_(); dv.zero_(); dq.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(dq, dq_e) and torch.equal(dk, dk_e) and torch.equal(dv, dv_e), f"replay {replay}"
