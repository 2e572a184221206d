"""GPU parity at the workloads' real widths, in the launch configuration bench.py times
(bf16, d=3584, 28q/4kv x128, F=18944, V=152064, chunk 2048).

The fp64 oracle cannot run a 32k-token layer (it is a plain full-sequence backprop), so:
  * layer and head are compared element by element against the oracle at the real widths AND the real chunk size
    (2048 rows; also 512 and no partition), at a sequence length the oracle finishes in tens of seconds
    (T = 4608 for the layer: two full chunks and a ragged one; 8792 rows for the head: four full chunks and a
    ragged one), so that the kernels' launch shapes - split-K factors, operand pairs, grouped multi-segment
    weight-gradient passes - are those of the benchmark;
  * at the full 32k length, chunk attention is compared element by element against the oracle
    for one whole KV group (the oracle's cost there is small), and the layer / head are checked
    through properties that hold at any size (chunk-size invariance, exact zeros of ignored
    rows, exact n_active, rows of dz summing to zero) plus oracle-computed sampled rows."""
import numpy as np
import pytest
import torch

from oracle import attn as o_attn
from oracle import head as o_head
from oracle import layer as o_layer
from paper_2506_03077_amd import binding as sb
from paper_2506_03077_amd import synth

from gpu_util import assert_close, dev, host, lib_layer_cfg, oracle_cfg, relerr

pytestmark = pytest.mark.gpu

C7B = synth.CONFIGS["7b"]
TOL = 2e-2


_LAYER_REF = {}


def layer_reference(cfg, T, seed):
    """Oracle gradients of one layer, computed once per (shape, T, seed) and shared by the chunk sizes compared with them."""
    key = (cfg["hidden"], cfg["mlp_width"], T, seed)
    if key not in _LAYER_REF:
        inp = synth.layer_inputs(cfg, seed=seed, seq_len=T)
        _, dx_ref, g_ref = o_layer.layer_forward_backward(inp["x"], inp["w"], oracle_cfg(cfg), inp["dy"])
        _LAYER_REF[key] = (inp, dx_ref, g_ref)
    return _LAYER_REF[key]


@pytest.mark.parametrize("chunk", [2048, 512, 4608])
def test_layer_7b_widths_vs_oracle(chunk):
    # 7B widths, T = 4608 = 2.25 chunks of 2048 (the chunk bench.py times; the last chunk ragged).  At chunk 2048 the layer
    # runs what the bench runs: the two-way XCD-pinned split-K input-gradient GEMMs over 112 output tiles, the operand-pair
    # dm GEMM, and ONE grouped weight-gradient launch with three reduction segments of 2048, 2048 and 512 rows; chunk 512
    # takes the 8-way split-K and groups of four chunks, chunk = T no partition at all.
    T = 4608
    assert sb.streambp_layer_fast_path(lib_layer_cfg(C7B, T, chunk)) == 1
    inp, dx_ref, g_ref = layer_reference(C7B, T, 0)
    w = {k: dev(v, "bf16") for k, v in inp["w"].items()}
    before = sb.streambp_generic_launches()
    dx, dw = sb.streambp_layer_backward(lib_layer_cfg(C7B, T, chunk), w, dev(inp["x"], "bf16"), dev(inp["dy"], "bf16"))
    torch.cuda.synchronize()
    assert sb.streambp_generic_launches() == before        # nothing left the MFMA kernels
    assert_close(host(dx), dx_ref, TOL, f"dx (chunk {chunk})")
    for n in sb.WEIGHT_NAMES:
        assert_close(host(dw[n]), g_ref[n], TOL, f"d{n} (chunk {chunk})")


_HEAD_REF = {}


@pytest.mark.parametrize("dw_group_rows", [0, 8192])
def test_head_full_vocab_vs_oracle(dw_group_rows):
    # V = 152064 at the bench's chunk of 2048 rows with 8792 active rows = four full chunks and a ragged fifth (600 rows).
    # Default grouping: their weight gradient is ONE five-segment pass over dW; with 8192 rows per pass a four-segment pass
    # and the ragged chunk as a pass of its own.  Every row of dh and every 256 x 256 tile of dW (8316 of them) is compared
    # with the oracle.
    T, chunk = 8792, 2048
    cfg = synth.CONFIGS["lmhead"]
    inp = synth.head_inputs(cfg, seed=0, seq_len=T, prompt_frac=0.0)
    n_act = int((inp["targets"] >= 0).sum())
    assert n_act == T
    if "ref" not in _HEAD_REF:
        _HEAD_REF["ref"] = o_head.sft(inp["h"], inp["w"], inp["targets"], 1.0 / n_act)
    ref = _HEAD_REF["ref"]
    hc = sb.head_cfg(sb.SBP_BF16, 1, T, chunk, cfg["hidden"], cfg["vocab"], sb.SBP_OBJ_SFT, 1.0 / n_act, dw_group_rows=dw_group_rows)
    assert sb.streambp_lmhead_fast_path(hc) == 1
    before = sb.streambp_generic_launches()
    dh, dw, loss, n_active = sb.streambp_lmhead_ce_backward(hc, dev(inp["w"], "bf16"), dev(inp["h"], "bf16"),
                                                            torch.from_numpy(inp["targets"]).cuda())
    torch.cuda.synchronize()
    assert sb.streambp_generic_launches() == before
    assert int(n_active.item()) == n_act
    assert_close(host(dh), ref["dh"], TOL, "dh")
    assert_close(host(dw), ref["dw"], TOL, "dw")
    assert abs(float(loss.item()) - ref["loss"]) < 2e-3 * ref["loss"]
    # random-init logits are ~N(0, 0.02^2 * d): mean loss ~ ln V + var/2
    assert abs(ref["loss"] - (np.log(cfg["vocab"]) + 0.5 * 0.02 ** 2 * cfg["hidden"])) < 0.1


def test_head_full_vocab_with_prompt_mask_vs_oracle():
    # the same with the first quarter of the rows ignored (the LM-head workload of the shape list): the active rows are
    # compacted, 2304 of them = one full chunk and a ragged one in ONE two-segment pass over dW
    T, chunk = 3072, 2048
    cfg = synth.CONFIGS["lmhead"]
    inp = synth.head_inputs(cfg, seed=1, seq_len=T)
    n_act = int((inp["targets"] >= 0).sum())
    ref = o_head.sft(inp["h"], inp["w"], inp["targets"], 1.0 / n_act)
    hc = sb.head_cfg(sb.SBP_BF16, 1, T, chunk, cfg["hidden"], cfg["vocab"], sb.SBP_OBJ_SFT, 1.0 / n_act)
    dh, dw, loss, n_active = sb.streambp_lmhead_ce_backward(hc, dev(inp["w"], "bf16"), dev(inp["h"], "bf16"),
                                                            torch.from_numpy(inp["targets"]).cuda())
    torch.cuda.synchronize()
    assert int(n_active.item()) == n_act == T - T // 4
    assert torch.all(dh[:, :T // 4] == 0)
    assert_close(host(dh), ref["dh"], TOL, "dh")
    assert_close(host(dw), ref["dw"], TOL, "dw")
    assert abs(float(loss.item()) - ref["loss"]) < 2e-3 * ref["loss"]


def test_head_with_a_151936_word_vocabulary_vs_oracle():
    # the vocabulary of the paper's own models: 593.5 output tiles - the logits GEMM, its row statistics and the weight
    # gradient end in a half tile; everything stays on the MFMA kernels
    T, chunk, V = 2304, 2048, 151936
    cfg = dict(synth.CONFIGS["lmhead"], vocab=V)
    inp = synth.head_inputs(cfg, seed=2, seq_len=T, prompt_frac=0.0)
    ref = o_head.sft(inp["h"], inp["w"], inp["targets"], 1.0 / T)
    hc = sb.head_cfg(sb.SBP_BF16, 1, T, chunk, cfg["hidden"], V, sb.SBP_OBJ_SFT, 1.0 / T)
    assert sb.streambp_lmhead_fast_path(hc) == 1
    before = sb.streambp_generic_launches()
    dh, dw, loss, n_active = sb.streambp_lmhead_ce_backward(hc, dev(inp["w"], "bf16"), dev(inp["h"], "bf16"),
                                                            torch.from_numpy(inp["targets"]).cuda())
    torch.cuda.synchronize()
    assert sb.streambp_generic_launches() == before
    assert int(n_active.item()) == T
    assert_close(host(dh), ref["dh"], TOL, "dh")
    assert_close(host(dw), ref["dw"], TOL, "dw")
    assert abs(float(loss.item()) - ref["loss"]) < 2e-3 * ref["loss"]


def test_attention_last_chunk_of_32k_one_kv_group_vs_oracle():
    Hq, Hkv, dh = C7B["n_q_heads"], C7B["n_kv_heads"], C7B["head_dim"]
    G = Hq // Hkv
    s, c = 32768 - 2048, 2048
    inp = synth.attn_inputs(Hq, Hkv, dh, s, c, "bf16", seed=0)
    scale = 1.0 / np.sqrt(dh)
    q, k, v, d_o = (dev(inp[n], "bf16") for n in ("q", "k", "v", "d_o"))
    ac = sb.attn_cfg(sb.SBP_BF16, Hq, Hkv, dh, s, c, scale)
    o, lse = sb.streambp_attn_chunk_forward(ac, q, k, v)
    dq, dk, dv = sb.streambp_attn_chunk_backward(ac, q, k, v, o, lse, d_o)
    torch.cuda.synchronize()
    g = 1                                              # KV head 1 and its 7 query heads
    hs = slice(g * G, (g + 1) * G)
    qg, kg, vg, dog = inp["q"][:, hs], inp["k"][:, g:g + 1], inp["v"][:, g:g + 1], inp["d_o"][:, hs]
    o_ref, lse_ref = o_attn.chunk_forward(qg, kg, vg, s, scale)
    dq_ref, dk_ref, dv_ref = o_attn.chunk_backward(qg, kg, vg, dog, s, scale)
    assert_close(host(o)[:, hs], o_ref, TOL, "o")
    assert_close(host(lse)[hs], lse_ref, 2e-3, "lse")
    assert_close(host(dq)[:, hs], dq_ref, TOL, "dq")
    assert_close(host(dk)[:, g], dk_ref[:, 0], TOL, "dk")
    assert_close(host(dv)[:, g], dv_ref[:, 0], TOL, "dv")


def test_layer_32k_chunk_invariance_and_structure():
    T = 32768
    gen = torch.Generator(device="cuda"); gen.manual_seed(1)
    bf = torch.bfloat16
    d, Hq, Hkv, dh, F = (C7B[k] for k in ("hidden", "n_q_heads", "n_kv_heads", "head_dim", "mlp_width"))
    rn = lambda shape, std, mean=0.0: (torch.randn(shape, generator=gen, device="cuda") * std + mean).to(bf)
    w = dict(wq=rn((Hq * dh, d), 0.02), wk=rn((Hkv * dh, d), 0.02), wv=rn((Hkv * dh, d), 0.02), wo=rn((d, Hq * dh), 0.02),
             wgate=rn((F, d), 0.02), wup=rn((F, d), 0.02), wdown=rn((d, F), 0.02), g1=rn((d,), 0.02, 1.0), g2=rn((d,), 0.02, 1.0))
    x, dy = rn((1, T, d), 1.0), rn((1, T, d), 1e-3)
    dy[:, T // 2:] = 0                                   # no loss on the second half ...
    dx_a, dw_a = sb.streambp_layer_backward(lib_layer_cfg(C7B, T, 2048), w, x, dy)
    dx_b, dw_b = sb.streambp_layer_backward(lib_layer_cfg(C7B, T, 4096), w, x, dy)
    torch.cuda.synchronize()
    assert torch.all(dx_a[:, T // 2:] == 0)              # ... so causality makes dx of those rows exactly zero
    assert bool(torch.isfinite(dx_a.float()).all())
    assert relerr(host(dx_b), host(dx_a)) < 1e-2         # chunk size only changes the rounding order
    for n in sb.WEIGHT_NAMES:
        assert relerr(host(dw_b[n]), host(dw_a[n])) < 1e-2, n


def test_head_32k_structure_and_sampled_rows():
    cfg = synth.CONFIGS["lmhead"]
    T, V, d = 32768, cfg["vocab"], cfg["hidden"]
    gen = torch.Generator(device="cuda"); gen.manual_seed(2)
    w = (torch.randn((V, d), generator=gen, device="cuda") * 0.02).to(torch.bfloat16)
    h = torch.randn((1, T, d), generator=gen, device="cuda").to(torch.bfloat16)
    tg = torch.randint(0, V, (1, T), generator=gen, device="cuda", dtype=torch.int32)
    tg[:, :T // 4] = -1
    n_act = T - T // 4
    hc = sb.head_cfg(sb.SBP_BF16, 1, T, 2048, d, V, sb.SBP_OBJ_SFT, 1.0 / n_act)
    dh, dw, loss, n_active = sb.streambp_lmhead_ce_backward(hc, w, h, tg)
    torch.cuda.synchronize()
    assert int(n_active.item()) == n_act                                   # integer: exact
    assert torch.all(dh[:, :T // 4] == 0)                                  # ignored rows: exact zeros
    col = dw.sum(dim=0).abs().max().item()                                 # rows of dz sum to zero
    assert col < 1e-3 * dw.abs().max().item() * np.sqrt(V)
    assert abs(float(loss.item()) - (np.log(V) + 0.5 * 0.02 ** 2 * d)) < 0.1
    # Eq. 1: the grouping of the per-chunk summands of dW is free.  The default adds eight chunks' worth (8 x 2048 rows) per
    # pass; chunk by chunk (the form compared with the oracle tile by tile above) must give the same dW up to fp32 rounding order
    lean = sb.head_cfg(sb.SBP_BF16, 1, T, 2048, d, V, sb.SBP_OBJ_SFT, 1.0 / n_act, dw_group_rows=2048)
    dh1, dw1, _, _ = sb.streambp_lmhead_ce_backward(lean, w, h, tg)
    torch.cuda.synchronize()
    assert torch.equal(dh1, dh)
    err = (dw1 - dw).abs().max().item()
    assert err < 1e-4 * dw.abs().max().item(), err
    del dh1, dw1
    # sampled rows, one by one with the oracle (dh_t needs only row t of h and W)
    w64 = w.double().cpu().numpy()
    rows = [T // 4, T // 4 + 1, 20000, T - 1]
    hs = h[0, rows].double().cpu().numpy()[None]
    ts = tg[0, rows].cpu().numpy()[None]
    ref = o_head.sft(hs, w64, ts, 1.0 / n_act)
    assert_close(host(dh[0, rows]), ref["dh"][0], TOL, "dh sampled rows")


# ---------------------------------------------------- the other workloads of the shape list ---
LLAMA = synth.CONFIGS["llama_layer"]


def test_llama_layer_widths_vs_oracle_and_8k_chunk_invariance():
    # Llama-style layer (d=4096, 32q/8kv x128, F=14336): element by element against the oracle at the config's own chunk
    # of 1024 rows (T = 2560: two chunks and a ragged third, one three-segment weight-gradient launch), then the real shape
    # (T=8192, chunk 1024) against itself at another chunk size.
    T, chunk = 2560, LLAMA["chunk"]
    inp, dx_ref, g_ref = layer_reference(LLAMA, T, 4)
    w = {k: dev(v, "bf16") for k, v in inp["w"].items()}
    dx, dw = sb.streambp_layer_backward(lib_layer_cfg(LLAMA, T, chunk), w, dev(inp["x"], "bf16"), dev(inp["dy"], "bf16"))
    torch.cuda.synchronize()
    assert_close(host(dx), dx_ref, TOL, "dx")
    for n in sb.WEIGHT_NAMES:
        assert_close(host(dw[n]), g_ref[n], TOL, f"d{n}")
    T = LLAMA["seq_len"]
    gen = torch.Generator(device="cuda"); gen.manual_seed(5)
    x = torch.randn((1, T, LLAMA["hidden"]), generator=gen, device="cuda").to(torch.bfloat16)
    dy = (torch.randn((1, T, LLAMA["hidden"]), generator=gen, device="cuda") * 1e-3).to(torch.bfloat16)
    dx_a, dw_a = sb.streambp_layer_backward(lib_layer_cfg(LLAMA, T, LLAMA["chunk"]), w, x, dy)
    dx_b, dw_b = sb.streambp_layer_backward(lib_layer_cfg(LLAMA, T, 3000), w, x, dy)       # ragged chunks
    torch.cuda.synchronize()
    assert bool(torch.isfinite(dx_a.float()).all())
    assert relerr(host(dx_b), host(dx_a)) < 1e-2
    for n in sb.WEIGHT_NAMES:
        assert relerr(host(dw_b[n]), host(dw_a[n])) < 1e-2, n


def test_grpo_group_of_8_structure_sampled_rows_and_batch_independence():
    # GRPO workload: 8 sequences x 16384 tokens, response = last 75 % of every sequence, on-policy, reference
    # log-probs N(-2, 0.5), one advantage per sequence.
    cfg = synth.CONFIGS["grpo"]
    B, T, V, d = cfg["batch"], cfg["seq_len"], cfg["vocab"], cfg["hidden"]
    gen = torch.Generator(device="cuda"); gen.manual_seed(6)
    w = (torch.randn((V, d), generator=gen, device="cuda") * 0.02).to(torch.bfloat16)
    h = torch.randn((B, T, d), generator=gen, device="cuda").to(torch.bfloat16)
    tg = torch.randint(0, V, (B, T), generator=gen, device="cuda", dtype=torch.int32)
    tg[:, :T // 4] = -1
    adv = torch.randn((B,), generator=gen, device="cuda")
    ref_logp = torch.randn((B, T), generator=gen, device="cuda") * 0.5 - 2.0
    T_o = T - T // 4
    hc = sb.head_cfg(sb.SBP_BF16, B, T, 2048, d, V, sb.SBP_OBJ_GRPO, 1.0, 0.2, 0.04, 1)
    dh, dw, loss, n_active = sb.streambp_lmhead_ce_backward(hc, w, h, tg, None, ref_logp, adv)
    torch.cuda.synchronize()
    assert int(n_active.item()) == B * T_o                                 # integer: exact
    assert torch.all(dh[:, :T // 4] == 0)                                  # prompt rows: exact zeros
    assert bool(torch.isfinite(dh.float()).all()) and bool(torch.isfinite(loss).all())
    assert dw.sum(dim=0).abs().max().item() < 1e-3 * dw.abs().max().item() * np.sqrt(V)   # rows of dz sum to zero
    # Two response rows per sequence, one by one with the oracle.  Given only those rows the oracle normalises by
    # T_o = 2 per sequence instead of the real count, so its gradient is scaled by 2 / T_o.
    rows = [T // 4, T - 1]
    ref = o_head.grpo(h[:, rows].double().cpu().numpy(), w.double().cpu().numpy(), tg[:, rows].cpu().numpy(),
                      adv.double().cpu().numpy(), ref_logp[:, rows].double().cpu().numpy(), None, 0.2, 0.04, 1)
    assert_close(host(dh[:, rows]), ref["dh"] * (len(rows) / T_o), TOL, "dh sampled rows")
    del dw, dh
    # Layer: the sequences of a batch do not interact, so sequence 3 alone reproduces its rows of dx bit for bit.
    Hq, Hkv, dhd, F = (cfg[k] for k in ("n_q_heads", "n_kv_heads", "head_dim", "mlp_width"))
    rn = lambda shape, std, mean=0.0: (torch.randn(shape, generator=gen, device="cuda") * std + mean).to(torch.bfloat16)
    lw = dict(wq=rn((Hq * dhd, d), 0.02), wk=rn((Hkv * dhd, d), 0.02), wv=rn((Hkv * dhd, d), 0.02), wo=rn((d, Hq * dhd), 0.02),
              wgate=rn((F, d), 0.02), wup=rn((F, d), 0.02), wdown=rn((d, F), 0.02), g1=rn((d,), 0.02, 1.0), g2=rn((d,), 0.02, 1.0))
    x, dy = rn((B, T, d), 1.0), rn((B, T, d), 1e-3)
    dx_all, dw_all = sb.streambp_layer_backward(lib_layer_cfg(cfg, T, 2048, batch=B), lw, x, dy)
    dx_one, dw_one = sb.streambp_layer_backward(lib_layer_cfg(cfg, T, 2048, batch=1), lw, x[3:4].contiguous(), dy[3:4].contiguous())
    torch.cuda.synchronize()
    assert torch.equal(dx_all[3], dx_one[0])
    assert bool(torch.isfinite(dx_all.float()).all())
    # Eq. 1 over sequences: the batch's weight gradient is the sum of the per-sequence ones
    assert dw_all["wdown"].norm().item() > dw_one["wdown"].norm().item()


NARROW = dict(dtype="bf16", hidden=256, n_q_heads=4, n_kv_heads=2, head_dim=128, mlp_width=512)


def test_attention_with_a_prefix_beyond_64k_vs_oracle():
    # a short chunk at the end of a 70001-token prefix: row and key indices beyond 2^16, element by element against the oracle
    Hq, Hkv, dh, s, c = 4, 2, 128, 69993, 8
    inp = synth.attn_inputs(Hq, Hkv, dh, s, c, "bf16", 11)
    scale = 1.0 / np.sqrt(dh)
    o_ref, lse_ref = o_attn.chunk_forward(inp["q"], inp["k"], inp["v"], s, scale)
    dq_ref, dk_ref, dv_ref = o_attn.chunk_backward(inp["q"], inp["k"], inp["v"], inp["d_o"], s, scale)
    q, k, v, d_o = (dev(inp[n], "bf16") for n in ("q", "k", "v", "d_o"))
    ac = sb.attn_cfg(sb.SBP_BF16, Hq, Hkv, dh, s, c, scale)
    o, lse = sb.streambp_attn_chunk_forward(ac, q, k, v)
    dq, dk, dv = sb.streambp_attn_chunk_backward(ac, q, k, v, o, lse, d_o)
    torch.cuda.synchronize()
    assert_close(host(o), o_ref, TOL, "o")
    assert_close(host(lse), lse_ref, 2e-3, "lse")
    assert_close(host(dq), dq_ref, TOL, "dq")
    assert_close(host(dk)[:s + c], dk_ref, TOL, "dk")
    assert_close(host(dv)[:s + c], dv_ref, TOL, "dv")


def test_layer_70k_tokens_chunk_invariance():
    # longer than 2^16 rows and not a multiple of anything: chunk 4096 (ragged tail) against chunk 25000
    T = 70001
    inp = synth.layer_inputs(NARROW, seed=4, seq_len=T)
    w = {k: dev(v, "bf16") for k, v in inp["w"].items()}
    x, dy = dev(inp["x"], "bf16"), dev(inp["dy"], "bf16")
    dy[:, T - 1000:] = 0
    dx_a, dw_a = sb.streambp_layer_backward(lib_layer_cfg(NARROW, T, 4096), w, x, dy)
    dx_b, dw_b = sb.streambp_layer_backward(lib_layer_cfg(NARROW, T, 25000), w, x, dy)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(dx_a.float()).all())
    assert torch.all(dx_a[:, T - 1000:] == 0) and torch.all(dx_b[:, T - 1000:] == 0)     # causality
    assert relerr(host(dx_b), host(dx_a)) < 1e-2
    for n in sb.WEIGHT_NAMES:
        assert relerr(host(dw_b[n]), host(dw_a[n])) < 1e-2, n
