"""The C-ABI library loads and exports every symbol include/*.h declares;
host-side validation returns the documented error codes (no GPU needed: every
check happens before the first HIP call)."""
import ctypes as C
import os
import re

import pytest

from paper_2506_03077_amd import binding as sb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions(header="streambp.h"):
    src = open(os.path.join(ROOT, "include", header)).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(streambp_\w+)\s*\(", src)))


def test_every_exported_symbol_is_declared_in_a_header():
    # nothing is exported behind the headers' back: the library's dynamic symbols named streambp_* are exactly
    # those of include/streambp.h plus the test hooks of include/streambp_debug.h
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", sb.LIB_PATH], capture_output=True, text=True, check=True).stdout
    exported = sorted({line.split()[-1] for line in out.splitlines() if line.split()[-1].startswith("streambp_")})
    declared = sorted(set(declared_functions()) | set(declared_functions("streambp_debug.h")))
    assert exported == declared
    assert all(n.startswith("streambp_debug_") for n in declared_functions("streambp_debug.h"))
    assert not any(n.startswith("streambp_debug_") for n in declared_functions())


def test_header_declares_the_three_named_entry_points():
    names = declared_functions()
    for n in ("streambp_layer_backward", "streambp_lmhead_ce_backward", "streambp_attn_chunk_backward"):
        assert n in names


def test_library_exports_every_declared_symbol():
    L = sb.lib()
    for n in declared_functions() + declared_functions("streambp_debug.h"):
        assert hasattr(L, n), n
    assert b"gfx950" in L.streambp_version()


def test_binding_mirrors_every_entry_point():
    # argument-marshalling wrappers carry the C names
    for n in declared_functions():
        if n in ("streambp_last_error",):
            continue
        assert hasattr(sb, n), f"binding lacks {n}"
    for n in ("layer_cfg", "head_cfg", "attn_cfg", "stack_cfg", "debug_gemm", "debug_profile_begin", "debug_profile_end"):
        assert hasattr(sb, n), n


def test_profile_kind_names_match_the_library():
    # the per-launch timing table of the binding names one entry per kind the library counts
    assert sb.lib().streambp_debug_profile_kinds() == len(sb.PROFILE_KINDS)
    assert "gemm_mfma_k<false, true, 5>" in sb.PROFILE_KINDS and "gemm_mfma_seg_k" in sb.PROFILE_KINDS


def good_layer_cfg(**kw):
    base = dict(dtype=sb.SBP_F32, batch=1, seq_len=256, chunk=64, hidden=64, n_q_heads=4, n_kv_heads=4,
                head_dim=16, mlp_width=172)
    base.update(kw)
    return sb.layer_cfg(**base)


def test_layer_workspace_has_no_full_sequence_activation_term():
    # bytes = alpha*min(c,T) + beta*T*Hkv*dh + const: linear in T through K/V-side terms only
    big = dict(dtype=sb.SBP_BF16, hidden=3584, n_q_heads=28, n_kv_heads=4, head_dim=128, mlp_width=18944, chunk=2048)
    w8, w16, w32 = (sb.streambp_layer_workspace_bytes(good_layer_cfg(seq_len=T, **big)) for T in (8192, 16384, 32768))
    assert w8 > 0 and (w32 - w16) == 2 * (w16 - w8) // 1 and (w16 - w8) > 0
    per_row = (w16 - w8) / 8192
    kv_row = 4 * 128 * (2 + 2 + 4 + 4) + 64 * 8      # K, V (bf16), dK, dV (fp32), RoPE table
    assert per_row == kv_row
    # chunk >= T: nothing grows past T
    assert sb.streambp_layer_workspace_bytes(good_layer_cfg(seq_len=100, chunk=10 ** 6)) == \
        sb.streambp_layer_workspace_bytes(good_layer_cfg(seq_len=100, chunk=100))


def test_head_workspace_is_per_chunk():
    a = sb.streambp_lmhead_workspace_bytes(sb.head_cfg(sb.SBP_BF16, 1, 32768, 2048, 3584, 152064))
    b = sb.streambp_lmhead_workspace_bytes(sb.head_cfg(sb.SBP_BF16, 1, 65536, 2048, 3584, 152064))
    # the only term that grows with T is the int32 list of active rows (+ one count per chunk); no T*V or T*d term
    assert 0 < b - a <= 32768 * 4 + 16 * 4 + 512
    # chunk logits fp32 + dz bf16 of the eight chunks (16384 rows) whose weight gradient is added in one pass + gathered h / dh
    # rows + split-K scratch + the (max, sum of exp) pair per row and block of 256 logits
    assert a < 2048 * 152064 * (4 + 8 * 2) + 9 * 2048 * 3584 * 2 + 4 * 2048 * 3584 * 4 + 2048 * (152064 // 256) * 8 + (1 << 20)
    assert a < 32768 * 152064 * 4 / 3        # a third of the full-sequence fp32 logits alone
    mid = sb.streambp_lmhead_workspace_bytes(sb.head_cfg(sb.SBP_BF16, 1, 32768, 2048, 3584, 152064, dw_group_rows=8192))
    assert mid < 32768 * 152064 * 4 / 5      # four chunks per pass: a fifth
    lean = sb.streambp_lmhead_workspace_bytes(sb.head_cfg(sb.SBP_BF16, 1, 32768, 2048, 3584, 152064, dw_group_rows=2048))
    assert lean < 32768 * 152064 * 4 / 9     # with the weight gradient added chunk by chunk: a ninth


def test_weight_gradient_group_rows_only_change_the_workspace():
    # dw_group_rows = 0 is the default (layer: 8192 rows, head: 16384); more rows keep more chunks' GEMM operands alive (at most eight chunks)
    big = dict(dtype=sb.SBP_BF16, hidden=3584, n_q_heads=28, n_kv_heads=4, head_dim=128, mlp_width=18944, chunk=2048, seq_len=32768)
    ws = {r: sb.streambp_layer_workspace_bytes(good_layer_cfg(dw_group_rows=r, **big))
          for r in (0, 1, 2048, 4096, 6144, 8192, 16384, 10 ** 6)}
    assert ws[0] == ws[8192] and ws[1] == ws[2048] and ws[16384] == ws[10 ** 6]
    assert ws[2048] < ws[4096] < ws[6144] < ws[8192] < ws[16384]
    per_chunk = ws[4096] - ws[2048]
    assert ws[8192] - ws[2048] == 3 * per_chunk                     # one copy of the ten operand buffers per further chunk
    assert ws[16384] - ws[2048] == 7 * per_chunk
    assert per_chunk <= 2048 * (3 * 18944 + 7 * 3584) * 2 + 16 * 256
    hw = {r: sb.streambp_lmhead_workspace_bytes(sb.head_cfg(sb.SBP_BF16, 1, 32768, 2048, 3584, 152064, dw_group_rows=r))
          for r in (0, 2048, 4096, 8192, 16384, 10 ** 6)}
    assert hw[0] == hw[16384] == hw[10 ** 6] and hw[2048] < hw[4096] < hw[8192] < hw[16384]
    assert hw[8192] - hw[4096] == 2 * (hw[4096] - hw[2048])         # dz + gathered h rows per further chunk
    assert hw[16384] - hw[8192] == 4 * (hw[4096] - hw[2048])
    assert sb.streambp_layer_workspace_bytes(good_layer_cfg(dw_group_rows=-1)) == 0
    assert sb.streambp_lmhead_workspace_bytes(sb.head_cfg(sb.SBP_F32, 1, 8, 4, 8, 16, dw_group_rows=-5)) == 0


@pytest.mark.parametrize("kw,code", [
    (dict(n_q_heads=4, n_kv_heads=3), -2), (dict(head_dim=15), -2), (dict(chunk=0), -2), (dict(seq_len=0), -2),
    (dict(dtype=7), -3), (dict(head_dim=512), -2),
    (dict(grad_dtype=7), -3), (dict(grad_dtype=sb.SBP_BF16), -3),      # bf16 gradients only next to bf16 weights
])
def test_layer_bad_config_codes(kw, code):
    cfg = good_layer_cfg(**kw)
    assert sb.streambp_layer_workspace_bytes(cfg) == 0
    w = sb.LayerWeights(*[1] * 9)
    g = sb.LayerGrads(*[1] * 9)
    rc = sb.lib().streambp_layer_backward(C.byref(cfg), C.byref(w), 256, 512, 768, C.byref(g), 1024, 1 << 40, None)
    assert rc == code
    assert len(sb.lib().streambp_last_error()) > 0


def test_layer_null_alias_and_workspace_codes():
    cfg = good_layer_cfg()
    L = sb.lib()
    w = sb.LayerWeights(*[256] * 9)
    g = sb.LayerGrads(*[256] * 9)
    need = sb.streambp_layer_workspace_bytes(cfg)
    assert L.streambp_layer_backward(C.byref(cfg), C.byref(w), None, 512, 768, C.byref(g), 1024, need, None) == -1
    assert L.streambp_layer_backward(C.byref(cfg), C.byref(w), 256, 512, 256, C.byref(g), 1024, need, None) == -2
    assert L.streambp_layer_backward(C.byref(cfg), C.byref(w), 256, 512, 768, C.byref(g), 1024, need - 1, None) == -4
    assert L.streambp_layer_backward(C.byref(cfg), C.byref(w), 256, 512, 768, C.byref(g), 1025, need, None) == -4
    w0 = sb.LayerWeights(*([256] * 8 + [None]))
    assert L.streambp_layer_backward(C.byref(cfg), C.byref(w0), 256, 512, 768, C.byref(g), 1024, need, None) == -1


def test_head_and_attn_codes():
    L = sb.lib()
    hc = sb.head_cfg(sb.SBP_F32, 1, 8, 4, 8, 16, objective=5)
    assert sb.streambp_lmhead_workspace_bytes(hc) == 0
    assert sb.streambp_lmhead_workspace_bytes(sb.head_cfg(sb.SBP_F32, 1, 8, 4, 8, 16, grad_dtype=sb.SBP_BF16)) == 0
    assert sb.streambp_lmhead_workspace_bytes(sb.head_cfg(sb.SBP_BF16, 1, 8, 4, 8, 16, grad_dtype=sb.SBP_BF16)) > 0
    hc = sb.head_cfg(sb.SBP_F32, 1, 8, 4, 8, 16, objective=sb.SBP_OBJ_GRPO)
    need = sb.streambp_lmhead_workspace_bytes(hc)
    args = [256] * 4
    assert L.streambp_lmhead_ce_backward(C.byref(hc), 256, 256, 256, None, None, None, 256, 256, 256, 256, 1024, need, None) == -1
    hc = sb.head_cfg(sb.SBP_F32, 3, 8, 4, 8, 16, objective=sb.SBP_OBJ_DPO)
    assert sb.streambp_lmhead_workspace_bytes(hc) == 0
    ac = sb.attn_cfg(sb.SBP_BF16, 8, 3, 128, 0, 64, 0.1)
    assert sb.streambp_attn_workspace_bytes(ac) == 0
    ac = sb.attn_cfg(sb.SBP_BF16, 8, 2, 128, -1, 64, 0.1)
    assert L.streambp_attn_chunk_forward(C.byref(ac), 256, 256, 256, 256, 256, None) == -2
    for bad_scale in (0.0, -0.1, float("nan"), float("inf")):     # the kernels order raw scores: scale must be > 0
        ac = sb.attn_cfg(sb.SBP_BF16, 8, 2, 128, 0, 64, bad_scale)
        assert L.streambp_attn_chunk_forward(C.byref(ac), 256, 256, 256, 256, 256, None) == -2


def test_noalloc_backward_rejects_what_the_builtin_scratch_cannot_hold():
    L = sb.lib()
    ac = sb.attn_cfg(sb.SBP_BF16, 128, 8, 128, 0, 2049, 0.1)      # 2049 x 128 pairs > 262144
    assert L.streambp_attn_chunk_backward_noalloc(C.byref(ac), 256, 256, 256, 256, 256, 256, 256, 256, 256, None) == -4
    assert "built-in scratch" in sb.streambp_last_error()
    ac = sb.attn_cfg(sb.SBP_BF16, 128, 8, 128, 0, 2048, 0.1)      # exactly at the limit: the NULL check is what stops it
    assert L.streambp_attn_chunk_backward_noalloc(C.byref(ac), None, 256, 256, 256, 256, 256, 256, 256, 256, None) == -1


def test_bad_mask_arguments_are_refused():
    ac = sb.attn_cfg(sb.SBP_BF16, 8, 2, 128, 0, 64, 0.1, window=-1)
    assert sb.lib().streambp_attn_chunk_forward(C.byref(ac), 256, 256, 256, 256, 256, None) == -2
    ac = sb.attn_cfg(sb.SBP_BF16, 8, 2, 128, 0, 64, 0.1, kv_first=-3)
    assert sb.lib().streambp_attn_chunk_forward(C.byref(ac), 256, 256, 256, 256, 256, None) == -2
    lc = sb.layer_cfg(sb.SBP_F32, 2, 64, 16, 64, 4, 4, 16, 172, seq_first=[0, 65])
    assert sb.streambp_layer_workspace_bytes(lc) == 0 and "seq_first" in sb.streambp_last_error()
    assert sb.streambp_layer_workspace_bytes(sb.layer_cfg(sb.SBP_F32, 2, 64, 16, 64, 4, 4, 16, 172, window=-2)) == 0
    assert sb.streambp_layer_workspace_bytes(sb.layer_cfg(sb.SBP_F32, 2, 64, 16, 64, 4, 4, 16, 172, window=8, seq_first=[0, 64])) > 0


def test_adapter_mode_validation_and_workspace():
    L = sb.lib()
    big = dict(dtype=sb.SBP_BF16, hidden=3584, n_q_heads=28, n_kv_heads=4, head_dim=128, mlp_width=18944, chunk=2048, seq_len=32768)
    cfg = good_layer_cfg(**big)
    ad = sb.LoraAdapters(32, 2.0, (C.c_void_p * 7)(*[256] * 7), (C.c_void_p * 7)(*[256] * 7))
    need = L.streambp_layer_lora_workspace_bytes(C.byref(cfg), C.byref(ad))
    plain = sb.streambp_layer_workspace_bytes(good_layer_cfg(dw_group_rows=2048, **big))
    p_lin = 3584 * 28 * 128 * 2 + 2 * 3584 * 4 * 128 + 3 * 3584 * 18944
    # one chunk's buffers + one copy of the adapted matrices + the padded adapter operands / accumulators (rank 32: a few % of that)
    assert plain + 2 * p_lin < need < plain + 2 * p_lin * 1.06
    only_qv = sb.LoraAdapters(32, 2.0, (C.c_void_p * 7)(256, None, 256, None, None, None, None), (C.c_void_p * 7)(256, None, 256, None, None, None, None))
    assert L.streambp_layer_lora_workspace_bytes(C.byref(cfg), C.byref(only_qv)) < plain + 2 * (3584 * 3584 + 512 * 3584) * 1.2     # only the adapted matrices are copied
    for bad in (sb.LoraAdapters(0, 1.0, ad.a, ad.b), sb.LoraAdapters(257, 1.0, ad.a, ad.b),
                sb.LoraAdapters(8, float("nan"), ad.a, ad.b),
                sb.LoraAdapters(8, 1.0, (C.c_void_p * 7)(256, *[None] * 6), (C.c_void_p * 7)(*[None] * 7)),     # A without B
                sb.LoraAdapters(8, 1.0, (C.c_void_p * 7)(*[None] * 7), (C.c_void_p * 7)(*[None] * 7))):        # nothing adapted
        assert L.streambp_layer_lora_workspace_bytes(C.byref(cfg), C.byref(bad)) == 0
    w = sb.LayerWeights(*[256] * 9)
    g = sb.LoraGrads((C.c_void_p * 7)(*[256] * 7), (C.c_void_p * 7)(*[256] * 7))
    assert L.streambp_layer_lora_backward(C.byref(cfg), C.byref(w), C.byref(ad), 256, 512, 768, C.byref(g), 1024, need - 1, None) == -4
    g0 = sb.LoraGrads((C.c_void_p * 7)(*[256] * 6, None), (C.c_void_p * 7)(*[256] * 7))
    assert L.streambp_layer_lora_backward(C.byref(cfg), C.byref(w), C.byref(ad), 256, 512, 768, C.byref(g0), 1024, need, None) == -1
    bf = good_layer_cfg(grad_dtype=sb.SBP_BF16, **big)
    assert L.streambp_layer_lora_backward(C.byref(bf), C.byref(w), C.byref(ad), 256, 512, 768, C.byref(g), 1024, need, None) == -3


def test_fast_path_query_names_the_configs_that_leave_the_mfma_kernels():
    big = dict(dtype=sb.SBP_BF16, hidden=3584, n_q_heads=28, n_kv_heads=4, head_dim=128, mlp_width=18944, chunk=2048, seq_len=32768)
    assert sb.streambp_layer_fast_path(good_layer_cfg(**big)) == 1
    assert sb.streambp_layer_fast_path(good_layer_cfg(**dict(big, mlp_width=18944 + 64))) == 1      # ragged last tile: still MFMA
    assert sb.streambp_layer_fast_path(good_layer_cfg(**dict(big, mlp_width=18944 + 32))) == 0
    assert "mlp_width" in sb.streambp_last_error()
    assert sb.streambp_layer_fast_path(good_layer_cfg(**dict(big, head_dim=64, n_q_heads=56, n_kv_heads=8))) == 0
    assert sb.streambp_layer_fast_path(good_layer_cfg()) == 0                       # fp32 storage
    assert sb.streambp_layer_fast_path(good_layer_cfg(chunk=0)) == -2
    assert sb.streambp_lmhead_fast_path(sb.head_cfg(sb.SBP_BF16, 1, 32768, 2048, 3584, 152064)) == 1
    assert sb.streambp_lmhead_fast_path(sb.head_cfg(sb.SBP_BF16, 1, 32768, 2048, 3584, 151936)) == 1   # 593.5 x 256: masked last tile
    assert sb.streambp_lmhead_fast_path(sb.head_cfg(sb.SBP_BF16, 1, 32768, 2048, 3584, 50257)) == 0
    assert "vocab" in sb.streambp_last_error()
    assert sb.streambp_generic_launches() >= 0


def test_attn_tile_pairs_follow_the_causal_count():
    # Sec. 3.2.2: chunked causal attention touches about (1+D)/(2D) of the T x T square.
    T, c = 32768, 2048
    D = T // c
    total = 0
    for i in range(D):
        n, tq, tk = sb.streambp_attn_tile_pairs(i * c, c)
        total += n * tq * tk
    exact = T * (T + 1) // 2
    chunk_dense = (1 + D) * T * T // (2 * D)
    assert exact <= total <= chunk_dense
    assert total <= exact * 1.01                                  # tile skipping is nearly exact
